/* Drives oracle/mask_scan.c over a list of shapes under AddressSanitizer / UBSan (CPU only).
 * Input lines on stdin: f s block sink num den extra qb_begin qb_end ; output: one total per line,
 * followed by a checksum of the bitmap, then (token mask of the first min(n, 40) rows x all columns) its sum. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int64_t radial_mask_scan(int32_t f, int32_t s, int32_t block, int32_t sink_frames, int32_t width_num, int32_t width_den,
                         int32_t extra_tokens, int32_t qb_begin, int32_t qb_end, uint8_t* bitmap);
void radial_token_mask(int32_t f, int32_t s, int32_t sink_frames, int32_t width_num, int32_t width_den, int64_t q_begin,
                       int64_t q_end, int64_t ncols, const int64_t* cols, uint8_t* out);

int main(void) {
  int f, s, block, sink, num, den, extra, qb0, qb1;
  while (scanf("%d %d %d %d %d %d %d %d %d", &f, &s, &block, &sink, &num, &den, &extra, &qb0, &qb1) == 9) {
    const int64_t n = (int64_t)f * s + extra, nkb = (n + block - 1) / block;
    /* exact-size heap buffers, so that any access past either end is caught */
    uint8_t* bitmap = (uint8_t*)malloc((size_t)(qb1 - qb0) * (size_t)nkb);
    const int64_t total = radial_mask_scan(f, s, block, sink, num, den, extra, qb0, qb1, bitmap);
    uint64_t sum = 0;
    for (int64_t i = 0; i < (int64_t)(qb1 - qb0) * nkb; ++i) sum = sum * 31 + bitmap[i];
    free(bitmap);
    const int64_t nv = (int64_t)f * s, rows = nv < 40 ? nv : 40;
    int64_t* cols = (int64_t*)malloc(sizeof(int64_t) * (size_t)nv);
    for (int64_t c = 0; c < nv; ++c) cols[c] = c;
    uint8_t* tm = (uint8_t*)malloc((size_t)rows * (size_t)nv);
    radial_token_mask(f, s, sink, num, den, nv - rows, nv, nv, cols, tm);
    int64_t tsum = 0;
    for (int64_t i = 0; i < rows * nv; ++i) tsum += tm[i];
    free(tm);
    free(cols);
    printf("%lld %llu %lld\n", (long long)total, (unsigned long long)sum, (long long)tsum);
  }
  return 0;
}
