/* Brute-force radial mask scan -- CPU oracle, TEST INFRASTRUCTURE ONLY.
 *
 * The 4-D token mask of the paper's Sec. 4.2 (formal definition), the attention sink
 * of App. A.1 ("or j = 0"), the flattening M[i*s+k, j*s+l] = M~[i,j,k,l], and the
 * reduction to blocks (a block pair is listed iff any token pair in it is visible),
 * as a plain loop over every (query token, key token) pair.  The sparsity knob (the paper
 * adjusts the mask's sparsity without defining how) is read as a rational width scale
 * c = num/den on frame pairs at distance >= 2: width floor(c*s/2^r), stride ceil(2^r/(c*s)).  No interval arithmetic,
 * no shortcuts: cost is O(n^2).  Shares nothing with the GPU library.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static int64_t pow2_floor(int64_t d) {            /* 2^floor(log2(max(d,1))) */
    if (d < 1) d = 1;
    int64_t b = 1;
    while (2 * b <= d) b *= 2;
    return b;
}

static int visible(int64_t s, int64_t sink_frames, int64_t num, int64_t den,
                   int64_t i, int64_t j, int64_t k, int64_t l) {
    if (j < sink_frames) return 1;                               /* sink */
    int64_t d = i > j ? i - j : j - i;
    int64_t b = pow2_floor(d);
    int64_t a = k > l ? k - l : l - k;
    if (d < 2) num = den = 1;                                    /* the knob leaves d = 0, 1 alone */
    if (b * den <= s * num && (a + 1) * b * den <= s * num) return 1;   /* case 1 */
    int64_t stride = (b * den + s * num - 1) / (s * num);        /* ceil(b/(c*s)) */
    if (d % stride == 0 && k == l) return 1;                     /* case 2 */
    return 0;
}

/* Scans query blocks [qb_begin, qb_end).  bitmap: (qb_end-qb_begin) x nkb bytes, row-major,
 * written 0/1.  Returns the number of visible token pairs among the scanned query rows. */
int64_t radial_mask_scan(int32_t f, int32_t s, int32_t block, int32_t sink_frames,
                         int32_t width_num, int32_t width_den, int32_t extra_tokens,
                         int32_t qb_begin, int32_t qb_end, uint8_t *bitmap) {
    /* extra_tokens text tokens follow the f*s video tokens; they see and are seen by everyone */
    const int64_t nv = (int64_t)f * s;
    const int64_t n = nv + extra_tokens;
    const int64_t nkb = (n + block - 1) / block;
    int64_t total = 0;
    memset(bitmap, 0, (size_t)(qb_end - qb_begin) * (size_t)nkb);
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : total)
    for (int32_t qb = qb_begin; qb < qb_end; ++qb) {
        uint8_t *row = bitmap + (size_t)(qb - qb_begin) * (size_t)nkb;
        int64_t q0 = (int64_t)qb * block, q1 = q0 + block;
        if (q1 > n) q1 = n;
        for (int64_t q = q0; q < q1; ++q) {
            int64_t i = q / s, k = q % s;
            for (int64_t c = 0; c < n; ++c) {
                int64_t j = c / s, l = c % s;
                if (q >= nv || c >= nv || visible(s, sink_frames, width_num, width_den, i, j, k, l)) {
                    row[c / block] = 1;
                    ++total;
                }
            }
        }
    }
    return total;
}

/* Token mask entries M[q, cols[c]] for query rows [q_begin, q_end) and the given key columns:
 * out is (q_end-q_begin) x ncols bytes, row-major, written 0/1.  Same visible() as the scan. */
void radial_token_mask(int32_t f, int32_t s, int32_t sink_frames, int32_t width_num, int32_t width_den,
                       int64_t q_begin, int64_t q_end, int64_t ncols, const int64_t *cols, uint8_t *out) {
    (void)f;
#pragma omp parallel for schedule(static)
    for (int64_t q = q_begin; q < q_end; ++q) {
        uint8_t *row = out + (size_t)(q - q_begin) * (size_t)ncols;
        int64_t i = q / s, k = q % s;
        for (int64_t c = 0; c < ncols; ++c)
            row[c] = (uint8_t)visible(s, sink_frames, width_num, width_den, i, cols[c] / s, k, cols[c] % s);
    }
}
