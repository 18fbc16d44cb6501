/* A plain C caller of libradial that does GPU work: no Python, no torch.
 *
 *   abi_forward <fixture file>
 *
 * Fills q, k, v on the host from a seeded generator, hipMallocs device copies, builds the radial
 * mask (Sec. 4.2 of the paper, blocks, sink of App. A.1) with radial_mask_build, runs
 * radial_attn_fwd (Eq. 2), copies the result back and compares the block lists (bit for bit)
 * and a few output rows and their log-sum-exp (|err| <= 1e-2 + 1e-2 |ref|) with the values the
 * CPU oracle wrote into the fixture file.  Exit status 0 = all checks passed. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "radial.h"

#define HIP_TRY(x)                                                                       \
  do {                                                                                   \
    hipError_t e_ = (x);                                                                 \
    if (e_ != hipSuccess) {                                                              \
      fprintf(stderr, "%s failed: %s (line %d)\n", #x, hipGetErrorString(e_), __LINE__); \
      return 2;                                                                          \
    }                                                                                    \
  } while (0)
#define RADIAL_TRY(x)                                                                     \
  do {                                                                                    \
    int rc_ = (x);                                                                        \
    if (rc_ != RADIAL_OK) {                                                               \
      fprintf(stderr, "%s returned %d: %s (line %d)\n", #x, rc_, radial_last_error(), __LINE__); \
      return 3;                                                                           \
    }                                                                                     \
  } while (0)

/* value in {-128..127}/64 (exact in bf16), from state' = state * 6364136223846793005 + 1442695040888963407 */
static uint16_t next_bf16(uint64_t* state) {
  *state = *state * 6364136223846793005ull + 1442695040888963407ull;
  const float x = (float)((int)((*state >> 40) & 0xFF) - 128) / 64.0f;
  uint32_t bits;
  memcpy(&bits, &x, 4);
  return (uint16_t)(bits >> 16); /* exact: the value has at most 8 significant bits */
}

static float bf16_to_float(uint16_t h) {
  const uint32_t bits = (uint32_t)h << 16;
  float x;
  memcpy(&x, &bits, 4);
  return x;
}

int main(int argc, char** argv) {
  if (argc != 2) {
    fprintf(stderr, "usage: %s <fixture file>\n", argv[0]);
    return 1;
  }
  FILE* fx = fopen(argv[1], "r");
  if (!fx) {
    perror(argv[1]);
    return 1;
  }
  static char line[1 << 17];
  int f = 0, s = 0, block = 0, D = 0, B = 0, H = 0, sink = 0, n_rows = 0;
  long long seed = 0, nnz = 0;
  int32_t* want_ptr = NULL;
  int32_t* want_idx = NULL;
  int n_blocks = 0;
  /* header */
  while (fgets(line, sizeof line, fx)) {
    if (line[0] == '#') continue;
    if (sscanf(line, "shape %d %d %d %d %d %d %d", &f, &s, &block, &D, &B, &H, &sink) == 7) continue;
    if (sscanf(line, "seed %lld", &seed) == 1) continue;
    if (sscanf(line, "nnz %lld", &nnz) == 1) continue;
    if (!strncmp(line, "row_ptr ", 8) || !strncmp(line, "col_idx ", 8)) {
      const int is_ptr = line[0] == 'r';
      const long long count = is_ptr ? ((long long)f * s + block - 1) / block + 1 : nnz;
      int32_t* dst = (int32_t*)malloc(sizeof(int32_t) * (size_t)count);
      char* p = line + 8;
      for (long long i = 0; i < count; ++i) dst[i] = (int32_t)strtol(p, &p, 10);
      if (is_ptr) {
        want_ptr = dst;
        n_blocks = (int)count - 1;
      } else {
        want_idx = dst;
      }
      continue;
    }
    if (sscanf(line, "rows %d", &n_rows) == 1) break;
  }
  if (!f || !want_ptr || !want_idx || !n_rows) {
    fprintf(stderr, "fixture header incomplete\n");
    return 1;
  }
  const int N = f * s;
  const size_t elems = (size_t)B * H * N * D;
  printf("abi_forward: f=%d s=%d block=%d D=%d B=%d H=%d sink=%d N=%d\n", f, s, block, D, B, H, sink, N);
  fflush(stdout);

  /* inputs */
  uint16_t* host[3];
  void* dev[4];
  for (int t = 0; t < 3; ++t) {
    host[t] = (uint16_t*)malloc(elems * 2);
    uint64_t state = (uint64_t)seed + (uint64_t)(t + 1);
    for (size_t i = 0; i < elems; ++i) host[t][i] = next_bf16(&state);
    HIP_TRY(hipMalloc(&dev[t], elems * 2));
    HIP_TRY(hipMemcpy(dev[t], host[t], elems * 2, hipMemcpyHostToDevice));
  }
  HIP_TRY(hipMalloc(&dev[3], elems * 2));
  float* d_lse = NULL;
  HIP_TRY(hipMalloc((void**)&d_lse, sizeof(float) * (size_t)B * H * N));

  /* mask: lists must equal the oracle's */
  radial_mask_params prm;
  memset(&prm, 0, sizeof prm);
  prm.frames = f; prm.tokens_per_frame = s; prm.block = block; prm.sink_frames = sink;
  prm.width_num = 1; prm.width_den = 1;
  radial_mask* mask = NULL;
  RADIAL_TRY(radial_mask_build(&prm, NULL, &mask));
  int32_t got_n = 0, got_block = 0, got_nb = 0;
  int64_t got_nnz = 0;
  RADIAL_TRY(radial_mask_info(mask, &got_n, &got_block, &got_nb, &got_nnz, NULL));
  if (got_n != N || got_block != block || got_nb != n_blocks || got_nnz != nnz) {
    fprintf(stderr, "mask info mismatch: N %d blocks %d nnz %lld, expected %d %d %lld\n", got_n, got_nb, (long long)got_nnz, N,
            n_blocks, nnz);
    return 4;
  }
  int32_t* got_ptr = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_blocks + 1));
  int32_t* got_idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)nnz);
  RADIAL_TRY(radial_mask_copy_to_host(mask, got_ptr, got_idx));
  if (memcmp(got_ptr, want_ptr, sizeof(int32_t) * (size_t)(n_blocks + 1)) || memcmp(got_idx, want_idx, sizeof(int32_t) * (size_t)nnz)) {
    fprintf(stderr, "block lists differ from the oracle's\n");
    return 4;
  }
  printf("abi_forward: %lld listed block pairs, lists bit-exact\n", nnz);
  fflush(stdout);

  /* forward */
  radial_tensor t[4];
  for (int i = 0; i < 4; ++i) {
    t[i].ptr = dev[i];
    t[i].stride_b = (int64_t)H * N * D;
    t[i].stride_h = (int64_t)N * D;
    t[i].stride_n = D;
  }
  RADIAL_TRY(radial_attn_fwd(B, H, N, D, t[0], t[1], t[2], t[3], d_lse, mask, 1.0f / sqrtf((float)D), NULL));
  HIP_TRY(hipDeviceSynchronize());
  uint16_t* out = (uint16_t*)malloc(elems * 2);
  float* lse = (float*)malloc(sizeof(float) * (size_t)B * H * N);
  HIP_TRY(hipMemcpy(out, dev[3], elems * 2, hipMemcpyDeviceToHost));
  HIP_TRY(hipMemcpy(lse, d_lse, sizeof(float) * (size_t)B * H * N, hipMemcpyDeviceToHost));

  /* rows against the fixture */
  double worst = 0.0;
  int checked = 0, bad = 0;
  while (fgets(line, sizeof line, fx)) {
    if (line[0] == '#' || line[0] == '\n') continue;
    char* p = line;
    const int b = (int)strtol(p, &p, 10), h = (int)strtol(p, &p, 10), r = (int)strtol(p, &p, 10);
    const double want_lse = strtod(p, &p);
    const size_t row = ((size_t)b * H + h) * N + r;
    if (fabs((double)lse[row] - want_lse) > 1e-4 + 1e-4 * fabs(want_lse)) {
      fprintf(stderr, "lse b%d h%d row %d: got %.7g want %.7g\n", b, h, r, lse[row], want_lse);
      ++bad;
    }
    for (int d = 0; d < D; ++d) {
      const double want = strtod(p, &p);
      const double got = bf16_to_float(out[row * D + d]);
      const double err = fabs(got - want);
      if (err > worst) worst = err;
      if (!(err <= 1e-2 + 1e-2 * fabs(want))) {
        if (bad < 10) fprintf(stderr, "out b%d h%d row %d d %d: got %.7g want %.7g\n", b, h, r, d, got, want);
        ++bad;
      }
    }
    ++checked;
  }
  fclose(fx);
  printf("abi_forward: %d rows checked, max |err| %.3e, %d values outside the tolerance\n", checked, worst, bad);
  radial_mask_free(mask);
  for (int i = 0; i < 4; ++i) HIP_TRY(hipFree(dev[i]));
  HIP_TRY(hipFree(d_lse));
  if (checked != n_rows) {
    fprintf(stderr, "fixture announced %d rows, %d read\n", n_rows, checked);
    return 5;
  }
  return bad ? 6 : 0;
}
