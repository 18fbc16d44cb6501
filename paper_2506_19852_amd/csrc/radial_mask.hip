// Radial block-mask construction on the GPU (integer kernels) and the radial_mask object.
//
// The token-level rule is the formal definition of Sec. 4.2 of the paper plus the attention
// sink of App. A.1.  For one query frame i and one key frame j it keeps, for the query
// positions k in [klo, khi], the key positions
//     sink (j < sink_frames):              the whole frame,
//     b = 2^floor(log2 max(|i-j|,1)) <= s:  l in [klo-(w-1), khi+(w-1)] clipped to the frame, w = floor(s/b),
//     b > s and |i-j| mod ceil(b/s) == 0:   l in [klo, khi]  (single diagonal k == l),
// so the key blocks touched by a query block are a union of contiguous block ranges, one per
// (query frame in the block, key frame).  Each workgroup ORs those ranges into a bitmap in
// LDS; a count pass, an exclusive scan and a fill pass turn the bitmaps into compressed lists.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "radial_internal.h"

namespace radial {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

namespace {

constexpr int kThreads = 256;
constexpr int kMaxWords = 15 * 1024;  // 60 KiB of LDS bitmap: up to 491 520 key blocks

struct MaskGeom {
  int32_t f, s, block, sink, n, nb;
  int32_t w0, den;  // sparsity knob c = num/den (frame distances >= 2): w0 = floor(s*num/den)
  int64_t s_num;    // s * num
  // banded patterns: device table [f + 1] of spatial half widths per frame distance (-1: none);
  // null for the radial mask
  const int32_t* half_width;
  int32_t nv;  // video tokens f*s; tokens nv .. n-1 are text tokens (dense rows and columns)
};

__device__ inline int32_t pow2_floor(int32_t d) {
  d = d < 1 ? 1 : d;
  return 1 << (31 - __clz(d));
}

// Bitmap of the key blocks listed for query block qb; words[] is LDS, nwords = ceil(nb/32).
__device__ void row_bitmap(const MaskGeom g, int32_t qb, uint32_t* words, int32_t nwords) {
  for (int32_t w = threadIdx.x; w < nwords; w += blockDim.x) words[w] = 0u;
  __syncthreads();
  const int64_t q0 = (int64_t)qb * g.block;
  int64_t q1 = q0 + g.block - 1;
  if (q1 > (int64_t)g.n - 1) q1 = (int64_t)g.n - 1;
  if (q1 >= g.nv) {  // the block holds a text token: it lists every key block
    for (int32_t w = threadIdx.x; w < nwords; w += blockDim.x) {
      const int32_t left = g.nb - w * 32;
      words[w] = left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
    }
    __syncthreads();
    return;
  }
  if (g.nv < g.n) {  // every video row lists the text tokens' key blocks
    for (int32_t kb = g.nv / g.block + threadIdx.x; kb < g.nb; kb += blockDim.x) atomicOr(&words[kb >> 5], 1u << (kb & 31));
  }
  const int32_t i0 = (int32_t)(q0 / g.s), i1 = (int32_t)(q1 / g.s);
  const int64_t npairs = (int64_t)(i1 - i0 + 1) * g.f;
  for (int64_t p = threadIdx.x; p < npairs; p += blockDim.x) {
    const int32_t i = i0 + (int32_t)(p / g.f);
    const int32_t j = (int32_t)(p % g.f);
    const int64_t fi = (int64_t)i * g.s;
    const int32_t klo = (int32_t)((q0 > fi ? q0 : fi) - fi);
    const int64_t fe = fi + g.s - 1;
    const int32_t khi = (int32_t)((q1 < fe ? q1 : fe) - fi);
    const int32_t d = i > j ? i - j : j - i;
    const int32_t b = pow2_floor(d);
    int64_t llo, lhi;
    if (j < g.sink) {
      llo = 0;
      lhi = g.s - 1;
    } else if (g.half_width) {
      const int64_t hw = g.half_width[d];
      if (hw < 0) continue;
      llo = klo - hw;
      if (llo < 0) llo = 0;
      lhi = khi + hw;
      if (lhi > g.s - 1) lhi = g.s - 1;
    } else if (d < 2 || g.w0 / b >= 1) {
      // diagonal of width floor(s/b), or floor(c*s/b) for the scaled distances d >= 2
      const int64_t w = d < 2 ? g.s : (g.w0 / b < g.s ? g.w0 / b : g.s);
      llo = klo - (w - 1);
      if (llo < 0) llo = 0;
      lhi = khi + (w - 1);
      if (lhi > g.s - 1) lhi = g.s - 1;
    } else {
      const int32_t stride = (int32_t)(((int64_t)b * g.den + g.s_num - 1) / g.s_num);
      if (d % stride != 0) continue;
      llo = klo;
      lhi = khi;
    }
    const int64_t t0 = (int64_t)j * g.s + llo, t1 = (int64_t)j * g.s + lhi;
    const int32_t b0 = (int32_t)(t0 / g.block), b1 = (int32_t)(t1 / g.block);
    for (int32_t w = b0 >> 5; w <= (b1 >> 5); ++w) {
      const int32_t lo = w == (b0 >> 5) ? (b0 & 31) : 0;
      const int32_t hi = w == (b1 >> 5) ? (b1 & 31) : 31;
      const uint32_t m = (hi == 31 ? 0xffffffffu : ((1u << (hi + 1)) - 1u)) & ~((1u << lo) - 1u);
      atomicOr(&words[w], m);
    }
  }
  __syncthreads();
}

// Exclusive scan of one value per thread across the workgroup (blockDim.x == kThreads).
__device__ int32_t block_exclusive_scan(int32_t v, int32_t* total) {
  __shared__ int32_t part[kThreads];
  part[threadIdx.x] = v;
  __syncthreads();
  for (int off = 1; off < kThreads; off <<= 1) {
    int32_t add = threadIdx.x >= off ? part[threadIdx.x - off] : 0;
    __syncthreads();
    part[threadIdx.x] += add;
    __syncthreads();
  }
  const int32_t incl = part[threadIdx.x];
  if (total) *total = part[kThreads - 1];
  __syncthreads();
  return incl - v;
}

__global__ void __launch_bounds__(kThreads) mask_count_kernel(MaskGeom g, int32_t nwords, int32_t* counts) {
  extern __shared__ uint32_t words[];
  row_bitmap(g, blockIdx.x, words, nwords);
  int32_t c = 0;
  for (int32_t w = threadIdx.x; w < nwords; w += blockDim.x) c += __popc(words[w]);
  int32_t total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) counts[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kThreads) mask_fill_kernel(MaskGeom g, int32_t nwords, const int32_t* row_ptr,
                                                            int32_t* col_idx) {
  extern __shared__ uint32_t words[];
  row_bitmap(g, blockIdx.x, words, nwords);
  const int32_t per = (nwords + kThreads - 1) / kThreads;
  const int32_t w0 = threadIdx.x * per;
  const int32_t w1 = w0 + per < nwords ? w0 + per : nwords;
  int32_t c = 0;
  for (int32_t w = w0; w < w1; ++w) c += __popc(words[w]);
  int32_t pos = row_ptr[blockIdx.x] + block_exclusive_scan(c, nullptr);
  for (int32_t w = w0; w < w1; ++w) {
    uint32_t m = words[w];
    while (m) {
      const int32_t bit = __ffs(m) - 1;
      m &= m - 1;
      col_idx[pos++] = w * 32 + bit;
    }
  }
}

// In place: counts[0..n) -> exclusive prefix, counts[n] = total (as int32), *total64 = exact total.
__global__ void __launch_bounds__(kThreads) scan_kernel(int32_t* counts, int32_t n, long long* total64) {
  const int32_t per = (n + kThreads - 1) / kThreads;
  const int32_t a = threadIdx.x * per;
  const int32_t b = a + per < n ? a + per : n;
  long long sum = 0;
  for (int32_t i = a; i < b; ++i) sum += counts[i];
  __shared__ long long part[kThreads];
  part[threadIdx.x] = sum;
  __syncthreads();
  if (threadIdx.x == 0) {
    long long run = 0;
    for (int t = 0; t < kThreads; ++t) {
      const long long v = part[t];
      part[t] = run;
      run += v;
    }
    *total64 = run;
    counts[n] = run > 0x7fffffffLL ? 0x7fffffff : (int32_t)run;
  }
  __syncthreads();
  long long run = part[threadIdx.x];
  for (int32_t i = a; i < b; ++i) {
    const int32_t v = counts[i];
    counts[i] = (int32_t)(run > 0x7fffffffLL ? 0x7fffffffLL : run);
    run += v;
  }
}

__global__ void dense_fill_kernel(int32_t nb, int32_t* row_ptr, int32_t* col_idx) {
  const int64_t total = (int64_t)nb * nb;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
    col_idx[i] = (int32_t)(i % nb);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i <= nb; i += (int64_t)gridDim.x * blockDim.x)
    row_ptr[i] = (int32_t)(i * nb);
}

__device__ inline bool row_contains(const int32_t* col_idx, int32_t lo, int32_t hi, int32_t key) {
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo) >> 1);
    const int32_t v = col_idx[mid];
    if (v == key) return true;
    if (v < key) lo = mid + 1; else hi = mid;
  }
  return false;
}

// Transposed lists: workgroup kb looks kb up in every (ascending) row.
__global__ void __launch_bounds__(kThreads) transpose_count_kernel(const int32_t* row_ptr, const int32_t* col_idx,
                                                                  int32_t nb, int32_t* tcounts) {
  const int32_t kb = blockIdx.x;
  int32_t c = 0;
  for (int32_t qb = threadIdx.x; qb < nb; qb += blockDim.x)
    c += row_contains(col_idx, row_ptr[qb], row_ptr[qb + 1], kb) ? 1 : 0;
  int32_t total;
  block_exclusive_scan(c, &total);
  if (threadIdx.x == 0) tcounts[kb] = total;
}

__global__ void __launch_bounds__(kThreads) transpose_fill_kernel(const int32_t* row_ptr, const int32_t* col_idx,
                                                                 int32_t nb, const int32_t* col_ptr, int32_t* row_idx) {
  const int32_t kb = blockIdx.x;
  int32_t pos = col_ptr[kb];
  for (int32_t base = 0; base < nb; base += kThreads) {
    const int32_t qb = base + threadIdx.x;
    const int32_t hit = (qb < nb && row_contains(col_idx, row_ptr[qb], row_ptr[qb + 1], kb)) ? 1 : 0;
    int32_t total;
    const int32_t off = block_exclusive_scan(hit, &total);
    if (hit) row_idx[pos + off] = qb;
    pos += total;
  }
}

// Launch partition: slice[k] = first block r whose weight prefix W(r) = ptr[r] + kItemCost*r
// reaches k/8 of the total (slice[0] = 0, slice[8] = nb): 8 runs of consecutive blocks with
// equal work, one per XCD.  kItemCost stands for the fixed cost of a work item (loading Q,
// storing O) in units of one listed block.
constexpr int kItemCost = 4;
__global__ void slice_kernel(const int32_t* ptr, int32_t nb, int32_t* slice) {
  const int k = threadIdx.x;
  if (k > 8) return;
  const long long total = (long long)ptr[nb] + (long long)kItemCost * nb;
  const long long target = (total * k + 7) / 8;
  int32_t lo = 0, hi = nb;  // smallest r in [0, nb] with W(r) >= target
  while (lo < hi) {
    const int32_t mid = lo + ((hi - lo) >> 1);
    if ((long long)ptr[mid] + (long long)kItemCost * mid >= target) hi = mid; else lo = mid + 1;
  }
  slice[k] = k == 8 ? nb : (k == 0 ? 0 : lo);
}

int check_common(int64_t n_tokens, int32_t block, uint32_t flags) {
  if (block != 64 && block != 128) return fail(RADIAL_EUNSUPPORTED, "block must be 64 or 128 (got %d)", block);
  if (flags & ~(RADIAL_MASK_TRANSPOSE | RADIAL_MASK_TOKEN_EXACT)) return fail(RADIAL_EINVAL, "unknown mask flag bits 0x%x", flags);
  if (n_tokens < 1 || n_tokens >= (int64_t)0x7fffffff - block)
    return fail(RADIAL_EINVAL, "token count %lld outside [1, 2^31 - block)", (long long)n_tokens);
  const int64_t nb = (n_tokens + block - 1) / block;
  if ((nb + 31) / 32 > kMaxWords) return fail(RADIAL_EUNSUPPORTED, "more than %d key blocks", kMaxWords * 32);
  return RADIAL_OK;
}

// Device storage of a mask is three allocations: `meta` (two 64-bit totals and the two launch
// partitions), `ptrs` (row_ptr and, with the transposed lists, col_ptr) and `idx` (col_idx and
// row_idx).  The views d_row_ptr, d_col_ptr, ... point into them at 256-byte aligned offsets.
constexpr int kMetaInts = 32;  // [0..1] total of rows, [2..3] total of columns, [8..16] slice, [20..28] slice_t
inline int64_t aligned_ints(int64_t n) { return (n + 63) & ~(int64_t)63; }

int alloc_meta_and_ptrs(radial_mask* m) {
  const int64_t np = aligned_ints((int64_t)m->n_blocks + 1);
  RADIAL_HIP_TRY(hipMalloc(&m->d_meta, sizeof(int32_t) * kMetaInts));
  RADIAL_HIP_TRY(hipMalloc(&m->d_ptrs, sizeof(int32_t) * np * ((m->flags & RADIAL_MASK_TRANSPOSE) ? 2 : 1)));
  m->d_row_ptr = m->d_ptrs;
  m->d_slice = m->d_meta + 8;
  if (m->flags & RADIAL_MASK_TRANSPOSE) {
    m->d_col_ptr = m->d_ptrs + np;
    m->d_slice_t = m->d_meta + 20;
  }
  return RADIAL_OK;
}

// Needs m->nnz.
int alloc_idx(radial_mask* m) {
  const int64_t ni = aligned_ints(m->nnz > 0 ? m->nnz : 1);
  RADIAL_HIP_TRY(hipMalloc(&m->d_idx, sizeof(int32_t) * ni * ((m->flags & RADIAL_MASK_TRANSPOSE) ? 2 : 1)));
  m->d_col_idx = m->d_idx;
  if (m->flags & RADIAL_MASK_TRANSPOSE) m->d_row_idx = m->d_idx + ni;
  return RADIAL_OK;
}

// Shared tail of the constructors: transposed lists (optional) and launch partitions, then the one
// wait of the call for everything queued on the stream (the partitions come back to the host).
int finish_mask(radial_mask* m, hipStream_t st) {
  const int32_t nb = m->n_blocks;
  int32_t h_meta[kMetaInts];
  slice_kernel<<<1, 64, 0, st>>>(m->d_row_ptr, nb, m->d_slice);
  if (m->flags & RADIAL_MASK_TRANSPOSE) {
    transpose_count_kernel<<<nb, kThreads, 0, st>>>(m->d_row_ptr, m->d_col_idx, nb, m->d_col_ptr);
    scan_kernel<<<1, kThreads, 0, st>>>(m->d_col_ptr, nb, (long long*)(m->d_meta + 2));
    transpose_fill_kernel<<<nb, kThreads, 0, st>>>(m->d_row_ptr, m->d_col_idx, nb, m->d_col_ptr, m->d_row_idx);
    slice_kernel<<<1, 64, 0, st>>>(m->d_col_ptr, nb, m->d_slice_t);
  }
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(h_meta, m->d_meta, sizeof h_meta, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  if (e != hipSuccess) return fail(RADIAL_EHIP, "mask kernels failed: %s", hipGetErrorString(e));
  for (int k = 0; k < 8; ++k) {
    const int32_t len = h_meta[8 + k + 1] - h_meta[8 + k];
    m->max_slice = len > m->max_slice ? len : m->max_slice;
    if (m->flags & RADIAL_MASK_TRANSPOSE) {
      const int32_t len_t = h_meta[20 + k + 1] - h_meta[20 + k];
      m->max_slice_t = len_t > m->max_slice_t ? len_t : m->max_slice_t;
    }
  }
  return RADIAL_OK;
}

}  // namespace
}  // namespace radial

using namespace radial;

extern "C" const char* radial_last_error(void) { return radial::g_err; }

extern "C" void radial_mask_free(radial_mask* m) {
  if (!m) return;
  (void)hipFree(m->d_meta);
  (void)hipFree(m->d_ptrs);
  (void)hipFree(m->d_idx);
  (void)hipFree(m->d_half_width);
  delete m;
}

static int new_mask(int64_t n_tokens, int32_t block, uint32_t flags, radial_mask** out, radial_mask** m) {
  if (!out) return fail(RADIAL_EINVAL, "out is NULL");
  *out = nullptr;
  if (int rc = check_common(n_tokens, block, flags)) return rc;
  radial_mask* mm = new (std::nothrow) radial_mask();
  if (!mm) return fail(RADIAL_ENOMEM, "host allocation failed");
  mm->n_tokens = (int32_t)n_tokens;
  mm->block = block;
  mm->n_blocks = (int32_t)((n_tokens + block - 1) / block);
  mm->flags = flags;
  if (hipGetDevice(&mm->device) != hipSuccess) {
    delete mm;
    return fail(RADIAL_EHIP, "hipGetDevice failed");
  }
  *m = mm;
  return RADIAL_OK;
}

// Lists of a radial mask (m->d_half_width null) or of a banded pattern (table already on the device).
static int build_radial(radial_mask* m, const radial_mask_params* p, hipStream_t st) {
  const int32_t nb = m->n_blocks;
  const int32_t nwords = (nb + 31) / 32;
  const int64_t s_num = (int64_t)p->tokens_per_frame * p->width_num;
  const MaskGeom g{p->frames, p->tokens_per_frame, p->block, p->sink_frames, m->n_tokens, nb,
                   (int32_t)(s_num / p->width_den), p->width_den, s_num, m->d_half_width,
                   (int32_t)((int64_t)p->frames * p->tokens_per_frame)};
  long long total = 0;
  if (int rc = alloc_meta_and_ptrs(m)) return rc;
  mask_count_kernel<<<nb, kThreads, nwords * sizeof(uint32_t), st>>>(g, nwords, m->d_row_ptr);
  scan_kernel<<<1, kThreads, 0, st>>>(m->d_row_ptr, nb, (long long*)m->d_meta);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(&total, m->d_meta, sizeof total, hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);   // the list storage is sized by the count
  if (e != hipSuccess) return fail(RADIAL_EHIP, "mask count failed: %s", hipGetErrorString(e));
  if (total > 0x7fffffffLL) return fail(RADIAL_EUNSUPPORTED, "%lld listed block pairs do not fit int32", total);
  m->nnz = total;
  if (int rc = alloc_idx(m)) return rc;
  mask_fill_kernel<<<nb, kThreads, nwords * sizeof(uint32_t), st>>>(g, nwords, m->d_row_ptr, m->d_col_idx);
  RADIAL_HIP_TRY(hipGetLastError());
  return finish_mask(m, st);
}

extern "C" int radial_mask_build(const radial_mask_params* p, void* hip_stream, radial_mask** out) {
  if (!p) return fail(RADIAL_EINVAL, "params is NULL");
  if (p->frames < 1 || p->tokens_per_frame < 1 || p->sink_frames < 0 || p->extra_tokens < 0)
    return fail(RADIAL_EINVAL, "need frames >= 1, tokens_per_frame >= 1, sink_frames >= 0, extra_tokens >= 0");
  if ((p->flags & RADIAL_MASK_TOKEN_EXACT) && p->tokens_per_frame < 64)
    return fail(RADIAL_EUNSUPPORTED, "RADIAL_MASK_TOKEN_EXACT needs tokens_per_frame >= 64");
  if (p->width_num < 1 || p->width_num > 32767 || p->width_den < 1 || p->width_den > 32767)
    return fail(RADIAL_EINVAL, "width_num and width_den must be in [1, 32767] (1, 1 for the paper's mask)");
  if ((int64_t)p->tokens_per_frame * p->width_num > 0x7fffffffLL)
    return fail(RADIAL_EINVAL, "tokens_per_frame * width_num must be below 2^31");
  radial_mask* m = nullptr;
  if (int rc = new_mask((int64_t)p->frames * p->tokens_per_frame + p->extra_tokens, p->block, p->flags, out, &m)) return rc;
  m->tokens_per_frame = p->tokens_per_frame;
  m->frames = p->frames;
  m->sink_frames = p->sink_frames;
  m->width_num = p->width_num;
  m->width_den = p->width_den;
  const int rc = build_radial(m, p, (hipStream_t)hip_stream);
  if (rc) {
    radial_mask_free(m);
    return rc;
  }
  *out = m;
  return RADIAL_OK;
}

extern "C" int radial_mask_build_banded(int32_t frames, int32_t tokens_per_frame, int32_t block, int32_t sink_frames,
                                        const int32_t* half_width, uint32_t flags, void* hip_stream,
                                        radial_mask** out) {
  if (frames < 1 || tokens_per_frame < 1 || sink_frames < 0)
    return fail(RADIAL_EINVAL, "need frames >= 1, tokens_per_frame >= 1, sink_frames >= 0");
  if (!half_width) return fail(RADIAL_EINVAL, "half_width is NULL");
  if ((flags & RADIAL_MASK_TOKEN_EXACT) && tokens_per_frame < 64)
    return fail(RADIAL_EUNSUPPORTED, "RADIAL_MASK_TOKEN_EXACT needs tokens_per_frame >= 64");
  radial_mask* m = nullptr;
  if (int rc = new_mask((int64_t)frames * tokens_per_frame, block, flags, out, &m)) return rc;
  m->tokens_per_frame = tokens_per_frame;
  m->frames = frames;
  m->sink_frames = sink_frames;
  // device table with one extra entry: the kernels also look up the distance to the frame after
  // the last one (a stage of keys may run past the end of the sequence)
  std::vector<int32_t> table((size_t)frames + 1, -1);
  for (int32_t d = 0; d < frames; ++d) table[d] = half_width[d] < -1 ? -1 : half_width[d];
  const hipStream_t st = (hipStream_t)hip_stream;
  int rc = RADIAL_OK;
  if (hipMalloc(&m->d_half_width, sizeof(int32_t) * table.size()) != hipSuccess ||
      hipMemcpyAsync(m->d_half_width, table.data(), sizeof(int32_t) * table.size(), hipMemcpyHostToDevice, st) != hipSuccess)
    rc = fail(RADIAL_EHIP, "copying the half-width table failed");
  if (!rc) {  // `table` stays alive until build_radial has waited for the stream
    const radial_mask_params p{frames, tokens_per_frame, block, sink_frames, flags, 1, 1, 0};
    rc = build_radial(m, &p, st);
  }
  if (rc) {
    radial_mask_free(m);
    return rc;
  }
  *out = m;
  return RADIAL_OK;
}

static int build_dense(radial_mask* m, hipStream_t st) {
  const int64_t nb = m->n_blocks;
  if (nb * nb > 0x7fffffffLL) return fail(RADIAL_EUNSUPPORTED, "%lld block pairs do not fit int32", (long long)(nb * nb));
  m->nnz = nb * nb;
  if (int rc = alloc_meta_and_ptrs(m)) return rc;
  if (int rc = alloc_idx(m)) return rc;
  dense_fill_kernel<<<1024, kThreads, 0, st>>>((int32_t)nb, m->d_row_ptr, m->d_col_idx);
  RADIAL_HIP_TRY(hipGetLastError());
  return finish_mask(m, st);
}

extern "C" int radial_mask_build_dense(int32_t n_tokens, int32_t block, uint32_t flags, void* hip_stream,
                                       radial_mask** out) {
  if (flags & RADIAL_MASK_TOKEN_EXACT) return fail(RADIAL_EINVAL, "RADIAL_MASK_TOKEN_EXACT applies to radial_mask_build only");
  radial_mask* m = nullptr;
  if (int rc = new_mask(n_tokens, block, flags, out, &m)) return rc;
  const int rc = build_dense(m, (hipStream_t)hip_stream);
  if (rc) {
    radial_mask_free(m);
    return rc;
  }
  *out = m;
  return RADIAL_OK;
}

static int build_from_csr(radial_mask* m, const int32_t* row_ptr, const int32_t* col_idx, hipStream_t st) {
  const int32_t nb = m->n_blocks;
  if (row_ptr[0] != 0) return fail(RADIAL_EINVAL, "row_ptr[0] must be 0");
  for (int32_t r = 0; r < nb; ++r) {
    if (row_ptr[r + 1] < row_ptr[r]) return fail(RADIAL_EINVAL, "row_ptr decreases at row %d", r);
    for (int32_t e = row_ptr[r]; e < row_ptr[r + 1]; ++e) {
      if (col_idx[e] < 0 || col_idx[e] >= nb) return fail(RADIAL_EINVAL, "row %d: key block %d out of range", r, col_idx[e]);
      if (e > row_ptr[r] && col_idx[e] <= col_idx[e - 1]) return fail(RADIAL_EINVAL, "row %d is not strictly ascending", r);
    }
  }
  m->nnz = row_ptr[nb];
  if (int rc = alloc_meta_and_ptrs(m)) return rc;
  if (int rc = alloc_idx(m)) return rc;
  // the caller's arrays are read until finish_mask has waited for the stream
  RADIAL_HIP_TRY(hipMemcpyAsync(m->d_row_ptr, row_ptr, sizeof(int32_t) * (nb + 1), hipMemcpyHostToDevice, st));
  if (m->nnz > 0)
    RADIAL_HIP_TRY(hipMemcpyAsync(m->d_col_idx, col_idx, sizeof(int32_t) * m->nnz, hipMemcpyHostToDevice, st));
  return finish_mask(m, st);
}

extern "C" int radial_mask_from_csr(int32_t n_tokens, int32_t block, uint32_t flags, const int32_t* row_ptr,
                                    const int32_t* col_idx, void* hip_stream, radial_mask** out) {
  if (!row_ptr) return fail(RADIAL_EINVAL, "row_ptr is NULL");
  if (flags & RADIAL_MASK_TOKEN_EXACT) return fail(RADIAL_EINVAL, "RADIAL_MASK_TOKEN_EXACT applies to radial_mask_build only");
  radial_mask* m = nullptr;
  if (int rc = new_mask(n_tokens, block, flags, out, &m)) return rc;
  int rc = RADIAL_OK;
  if (!col_idx && row_ptr[m->n_blocks] != 0) rc = fail(RADIAL_EINVAL, "col_idx is NULL");
  if (!rc) rc = build_from_csr(m, row_ptr, col_idx, (hipStream_t)hip_stream);
  if (rc) {
    radial_mask_free(m);
    return rc;
  }
  *out = m;
  return RADIAL_OK;
}

extern "C" int radial_mask_info(const radial_mask* m, int32_t* n_tokens, int32_t* block, int32_t* n_blocks,
                                int64_t* nnz, uint32_t* flags) {
  if (!m) return fail(RADIAL_EINVAL, "mask is NULL");
  if (n_tokens) *n_tokens = m->n_tokens;
  if (block) *block = m->block;
  if (n_blocks) *n_blocks = m->n_blocks;
  if (nnz) *nnz = m->nnz;
  if (flags) *flags = m->flags;
  return RADIAL_OK;
}

extern "C" int radial_mask_copy_to_host(const radial_mask* m, int32_t* row_ptr, int32_t* col_idx) {
  if (!m) return fail(RADIAL_EINVAL, "mask is NULL");
  if (row_ptr) RADIAL_HIP_TRY(hipMemcpy(row_ptr, m->d_row_ptr, sizeof(int32_t) * (m->n_blocks + 1), hipMemcpyDeviceToHost));
  if (col_idx && m->nnz > 0) RADIAL_HIP_TRY(hipMemcpy(col_idx, m->d_col_idx, sizeof(int32_t) * m->nnz, hipMemcpyDeviceToHost));
  return RADIAL_OK;
}

extern "C" int radial_mask_copy_transpose_to_host(const radial_mask* m, int32_t* col_ptr, int32_t* row_idx) {
  if (!m) return fail(RADIAL_EINVAL, "mask is NULL");
  if (!(m->flags & RADIAL_MASK_TRANSPOSE)) return fail(RADIAL_ESHAPE, "mask was built without RADIAL_MASK_TRANSPOSE");
  if (col_ptr) RADIAL_HIP_TRY(hipMemcpy(col_ptr, m->d_col_ptr, sizeof(int32_t) * (m->n_blocks + 1), hipMemcpyDeviceToHost));
  if (row_idx && m->nnz > 0) RADIAL_HIP_TRY(hipMemcpy(row_idx, m->d_row_idx, sizeof(int32_t) * m->nnz, hipMemcpyDeviceToHost));
  return RADIAL_OK;
}
