// Per-tensor scaling kernels: abs-max, scale, FP8 cast (optionally fused with a transpose).
//
// What they compute (Appendix E of the paper): rho = FP8MaxValue / (2^m max H) and
// FP8cast(rho X); Section 2 calls the two-pass flow (abs-max, then cast) just-in-time scaling
// and the one-pass flow (cast with last iteration's scale, abs-max as a by-product) delayed
// scaling.  All of these are HBM-bound: every element is read once with 16-byte loads and
// every output byte is written once with 8- or 16-byte stores.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

__global__ void zero_u32_kernel(uint32_t* p) { *p = 0u; }

// ---------------------------------------------------------------- abs-max
// bf16 magnitudes order like unsigned 16-bit integers, so the running maximum is a packed
// u16 max over the sign-cleared bit patterns; the result is the float whose upper half is it.
//
// PARTIALS: the form used by the one-call just-in-time flow.  Every workgroup stores its maximum in
// its own word of the caller's workspace (no atomics, no zero-initialisation, no fence); a
// one-workgroup kernel then reduces the words and derives the scale.  This form reads with ordinary
// (cache-retaining) loads, because the cast pass re-reads the tensor right away, back to front.
FOG_DEVICE void scale_from_amax(float a, int fmt, int margin, float* scale, float* scale_inv);
FOG_DEVICE void publish_block_max(uint32_t r, uint32_t* out, bool partials, int bid) {
  if (partials) {
    out[bid] = r << 16;
    return;
  }
  // same-address atomics are served one at a time: skip the ones that cannot raise the maximum
  if (r && (r << 16) > __hip_atomic_load(out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(out, r << 16);
}

// Workgroup `bid` of `nb` over one contiguous tensor (a whole launch, or one job's share of a batched launch).
template <bool PARTIALS>
FOG_DEVICE void amax_span(const uint4* __restrict__ x, int64_t nvec, const uint16_t* __restrict__ tail, int ntail,
                          uint32_t* __restrict__ out, int bid, int nb) {
  // Every workgroup owns one contiguous span and walks it in batches of eight 16-byte loads per
  // thread; the next batch is requested before the current one is reduced, so loads never stop.
  constexpr int NL = 8;
  const int64_t per = (nvec + nb - 1) / nb;
  const int64_t b0 = per * bid, b1 = b0 + per < nvec ? b0 + per : nvec;
  uint32_t m[4] = {0, 0, 0, 0};
  int64_t i = b0 + threadIdx.x;
  uint4 v[NL];
  bool have = i + (NL - 1) * kThreads < b1;
  if (have) {
#pragma unroll
    for (int k = 0; k < NL; ++k) v[k] = PARTIALS ? x[i + k * kThreads] : ld_nt16(x + i + k * kThreads);
  }
  while (have) {
    const int64_t n = i + NL * kThreads;
    const bool more = n + (NL - 1) * kThreads < b1;
    uint4 nx[NL];
    if (more) {
#pragma unroll
      for (int k = 0; k < NL; ++k) nx[k] = PARTIALS ? x[n + k * kThreads] : ld_nt16(x + n + k * kThreads);
    }
#pragma unroll
    for (int k = 0; k < NL; ++k) {
      m[0] = pkmax_abs_bf16(m[0], v[k].x); m[1] = pkmax_abs_bf16(m[1], v[k].y);
      m[2] = pkmax_abs_bf16(m[2], v[k].z); m[3] = pkmax_abs_bf16(m[3], v[k].w);
    }
    if (more) {
#pragma unroll
      for (int k = 0; k < NL; ++k) v[k] = nx[k];
    }
    i = n;
    have = more;
  }
  for (; i < b1; i += kThreads) {
    uint4 a = ld_nt16(x + i);
    m[0] = pkmax_abs_bf16(m[0], a.x); m[1] = pkmax_abs_bf16(m[1], a.y);
    m[2] = pkmax_abs_bf16(m[2], a.z); m[3] = pkmax_abs_bf16(m[3], a.w);
  }
  uint32_t mm = pkmax_abs_bf16(pkmax_abs_bf16(m[0], m[1]), pkmax_abs_bf16(m[2], m[3]));
  uint32_t h = (mm >> 16) > (mm & 0xFFFFu) ? (mm >> 16) : (mm & 0xFFFFu);
  if (bid == 0 && (int)threadIdx.x < ntail) {
    uint32_t t = tail[threadIdx.x] & 0x7FFFu;
    h = h > t ? h : t;
  }
  h = wave_max_u32(h);
  __shared__ uint32_t part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = h;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = part[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = r > part[w] ? r : part[w];
    publish_block_max(r, out, PARTIALS, bid);
  }
}

template <bool PARTIALS>
__global__ __launch_bounds__(kThreads) void amax_kernel(const uint4* __restrict__ x, int64_t nvec,
                                                        const uint16_t* __restrict__ tail, int ntail,
                                                        uint32_t* __restrict__ out) {
  amax_span<PARTIALS>(x, nvec, tail, ntail, out, (int)blockIdx.x, (int)gridDim.x);
}

// Abs-max of a matrix whose rows are not contiguous or not 16-byte aligned (slow, same result).
template <bool PARTIALS>
__global__ __launch_bounds__(kThreads) void amax_strided_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                                int64_t ldx, uint32_t* __restrict__ out) {
  const int64_t total = rows * cols;
  uint32_t m = 0;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / cols, c = i - r * cols;
    const uint32_t a = x[r * ldx + c] & 0x7FFFu;
    m = m > a ? m : a;
  }
  m = wave_max_u32(m);
  __shared__ uint32_t part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = part[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = r > part[w] ? r : part[w];
    publish_block_max(r, out, PARTIALS, (int)blockIdx.x);
  }
}

// ---------------------------------------------------------------- scale
FOG_DEVICE void scale_from_amax(float a, int fmt, int margin, float* scale, float* scale_inv) {
  const float fmax = fmt == FOG_E4M3 ? 448.0f : 57344.0f;
  float rho = 1.0f;
  if (a > 0.0f && a <= 3.402823466e38f) {
    float denom = ldexpf(a, margin);
    rho = fmax / denom;  // correctly rounded binary32 division
    if (rho > 3.402823466e38f) rho = 3.402823466e38f;
    if (!(rho > 0.0f)) rho = 1.0f;
  }
  *scale = rho;
  if (scale_inv) *scale_inv = 1.0f / rho;
}

__global__ void scale_kernel(const float* amax, int fmt, int margin, float* scale, float* scale_inv) {
  scale_from_amax(*amax, fmt, margin, scale, scale_inv);
}

// One workgroup: maximum of the per-workgroup maxima of the abs-max pass, then the scale.
__global__ __launch_bounds__(kThreads) void scale_partials_kernel(const uint32_t* __restrict__ part, int n, int fmt, int margin,
                                                                 float* amax, float* scale, float* scale_inv) {
  uint32_t m = 0;
  for (int i = threadIdx.x; i < n; i += kThreads) m = m > part[i] ? m : part[i];   // non-negative floats order like their bits
  m = wave_max_u32(m);
  __shared__ uint32_t wmax[kThreads / 64];
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = wmax[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = r > wmax[w] ? r : wmax[w];
    const float a = __uint_as_float(r);
    *amax = a;
    scale_from_amax(a, fmt, margin, scale, scale_inv);
  }
}

// The same reduction inside a cast kernel: under just-in-time scaling every workgroup of the cast pass
// derives the scale itself from the per-workgroup maxima of the abs-max pass (at most 4 KB, served from
// L2), so no launch sits between the two passes; workgroup 0 publishes abs-max, scale and 1/scale.
// Under delayed scaling in one launch (fog_quantize_delayed) the maxima are those the PREVIOUS cast of
// this tensor left behind: their maximum enters the abs-max history (a ring: entry `slot` is replaced,
// every workgroup takes the maximum over the other entries and the new value, workgroup 0 stores it),
// the scale comes from the history's maximum, and this pass's own maxima go to `cur`, 1024 words that
// the previous pass cleared; workgroup 0 clears `next` for the pass after this one.  Three buffers in
// rotation: no word is read and written by different workgroups of one launch.
struct ScaleSource {
  const uint32_t* part;   // NULL: the scale is read from memory instead
  int n, fmt, margin;
  float* amax;
  float* scale;
  float* scale_inv;
  float* hist;            // delayed scaling only (else NULL): the history, hlen entries, entry `slot` is replaced
  int hlen, slot;
  uint32_t* cur;          // delayed scaling only: where this pass's workgroup maxima are raised (atomic max)
  uint32_t* next;         // delayed scaling only: cleared by workgroup 0
};
constexpr int kDelayedSlots = 1024;
FOG_DEVICE float scale_from_partials(const ScaleSource& js, bool publisher) {
  uint32_t m = 0;
  for (int i = threadIdx.x; i < js.n; i += kThreads) m = m > js.part[i] ? m : js.part[i];
  uint32_t h = 0;   // maximum of the history entries that stay
  if (js.hist) {
    for (int i = threadIdx.x; i < js.hlen; i += kThreads) {
      const uint32_t v = i == js.slot ? 0u : __float_as_uint(js.hist[i]);   // abs-maxes: non-negative floats order like their bits
      h = h > v ? h : v;
    }
    if (publisher)
      for (int i = threadIdx.x; i < kDelayedSlots; i += kThreads) js.next[i] = 0u;
  }
  m = wave_max_u32(m);
  h = wave_max_u32(h);
  __shared__ uint32_t wmax[kThreads / 64], hmax[kThreads / 64];
  __shared__ float rho_shared;
  if ((threadIdx.x & 63) == 0) {
    wmax[threadIdx.x >> 6] = m;
    hmax[threadIdx.x >> 6] = h;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = wmax[0], rh = hmax[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) {
      r = r > wmax[w] ? r : wmax[w];
      rh = rh > hmax[w] ? rh : hmax[w];
    }
    const float a = __uint_as_float(r);                       // abs-max of the tensor the maxima belong to
    const float basis = __uint_as_float(r > rh ? r : rh);     // what the scale is derived from
    float sc, si;
    scale_from_amax(basis, js.fmt, js.margin, &sc, &si);
    rho_shared = sc;
    if (publisher) {
      if (js.amax) *js.amax = a;
      if (js.hist) js.hist[js.slot] = a;
      *js.scale = sc;
      if (js.scale_inv) *js.scale_inv = si;
    }
  }
  __syncthreads();
  return rho_shared;
}

// One workgroup of the above without a cast (empty tensors), and the maximum of one buffer of maxima.
__global__ __launch_bounds__(kThreads) void delayed_scale_only_kernel(ScaleSource js) { scale_from_partials(js, true); }
__global__ __launch_bounds__(kThreads) void partials_max_kernel(const uint32_t* __restrict__ part, int n, float* __restrict__ amax) {
  uint32_t m = 0;
  for (int i = threadIdx.x; i < n; i += kThreads) m = m > part[i] ? m : part[i];
  m = wave_max_u32(m);
  __shared__ uint32_t wmax[kThreads / 64];
  if ((threadIdx.x & 63) == 0) wmax[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = wmax[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = r > wmax[w] ? r : wmax[w];
    *amax = __uint_as_float(r);
  }
}

// One workgroup: roll the history by one (newest first), then scale from its maximum.
__global__ __launch_bounds__(kThreads) void scale_delayed_kernel(float* hist, int len, const float* new_amax, int fmt,
                                                                int margin, float* scale, float* scale_inv) {
  __shared__ float part[kThreads / 64];
  const float na = *new_amax;
  float m = 0.0f;
  // Walk the history from the back in blocks so that every element is read before it is overwritten.
  for (int base = ((len - 1) / kThreads) * kThreads; base >= 0; base -= kThreads) {
    int i = base + threadIdx.x;
    float v = 0.0f;
    bool in = i < len;
    if (in) v = i == 0 ? na : hist[i - 1];
    __syncthreads();
    if (in) hist[i] = v;
    m = fmaxf(m, v);
    __syncthreads();
  }
  m = wave_max_f32(m);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = part[0];
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, part[w]);
    scale_from_amax(r, fmt, margin, scale, scale_inv);
  }
}

// ---------------------------------------------------------------- cast, row-major output only
template <int FMT>
FOG_DEVICE uint2 cast8(uint4 v, float rho) {
  uint2 o;
  o.x = cvt4_fp8_nan<FMT>(bf16lo(v.x) * rho, bf16hi(v.x) * rho, bf16lo(v.y) * rho, bf16hi(v.y) * rho);
  o.y = cvt4_fp8_nan<FMT>(bf16lo(v.z) * rho, bf16hi(v.z) * rho, bf16lo(v.w) * rho, bf16hi(v.w) * rho);
  return o;
}

// Each thread turns 16 bf16 (two 16-byte loads) into 16 FP8 codes (one 16-byte store), two such
// chunks per trip so that four loads are in flight.
// Workgroup `bid` of `nb` over one tensor (a whole launch, or one job's share of a batched launch).
template <int FMT, bool AMAX>
FOG_DEVICE void quantize_rows_body(const uint16_t* __restrict__ x, int64_t rows, int64_t chunks_per_row, int64_t ldx,
                                   const float* __restrict__ scale, uint8_t* __restrict__ q, int64_t ldq,
                                   uint32_t* __restrict__ amax_out, const ScaleSource& js, int bid, int nb) {
  const float rho = js.part ? scale_from_partials(js, bid == 0) : *scale;
  const int64_t total = rows * chunks_per_row;
  const int64_t stride = (int64_t)nb * kThreads;
  uint32_t m = 0;
  // Chunks are visited back to front: under just-in-time scaling the abs-max pass ran front to back
  // just before, so the END of the tensor is what the caches still hold.
  auto src_of = [&](int64_t i) {
    i = total - 1 - i;
    if (rows == 1) return x + i * 16;
    const int64_t r = i / chunks_per_row, c = i - r * chunks_per_row;
    return x + r * ldx + c * 16;
  };
  auto dst_of = [&](int64_t i) {
    i = total - 1 - i;
    if (rows == 1) return q + i * 16;
    const int64_t r = i / chunks_per_row, c = i - r * chunks_per_row;
    return q + r * ldq + c * 16;
  };
  auto emit = [&](uint4 a, uint4 b, uint8_t* dst) {
    if (AMAX) {
      m = pkmax_abs_bf16(pkmax_abs_bf16(pkmax_abs_bf16(pkmax_abs_bf16(m, a.x), a.y), a.z), a.w);
      m = pkmax_abs_bf16(pkmax_abs_bf16(pkmax_abs_bf16(pkmax_abs_bf16(m, b.x), b.y), b.z), b.w);
    }
    uint2 lo = cast8<FMT>(a, rho), hi = cast8<FMT>(b, rho);
    st_nt16(dst, make_uint4(lo.x, lo.y, hi.x, hi.y));
  };
  int64_t i = (int64_t)bid * kThreads + threadIdx.x;
  for (; i + stride < total; i += 2 * stride) {
    const uint16_t* s0 = src_of(i);
    const uint16_t* s1 = src_of(i + stride);
    uint4 a0 = ld_nt16(s0), b0 = ld_nt16(s0 + 8), a1 = ld_nt16(s1), b1 = ld_nt16(s1 + 8);
    emit(a0, b0, dst_of(i));
    emit(a1, b1, dst_of(i + stride));
  }
  if (i < total) {
    const uint16_t* s0 = src_of(i);
    emit(ld_nt16(s0), ld_nt16(s0 + 8), dst_of(i));
  }
  if (AMAX) {
    uint32_t h = (m >> 16) > (m & 0xFFFFu) ? (m >> 16) : (m & 0xFFFFu);
    h = wave_max_u32(h);
    __shared__ uint32_t part[kThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = h;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t r = part[0];
#pragma unroll
      for (int w = 1; w < kThreads / 64; ++w) r = r > part[w] ? r : part[w];
      if (r) atomicMax(js.cur ? js.cur + (bid & (kDelayedSlots - 1)) : amax_out, r << 16);
    }
  }
}

template <int FMT, bool AMAX>
__global__ __launch_bounds__(kThreads) void quantize_rows_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                 int64_t chunks_per_row, int64_t ldx,
                                                                 const float* __restrict__ scale, uint8_t* __restrict__ q,
                                                                 int64_t ldq, uint32_t* __restrict__ amax_out, ScaleSource js) {
  quantize_rows_body<FMT, AMAX>(x, rows, chunks_per_row, ldx, scale, q, ldq, amax_out, js, (int)blockIdx.x, (int)gridDim.x);
}

// ---------------------------------------------------------------- several tensors per launch (just-in-time scaling)
// A launch costs about 4 us of ramp and tail whatever it does, a fifth of what the abs-max or the cast of a
// 100 MB tensor takes; fog_quantize_jit_batch therefore runs the abs-max pass of up to kBatchMax contiguous
// tensors as ONE launch and their cast pass as another.  Workgroups are dealt to the jobs in proportion to
// their sizes; inside its job a workgroup does exactly what it does in the one-tensor kernels.
constexpr int kBatchMax = FOG_CAST_BATCH_MAX;
struct BatchJobs {
  int count;
  int amax_first[kBatchMax + 1];   // first workgroup of each job in the abs-max launch (prefix sums)
  int cast_first[kBatchMax + 1];   // ... and in the cast launch, where the jobs run in reverse order
  const uint16_t* x[kBatchMax];
  int64_t n[kBatchMax];            // elements, a multiple of 16
  uint8_t* q[kBatchMax];
  int fmt[kBatchMax], margin[kBatchMax];
  float* amax[kBatchMax];
  float* scale[kBatchMax];
  float* scale_inv[kBatchMax];
};
constexpr int kJitSlots = 1024;    // workspace words per job = most workgroups a job gets in the abs-max launch

__global__ __launch_bounds__(kThreads) void amax_batch_kernel(BatchJobs b, uint32_t* __restrict__ ws) {
  int j = 0;
  for (int k = 1; k < b.count; ++k)
    if ((int)blockIdx.x >= b.amax_first[k]) j = k;
  const int nb = b.amax_first[j + 1] - b.amax_first[j];
  amax_span<true>(reinterpret_cast<const uint4*>(b.x[j]), b.n[j] / 8, nullptr, 0, ws + j * kJitSlots, (int)blockIdx.x - b.amax_first[j], nb);
}

__global__ __launch_bounds__(kThreads) void quantize_batch_kernel(BatchJobs b, const uint32_t* __restrict__ ws) {
  // position p in the launch order is job count - 1 - p: the tensor whose abs-max pass ran last is cast first
  int p = 0;
  for (int k = 1; k < b.count; ++k)
    if ((int)blockIdx.x >= b.cast_first[k]) p = k;
  const int j = b.count - 1 - p;
  const int bid = (int)blockIdx.x - b.cast_first[p], nb = b.cast_first[p + 1] - b.cast_first[p];
  const ScaleSource js{ws + j * kJitSlots, b.amax_first[j + 1] - b.amax_first[j], b.fmt[j], b.margin[j], b.amax[j], b.scale[j], b.scale_inv[j],
                    nullptr, 0, 0, nullptr, nullptr};
  const int64_t chunks = b.n[j] / 16;
  if (b.fmt[j] == FOG_E4M3) quantize_rows_body<FOG_E4M3, false>(b.x[j], 1, chunks, chunks * 16, nullptr, b.q[j], chunks * 16, nullptr, js, bid, nb);
  else                      quantize_rows_body<FOG_E5M2, false>(b.x[j], 1, chunks, chunks * 16, nullptr, b.q[j], chunks * 16, nullptr, js, bid, nb);
}

// ---------------------------------------------------------------- several tensors per launch (delayed scaling)
// fog_quantize_delayed for up to kBatchMax contiguous tensors in ONE launch: a workgroup finds its job from the prefix
// sums and does, inside it, exactly what it does in the one-tensor launch (the history update and the scale from the
// previous pass's maxima, the cast, this pass's maxima into the job's own state).
struct DelayedJobs {
  int count;
  int first[kBatchMax + 1];        // first workgroup of each job (prefix sums)
  int prev_off, cur_off, next_off; // word offsets of the three rotating buffers inside a job's state (the same for every job)
  const uint16_t* x[kBatchMax];
  int64_t n[kBatchMax];            // elements, a multiple of 16
  uint8_t* q[kBatchMax];
  int fmt[kBatchMax], margin[kBatchMax];
  float* amax_prev[kBatchMax];
  float* scale[kBatchMax];
  float* scale_inv[kBatchMax];
  float* hist[kBatchMax];
  int hlen[kBatchMax], slot[kBatchMax];
  uint32_t* state[kBatchMax];
};

__global__ __launch_bounds__(kThreads) void quantize_delayed_batch_kernel(DelayedJobs b) {
  int j = 0;
  for (int k = 1; k < b.count; ++k)
    if ((int)blockIdx.x >= b.first[k]) j = k;
  const int bid = (int)blockIdx.x - b.first[j], nb = b.first[j + 1] - b.first[j];
  uint32_t* st = b.state[j];
  const ScaleSource js{st + b.prev_off, kDelayedSlots, b.fmt[j], b.margin[j], b.amax_prev[j], b.scale[j], b.scale_inv[j],
                       b.hist[j], b.hlen[j], b.slot[j], st + b.cur_off, st + b.next_off};
  const int64_t chunks = b.n[j] / 16;
  if (b.fmt[j] == FOG_E4M3) quantize_rows_body<FOG_E4M3, true>(b.x[j], 1, chunks, chunks * 16, nullptr, b.q[j], chunks * 16, st + b.cur_off, js, bid, nb);
  else                      quantize_rows_body<FOG_E5M2, true>(b.x[j], 1, chunks, chunks * 16, nullptr, b.q[j], chunks * 16, st + b.cur_off, js, bid, nb);
}

// ---------------------------------------------------------------- cast fused with transpose
// One workgroup handles a 128 x 128 element tile.  A thread owns units of 4 rows x 8 columns:
// it loads 16 bytes from each of four consecutive rows, casts, stores 8 code bytes per row to q,
// transposes the 4 x 8 code block in registers (byte permutes) and parks the eight resulting
// dwords (4 rows of one column each) in an LDS tile that is column-major; the tile is then
// streamed out to qT in 16-byte pieces.  LDS 16-byte chunks are XOR-swizzled by column group so
// that neither the dword writes nor the 16-byte reads pile onto the same banks.
constexpr int kTile = 128;

FOG_DEVICE void transpose4x4(uint32_t r0, uint32_t r1, uint32_t r2, uint32_t r3, uint32_t* t) {
  uint32_t lo01 = __builtin_amdgcn_perm(r1, r0, 0x05010400u);  // r0.b0 r1.b0 r0.b1 r1.b1
  uint32_t hi01 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);  // r0.b2 r1.b2 r0.b3 r1.b3
  uint32_t lo23 = __builtin_amdgcn_perm(r3, r2, 0x05010400u);
  uint32_t hi23 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
  t[0] = __builtin_amdgcn_perm(lo23, lo01, 0x05040100u);
  t[1] = __builtin_amdgcn_perm(lo23, lo01, 0x07060302u);
  t[2] = __builtin_amdgcn_perm(hi23, hi01, 0x05040100u);
  t[3] = __builtin_amdgcn_perm(hi23, hi01, 0x07060302u);
}

template <int FMT, bool AMAX, bool WRITE_Q>
__global__ __launch_bounds__(kThreads) void quantize_transpose_kernel(const uint16_t* __restrict__ x, int64_t rows,
                                                                      int64_t cols, int64_t ldx,
                                                                      const float* __restrict__ scale,
                                                                      uint8_t* __restrict__ q, int64_t ldq,
                                                                      uint8_t* __restrict__ qT, int64_t ldqT,
                                                                      uint32_t* __restrict__ amax_out, int tiles_c, ScaleSource js) {
  __shared__ __attribute__((aligned(16))) uint8_t tile[kTile * kTile];  // [col][row], chunk-swizzled
  const float rho = js.part ? scale_from_partials(js, blockIdx.x == 0) : *scale;
  const int bid = gridDim.x - 1 - blockIdx.x;   // tiles back to front (see quantize_rows_kernel)
  const int64_t r0 = (int64_t)(bid / tiles_c) * kTile;
  const int64_t c0 = (int64_t)(bid % tiles_c) * kTile;
  uint32_t m = 0;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int u = threadIdx.x + it * kThreads;  // 512 units: 32 row groups x 16 column chunks
    const int cc = u & 15, rg = u >> 4;
    const int64_t r = r0 + rg * 4, c = c0 + cc * 8;
    uint2 code[4];
    const bool in = r < rows && c < cols;  // rows % 4 == 0 and cols % 8 == 0 on this path
    if (in) {
      uint4 v[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) v[k] = ld_nt16(x + (r + k) * ldx + c);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (AMAX) m = pkmax_abs_bf16(pkmax_abs_bf16(pkmax_abs_bf16(pkmax_abs_bf16(m, v[k].x), v[k].y), v[k].z), v[k].w);
        code[k] = cast8<FMT>(v[k], rho);
        if (WRITE_Q) st_nt8(q + (r + k) * ldq + c, code[k]);
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) code[k] = make_uint2(0u, 0u);
    }
    uint32_t t[8];
    transpose4x4(code[0].x, code[1].x, code[2].x, code[3].x, t);
    transpose4x4(code[0].y, code[1].y, code[2].y, code[3].y, t + 4);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int col = cc * 8 + j;
      const int chunk = (rg >> 2) ^ (cc & 7);
      *reinterpret_cast<uint32_t*>(tile + col * kTile + chunk * 16 + (rg & 3) * 4) = t[j];
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int idx = threadIdx.x + it * kThreads;  // 1024 pieces: 128 columns x 8 chunks of 16 rows
    const int col = idx >> 3, ch = idx & 7;
    const int64_t c = c0 + col, r = r0 + ch * 16;
    if (c < cols && r < rows) {  // rows % 16 == 0 on this path
      uint4 v = *reinterpret_cast<const uint4*>(tile + col * kTile + ((ch ^ ((col >> 3) & 7)) * 16));
      st_nt16(qT + c * ldqT + r, v);
    }
  }
  if (AMAX) {
    uint32_t h = (m >> 16) > (m & 0xFFFFu) ? (m >> 16) : (m & 0xFFFFu);
    h = wave_max_u32(h);
    __shared__ uint32_t part[kThreads / 64];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = h;
    __syncthreads();
    if (threadIdx.x == 0) {
      uint32_t r = part[0];
#pragma unroll
      for (int w = 1; w < kThreads / 64; ++w) r = r > part[w] ? r : part[w];
      if (r) atomicMax(js.cur ? js.cur + (blockIdx.x & (kDelayedSlots - 1)) : amax_out, r << 16);
    }
  }
}

// ---------------------------------------------------------------- general shapes (slow, same results)
template <int FMT>
__global__ __launch_bounds__(kThreads) void quantize_general_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols,
                                                                    int64_t ldx, const float* __restrict__ scale,
                                                                    uint8_t* __restrict__ q, int64_t ldq,
                                                                    uint8_t* __restrict__ qT, int64_t ldqT,
                                                                    uint32_t* __restrict__ amax_out, ScaleSource js) {
  const float rho = js.part ? scale_from_partials(js, blockIdx.x == 0) : *scale;
  const int64_t total = rows * cols;
  uint32_t m = 0;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
    int64_t r = i / cols, c = i - r * cols;
    uint32_t w = x[r * ldx + c];
    uint32_t a = w & 0x7FFFu;
    m = m > a ? m : a;
    float t = bf16lo(w) * rho;
    uint8_t code = (uint8_t)(cvt4_fp8_nan<FMT>(t, t, t, t) & 0xFFu);
    if (q) q[r * ldq + c] = code;
    if (qT) qT[c * ldqT + r] = code;
  }
  if (amax_out) {
    m = wave_max_u32(m);
    if ((threadIdx.x & 63) == 0 && m) atomicMax(js.cur ? js.cur + (blockIdx.x & (kDelayedSlots - 1)) : amax_out, m << 16);
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

// ---------------------------------------------------------------- host entry points
extern "C" fog_status fog_amax(const void* x_bf16, int64_t n, float* amax, void* stream) {
  if (!amax || (!x_bf16 && n > 0)) return FOG_ERR_NULL;
  if (n < 0) return FOG_ERR_SHAPE;
  if (n > 0 && !aligned16(x_bf16)) return FOG_ERR_ALIGN;
  hipStream_t s = (hipStream_t)stream;
  zero_u32_kernel<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax));
  if (n > 0) {
    const int64_t nvec = n / 8;
    const int ntail = (int)(n - nvec * 8);
    int64_t blocks = (nvec + kThreads * 8 - 1) / (kThreads * 8);
    if (blocks > 1024) blocks = 1024;   // 4 workgroups per CU; one atomic per workgroup
    if (blocks < 1) blocks = 1;
    amax_kernel<false><<<(int)blocks, kThreads, 0, s>>>(reinterpret_cast<const uint4*>(x_bf16), nvec,
                                                        reinterpret_cast<const uint16_t*>(x_bf16) + nvec * 8, ntail,
                                                        reinterpret_cast<uint32_t*>(amax));
  }
  return fog_launch_status();
}

extern "C" fog_status fog_scale(const float* amax, fog_fp8 fmt, int margin, float* scale, float* scale_inv, void* stream) {
  if (!amax || !scale) return FOG_ERR_NULL;
  if (fmt != FOG_E4M3 && fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
  if (margin < -64 || margin > 64) return FOG_ERR_SHAPE;
  scale_kernel<<<1, 1, 0, (hipStream_t)stream>>>(amax, (int)fmt, margin, scale, scale_inv);
  return fog_launch_status();
}

extern "C" fog_status fog_scale_delayed(float* history, int len, const float* new_amax, fog_fp8 fmt, int margin,
                                        float* scale, float* scale_inv, void* stream) {
  if (!history || !new_amax || !scale) return FOG_ERR_NULL;
  if (len < 1 || margin < -64 || margin > 64) return FOG_ERR_SHAPE;
  if (fmt != FOG_E4M3 && fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
  scale_delayed_kernel<<<1, kThreads, 0, (hipStream_t)stream>>>(history, len, new_amax, (int)fmt, margin, scale, scale_inv);
  return fog_launch_status();
}

template <int FMT>
static void launch_quantize(const uint16_t* x, int64_t rows, int64_t cols, int64_t ldx, const float* scale, uint8_t* q,
                            int64_t ldq, uint8_t* qT, int64_t ldqT, uint32_t* amax_out, hipStream_t s, ScaleSource js = ScaleSource{}) {
  const bool base_ok = cols % 16 == 0 && ldx % 16 == 0 && aligned16(x) && (!q || (ldq % 16 == 0 && aligned16(q)));
  if (!qT && base_ok) {
    int64_t r = rows, cpr = cols / 16, lx = ldx, lq = ldq;
    if (ldx == cols && ldq == cols) { cpr = rows * cpr; r = 1; }  // contiguous: one long row
    int64_t total = r * cpr;
    int64_t blocks = (total + 2 * kThreads - 1) / (2 * kThreads);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    if (amax_out)
      quantize_rows_kernel<FMT, true><<<(int)blocks, kThreads, 0, s>>>(x, r, cpr, lx, scale, q, lq, amax_out, js);
    else
      quantize_rows_kernel<FMT, false><<<(int)blocks, kThreads, 0, s>>>(x, r, cpr, lx, scale, q, lq, amax_out, js);
    return;
  }
  if (qT && base_ok && rows % 16 == 0 && ldqT % 16 == 0 && aligned16(qT)) {
    const int64_t tr = (rows + kTile - 1) / kTile, tc = (cols + kTile - 1) / kTile;
    if (tr * tc <= 0x7FFFFFFF) {
      const int grid = (int)(tr * tc);
#define FOG_QT(AM, WQ) quantize_transpose_kernel<FMT, AM, WQ><<<grid, kThreads, 0, s>>>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, amax_out, (int)tc, js)
      if (amax_out) { if (q) FOG_QT(true, true); else FOG_QT(true, false); }
      else          { if (q) FOG_QT(false, true); else FOG_QT(false, false); }
#undef FOG_QT
      return;
    }
  }
  int64_t total = rows * cols;
  int64_t blocks = (total + kThreads - 1) / kThreads;
  if (blocks > 8192) blocks = 8192;
  quantize_general_kernel<FMT><<<(int)blocks, kThreads, 0, s>>>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, amax_out, js);
}

static fog_status quantize_checks(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt,
                                  const uint8_t* q, int64_t ldq, const uint8_t* qT, int64_t ldqT) {
  if (rows < 0 || cols < 0) return FOG_ERR_SHAPE;
  if (fmt != FOG_E4M3 && fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
  if (rows != 0 && cols != 0) {
    if (!x_bf16 || (!q && !qT)) return FOG_ERR_NULL;
    if (ldx < cols || (q && ldq < cols) || (qT && ldqT < rows)) return FOG_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(x_bf16) & 1u) != 0) return FOG_ERR_ALIGN;
  }
  return FOG_OK;
}

extern "C" fog_status fog_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt,
                                   const float* scale, uint8_t* q, int64_t ldq, uint8_t* qT, int64_t ldqT,
                                   float* amax_out, void* stream) {
  if (!scale) return FOG_ERR_NULL;
  const fog_status st = quantize_checks(x_bf16, rows, cols, ldx, fmt, q, ldq, qT, ldqT);
  if (st != FOG_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if (amax_out) zero_u32_kernel<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_out));
  if (rows != 0 && cols != 0) {
    const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
    uint32_t* am = reinterpret_cast<uint32_t*>(amax_out);
    if (fmt == FOG_E4M3) launch_quantize<FOG_E4M3>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, am, s);
    else                 launch_quantize<FOG_E5M2>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, am, s);
  }
  return fog_launch_status();
}

constexpr int kJitBlocks = 1024;   // workgroups of the abs-max pass = words of workspace

extern "C" size_t fog_quantize_jit_workspace(void) { return kJitBlocks * sizeof(uint32_t); }

extern "C" fog_status fog_quantize_jit(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt, int margin,
                                       uint8_t* q, int64_t ldq, uint8_t* qT, int64_t ldqT,
                                       float* amax, float* scale, float* scale_inv,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!amax || !scale || !workspace) return FOG_ERR_NULL;
  if (workspace_bytes < fog_quantize_jit_workspace()) return FOG_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 3u) != 0) return FOG_ERR_ALIGN;
  if (margin < -64 || margin > 64) return FOG_ERR_SHAPE;
  const fog_status st = quantize_checks(x_bf16, rows, cols, ldx, fmt, q, ldq, qT, ldqT);
  if (st != FOG_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
  uint32_t* ws = reinterpret_cast<uint32_t*>(workspace);
  const int64_t n = rows * cols;
  int64_t blocks = 0;   // an empty tensor: no partial maxima, abs-max 0, scale 1
  if (n > 0) {
    if ((ldx == cols || rows == 1) && aligned16(x_bf16)) {
      const int64_t nvec = n / 8;
      const int ntail = (int)(n - nvec * 8);
      blocks = (nvec + kThreads * 8 - 1) / (kThreads * 8);
      if (blocks > kJitBlocks) blocks = kJitBlocks;
      if (blocks < 1) blocks = 1;
      amax_kernel<true><<<(int)blocks, kThreads, 0, s>>>(reinterpret_cast<const uint4*>(x), nvec, x + nvec * 8, ntail, ws);
    } else {
      blocks = (n + kThreads - 1) / kThreads;
      if (blocks > kJitBlocks) blocks = kJitBlocks;
      amax_strided_kernel<true><<<(int)blocks, kThreads, 0, s>>>(x, rows, cols, ldx, ws);
    }
  }
  if (n == 0) {   // nothing to cast: abs-max 0, scale 1
    scale_partials_kernel<<<1, kThreads, 0, s>>>(ws, 0, (int)fmt, margin, amax, scale, scale_inv);
    return fog_launch_status();
  }
  const ScaleSource js{ws, (int)blocks, (int)fmt, margin, amax, scale, scale_inv, nullptr, 0, 0, nullptr, nullptr};
  if (fmt == FOG_E4M3) launch_quantize<FOG_E4M3>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, nullptr, s, js);
  else                 launch_quantize<FOG_E5M2>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, nullptr, s, js);
  return fog_launch_status();
}

extern "C" size_t fog_quantize_delayed_state(void) { return 3 * kDelayedSlots * sizeof(uint32_t); }

extern "C" fog_status fog_quantize_delayed(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt, int margin,
                                           float* history, int history_len, int64_t step, void* state, size_t state_bytes,
                                           uint8_t* q, int64_t ldq, uint8_t* qT, int64_t ldqT,
                                           float* amax_prev, float* scale, float* scale_inv, void* stream) {
  if (!history || !state || !scale) return FOG_ERR_NULL;
  if (state_bytes < fog_quantize_delayed_state()) return FOG_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(state) & 3u) != 0) return FOG_ERR_ALIGN;
  if (history_len < 1 || step < 0 || margin < -64 || margin > 64) return FOG_ERR_SHAPE;
  const fog_status st = quantize_checks(x_bf16, rows, cols, ldx, fmt, q, ldq, qT, ldqT);
  if (st != FOG_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  uint32_t* base = reinterpret_cast<uint32_t*>(state);
  uint32_t* prev = base + ((step + 2) % 3) * kDelayedSlots;
  uint32_t* cur = base + (step % 3) * kDelayedSlots;
  uint32_t* next = base + ((step + 1) % 3) * kDelayedSlots;
  const ScaleSource js{prev, kDelayedSlots, (int)fmt, margin, amax_prev, scale, scale_inv,
                    history, history_len, (int)(step % history_len), cur, next};
  if (rows == 0 || cols == 0) {   // nothing to cast: the history still advances, this pass's abs-max stays 0
    delayed_scale_only_kernel<<<1, kThreads, 0, s>>>(js);
    return fog_launch_status();
  }
  const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
  if (fmt == FOG_E4M3) launch_quantize<FOG_E4M3>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, cur, s, js);
  else                 launch_quantize<FOG_E5M2>(x, rows, cols, ldx, scale, q, ldq, qT, ldqT, cur, s, js);
  return fog_launch_status();
}

extern "C" fog_status fog_delayed_amax(const void* state, int64_t step, float* amax, void* stream) {
  if (!state || !amax) return FOG_ERR_NULL;
  if (step < 0) return FOG_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(state) & 3u) != 0) return FOG_ERR_ALIGN;
  const uint32_t* cur = reinterpret_cast<const uint32_t*>(state) + (step % 3) * kDelayedSlots;
  partials_max_kernel<<<1, kThreads, 0, (hipStream_t)stream>>>(cur, kDelayedSlots, amax);
  return fog_launch_status();
}

extern "C" size_t fog_quantize_jit_batch_workspace(int count) {
  return count > 0 ? (size_t)count * kJitSlots * sizeof(uint32_t) : 0;
}

extern "C" fog_status fog_quantize_jit_batch(const fog_cast_job* jobs, int count, void* workspace, size_t workspace_bytes,
                                             void* stream) {
  if (count == 0) return FOG_OK;
  if (!jobs || !workspace) return FOG_ERR_NULL;
  if (count < 0 || count > kBatchMax) return FOG_ERR_SHAPE;
  if (workspace_bytes < fog_quantize_jit_batch_workspace(count)) return FOG_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 3u) != 0) return FOG_ERR_ALIGN;
  BatchJobs b;
  b.count = count;
  b.amax_first[0] = 0;
  for (int j = 0; j < count; ++j) {
    const fog_cast_job& t = jobs[j];
    if (!t.x_bf16 || !t.q || !t.amax || !t.scale) return FOG_ERR_NULL;
    if (t.rows <= 0 || t.cols <= 0 || t.margin < -64 || t.margin > 64) return FOG_ERR_SHAPE;
    if (t.fmt != FOG_E4M3 && t.fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
    if (!aligned16(t.x_bf16) || !aligned16(t.q)) return FOG_ERR_ALIGN;
    const int64_t n = t.rows * t.cols;
    if (n % 16 != 0) return FOG_ERR_UNSUPPORTED;
    int64_t ab = (n / 8 + kThreads * 8 - 1) / (kThreads * 8);
    if (ab > kJitSlots) ab = kJitSlots;
    b.amax_first[j + 1] = b.amax_first[j] + (int)ab;
    b.x[j] = reinterpret_cast<const uint16_t*>(t.x_bf16);
    b.n[j] = n;
    b.q[j] = t.q;
    b.fmt[j] = (int)t.fmt;
    b.margin[j] = t.margin;
    b.amax[j] = t.amax;
    b.scale[j] = t.scale;
    b.scale_inv[j] = t.scale_inv;
  }
  b.cast_first[0] = 0;
  for (int p = 0; p < count; ++p) {   // launch position p casts job count - 1 - p
    const int64_t chunks = b.n[count - 1 - p] / 16;
    int64_t cb = (chunks + 2 * kThreads - 1) / (2 * kThreads);
    if (cb > 2048) cb = 2048;
    b.cast_first[p + 1] = b.cast_first[p] + (int)cb;
  }
  for (int j = count; j < kBatchMax; ++j) {
    b.amax_first[j + 1] = b.amax_first[count];
    b.cast_first[j + 1] = b.cast_first[count];
    b.x[j] = nullptr; b.n[j] = 0; b.q[j] = nullptr; b.fmt[j] = 0; b.margin[j] = 0;
    b.amax[j] = b.scale[j] = b.scale_inv[j] = nullptr;
  }
  hipStream_t s = (hipStream_t)stream;
  uint32_t* ws = reinterpret_cast<uint32_t*>(workspace);
  amax_batch_kernel<<<b.amax_first[count], kThreads, 0, s>>>(b, ws);
  quantize_batch_kernel<<<b.cast_first[count], kThreads, 0, s>>>(b, ws);
  return fog_launch_status();
}

extern "C" fog_status fog_quantize_delayed_batch(const fog_delayed_job* jobs, int count, int64_t step, void* stream) {
  if (count == 0) return FOG_OK;
  if (!jobs) return FOG_ERR_NULL;
  if (count < 0 || count > kBatchMax || step < 0) return FOG_ERR_SHAPE;
  DelayedJobs b;
  b.count = count;
  b.first[0] = 0;
  b.prev_off = (int)((step + 2) % 3) * kDelayedSlots;
  b.cur_off = (int)(step % 3) * kDelayedSlots;
  b.next_off = (int)((step + 1) % 3) * kDelayedSlots;
  for (int j = 0; j < count; ++j) {
    const fog_delayed_job& t = jobs[j];
    if (!t.x_bf16 || !t.q || !t.history || !t.state || !t.scale) return FOG_ERR_NULL;
    if (t.rows <= 0 || t.cols <= 0 || t.history_len < 1 || t.margin < -64 || t.margin > 64) return FOG_ERR_SHAPE;
    if (t.fmt != FOG_E4M3 && t.fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
    if (!aligned16(t.x_bf16) || !aligned16(t.q) || (reinterpret_cast<uintptr_t>(t.state) & 3u) != 0) return FOG_ERR_ALIGN;
    if (t.state_bytes < fog_quantize_delayed_state()) return FOG_ERR_WORKSPACE;
    const int64_t n = t.rows * t.cols;
    if (n % 16 != 0) return FOG_ERR_UNSUPPORTED;
    int64_t cb = (n / 16 + 2 * kThreads - 1) / (2 * kThreads);
    if (cb > 2048) cb = 2048;
    b.first[j + 1] = b.first[j] + (int)cb;
    b.x[j] = reinterpret_cast<const uint16_t*>(t.x_bf16);
    b.n[j] = n;
    b.q[j] = t.q;
    b.fmt[j] = (int)t.fmt;
    b.margin[j] = t.margin;
    b.amax_prev[j] = t.amax_prev;
    b.scale[j] = t.scale;
    b.scale_inv[j] = t.scale_inv;
    b.hist[j] = t.history;
    b.hlen[j] = t.history_len;
    b.slot[j] = (int)(step % t.history_len);
    b.state[j] = reinterpret_cast<uint32_t*>(t.state);
  }
  for (int j = count; j < kBatchMax; ++j) {
    b.first[j + 1] = b.first[count];
    b.x[j] = nullptr; b.n[j] = 0; b.q[j] = nullptr; b.fmt[j] = 0; b.margin[j] = 0;
    b.amax_prev[j] = b.scale[j] = b.scale_inv[j] = b.hist[j] = nullptr;
    b.hlen[j] = 1; b.slot[j] = 0; b.state[j] = nullptr;
  }
  quantize_delayed_batch_kernel<<<b.first[count], kThreads, 0, (hipStream_t)stream>>>(b);
  return fog_launch_status();
}
