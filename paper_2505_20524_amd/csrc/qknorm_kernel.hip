// QK RMS normalisation with a frozen scalar gain, fused with the FP8 cast (Section 3 of the paper:
// N_gamma(x) = gamma x / rms(x), rms(x) = ||x||_2 / sqrt(D), gains frozen in the FOG variants;
// cast of Appendix E with a caller-provided scale, as under delayed scaling).  The normalised
// tensor is never stored: every bf16 element is read once and one FP8 byte is written, against
// 2 + 2 + 2 + 2 + 1 bytes per element for normalise -> abs-max -> cast as separate passes.
// HBM-bound.  A row of D elements is handled by D / 8 adjacent lanes (16 for the head size 128,
// four rows per wave); longer or odd rows take one wave per row and read the row twice.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

__global__ void zero_u32q(uint32_t* p) { *p = 0u; }

FOG_DEVICE float inv_rms(float sumsq, float cols, float gain) {
  // gain / sqrt(sumsq / D), correctly rounded square root and divisions; 0 for a row of zeros
  return sumsq > 0.0f ? gain / __builtin_sqrtf(sumsq / cols) : 0.0f;
}

// Workgroup maximum raised into *amax_out; reduced on bit patterns (non-negative floats order like them,
// and the NaN pattern of a thread that saw a NaN orders above everything).
FOG_DEVICE void block_amax(float m, bool nan, uint32_t* amax_out) {
  const uint32_t h = wave_max_u32(amax_bits(m, nan));
  __shared__ uint32_t part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = h;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t b = part[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) b = b > part[w] ? b : part[w];
    if (b > __hip_atomic_load(amax_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_out, b);
  }
}

// LPR lanes per row, each holding 8 consecutive elements (cols = 8 LPR); 64 / LPR rows per wave.
template <int FMT, int LPR>
__global__ __launch_bounds__(kThreads) void qknorm_rows_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t ldx, float gain,
                                                               const float* __restrict__ scale, uint8_t* __restrict__ q, int64_t ldq,
                                                               uint32_t* __restrict__ amax_out) {
  constexpr int RPB = kThreads / LPR;   // rows per workgroup and load
  constexpr int U = 4;                  // rows per lane group and trip: four loads in flight
  const float rho = *scale;
  const int sub = threadIdx.x % LPR, rloc = threadIdx.x / LPR;
  float m = 0.0f;
  bool nan = false;
  auto fetch = [&](int64_t r0, uint4 (&v)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = r0 + u * RPB + rloc;
      v[u] = make_uint4(0u, 0u, 0u, 0u);
      if (r < rows) v[u] = ld_nt16(x + r * ldx + 8 * sub);
    }
  };
  auto process = [&](int64_t r0, const uint4 (&v)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t r = r0 + u * RPB + rloc;
      float f[8] = {bf16lo(v[u].x), bf16hi(v[u].x), bf16lo(v[u].y), bf16hi(v[u].y), bf16lo(v[u].z), bf16hi(v[u].z), bf16lo(v[u].w), bf16hi(v[u].w)};
      float s = 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) s = __builtin_fmaf(f[k], f[k], s);
#pragma unroll
      for (int o = 1; o < LPR; o <<= 1) s += __shfl_xor(s, o, 64);
      const float inv = inv_rms(s, (float)(8 * LPR), gain);
      float y[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        y[k] = f[k] * inv;
        m = fmaxf(m, fabsf(y[k]));
      }
      if (r < rows) {
        uint2 o;
        o.x = cvt4_fp8_nan<FMT>(y[0] * rho, y[1] * rho, y[2] * rho, y[3] * rho, &nan);
        o.y = cvt4_fp8_nan<FMT>(y[4] * rho, y[5] * rho, y[6] * rho, y[7] * rho, &nan);
        st_nt8(q + r * ldq + 8 * sub, o);
      }
    }
  };
  // the next trip's loads are requested before the current trip is normalised
  const int64_t step = (int64_t)gridDim.x * (RPB * U);
  int64_t r0 = (int64_t)blockIdx.x * (RPB * U);
  uint4 va[U], vb[U];
  if (r0 < rows) fetch(r0, va);
  while (r0 < rows) {
    const int64_t r1 = r0 + step;
    if (r1 < rows) fetch(r1, vb);
    process(r0, va);
    if (r1 >= rows) break;
    const int64_t r2 = r1 + step;
    if (r2 < rows) fetch(r2, va);
    process(r1, vb);
    r0 = r2;
  }
  if (amax_out) block_amax(m, nan, amax_out);
}

// Any row length: one wave per row, two passes over the row (the second is served from cache).
template <int FMT>
__global__ __launch_bounds__(kThreads) void qknorm_general_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx,
                                                                  float gain, const float* __restrict__ scale, uint8_t* __restrict__ q,
                                                                  int64_t ldq, uint32_t* __restrict__ amax_out) {
  const float rho = *scale;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float m = 0.0f;
  bool nan = false;
  for (int64_t r = (int64_t)blockIdx.x * 4 + w; r < rows; r += (int64_t)gridDim.x * 4) {
    const uint16_t* row = x + r * ldx;
    float s = 0.0f;
    for (int64_t i = lane; i < cols; i += 64) {
      const float a = bf16lo(row[i]);
      s = __builtin_fmaf(a, a, s);
    }
    s = wave_sum_f32(s);
    const float inv = inv_rms(s, (float)cols, gain);
    for (int64_t i = lane; i < cols; i += 64) {
      const float y = bf16lo(row[i]) * inv;
      m = fmaxf(m, fabsf(y));
      const float t = y * rho;
      q[r * ldq + i] = (uint8_t)(cvt4_fp8_nan<FMT>(t, t, t, t, &nan) & 0xFFu);
    }
  }
  if (amax_out) block_amax(m, nan, amax_out);
}

template <int FMT>
void launch_qknorm(const uint16_t* x, int64_t rows, int64_t cols, int64_t ldx, float gain, const float* scale, uint8_t* q, int64_t ldq,
                   uint32_t* amax_out, hipStream_t s) {
  const bool vec = (reinterpret_cast<uintptr_t>(x) & 15u) == 0 && (reinterpret_cast<uintptr_t>(q) & 7u) == 0 && ldx % 8 == 0 && ldq % 8 == 0;
#define FOG_QKN(LPR)                                                                                            \
  do {                                                                                                          \
    int64_t blocks = (rows + 4 * (kThreads / LPR) - 1) / (4 * (kThreads / LPR));                                \
    if (blocks > 2048) blocks = 2048;                                                                           \
    qknorm_rows_kernel<FMT, LPR><<<(int)blocks, kThreads, 0, s>>>(x, rows, ldx, gain, scale, q, ldq, amax_out); \
    return;                                                                                                     \
  } while (0)
  if (vec && cols == 128) FOG_QKN(16);
  if (vec && cols == 64) FOG_QKN(8);
  if (vec && cols == 256) FOG_QKN(32);
  if (vec && cols == 512) FOG_QKN(64);
#undef FOG_QKN
  int64_t blocks = (rows + 3) / 4;
  if (blocks > 4096) blocks = 4096;
  qknorm_general_kernel<FMT><<<(int)blocks, kThreads, 0, s>>>(x, rows, cols, ldx, gain, scale, q, ldq, amax_out);
}

}  // namespace

extern "C" fog_status fog_rmsnorm_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float gain, fog_fp8 fmt,
                                           const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream) {
  if (!scale) return FOG_ERR_NULL;
  if (rows < 0 || cols < 0) return FOG_ERR_SHAPE;
  if (fmt != FOG_E4M3 && fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
  if (!(gain > 0.0f) || !(gain <= 3.402823466e38f)) return FOG_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (amax_out) zero_u32q<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_out));
  if (rows == 0 || cols == 0) return fog_launch_status();
  if (!x_bf16 || !q) return FOG_ERR_NULL;
  if (ldx < cols || ldq < cols) return FOG_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(x_bf16) & 1u) return FOG_ERR_ALIGN;
  const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
  uint32_t* am = reinterpret_cast<uint32_t*>(amax_out);
  if (fmt == FOG_E4M3) launch_qknorm<FOG_E4M3>(x, rows, cols, ldx, gain, scale, q, ldq, am, s);
  else                 launch_qknorm<FOG_E5M2>(x, rows, cols, ldx, gain, scale, q, ldq, am, s);
  return fog_launch_status();
}
