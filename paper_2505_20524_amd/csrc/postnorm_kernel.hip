// Post-RMSNorm with its residual connection, fused with the FP8 cast of the new residual stream
// (Section 3 of the paper: the sub-layer output y goes through N_gamma(y) = gamma (.) y / rms(y),
// rms(y) = ||y||_2 / sqrt(D), gamma a trainable vector, before it is added to the residual stream x;
// the block has no pre-normalisation, so x + N_gamma(y) is also the next GEMM's input and gets the
// cast of Appendix E with a caller-provided scale, as under delayed scaling).
// One pass: y and x are read once (2 + 2 B per element), the new stream is written as bf16 (2 B) and
// as FP8 codes (1 B); the abs-max of the stored bf16 tensor comes with it.  Done as separate passes
// the same work moves 2+2 (norm) + 2+2+2 (add) + 2 (abs-max) + 2+1 (cast) bytes.  HBM-bound.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

__global__ void zero_u32p(uint32_t* p) { *p = 0u; }

FOG_DEVICE float inv_rms(float sumsq, float cols) {
  // 1 / sqrt(sumsq / D), correctly rounded square root and divisions; 0 for a vector of zeros
  return sumsq > 0.0f ? 1.0f / __builtin_sqrtf(sumsq / cols) : 0.0f;
}

// abs-max of bf16 values kept as their 15-bit magnitude patterns (ordered like the values)
FOG_DEVICE void block_amax_bits(uint32_t m, uint32_t* amax_out) {
  m = wave_max_u32(m);
  __shared__ uint32_t part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t r = part[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = r > part[w] ? r : part[w];
    r <<= 16;   // the float with that bf16 pattern
    if (r > __hip_atomic_load(amax_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_out, r);
  }
}

// One element: binary32 sum, one rounding to bf16; returns the bf16 bits.
FOG_DEVICE uint32_t residual_bf16(float x, float y, float g, float inv) { return f32_to_bf16(__builtin_fmaf(g * y, inv, x)); }

// One wave per row; a lane owns C <= CMAX chunks of 8 consecutive elements (chunk c of lane l is
// elements [8 (64 c + l), +8): consecutive lanes read consecutive 16 bytes).  All loads of y and x
// of a row are issued before the first is used.
template <int FMT, int CMAX>
__global__ __launch_bounds__(kThreads) void postnorm_rows_kernel(const uint16_t* x, int64_t ldx, const uint16_t* __restrict__ y,
                                                                 int64_t ldy, int64_t rows, int C, const float* __restrict__ gamma,
                                                                 const float* __restrict__ scale, uint16_t* out, int64_t ldo,
                                                                 uint8_t* __restrict__ q, int64_t ldq, uint32_t* __restrict__ amax_out) {
  const float rho = *scale;
  const float cols = (float)(C * 512);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t m = 0u;
  for (int64_t r = (int64_t)blockIdx.x * 4 + w; r < rows; r += (int64_t)gridDim.x * 4) {
    uint4 vy[CMAX], vx[CMAX];
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
      if (c < C) vy[c] = ld_nt16(y + r * ldy + 8 * (64 * c + lane));
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
      if (c < C) vx[c] = ld_nt16(x + r * ldx + 8 * (64 * c + lane));
    float s = 0.0f;
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
      if (c < C) {
        const float f[8] = {bf16lo(vy[c].x), bf16hi(vy[c].x), bf16lo(vy[c].y), bf16hi(vy[c].y),
                            bf16lo(vy[c].z), bf16hi(vy[c].z), bf16lo(vy[c].w), bf16hi(vy[c].w)};
#pragma unroll
        for (int k = 0; k < 8; ++k) s = __builtin_fmaf(f[k], f[k], s);
      }
    s = wave_sum_f32(s);
    const float inv = inv_rms(s, cols);
#pragma unroll
    for (int c = 0; c < CMAX; ++c)
      if (c < C) {
        const int64_t col = 8 * (64 * c + lane);
        const float4 g0 = *reinterpret_cast<const float4*>(gamma + col), g1 = *reinterpret_cast<const float4*>(gamma + col + 4);
        const uint32_t b0 = residual_bf16(bf16lo(vx[c].x), bf16lo(vy[c].x), g0.x, inv), b1 = residual_bf16(bf16hi(vx[c].x), bf16hi(vy[c].x), g0.y, inv);
        const uint32_t b2 = residual_bf16(bf16lo(vx[c].y), bf16lo(vy[c].y), g0.z, inv), b3 = residual_bf16(bf16hi(vx[c].y), bf16hi(vy[c].y), g0.w, inv);
        const uint32_t b4 = residual_bf16(bf16lo(vx[c].z), bf16lo(vy[c].z), g1.x, inv), b5 = residual_bf16(bf16hi(vx[c].z), bf16hi(vy[c].z), g1.y, inv);
        const uint32_t b6 = residual_bf16(bf16lo(vx[c].w), bf16lo(vy[c].w), g1.z, inv), b7 = residual_bf16(bf16hi(vx[c].w), bf16hi(vy[c].w), g1.w, inv);
        const uint4 o = make_uint4(b0 | (b1 << 16), b2 | (b3 << 16), b4 | (b5 << 16), b6 | (b7 << 16));
        m = pkmax_abs_bf16(m, o.x); m = pkmax_abs_bf16(m, o.y); m = pkmax_abs_bf16(m, o.z); m = pkmax_abs_bf16(m, o.w);
        st_nt16(out + r * ldo + col, o);
        if (q) {
          uint2 c8;
          c8.x = cvt4_fp8_nan<FMT>(bf16lo(o.x) * rho, bf16hi(o.x) * rho, bf16lo(o.y) * rho, bf16hi(o.y) * rho);
          c8.y = cvt4_fp8_nan<FMT>(bf16lo(o.z) * rho, bf16hi(o.z) * rho, bf16lo(o.w) * rho, bf16hi(o.w) * rho);
          st_nt8(q + r * ldq + col, c8);
        }
      }
  }
  if (amax_out) {
    const uint32_t mm = (m & 0xFFFFu) > (m >> 16) ? (m & 0xFFFFu) : (m >> 16);
    block_amax_bits(mm, amax_out);
  }
}

// Any row length and alignment: one wave per row, two passes over y (the second is served from cache).
template <int FMT>
__global__ __launch_bounds__(kThreads) void postnorm_general_kernel(const uint16_t* x, int64_t ldx, const uint16_t* __restrict__ y,
                                                                    int64_t ldy, int64_t rows, int64_t cols, const float* __restrict__ gamma,
                                                                    const float* __restrict__ scale, uint16_t* out, int64_t ldo,
                                                                    uint8_t* __restrict__ q, int64_t ldq, uint32_t* __restrict__ amax_out) {
  const float rho = *scale;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t m = 0u;
  for (int64_t r = (int64_t)blockIdx.x * 4 + w; r < rows; r += (int64_t)gridDim.x * 4) {
    const uint16_t* yr = y + r * ldy;
    float s = 0.0f;
    for (int64_t i = lane; i < cols; i += 64) {
      const float a = bf16lo(yr[i]);
      s = __builtin_fmaf(a, a, s);
    }
    s = wave_sum_f32(s);
    const float inv = inv_rms(s, (float)cols);
    for (int64_t i = lane; i < cols; i += 64) {
      const uint32_t b = residual_bf16(bf16lo(x[r * ldx + i]), bf16lo(yr[i]), gamma[i], inv);
      out[r * ldo + i] = (uint16_t)b;
      const uint32_t mag = b & 0x7FFFu;
      m = m > mag ? m : mag;
      if (q) {
        const float t = bf16lo(b) * rho;
        q[r * ldq + i] = (uint8_t)(cvt4_fp8_nan<FMT>(t, t, t, t) & 0xFFu);
      }
    }
  }
  if (amax_out) block_amax_bits(m, amax_out);
}

template <int FMT>
void launch_postnorm(const uint16_t* x, int64_t ldx, const uint16_t* y, int64_t ldy, int64_t rows, int64_t cols, const float* gamma,
                     const float* scale, uint16_t* out, int64_t ldo, uint8_t* q, int64_t ldq, uint32_t* amax_out, hipStream_t s) {
  auto al = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; };
  const bool vec = cols % 512 == 0 && cols <= 8192 && al(x, 16) && al(y, 16) && al(out, 16) && al(gamma, 16) && (!q || al(q, 8)) &&
                   ldx % 8 == 0 && ldy % 8 == 0 && ldo % 8 == 0 && ldq % 8 == 0;
  int64_t blocks = (rows + 3) / 4;
  if (blocks > 8192) blocks = 8192;
  if (vec) {
    const int C = (int)(cols / 512);
    if (C <= 4)      postnorm_rows_kernel<FMT, 4><<<(int)blocks, kThreads, 0, s>>>(x, ldx, y, ldy, rows, C, gamma, scale, out, ldo, q, ldq, amax_out);
    else if (C <= 8) postnorm_rows_kernel<FMT, 8><<<(int)blocks, kThreads, 0, s>>>(x, ldx, y, ldy, rows, C, gamma, scale, out, ldo, q, ldq, amax_out);
    else             postnorm_rows_kernel<FMT, 16><<<(int)blocks, kThreads, 0, s>>>(x, ldx, y, ldy, rows, C, gamma, scale, out, ldo, q, ldq, amax_out);
    return;
  }
  postnorm_general_kernel<FMT><<<(int)blocks, kThreads, 0, s>>>(x, ldx, y, ldy, rows, cols, gamma, scale, out, ldo, q, ldq, amax_out);
}

}  // namespace

extern "C" fog_status fog_postnorm_residual_quantize(const void* x_bf16, int64_t ldx, const void* y_bf16, int64_t ldy, int64_t rows,
                                                     int64_t cols, const float* gamma, fog_fp8 fmt, const float* scale, void* xnew_bf16,
                                                     int64_t ldo, uint8_t* q, int64_t ldq, float* amax_out, void* stream) {
  if (!scale) return FOG_ERR_NULL;
  if (rows < 0 || cols < 0) return FOG_ERR_SHAPE;
  if (fmt != FOG_E4M3 && fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (amax_out) zero_u32p<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_out));
  if (rows == 0 || cols == 0) return fog_launch_status();
  if (!x_bf16 || !y_bf16 || !gamma || !xnew_bf16) return FOG_ERR_NULL;
  if (ldx < cols || ldy < cols || ldo < cols || (q && ldq < cols)) return FOG_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(x_bf16) | reinterpret_cast<uintptr_t>(y_bf16) | reinterpret_cast<uintptr_t>(xnew_bf16)) & 1u) return FOG_ERR_ALIGN;
  if (reinterpret_cast<uintptr_t>(gamma) & 3u) return FOG_ERR_ALIGN;
  const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
  const uint16_t* y = reinterpret_cast<const uint16_t*>(y_bf16);
  uint16_t* out = reinterpret_cast<uint16_t*>(xnew_bf16);
  uint32_t* am = reinterpret_cast<uint32_t*>(amax_out);
  if (fmt == FOG_E4M3) launch_postnorm<FOG_E4M3>(x, ldx, y, ldy, rows, cols, gamma, scale, out, ldo, q, ldq, am, s);
  else                 launch_postnorm<FOG_E5M2>(x, ldx, y, ldy, rows, cols, gamma, scale, out, ldo, q, ldq, am, s);
  return fog_launch_status();
}
