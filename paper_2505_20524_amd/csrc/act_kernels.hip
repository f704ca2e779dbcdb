// Element-wise producers of a GEMM or attention operand, fused with the FP8 cast (cast of Appendix E
// of the paper with a caller-provided scale, as under delayed scaling):
//   xIELU (Appendix B, equation xIELU: alpha_p x^2 + 0.5 x for x > 0,
//          alpha_n (e^x - 1) - alpha_n x + 0.5 x for x <= 0), the FOG-max activation;
//   GeLU  (Section 3, architecture table; read as x Phi(x), the exact form);
//   tanh_alpha(x) = tanh(alpha x) (Section 3), the query / key regulariser of the FOG-flash variant.
// The first two produce the second feed-forward GEMM's input, the third the attention's Q and K.
// The activated tensor is never stored as bf16: every element is read once (2 B) and one FP8 byte
// is written.  HBM-bound.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

__global__ void zero_u32a(uint32_t* p) { *p = 0u; }

enum { ACT_XIELU = 0, ACT_GELU = 1, ACT_TANH = 2 };

// binary32 evaluation.  e^x - 1 comes from expm1f (accurate near 0, where a plain exponential minus
// one would lose every significant bit of the quadratic term); the remaining operations are single
// multiplies and adds, so the result is within a few units in the last place of the exact value.
FOG_DEVICE float xielu(float x, float ap, float an) {
  const float pos = __builtin_fmaf(ap * x, x, 0.5f * x);
  const float neg = __builtin_fmaf(an, expm1f(fminf(x, 0.0f)), (0.5f - an) * x);
  return x > 0.0f ? pos : neg;
}

// x Phi(x) with Phi(x) = erfc(-x / sqrt 2) / 2: the complementary form keeps its relative accuracy
// in the negative tail, where 1 + erf would cancel.
FOG_DEVICE float gelu(float x) { return 0.5f * x * erfcf(-0.70710678118654752f * x); }

template <int ACT>
FOG_DEVICE float act(float x, float p0, float p1) {
  if (ACT == ACT_XIELU) return xielu(x, p0, p1);
  if (ACT == ACT_GELU) return gelu(x);
  return tanhf(p0 * x);
}

template <int ACT, int FMT>
FOG_DEVICE uint2 act_cast8(uint4 v, float ap, float an, float rho, float& m) {
  float y[8] = {act<ACT>(bf16lo(v.x), ap, an), act<ACT>(bf16hi(v.x), ap, an), act<ACT>(bf16lo(v.y), ap, an), act<ACT>(bf16hi(v.y), ap, an),
                act<ACT>(bf16lo(v.z), ap, an), act<ACT>(bf16hi(v.z), ap, an), act<ACT>(bf16lo(v.w), ap, an), act<ACT>(bf16hi(v.w), ap, an)};
#pragma unroll
  for (int k = 0; k < 8; ++k) m = fmaxf(m, fabsf(y[k]));
  uint2 o;
  o.x = cvt4_fp8<FMT>(y[0] * rho, y[1] * rho, y[2] * rho, y[3] * rho);
  o.y = cvt4_fp8<FMT>(y[4] * rho, y[5] * rho, y[6] * rho, y[7] * rho);
  return o;
}

FOG_DEVICE void block_amax(float m, uint32_t* amax_out) {
  m = wave_max_f32(m);
  __shared__ float part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    float r = part[0];
#pragma unroll
    for (int w = 1; w < kThreads / 64; ++w) r = fmaxf(r, part[w]);
    const uint32_t b = __float_as_uint(r);   // non-negative floats order like their bit patterns
    if (b > __hip_atomic_load(amax_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_out, b);
  }
}

// Each thread turns 16 bf16 (two 16-byte loads) into 16 FP8 codes (one 16-byte store), two such chunks per trip.
template <int ACT, int FMT>
__global__ __launch_bounds__(kThreads) void act_rows_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t chunks_per_row,
                                                            int64_t ldx, float ap, float an, const float* __restrict__ scale,
                                                            uint8_t* __restrict__ q, int64_t ldq, uint32_t* __restrict__ amax_out) {
  const float rho = *scale;
  const int64_t total = rows * chunks_per_row;
  const int64_t stride = (int64_t)gridDim.x * kThreads;
  float m = 0.0f;
  auto src_of = [&](int64_t i) {
    const int64_t r = i / chunks_per_row, c = i - r * chunks_per_row;
    return x + r * ldx + c * 16;
  };
  auto dst_of = [&](int64_t i) {
    const int64_t r = i / chunks_per_row, c = i - r * chunks_per_row;
    return q + r * ldq + c * 16;
  };
  auto emit = [&](uint4 a, uint4 b, uint8_t* dst) {
    const uint2 lo = act_cast8<ACT, FMT>(a, ap, an, rho, m), hi = act_cast8<ACT, FMT>(b, ap, an, rho, m);
    st_nt16(dst, make_uint4(lo.x, lo.y, hi.x, hi.y));
  };
  int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
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
  if (amax_out) block_amax(m, amax_out);
}

template <int ACT, int FMT>
__global__ __launch_bounds__(kThreads) void act_general_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx,
                                                               float ap, float an, const float* __restrict__ scale,
                                                               uint8_t* __restrict__ q, int64_t ldq, uint32_t* __restrict__ amax_out) {
  const float rho = *scale;
  const int64_t total = rows * cols;
  float m = 0.0f;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / cols, c = i - r * cols;
    const float y = act<ACT>(bf16lo(x[r * ldx + c]), ap, an);
    m = fmaxf(m, fabsf(y));
    const float t = y * rho;
    q[r * ldq + c] = (uint8_t)(cvt4_fp8<FMT>(t, t, t, t) & 0xFFu);
  }
  if (amax_out) block_amax(m, amax_out);
}

template <int ACT, int FMT>
void launch_act(const uint16_t* x, int64_t rows, int64_t cols, int64_t ldx, float ap, float an, const float* scale, uint8_t* q,
                  int64_t ldq, uint32_t* amax_out, hipStream_t s) {
  const bool vec = cols % 16 == 0 && ldx % 16 == 0 && ldq % 16 == 0 && (reinterpret_cast<uintptr_t>(x) & 15u) == 0 &&
                   (reinterpret_cast<uintptr_t>(q) & 15u) == 0;
  if (vec) {
    int64_t r = rows, cpr = cols / 16, lx = ldx, lq = ldq;
    if (ldx == cols && ldq == cols) { cpr = rows * cpr; r = 1; lx = lq = cpr * 16; }  // contiguous: one long row
    int64_t blocks = (r * cpr + 2 * kThreads - 1) / (2 * kThreads);
    if (blocks > 2048) blocks = 2048;
    act_rows_kernel<ACT, FMT><<<(int)blocks, kThreads, 0, s>>>(x, r, cpr, lx, ap, an, scale, q, lq, amax_out);
    return;
  }
  int64_t blocks = (rows * cols + kThreads - 1) / kThreads;
  if (blocks > 8192) blocks = 8192;
  act_general_kernel<ACT, FMT><<<(int)blocks, kThreads, 0, s>>>(x, rows, cols, ldx, ap, an, scale, q, ldq, amax_out);
}

// Argument checks and dispatch shared by the three entry points (p0, p1: the activation's parameters).
template <int ACT>
fog_status act_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float p0, float p1, fog_fp8 fmt,
                        const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream) {
  if (!scale) return FOG_ERR_NULL;
  if (rows < 0 || cols < 0) return FOG_ERR_SHAPE;
  if (fmt != FOG_E4M3 && fmt != FOG_E5M2) return FOG_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (amax_out) zero_u32a<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_out));
  if (rows == 0 || cols == 0) return fog_launch_status();
  if (!x_bf16 || !q) return FOG_ERR_NULL;
  if (ldx < cols || ldq < cols) return FOG_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(x_bf16) & 1u) return FOG_ERR_ALIGN;
  const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
  uint32_t* am = reinterpret_cast<uint32_t*>(amax_out);
  if (fmt == FOG_E4M3) launch_act<ACT, FOG_E4M3>(x, rows, cols, ldx, p0, p1, scale, q, ldq, am, s);
  else                 launch_act<ACT, FOG_E5M2>(x, rows, cols, ldx, p0, p1, scale, q, ldq, am, s);
  return fog_launch_status();
}

}  // namespace

extern "C" fog_status fog_xielu_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float alpha_p, float alpha_n,
                                         fog_fp8 fmt, const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream) {
  if (!(alpha_p >= 0.0f) || !(alpha_n >= 0.0f) || !(alpha_p <= 3.402823466e38f) || !(alpha_n <= 3.402823466e38f)) return FOG_ERR_UNSUPPORTED;
  return act_quantize<ACT_XIELU>(x_bf16, rows, cols, ldx, alpha_p, alpha_n, fmt, scale, q, ldq, amax_out, stream);
}

extern "C" fog_status fog_gelu_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, fog_fp8 fmt, const float* scale,
                                        uint8_t* q, int64_t ldq, float* amax_out, void* stream) {
  return act_quantize<ACT_GELU>(x_bf16, rows, cols, ldx, 0.0f, 0.0f, fmt, scale, q, ldq, amax_out, stream);
}

extern "C" fog_status fog_tanh_quantize(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float alpha, fog_fp8 fmt,
                                        const float* scale, uint8_t* q, int64_t ldq, float* amax_out, void* stream) {
  if (!(alpha >= -3.402823466e38f) || !(alpha <= 3.402823466e38f)) return FOG_ERR_UNSUPPORTED;
  return act_quantize<ACT_TANH>(x_bf16, rows, cols, ldx, alpha, 0.0f, fmt, scale, q, ldq, amax_out, stream);
}
