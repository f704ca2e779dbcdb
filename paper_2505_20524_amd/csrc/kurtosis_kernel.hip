// Activation kurtosis (Section 4 of the paper): kurt(x) = mu[x^4] / (mu[x^2])^2 per token vector,
// averaged over the token vectors of a tensor.  The denominator is read as the squared un-centred
// second moment (the printed sigma^2[x^2] cannot be the variance of x^2: that would fall as an
// outlier grows).  HBM-bound: every element is read once with 16-byte loads (eight to sixteen in flight); one wave per row,
// binary32 sums of x^2 and x^4, one float atomic per workgroup.  The same read can also deliver the
// tensor's abs-max (Appendix E: what the scaling history of the next cast needs), so that monitoring
// and delayed scaling share one pass over the activations.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;

__global__ void zero_f32_kernel(float* p, uint32_t* amax) {
  *p = 0.0f;
  if (amax) *amax = 0u;
}

template <bool AMAX>
FOG_DEVICE void acc_pair(uint32_t w, float& s2, float& s4, uint32_t& mx) {
  if (AMAX) mx = pkmax_abs_bf16(mx, w);
  const float a = bf16lo(w), b = bf16hi(w);
  const float a2 = a * a, b2 = b * b;
  s2 += a2 + b2;
  s4 = __builtin_fmaf(a2, a2, __builtin_fmaf(b2, b2, s4));
}

// VEC: rows are 16-byte aligned and cols % 8 == 0.  RB > 1 (VEC only): cols == 4096 / RB exactly, a batch of
// eight loads per lane then covers RB whole rows, so that short rows keep as many loads in flight as long ones.
template <bool VEC, bool AMAX, int RB>
__global__ __launch_bounds__(kThreads) void kurtosis_kernel(const uint16_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx,
                                                            float inv_rows, float* __restrict__ out, uint32_t* __restrict__ amax_out) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float local = 0.0f;   // sum of this wave's row kurtoses
  uint32_t mx = 0u;     // running max of |x| as two packed 15-bit bf16 magnitudes
  const int64_t rstep = (int64_t)gridDim.x * 4;
  const float fcols = (float)cols;
  // mu4 / mu2^2 = cols * s4 / s2^2; an all-zero row contributes 0
  auto close_row = [&](float s2, float s4) {
    s2 = wave_sum_f32(s2);
    s4 = wave_sum_f32(s4);
    if (s2 > 0.0f) local += fcols * (s4 / (s2 * s2));
  };
  if (VEC) {
    // A row is cut into batches of up to eight 16-byte loads per lane; the wave walks its (row, batch)
    // sequence with the next batch requested before the current one is summed, across row ends too.
    const int64_t nvec = cols >> 3;
    const int64_t nb = (nvec + 511) >> 9;
    constexpr int LPR = 8 / RB;   // loads per lane and row when RB > 1
    auto fetch = [&](int64_t r, int64_t b, uint4 (&v)[8]) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        v[k] = make_uint4(0u, 0u, 0u, 0u);   // zeros add nothing to the sums or the maximum
        if (RB == 1) {
          const int64_t i = (b << 9) + 64 * k + lane;
          if (i < nvec) v[k] = ld_nt16(x + r * ldx + 8 * i);
        } else {
          const int64_t row = r * RB + k / LPR;
          if (row < rows) v[k] = ld_nt16(x + row * ldx + 8 * (64 * (k % LPR) + lane));
        }
      }
    };
    float s2 = 0.0f, s4 = 0.0f;
    auto consume = [&](const uint4 (&v)[8], bool last) {
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        acc_pair<AMAX>(v[k].x, s2, s4, mx); acc_pair<AMAX>(v[k].y, s2, s4, mx); acc_pair<AMAX>(v[k].z, s2, s4, mx); acc_pair<AMAX>(v[k].w, s2, s4, mx);
        if (RB > 1 && k % LPR == LPR - 1) {   // a row of the batch is complete (rows past the end sum to 0 and add nothing)
          close_row(s2, s4);
          s2 = s4 = 0.0f;
        }
      }
      if (RB == 1 && last) {
        close_row(s2, s4);
        s2 = s4 = 0.0f;
      }
    };
    // with RB > 1 "r" counts groups of RB rows and a group is one batch
    const int64_t units = RB == 1 ? rows : (rows + RB - 1) / RB;
    int64_t r = (int64_t)blockIdx.x * 4 + w, b = 0;
    uint4 va[8], vb[8];
    if (r < units) fetch(r, b, va);
    while (r < units) {
      // (r1, b1): what follows (r, b)
      int64_t r1 = r, b1 = b + 1;
      if (b1 == nb) { r1 = r + rstep; b1 = 0; }
      if (r1 < units) fetch(r1, b1, vb);
      consume(va, b + 1 == nb);
      if (r1 >= units) break;
      int64_t r2 = r1, b2 = b1 + 1;
      if (b2 == nb) { r2 = r1 + rstep; b2 = 0; }
      if (r2 < units) fetch(r2, b2, va);
      consume(vb, b1 + 1 == nb);
      r = r2;
      b = b2;
    }
  } else {
    for (int64_t r = (int64_t)blockIdx.x * 4 + w; r < rows; r += rstep) {
      const uint16_t* row = x + r * ldx;
      float s2 = 0.0f, s4 = 0.0f;
      for (int64_t i = lane; i < cols; i += 64) {
        const float a = bf16lo(row[i]), a2 = a * a;
        if (AMAX) mx = pkmax_abs_bf16(mx, row[i]);
        s2 += a2;
        s4 = __builtin_fmaf(a2, a2, s4);
      }
      close_row(s2, s4);
    }
  }
  __shared__ float part[4];
  __shared__ uint32_t pmax[4];
  if (AMAX) mx = wave_max_u32((mx & 0xFFFFu) > (mx >> 16) ? (mx & 0xFFFFu) : (mx >> 16));
  if (lane == 0) {
    part[w] = local;
    if (AMAX) pmax[w] = mx;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const float t = (part[0] + part[1]) + (part[2] + part[3]);
    if (t != 0.0f) atomicAdd(out, t * inv_rows);
    if (AMAX) {
      uint32_t r = pmax[0];
#pragma unroll
      for (int k = 1; k < 4; ++k) r = r > pmax[k] ? r : pmax[k];
      r <<= 16;   // the float with that bf16 pattern; non-negative floats order like their bits
      if (r > __hip_atomic_load(amax_out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(amax_out, r);
    }
  }
}

}  // namespace

extern "C" fog_status fog_kurtosis(const void* x_bf16, int64_t rows, int64_t cols, int64_t ldx, float* kurt, float* amax_out,
                                   void* stream) {
  if (!kurt) return FOG_ERR_NULL;
  if (rows < 0 || cols < 0) return FOG_ERR_SHAPE;
  hipStream_t s = (hipStream_t)stream;
  uint32_t* am = reinterpret_cast<uint32_t*>(amax_out);
  zero_f32_kernel<<<1, 1, 0, s>>>(kurt, am);
  if (rows == 0 || cols == 0) return fog_launch_status();
  if (!x_bf16) return FOG_ERR_NULL;
  if (ldx < cols) return FOG_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(x_bf16) & 1u) return FOG_ERR_ALIGN;
  const bool vec = (reinterpret_cast<uintptr_t>(x_bf16) & 15u) == 0 && cols % 8 == 0 && ldx % 8 == 0;
  const int rb = !vec ? 1 : cols == 2048 ? 2 : cols == 1024 ? 4 : cols == 512 ? 8 : 1;
  int64_t blocks = ((rows + rb - 1) / rb + 3) / 4;
  if (blocks > 1024) blocks = 1024;   // four workgroups per CU are resident
  const uint16_t* x = reinterpret_cast<const uint16_t*>(x_bf16);
  const float inv = 1.0f / (float)rows;
#define FOG_KURT(V, A, RB) kurtosis_kernel<V, A, RB><<<(int)blocks, kThreads, 0, s>>>(x, rows, cols, ldx, inv, kurt, am)
#define FOG_KURT_A(V, RB) do { if (am) FOG_KURT(V, true, RB); else FOG_KURT(V, false, RB); } while (0)
  if (!vec)         FOG_KURT_A(false, 1);
  else if (rb == 2) FOG_KURT_A(true, 2);
  else if (rb == 4) FOG_KURT_A(true, 4);
  else if (rb == 8) FOG_KURT_A(true, 8);
  else              FOG_KURT_A(true, 1);
#undef FOG_KURT_A
#undef FOG_KURT
  return fog_launch_status();
}
