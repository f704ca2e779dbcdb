// Measurement helpers of the benchmark (include/fog_probe.h): what the GPU sustains in a register-resident
// FP8 matrix-instruction loop, as a function of the operand bit patterns.  Not part of the hot path.
#include "common.h"
#include "launch.h"
#include "../../include/fog_probe.h"

namespace {

// Four A fragments and four B fragments per wave (the register picture of the GEMM's 4 x 4 tile), loaded once;
// 16 independent accumulators, so the matrix core always has an instruction ready.
__global__ __launch_bounds__(256) void mfma_rate_kernel(const uint8_t* __restrict__ bytes, int iters, float* __restrict__ sink) {
  const int t = threadIdx.x;
  v8i fa[4], fb[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // 32 bytes per lane and fragment, taken from different places of the 64 KB pattern per lane, wave and workgroup
    const uint32_t oa = ((blockIdx.x * 1031u + t * 67u + i * 8209u) * 32u) & 0xFFE0u;
    const uint32_t ob = ((blockIdx.x * 2053u + t * 131u + i * 4099u + 17u) * 32u) & 0xFFE0u;
    const uint4 a0 = *reinterpret_cast<const uint4*>(bytes + oa), a1 = *reinterpret_cast<const uint4*>(bytes + oa + 16);
    const uint4 b0 = *reinterpret_cast<const uint4*>(bytes + ob), b1 = *reinterpret_cast<const uint4*>(bytes + ob + 16);
    fa[i][0] = a0.x; fa[i][1] = a0.y; fa[i][2] = a0.z; fa[i][3] = a0.w; fa[i][4] = a1.x; fa[i][5] = a1.y; fa[i][6] = a1.z; fa[i][7] = a1.w;
    fb[i][0] = b0.x; fb[i][1] = b0.y; fb[i][2] = b0.z; fb[i][3] = b0.w; fb[i][4] = b1.x; fb[i][5] = b1.y; fb[i][6] = b1.z; fb[i][7] = b1.w;
  }
  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], acc[i][j], 0, 0, 0, 0, 0, 0);
  }
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  sink[(size_t)blockIdx.x * 256 + t] = s;
}

// WHAT 0: score products, softmax arithmetic, P V products; 1: the products only; 2: the arithmetic only.
template <int WHAT>
__global__ __launch_bounds__(256) void attention_loop_kernel(float* __restrict__ sink, int iters) {
  const int t = threadIdx.x;
  v8i kf[2], qf[2], vf[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    kf[0][i] = 0x30313233 + t * (i + 1); kf[1][i] = 0x2c2d2e2f + t * (i + 3);
    qf[0][i] = 0x34353637 ^ (t << i); qf[1][i] = 0x31323334 ^ (t << (i + 1));
#pragma unroll
    for (int d = 0; d < 4; ++d) vf[d][i] = 0x38393a3b + i * 0x01010101 + d * 0x02020202;
  }
  v16f o[4], sc[2], sn[2], zero16;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    zero16[r] = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) o[d][r] = 0.0f;
    sc[0][r] = 0.001f * (r + t); sc[1][r] = 0.002f * (r + t);
    sn[0][r] = sc[0][r]; sn[1][r] = sc[1][r];
  }
  float l_run = 0.0f, m_run = 0.0f;
  const float c = 1e-6f;
  for (int it = 0; it < iters; ++it) {
    if (WHAT != 2) {   // the next block's scores
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        sn[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[kt], qf[0], zero16, 0, 0, 0, 0, 0, 0);
        sn[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[kt], qf[1], sn[kt], 0, 0, 0, 0, 0, 0);
      }
    }
    v8i pf;
    if (WHAT != 1) {   // this block's softmax arithmetic
      float bm = fmaxf(fmaxf(sc[0][0], sc[0][1]), sc[1][0]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) bm = fmaxf(fmaxf(bm, sc[0][r]), sc[0][r + 1]);
#pragma unroll
      for (int r = 1; r < 15; r += 2) bm = fmaxf(fmaxf(bm, sc[1][r]), sc[1][r + 1]);
      m_run = fmaxf(m_run, bm * c);
      const float shift = 3.0f - m_run;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 0], c, shift));
          const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 1], c, shift));
          const float e2 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 2], c, shift));
          const float e3 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 3], c, shift));
          l_run += (e0 + e1) + (e2 + e3);
          const uint32_t pk = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, 0u, false);
          pf[4 * kt + qd] = (int)__builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, pk, true);
        }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) pf[i] = __float_as_int(sc[i >> 2][i & 3]);
    }
    if (WHAT != 2) {
#pragma unroll
      for (int d = 0; d < 4; ++d) o[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf[d], pf, o[d], 0, 0, 0, 0, 0, 0);
      sc[0] = sn[0]; sc[1] = sn[1];
    } else {
      asm volatile("" ::"v"(pf));
      sc[0][it & 15] += 1e-3f;   // keeps the arithmetic loop-variant
    }
  }
  float s = l_run + m_run;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += o[d][r];
  sink[(size_t)blockIdx.x * 256 + t] = s;
}

}  // namespace

extern "C" fog_status fog_probe_attention_loop(int what, int waves_per_simd, int iters, float* sink, size_t sink_bytes,
                                               double* ns_per_block, void* stream) {
  if (!sink || !ns_per_block) return FOG_ERR_NULL;
  if (iters < 1 || waves_per_simd < 1 || waves_per_simd > 3 || what < 0 || what > 2) return FOG_ERR_SHAPE;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return FOG_ERR_HIP;
  const int grid = cus * waves_per_simd;
  if (sink_bytes < (size_t)grid * 256 * sizeof(float)) return FOG_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return FOG_ERR_HIP;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FOG_ERR_HIP; }
  auto launch = [&](int n) {
    if (what == 0) attention_loop_kernel<0><<<grid, 256, 0, s>>>(sink, n);
    else if (what == 1) attention_loop_kernel<1><<<grid, 256, 0, s>>>(sink, n);
    else attention_loop_kernel<2><<<grid, 256, 0, s>>>(sink, n);
  };
  launch(iters < 32 ? iters : 32);   // warm-up
  (void)hipEventRecord(e0, s);
  launch(iters);
  (void)hipEventRecord(e1, s);
  fog_status st = fog_launch_status();
  float ms = 0.0f;
  if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.0f)) st = FOG_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != FOG_OK) return st;
  *ns_per_block = (double)ms * 1e6 / ((double)iters * waves_per_simd);
  return FOG_OK;
}

extern "C" fog_status fog_probe_mfma_rate(const uint8_t* operand_bytes, int iters, float* sink, size_t sink_bytes,
                                          double* tflops, double* mfma_clock_ghz, void* stream) {
  if (!operand_bytes || !sink || !tflops) return FOG_ERR_NULL;
  if (iters < 1) return FOG_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(operand_bytes) & 15u) != 0 || (reinterpret_cast<uintptr_t>(sink) & 3u) != 0) return FOG_ERR_ALIGN;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return FOG_ERR_HIP;
  if (sink_bytes < (size_t)cus * 256 * sizeof(float)) return FOG_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return FOG_ERR_HIP;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return FOG_ERR_HIP; }
  mfma_rate_kernel<<<cus, 256, 0, s>>>(operand_bytes, iters < 64 ? iters : 64, sink);   // warm-up
  (void)hipEventRecord(e0, s);
  mfma_rate_kernel<<<cus, 256, 0, s>>>(operand_bytes, iters, sink);
  (void)hipEventRecord(e1, s);
  fog_status st = fog_launch_status();
  float ms = 0.0f;
  if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || !(ms > 0.0f)) st = FOG_ERR_HIP;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != FOG_OK) return st;
  const double per_wave = 16.0 * iters;                        // instructions per wave
  *tflops = per_wave * 131072.0 * 4.0 * cus / (ms * 1e-3) / 1e12;
  if (mfma_clock_ghz) *mfma_clock_ghz = per_wave * 64.0 / (ms * 1e-3) / 1e9;
  return FOG_OK;
}
