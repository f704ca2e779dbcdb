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

// the hardware's NaN-propagating maximum, as in the forward kernel (no quieting max(x, x) of the operands)
__device__ __forceinline__ float vmax(float a, float b) { return __builtin_elementwise_maximum(a, b); }

// WHAT 0: score products, softmax arithmetic, P V products; 1: the products only; 2: the arithmetic only.
// One key block the way the forward kernel takes it: scores into the one set of score registers, softmax, P V.
template <int WHAT>
__device__ __forceinline__ void attention_block(v8i* kf, const v8i* qf, const v8i* vf, const v16f& zero16, v16f* sc,
                                                v16f* o, float& l_run, float& m_run, float c, int it) {
  if (WHAT != 2) {
    asm volatile("" : "+v"(kf[0]), "+v"(kf[1]));   // the fragments "change" every block: the products stay in the loop
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      sc[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[kt], qf[0], zero16, 0, 0, 0, 0, 0, 0);
      sc[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[kt], qf[1], sc[kt], 0, 0, 0, 0, 0, 0);
    }
  } else {
    sc[0][it & 15] += 1e-3f;   // keeps the arithmetic loop-variant
  }
  v8i pf;
  if (WHAT != 1) {
    float cm[4];
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) {
      const v16f& x = sc[ch >> 1];
      const int b = 8 * (ch & 1);
      float m = vmax(vmax(x[b], x[b + 1]), x[b + 2]);
      m = vmax(vmax(m, x[b + 3]), x[b + 4]);
      m = vmax(vmax(m, x[b + 5]), x[b + 6]);
      cm[ch] = vmax(m, x[b + 7]);
    }
    m_run = vmax(m_run, vmax(vmax(vmax(cm[0], cm[1]), cm[2]), cm[3]) * c);
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
        const uint32_t pk = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, any_u32(), false);
        pf[4 * kt + qd] = (int)__builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, pk, true);
      }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) pf[i] = 0x38383838 + it;
  }
  if (WHAT != 2) {
#pragma unroll
    for (int d = 0; d < 4; ++d) o[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf[d], pf, o[d], 0, 0, 0, 0, 0, 0);
  } else {
    asm volatile("" ::"v"(pf));
  }
}

// WHAT 3: the same work with the P V products of the PREVIOUS block dealt out between the four groups of eight scores of
// this block's softmax (order pinned): a matrix instruction, then the exponentials, sums and converts of eight scores.
__device__ __forceinline__ void attention_block_interleaved(v8i* kf, const v8i* qf, const v8i* vf, const v16f& zero16, v16f* sc,
                                                            v16f* o, v8i& pf_prev, float& l_run, float& m_run, float c) {
  asm volatile("" : "+v"(kf[0]), "+v"(kf[1]));
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    sc[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[kt], qf[0], zero16, 0, 0, 0, 0, 0, 0);
    sc[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf[kt], qf[1], sc[kt], 0, 0, 0, 0, 0, 0);
  }
  float cm[4];
#pragma unroll
  for (int ch = 0; ch < 4; ++ch) {
    const v16f& x = sc[ch >> 1];
    const int b = 8 * (ch & 1);
    float m = vmax(vmax(x[b], x[b + 1]), x[b + 2]);
    m = vmax(vmax(m, x[b + 3]), x[b + 4]);
    m = vmax(vmax(m, x[b + 5]), x[b + 6]);
    cm[ch] = vmax(m, x[b + 7]);
  }
  m_run = vmax(m_run, vmax(vmax(vmax(cm[0], cm[1]), cm[2]), cm[3]) * c);
  const float shift = 3.0f - m_run;
  v8i pf;
#pragma unroll
  for (int grp = 0; grp < 4; ++grp) {
    __builtin_amdgcn_sched_barrier(0);
    o[grp] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf[grp], pf_prev, o[grp], 0, 0, 0, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    const int kt = grp >> 1;
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
      const int qd = 2 * (grp & 1) + qq;
      const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 0], c, shift));
      const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 1], c, shift));
      const float e2 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 2], c, shift));
      const float e3 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 3], c, shift));
      l_run += (e0 + e1) + (e2 + e3);
      const uint32_t pk = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, any_u32(), false);
      pf[4 * kt + qd] = (int)__builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, pk, true);
    }
    asm volatile("" : "+v"(pf[4 * kt + 2 * (grp & 1)]), "+v"(pf[4 * kt + 2 * (grp & 1) + 1]), "+v"(l_run));
  }
  __builtin_amdgcn_sched_barrier(0);
  pf_prev = pf;
}

template <int WHAT>
__global__ __launch_bounds__(256, 3) void attention_loop_kernel(float* __restrict__ sink, int iters) {
  const int t = threadIdx.x;
  v8i kf[2], qf[2], vf[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    kf[0][i] = 0x30313233 + t * (i + 1); kf[1][i] = 0x2c2d2e2f + t * (i + 3);
    qf[0][i] = 0x34353637 ^ (t << i); qf[1][i] = 0x31323334 ^ (t << (i + 1));
#pragma unroll
    for (int d = 0; d < 4; ++d) vf[d][i] = 0x38393a3b + i * 0x01010101 + d * 0x02020202;
  }
  v16f o[4], sc[2], zero16;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    zero16[r] = 0.0f;
#pragma unroll
    for (int d = 0; d < 4; ++d) o[d][r] = 0.0f;
    sc[0][r] = 0.001f * (r + t); sc[1][r] = 0.002f * (r + t);
  }
  float l_run = 0.0f, m_run = 0.0f;
  const float c = 1e-6f;
  if (WHAT == 3) {
    v8i pf_prev;
#pragma unroll
    for (int i = 0; i < 8; ++i) pf_prev[i] = 0x38383838;
    for (int it = 0; it < iters; ++it) attention_block_interleaved(kf, qf, vf, zero16, sc, o, pf_prev, l_run, m_run, c);
    asm volatile("" ::"v"(pf_prev));
  } else {
    for (int it = 0; it < iters; ++it) attention_block<(WHAT == 3 ? 0 : WHAT)>(kf, qf, vf, zero16, sc, o, l_run, m_run, c, it);
  }
  float s = l_run + m_run;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += o[d][r] + sc[d & 1][r];
  sink[(size_t)blockIdx.x * 256 + t] = s;
}

// One wave per SIMD; per trip eight independent matrix instructions, each followed (order pinned) by NV vector
// operations on registers of their own.  OP 0: v_fma_f32, 1: v_exp_f32, 2: v_cvt_pk_fp8_f32, 3: a quarter of a softmax
// group (fma, exp, add, and a max3 or a packed convert in turn).  MFMA false: the vector operations alone.
template <int OP, int NV, bool MFMA>
__global__ __launch_bounds__(256) void coissue_kernel(float* __restrict__ sink, int iters, long long* __restrict__ cycles) {
  const int t = threadIdx.x;
  v8i a[2], b[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[0][i] = 0x30313233 + t * (i + 1); a[1][i] = 0x2c2d2e2f + t * (i + 3);
    b[0][i] = 0x34353637 ^ (t << i); b[1][i] = 0x31323334 ^ (t << (i + 1));
  }
  v16f acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
  float x[8], y[4] = {0, 0, 0, 0}, z[4] = {1, 1, 1, 1}, u[4] = {0, 0, 0, 0}, m3[2] = {0, 0};
  uint32_t pq[4] = {0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = 0.001f * (t + i);
  const long long c0 = __builtin_readcyclecounter();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      __builtin_amdgcn_sched_barrier(0);
      if (MFMA) acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j & 1], b[(j >> 1) & 1], acc[j], 0, 0, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        if (OP == 0) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(x[v & 7]) : "v"(x[(v + 1) & 7]));
        if (OP == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(x[v & 7]));
        if (OP == 2) asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "=v"(pq[v & 3]) : "v"(x[v & 7]), "v"(x[(v + 1) & 7]));
        if (OP == 3) {
          asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(y[v & 3]) : "v"(x[v & 7]), "v"(x[(v + 1) & 7]), "v"(x[(v + 2) & 7]));
          asm volatile("v_exp_f32 %0, %1" : "=v"(z[v & 3]) : "v"(y[(v + 2) & 3]));
          asm volatile("v_add_f32 %0, %1, %2" : "=v"(u[v & 3]) : "v"(z[(v + 2) & 3]), "v"(u[(v + 1) & 3]));
          if (v & 1) asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(m3[(v >> 1) & 1]) : "v"(x[v & 7]), "v"(x[(v + 3) & 7]), "v"(m3[((v >> 1) + 1) & 1]));
          else asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "=v"(pq[(v >> 1) & 3]) : "v"(z[v & 3]), "v"(z[(v + 1) & 3]));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const long long c1 = __builtin_readcyclecounter();
  float s = y[0] + y[1] + y[2] + y[3] + z[0] + z[1] + z[2] + z[3] + u[0] + u[1] + u[2] + u[3] + m3[0] + m3[1];
  s += (float)(pq[0] ^ pq[1] ^ pq[2] ^ pq[3]);
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  sink[(size_t)blockIdx.x * 256 + t] = s;
  if (t == 0) cycles[blockIdx.x] = c1 - c0;
}

template <int OP, bool MFMA>
void coissue_launch(int nv, int grid, float* sink, int iters, long long* cycles, hipStream_t s) {
  switch (nv) {
    case 0:  coissue_kernel<OP, 0, MFMA><<<grid, 256, 0, s>>>(sink, iters, cycles); break;
    case 4:  coissue_kernel<OP, 4, MFMA><<<grid, 256, 0, s>>>(sink, iters, cycles); break;
    case 8:  coissue_kernel<OP, 8, MFMA><<<grid, 256, 0, s>>>(sink, iters, cycles); break;
    case 16: coissue_kernel<OP, 16, MFMA><<<grid, 256, 0, s>>>(sink, iters, cycles); break;
    default: coissue_kernel<OP, 32, MFMA><<<grid, 256, 0, s>>>(sink, iters, cycles); break;
  }
}

// Two waves per SIMD with separate roles (waves w and w + 4 of a workgroup share a SIMD): waves 0-3 issue nothing but
// independent matrix instructions, waves 4-7 nothing but the vector operations.  Each role counts its own cycles.
template <int OP, int NV>
__global__ __launch_bounds__(512) void cross_wave_kernel(float* __restrict__ sink, int iters_matrix, int iters_vector,
                                                         long long* __restrict__ cycles) {
  const int t = threadIdx.x;
  const bool vector_role = __builtin_amdgcn_readfirstlane(t >> 8) != 0;
  float s = 0.0f;
  long long c0 = 0, c1 = 0;
  if (!vector_role) {
    v8i a[2], b[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[0][i] = 0x30313233 + t * (i + 1); a[1][i] = 0x2c2d2e2f + t * (i + 3);
      b[0][i] = 0x34353637 ^ (t << i); b[1][i] = 0x31323334 ^ (t << (i + 1));
    }
    v16f acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    c0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters_matrix; ++it) {
#pragma unroll
      for (int j = 0; j < 8; ++j)
        acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[j & 1], b[(j >> 1) & 1], acc[j], 0, 0, 0, 0, 0, 0);
    }
    c1 = __builtin_readcyclecounter();
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[j][r];
  } else {
    float x[8], y[4] = {0, 0, 0, 0}, z[4] = {1, 1, 1, 1}, u[4] = {0, 0, 0, 0}, m3[2] = {0, 0};
    uint32_t pq[4] = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * (t + i);
    c0 = __builtin_readcyclecounter();
    for (int it = 0; it < iters_vector; ++it) {
#pragma unroll
      for (int v = 0; v < 8 * NV; ++v) {
        if (OP == 0) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(x[v & 7]) : "v"(x[(v + 1) & 7]));
        if (OP == 1) asm volatile("v_exp_f32 %0, %0" : "+v"(x[v & 7]));
        if (OP == 2) asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "=v"(pq[v & 3]) : "v"(x[v & 7]), "v"(x[(v + 1) & 7]));
        if (OP == 3) {
          asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(y[v & 3]) : "v"(x[v & 7]), "v"(x[(v + 1) & 7]), "v"(x[(v + 2) & 7]));
          asm volatile("v_exp_f32 %0, %1" : "=v"(z[v & 3]) : "v"(y[(v + 2) & 3]));
          asm volatile("v_add_f32 %0, %1, %2" : "=v"(u[v & 3]) : "v"(z[(v + 2) & 3]), "v"(u[(v + 1) & 3]));
          if (v & 1) asm volatile("v_max3_f32 %0, %1, %2, %3" : "=v"(m3[(v >> 1) & 1]) : "v"(x[v & 7]), "v"(x[(v + 3) & 7]), "v"(m3[((v >> 1) + 1) & 1]));
          else asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "=v"(pq[(v >> 1) & 3]) : "v"(z[v & 3]), "v"(z[(v + 1) & 3]));
        }
      }
    }
    c1 = __builtin_readcyclecounter();
    s = y[0] + y[1] + y[2] + y[3] + z[0] + z[1] + z[2] + z[3] + u[0] + u[1] + u[2] + u[3] + m3[0] + m3[1];
    s += (float)(pq[0] ^ pq[1] ^ pq[2] ^ pq[3]);
#pragma unroll
    for (int i = 0; i < 8; ++i) s += x[i];
  }
  sink[(size_t)blockIdx.x * 512 + t] = s;
  if ((t & 255) == 0) cycles[2 * blockIdx.x + (t >> 8)] = c1 - c0;
}

}  // namespace

extern "C" fog_status fog_probe_attention_loop(int what, int waves_per_simd, int iters, float* sink, size_t sink_bytes,
                                               double* ns_per_block, void* stream) {
  if (!sink || !ns_per_block) return FOG_ERR_NULL;
  if (iters < 1 || waves_per_simd < 1 || waves_per_simd > 3 || what < 0 || what > 3) return FOG_ERR_SHAPE;
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
    else if (what == 2) attention_loop_kernel<2><<<grid, 256, 0, s>>>(sink, n);
    else attention_loop_kernel<3><<<grid, 256, 0, s>>>(sink, n);
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

extern "C" fog_status fog_probe_mfma_coissue(int op, int vector_ops, int with_mfma, int iters, float* sink, size_t sink_bytes,
                                             double* cycles_per_slot, void* stream) {
  if (!sink || !cycles_per_slot) return FOG_ERR_NULL;
  if (iters < 1 || op < 0 || op > 3) return FOG_ERR_SHAPE;
  if (vector_ops != 0 && vector_ops != 4 && vector_ops != 8 && vector_ops != 16 && vector_ops != 32) return FOG_ERR_SHAPE;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return FOG_ERR_HIP;
  // the sink's tail holds one cycle count per workgroup (8 bytes each, 8-byte aligned)
  const size_t sink_floats = (size_t)cus * 256;
  const size_t cyc_off = (sink_floats * sizeof(float) + 7) & ~(size_t)7;
  if (sink_bytes < cyc_off + (size_t)cus * sizeof(long long)) return FOG_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(sink) & 7u) != 0) return FOG_ERR_ALIGN;
  long long* cycles = reinterpret_cast<long long*>(reinterpret_cast<char*>(sink) + cyc_off);
  hipStream_t s = (hipStream_t)stream;
  auto launch = [&](int n) {
    if (with_mfma) {
      if (op == 0) coissue_launch<0, true>(vector_ops, cus, sink, n, cycles, s);
      else if (op == 1) coissue_launch<1, true>(vector_ops, cus, sink, n, cycles, s);
      else if (op == 2) coissue_launch<2, true>(vector_ops, cus, sink, n, cycles, s);
      else coissue_launch<3, true>(vector_ops, cus, sink, n, cycles, s);
    } else {
      if (op == 0) coissue_launch<0, false>(vector_ops, cus, sink, n, cycles, s);
      else if (op == 1) coissue_launch<1, false>(vector_ops, cus, sink, n, cycles, s);
      else if (op == 2) coissue_launch<2, false>(vector_ops, cus, sink, n, cycles, s);
      else coissue_launch<3, false>(vector_ops, cus, sink, n, cycles, s);
    }
  };
  launch(iters < 32 ? iters : 32);   // warm-up
  launch(iters);
  fog_status st = fog_launch_status();
  if (st != FOG_OK) return st;
  if (hipStreamSynchronize(s) != hipSuccess) return FOG_ERR_HIP;
  static thread_local long long host[1024];
  const int n = cus < 1024 ? cus : 1024;
  if (hipMemcpy(host, cycles, (size_t)n * sizeof(long long), hipMemcpyDeviceToHost) != hipSuccess) return FOG_ERR_HIP;
  double sum = 0.0;
  for (int i = 0; i < n; ++i) sum += (double)host[i];
  *cycles_per_slot = sum / n / iters / 8.0;
  return FOG_OK;
}

extern "C" fog_status fog_probe_mfma_cross_wave(int op, int vector_ops, int iters_matrix, int iters_vector, float* sink, size_t sink_bytes,
                                                double* matrix_cycles_per_instruction, double* vector_cycles_per_group, void* stream) {
  if (!sink || !matrix_cycles_per_instruction || !vector_cycles_per_group) return FOG_ERR_NULL;
  if (iters_matrix < 0 || iters_vector < 0 || iters_matrix + iters_vector < 1 || op < 0 || op > 3) return FOG_ERR_SHAPE;
  if (vector_ops != 8 && vector_ops != 32) return FOG_ERR_SHAPE;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
    return FOG_ERR_HIP;
  // the sink's tail holds two cycle counts per workgroup (8 bytes each, 8-byte aligned)
  const size_t cyc_off = ((size_t)cus * 512 * sizeof(float) + 7) & ~(size_t)7;
  if (sink_bytes < cyc_off + (size_t)cus * 2 * sizeof(long long)) return FOG_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(sink) & 7u) != 0) return FOG_ERR_ALIGN;
  long long* cycles = reinterpret_cast<long long*>(reinterpret_cast<char*>(sink) + cyc_off);
  hipStream_t s = (hipStream_t)stream;
  auto launch = [&](int nm, int nv) {
    if (vector_ops == 8) {
      if (op == 0) cross_wave_kernel<0, 8><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
      else if (op == 1) cross_wave_kernel<1, 8><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
      else if (op == 2) cross_wave_kernel<2, 8><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
      else cross_wave_kernel<3, 8><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
    } else {
      if (op == 0) cross_wave_kernel<0, 32><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
      else if (op == 1) cross_wave_kernel<1, 32><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
      else if (op == 2) cross_wave_kernel<2, 32><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
      else cross_wave_kernel<3, 32><<<cus, 512, 0, s>>>(sink, nm, nv, cycles);
    }
  };
  launch(iters_matrix < 32 ? iters_matrix : 32, iters_vector < 32 ? iters_vector : 32);   // warm-up
  launch(iters_matrix, iters_vector);
  fog_status st = fog_launch_status();
  if (st != FOG_OK) return st;
  if (hipStreamSynchronize(s) != hipSuccess) return FOG_ERR_HIP;
  static thread_local long long host[2048];
  const int n = cus < 1024 ? cus : 1024;
  if (hipMemcpy(host, cycles, (size_t)n * 2 * sizeof(long long), hipMemcpyDeviceToHost) != hipSuccess) return FOG_ERR_HIP;
  double sm = 0.0, sv = 0.0;
  for (int i = 0; i < n; ++i) { sm += (double)host[2 * i]; sv += (double)host[2 * i + 1]; }
  *matrix_cycles_per_instruction = iters_matrix ? sm / n / iters_matrix / 8.0 : 0.0;
  *vector_cycles_per_group = iters_vector ? sv / n / iters_vector / 8.0 : 0.0;
  return FOG_OK;
}
