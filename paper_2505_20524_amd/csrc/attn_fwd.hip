// FP8 dot-product attention, forward (gfx950).
//
// Computes, per (batch, head), O = Softmax(s Q K^T + M) V (Appendix B of the paper, eq. P) with
// both products in FP8 (Appendix E, FP8DPA row of the table of FP8 methods): Q~, K~, V~ arrive as
// E4M3 codes, the probabilities are cast to E4M3 for the P V product, the softmax runs in binary32.
//
// One pass over the keys (online softmax).  The row reference is the INTEGER m = ceil(running max)
// in the log2 domain, so a later change of the reference rescales earlier probabilities by an
// exact power of two: the E4M3 codes of P do not depend on the order or size of the key blocks.
//
// Mapping.  A workgroup of 4 waves takes 128 queries of one head; a wave takes 32 queries and
// walks the keys in blocks of 64.  The scores are produced TRANSPOSED, S^T = K Q^T, with
// v_mfma_f32_32x32x64_f8f6f4: lane l then holds query (l & 31) and, per 32-key tile, the 16 keys
// 8 (r / 4) + 4 (l / 32) + (r % 4), r = 0..15.  That is exactly the shape of a B operand of the
// next MFMA, O^T += V^T P^T (32 contraction bytes per lane), so P never leaves registers: the
// cast packs the lane's 32 probabilities into 8 dwords.  The order in which those bytes list the
// keys is a permutation of 0..63, and the V^T fragments are gathered from LDS in the same order
// with the byte-transposing read (ds_read_b64_tr_b8) from the row-major V tile.
// Row statistics are per lane (a lane owns one query) plus one exchange with lane ^ 32.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int BQ = 128;        // queries per workgroup
constexpr int BKV = 64;        // keys per step
constexpr int HD = 128;        // head dimension
constexpr int K_BYTES = BKV * HD;            // K tile, 16-byte chunks swizzled by (row & 7)
constexpr int V_STRIDE = HD + 16;            // V tile row stride (padding spreads the transposing reads over banks)
constexpr int V_BYTES = BKV * V_STRIDE;
constexpr int STAGE = K_BYTES + V_BYTES;

typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

struct FwdArgs {
  const uint8_t* Q; const uint8_t* K; const uint8_t* V;
  const float* sinv_q; const float* sinv_k; const float* sinv_v; const float* scale_p;
  uint16_t* O; float* lse; uint32_t* amax_p;
  float softmax_scale;
  int BH, S, nqb;
};

FOG_DEVICE float lane_xor32(float v) { return __shfl_xor(v, 32, 64); }

template <bool CAUSAL>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(FwdArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t smem[2 * STAGE];
  const int bh = blockIdx.x % a.BH;
  const int qb = a.nqb - 1 - blockIdx.x / a.BH;   // long rows (late query blocks) are launched first
  const int t = threadIdx.x, w = t >> 6, l = t & 63, g = l >> 5;
  const int S = a.S;
  const uint8_t* Qh = a.Q + (int64_t)bh * S * HD;
  const uint8_t* Kh = a.K + (int64_t)bh * S * HD;
  const uint8_t* Vh = a.V + (int64_t)bh * S * HD;

  const int q0 = qb * BQ + 32 * w;           // first query of this wave
  const int q = q0 + (l & 31);
  const bool wave_on = q0 < S;               // S is a multiple of 64, so a wave is all in or all out

  // Q fragments (B operand of S^T = K Q^T): row q, contraction bytes 64 h + 32 g .. + 32.
  v8i qf[2];
  {
    const uint8_t* p = Qh + (int64_t)(wave_on ? q : 0) * HD + 32 * g;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      uint4 lo = *reinterpret_cast<const uint4*>(p + 64 * h), hi = *reinterpret_cast<const uint4*>(p + 64 * h + 16);
      qf[h][0] = lo.x; qf[h][1] = lo.y; qf[h][2] = lo.z; qf[h][3] = lo.w;
      qf[h][4] = hi.x; qf[h][5] = hi.y; qf[h][6] = hi.z; qf[h][7] = hi.w;
    }
  }

  const float rho_p = *a.scale_p;
  const float lg_rho_p = __log2f(rho_p);
  const float c = a.softmax_scale * 1.44269504088896340736f * (*a.sinv_q) * (*a.sinv_k);

  // keys needed by the workgroup / by this wave
  const int kv_end_wg = CAUSAL ? min(S, qb * BQ + BQ) : S;
  const int nkb = (kv_end_wg + BKV - 1) / BKV;

  v16f o[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.0f;
  float m_run = -INFINITY;    // integer-valued row reference (log2 domain)
  float l_run = 0.0f;         // this lane's share of sum_j rho_p p_ij
  float raw_max = -INFINITY;  // this lane's share of max_j (Q K^T)_ij, before scaling

  // global -> LDS staging: 2 chunks of K and 2 of V per thread and step
  uint4 rk[2], rv[2];
  auto gload = [&](int kb) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int ch = t + kThreads * i, row = ch >> 3, cc = ch & 7;
      const int64_t off = (int64_t)(kb * BKV + row) * HD + cc * 16;
      rk[i] = *reinterpret_cast<const uint4*>(Kh + off);
      rv[i] = *reinterpret_cast<const uint4*>(Vh + off);
    }
  };
  auto swrite = [&](int stage) {
    uint8_t* sk = smem + stage * STAGE;
    uint8_t* sv = sk + K_BYTES;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int ch = t + kThreads * i, row = ch >> 3, cc = ch & 7;
      *reinterpret_cast<uint4*>(sk + row * HD + ((cc ^ (row & 7)) << 4)) = rk[i];
      *reinterpret_cast<uint4*>(sv + row * V_STRIDE + cc * 16) = rv[i];
    }
  };

  gload(0);
  swrite(0);
  __syncthreads();

  for (int kb = 0; kb < nkb; ++kb) {
    const int cur = kb & 1;
    if (kb + 1 < nkb) gload(kb + 1);
    const uint8_t* sk = smem + cur * STAGE;
    const uint8_t* sv = sk + K_BYTES;
    const int key0 = kb * BKV;
    const bool need = wave_on && (!CAUSAL || key0 <= q0 + 31);
    if (need) {
      // ---- S^T tiles: st[kt][r] = sum_d K[key][d] Q[q][d], key = key0 + 32 kt + 8 (r/4) + 4 g + (r%4)
      v16f st[2];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) st[kt][r] = 0.0f;
        const int row = 32 * kt + (l & 31);
        const uint8_t* pr = sk + row * HD;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int chunk = 4 * h + 2 * g;
          v4i lo = *reinterpret_cast<const v4i*>(pr + ((chunk ^ (row & 7)) << 4));
          v4i hi = *reinterpret_cast<const v4i*>(pr + (((chunk + 1) ^ (row & 7)) << 4));
          v8i kf;
          kf[0] = lo[0]; kf[1] = lo[1]; kf[2] = lo[2]; kf[3] = lo[3];
          kf[4] = hi[0]; kf[5] = hi[1]; kf[6] = hi[2]; kf[7] = hi[3];
          st[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[h], st[kt], 0, 0, 0, 0, 0, 0);
        }
      }
      // ---- causal mask on blocks that reach past the wave's first query
      if (CAUSAL && key0 + BKV - 1 > q0) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3);
            if (key > q) st[kt][r] = -INFINITY;
          }
      }
      // ---- running integer reference
      float bm = st[0][0];
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) bm = fmaxf(bm, st[kt][r]);
      raw_max = fmaxf(raw_max, bm);
      bm = fmaxf(bm, lane_xor32(bm));
      const float m_new = fmaxf(m_run, ceilf(bm * c));
      if (__any(m_new != m_run)) {
        const float alpha = exp2f(m_run - m_new);   // exact power of two (0 on the first block)
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
        m_run = m_new;
      }
      // ---- t = rho_p 2^(x - m), summed in binary32 and cast to E4M3; 32 codes per lane = one B operand
      const float shift = lg_rho_p - m_run;
      v8i pf;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][4 * qd + 0], c, shift));
          float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][4 * qd + 1], c, shift));
          float e2 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][4 * qd + 2], c, shift));
          float e3 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][4 * qd + 3], c, shift));
          l_run += (e0 + e1) + (e2 + e3);
          pf[4 * kt + qd] = (int)cvt4_fp8<FOG_E4M3>(e0, e1, e2, e3);
        }
      }
      // ---- O^T += V^T P^T.  Byte 4 qd' + b of dword (4 kt + qd') of pf is key
      //      key0 + 32 kt + 8 qd' + 4 g + b; the V^T fragment lists its 32 keys in the same order.
      const int i16 = l & 15;
      const int jj = i16 >> 1;                         // row this lane addresses inside a transposing read
      const int vrow = 8 * (jj >> 2) + 4 * g + (jj & 3);
      const int vcol = (l & 16) + 8 * (i16 & 1);
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        v8i vf;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v2i v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(sv + (16 * r + vrow) * V_STRIDE + 32 * d + vcol));
          vf[2 * r] = v[0];
          vf[2 * r + 1] = v[1];
        }
        o[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf, pf, o[d], 0, 0, 0, 0, 0, 0);
      }
    }
    if (kb + 1 < nkb) swrite(cur ^ 1);
    __syncthreads();
  }

  if (!wave_on) return;
  // ---- epilogue: O = sinv_v O^T / (rho_p l);  lse = m + log2 l  (l_run holds rho_p l, split over two lanes)
  const float l_tot = l_run + lane_xor32(l_run);
  const float scale_o = (*a.sinv_v) / l_tot;
  uint16_t* orow = a.O + ((int64_t)bh * S + q) * HD;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      const int col = 32 * d + 8 * qd + 4 * g;
      uint2 v = make_uint2(pack_bf16x2(o[d][4 * qd + 0] * scale_o, o[d][4 * qd + 1] * scale_o),
                           pack_bf16x2(o[d][4 * qd + 2] * scale_o, o[d][4 * qd + 3] * scale_o));
      *reinterpret_cast<uint2*>(orow + col) = v;
    }
  if (g == 0) a.lse[(int64_t)bh * S + q] = m_run + (__log2f(l_tot) - lg_rho_p);
  if (a.amax_p) {
    float rm = fmaxf(raw_max, lane_xor32(raw_max));
    float pm = exp2f(rm * c - m_run);                 // largest p of this row, in (1/2, 1]
    pm = wave_max_f32(pm);
    if (l == 0) atomicMax(a.amax_p, __float_as_uint(pm));
  }
}

__global__ void zero_u32(uint32_t* p) { *p = 0u; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" fog_status fog_fp8_attn_fwd(int B, int H, int S, int D, float softmax_scale, int causal,
                                       const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                                       const float* sinv_q, const float* sinv_k, const float* sinv_v, const float* scale_p,
                                       void* O_bf16, float* lse, float* amax_p,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (B < 0 || H < 0 || S < 0 || D < 0) return FOG_ERR_SHAPE;
  if (!(softmax_scale > 0.0f)) return FOG_ERR_UNSUPPORTED;
  if (D != HD || S % BKV != 0) return FOG_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (amax_p) zero_u32<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_p));
  if (B == 0 || H == 0 || S == 0) return fog_launch_status();
  if (!Q || !K || !V || !sinv_q || !sinv_k || !sinv_v || !scale_p || !O_bf16 || !lse) return FOG_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O_bf16)) return FOG_ERR_ALIGN;
  if ((int64_t)B * H > 0x7FFFFF || (int64_t)B * H * ((S + BQ - 1) / BQ) > 0x7FFFFFF0) return FOG_ERR_UNSUPPORTED;
  FwdArgs a;
  a.Q = Q; a.K = K; a.V = V;
  a.sinv_q = sinv_q; a.sinv_k = sinv_k; a.sinv_v = sinv_v; a.scale_p = scale_p;
  a.O = reinterpret_cast<uint16_t*>(O_bf16); a.lse = lse; a.amax_p = reinterpret_cast<uint32_t*>(amax_p);
  a.softmax_scale = softmax_scale;
  a.BH = B * H; a.S = S; a.nqb = (S + BQ - 1) / BQ;
  const int grid = a.BH * a.nqb;
  if (causal) attn_fwd_kernel<true><<<grid, kThreads, 0, s>>>(a);
  else        attn_fwd_kernel<false><<<grid, kThreads, 0, s>>>(a);
  return fog_launch_status();
}
