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
//
// Pipeline.  K and V blocks stream from global memory straight into a 3-stage LDS ring (buffer_load ... lds), two
// blocks in flight.  A wave takes a block through scores, softmax and P V one after the other and keeps a single
// set of score registers: under 168 registers per lane, so THREE workgroups share a CU (three waves per SIMD) and one
// wave's exponentials and converts run under another's matrix instructions and LDS waits.  (Producing the next
// block's scores ahead of the softmax needs a second score set, 229 registers and two waves per SIMD: 5 % slower.)
// The softmax costs about 4 vector instructions per score (max3, fma, exp2, add, half a convert): with FP8 the
// kernel is bound by the vector ALU's issue, not by the matrix core, and every vector instruction that is not
// arithmetic (address adds, quieting moves) counts: see the notes at Stg and vmax.
#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int BQ = 128;        // queries per workgroup
constexpr int BKV = 64;        // keys per step
constexpr int HD = 128;        // head dimension
constexpr int TILE_BYTES = BKV * HD;         // 8 KB: one K or V block, 16-byte chunks swizzled (see below)
constexpr int STAGE = 2 * TILE_BYTES;        // K then V
constexpr int NSTAGE = 3;
constexpr uint32_t OOB = 0x80000000u;
template <int N> struct Stg { static constexpr int value = N; };

typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

struct FwdArgs {
  const uint8_t* Q; const uint8_t* K; const uint8_t* V;
  const float* sinv_q; const float* sinv_k; const float* sinv_v; const float* scale_p;
  uint16_t* O; float* lse; uint32_t* amax_p;
  float softmax_scale;
  int BH, S, nqb;
  int G;   // query heads per key/value head (grouped-query attention); 1 = multi-head
};

FOG_DEVICE float lane_xor32(float v) { return __shfl_xor(v, 32, 64); }
// The larger of two values as the hardware's NaN-propagating maximum (v_maximum3_f32 takes three operands).  fmaxf has
// to return the other operand when one is a NaN, and for that the compiler first passes every operand that comes
// straight from a matrix instruction or a lane exchange through a quieting max(x, x): a dozen extra vector
// instructions per key block.  On numbers the two agree; a NaN score makes its row NaN either way.
FOG_DEVICE float vmax(float a, float b) { return __builtin_elementwise_maximum(a, b); }
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
// max of a lane's value and that of lane ^ 32 (both lanes get it), exchanged inside the vector ALU
// (v_permlane32_swap: no trip through LDS in the middle of the softmax's dependency chain)
FOG_DEVICE float pair_max32(float v) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return vmax(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// LDS chunk swizzles (16-byte chunks inside a 128-byte row), applied by choosing which global chunk
// a lane of the direct load fetches.  K rows are read 32 consecutive rows at a time (same chunk):
// key (row & 7).  V rows are read by the transposing read 8 rows {r..r+3, r+8..r+11} at a time:
// key (row & 3) | ((row >> 3) & 1) << 2.
FOG_DEVICE int swz_k(int row) { return row & 7; }
FOG_DEVICE int swz_v(int row) { return (row & 3) | (((row >> 3) & 1) << 2); }

FOG_DEVICE void load_to_lds(v4i rsrc, uint32_t voff, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
               :
               : "v"(voff), "s"(rsrc), "s"(lds_addr_uniform)
               : "memory", "m0");
}
FOG_DEVICE v4i make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t b = reinterpret_cast<uint64_t>(base);
  v4i r;
  r[0] = (int)(uint32_t)b;
  r[1] = (int)((uint32_t)(b >> 32) & 0xFFFFu);
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}

template <bool CAUSAL>
__global__ __launch_bounds__(kThreads, 3) void attn_fwd_kernel(FwdArgs a) {
  __shared__ __attribute__((aligned(1024))) uint8_t smem[NSTAGE * STAGE];
  const int bh = blockIdx.x % a.BH;
  const int qb = a.nqb - 1 - blockIdx.x / a.BH;   // long rows (late query blocks) are launched first
  const int t = threadIdx.x, w = t >> 6, l = t & 63, g = l >> 5;
  const int S = a.S;
  const uint8_t* Qh = a.Q + (int64_t)bh * S * HD;
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

  // p <= 1, so 448 is the largest scale that cannot overflow E4M3.  A larger one is used as 448: it could
  // only saturate, and because p is taken against the RUNNING row reference, which of the entries saturate
  // would depend on the order in which the key blocks are visited.
  const float rho_p = fminf(*a.scale_p, 448.0f);
  const float lg_rho_p = __log2f(rho_p);
  const float c = a.softmax_scale * 1.44269504088896340736f * (*a.sinv_q) * (*a.sinv_k);

  // key blocks needed by the workgroup / by this wave
  const int kv_end_wg = CAUSAL ? min(S, qb * BQ + BQ) : S;
  const int nkb = (kv_end_wg + BKV - 1) / BKV;
  const int nkb_wave = !wave_on ? 0 : (CAUSAL ? min(nkb, (q0 + 31) / BKV + 1) : nkb);

  // ---- direct loads: 2 pieces of K and 2 of V (1 KB = 8 rows each) per wave and block
  const uint32_t head_bytes = (uint32_t)S * HD;
  const int kvh = bh / a.G;   // heads are laid out [B][H]: the G query heads of a group are consecutive and share one K/V head
  const v4i rsrc_k = make_rsrc(a.K + (int64_t)kvh * S * HD, head_bytes);
  const v4i rsrc_v = make_rsrc(a.V + (int64_t)kvh * S * HD, head_bytes);
  uint32_t off_k[2], off_v[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 8 * (2 * w + j) + (l >> 3), cpos = l & 7;
    off_k[j] = (uint32_t)(row * HD + ((cpos ^ swz_k(row)) << 4));
    off_v[j] = (uint32_t)(row * HD + ((cpos ^ swz_v(row)) << 4));
  }
  const uint32_t lds_w = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(uintptr_t)smem + 2048u * w));
  // The ring stage of a block is a compile-time constant (the loop below is unrolled over the ring), so that every LDS
  // address is a per-lane constant plus an immediate offset: a stage taken from kb at run time costs an integer add per
  // fragment read, a sixth of the loop's vector instructions.
  auto issue = [&](int kb, auto stg) {   // block kb -> stage kb % NSTAGE = stg; blocks past the end fetch zeros (keeps the wait counts uniform)
    const uint32_t adv = kb < nkb ? (uint32_t)kb * (BKV * HD) : OOB;
    const uint32_t base = lds_w + (uint32_t)decltype(stg)::value * STAGE;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      load_to_lds(rsrc_k, off_k[j] + adv, base + 1024u * j);
      load_to_lds(rsrc_v, off_v[j] + adv, base + TILE_BYTES + 1024u * j);
    }
  };

  // ---- fragment addresses (bytes inside a K / V tile), computed once
  // K (A operand of S^T): row 32 kt + (l & 31), chunks 4 h + 2 g, + 1
  uint32_t ka[2][2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = l & 31;   // + 32 kt: swizzle key unchanged
    ka[h][0] = (uint32_t)(row * HD + (((4 * h + 2 * g) ^ swz_k(row)) << 4));
    ka[h][1] = (uint32_t)(row * HD + (((4 * h + 2 * g + 1) ^ swz_k(row)) << 4));
  }
  // V^T (A operand of O^T += V^T P^T): lane p of a 16-lane block addresses row 16 r + vrow (r = read
  // number) and the 8-byte column group (p & 1) of chunk 2 d + ((l & 16) >> 4) of head-dim tile d.
  uint32_t va[4];
  {
    const int i16 = l & 15, jj = i16 >> 1;
    const int vrow = 8 * (jj >> 2) + 4 * g + (jj & 3);   // + 16 r per read: leaves the swizzle key unchanged
    const int cbase = (l & 16) >> 4;
#pragma unroll
    for (int d = 0; d < 4; ++d) va[d] = (uint32_t)(vrow * HD + (((2 * d + cbase) ^ swz_v(vrow)) << 4) + 8 * (i16 & 1));
  }

  v16f o[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.0f;
  float m_run = -INFINITY;    // integer-valued row reference (log2 domain)
  float l_run = 0.0f;         // this lane's share of sum_j rho_p p_ij
  float raw_max = -INFINITY;  // this lane's share of max_j (Q K^T)_ij, before scaling

  auto scores = [&](v16f* st, auto stg) {   // st[kt][r] = sum_d K[key][d] Q[q][d], key = 64 kb + 32 kt + 8 (r/4) + 4 g + (r%4)
    const uint8_t* sk = smem + decltype(stg)::value * STAGE;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) st[kt][r] = 0.0f;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        v4i lo = *reinterpret_cast<const v4i*>(sk + ka[h][0] + 4096 * kt);
        v4i hi = *reinterpret_cast<const v4i*>(sk + ka[h][1] + 4096 * kt);
        v8i kf;
        kf[0] = lo[0]; kf[1] = lo[1]; kf[2] = lo[2]; kf[3] = lo[3];
        kf[4] = hi[0]; kf[5] = hi[1]; kf[6] = hi[2]; kf[7] = hi[3];
        st[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(kf, qf[h], st[kt], 0, 0, 0, 0, 0, 0);
      }
    }
  };

  FOG_SETTLE(qf[0]); FOG_SETTLE(qf[1]);
  issue(0, Stg<0>{});
  issue(1, Stg<1>{});
  v16f sc[2];

  // One key block.
  auto block = [&](int kb, v16f* sc, auto stg) {
    constexpr int STG = decltype(stg)::value;
    // block kb landed (block kb + 1 may be in flight: vmcnt = 4), own LDS reads done (lgkmcnt = 0)
    __builtin_amdgcn_s_waitcnt(0x0074);
    __syncthreads();
    issue(kb + 2, Stg<(STG + 2) % NSTAGE>{});   // into the stage of block kb - 1, which every wave finished reading before the barrier
    if (kb < nkb_wave) {               // this wave needs the block: scores, softmax, P V
      scores(sc, stg);
      const int key0 = kb * BKV;
      if (CAUSAL && key0 + BKV - 1 > q0) {   // causal mask on blocks that reach past the wave's first query
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3);
            if (key > q) sc[kt][r] = -INFINITY;
          }
      }
      float cm[4];   // four independent chains of eight scores (one chain of 32 is latency-bound)
#pragma unroll
      for (int ch = 0; ch < 4; ++ch) {
        const v16f& x = sc[ch >> 1];
        const int b = 8 * (ch & 1);
        float m = vmax(vmax(x[b], x[b + 1]), x[b + 2]);
        m = vmax(vmax(m, x[b + 3]), x[b + 4]);
        m = vmax(vmax(m, x[b + 5]), x[b + 6]);
        cm[ch] = vmax(m, x[b + 7]);
      }
      float bm = vmax(vmax(vmax(cm[0], cm[1]), cm[2]), cm[3]);
      raw_max = vmax(raw_max, bm);
      bm = pair_max32(bm);
      const float m_new = vmax(m_run, ceilf(bm * c));
      if (__any(m_new != m_run)) {
        const float alpha = exp2f(m_run - m_new);   // exact power of two (0 on the first block)
        l_run *= alpha;
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
        m_run = m_new;
      }
      // t = rho_p 2^(x - m) <= 448 (1 + eps): summed in binary32 and cast to E4M3 (no clamp needed: values
      // up to 464 round to 448); 32 codes per lane = one B operand.
      const float shift = lg_rho_p - m_run;
      v8i pf;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 0], c, shift));
          const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 1], c, shift));
          const float e2 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 2], c, shift));
          const float e3 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[kt][4 * qd + 3], c, shift));
          l_run += (e0 + e1) + (e2 + e3);
          uint32_t pk = __builtin_amdgcn_cvt_pk_fp8_f32(e0, e1, any_u32(), false);
          pf[4 * kt + qd] = (int)__builtin_amdgcn_cvt_pk_fp8_f32(e2, e3, pk, true);
        }
      }
      // O^T += V^T P^T.  Byte 4 qd' + b of dword (4 kt + qd') of pf is key key0 + 32 kt + 8 qd' + 4 g + b;
      // the V^T fragment lists its 32 keys in the same order (read r covers rows 16 r + vrow).
      const uint8_t* sv = smem + STG * STAGE + TILE_BYTES;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        v8i vf;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          v2i v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(sv + va[d] + 16 * r * HD));
          vf[2 * r] = v[0];
          vf[2 * r + 1] = v[1];
        }
        o[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vf, pf, o[d], 0, 0, 0, 0, 0, 0);
      }
    }
  };
  static_assert(NSTAGE == 3, "the loop is unrolled over a ring of three stages");
  int kb = 0;
  for (; kb + NSTAGE <= nkb; kb += NSTAGE) {
    block(kb, sc, Stg<0>{});
    block(kb + 1, sc, Stg<1>{});
    block(kb + 2, sc, Stg<2>{});
  }
  if (kb < nkb) {
    block(kb, sc, Stg<0>{});
    if (kb + 1 < nkb) block(kb + 1, sc, Stg<1>{});
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no direct load may still be writing LDS when the workgroup retires

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
    // every wave of the launch ends here: only a wave that would raise the maximum pays for the atomic (a stale read can
    // only be too small, which costs an atomic that changes nothing)
    if (l == 0 && __float_as_uint(pm) > __hip_atomic_load(a.amax_p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(a.amax_p, __float_as_uint(pm));
  }
}

__global__ void zero_u32(uint32_t* p) { *p = 0u; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" fog_status fog_fp8_attn_fwd(int B, int H, int H_kv, int S, int D, float softmax_scale, int causal,
                                       const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                                       const float* sinv_q, const float* sinv_k, const float* sinv_v, const float* scale_p,
                                       void* O_bf16, float* lse, float* amax_p,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (B < 0 || H < 0 || H_kv < 0 || S < 0 || D < 0) return FOG_ERR_SHAPE;
  if ((H > 0) != (H_kv > 0) || (H_kv > 0 && H % H_kv != 0)) return FOG_ERR_SHAPE;
  if (!(softmax_scale > 0.0f)) return FOG_ERR_UNSUPPORTED;
  if (D != HD || S % BKV != 0) return FOG_ERR_UNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  const bool empty = B == 0 || H == 0 || S == 0;
  // every argument check comes before the first launch: a failing call leaves device memory untouched
  if (!empty) {
    if (!Q || !K || !V || !sinv_q || !sinv_k || !sinv_v || !scale_p || !O_bf16 || !lse) return FOG_ERR_NULL;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O_bf16)) return FOG_ERR_ALIGN;
    if ((int64_t)S * HD >= 0x7FFFFFFF) return FOG_ERR_UNSUPPORTED;
    if ((int64_t)B * H > 0x7FFFFF || (int64_t)B * H * ((S + BQ - 1) / BQ) > 0x7FFFFFF0) return FOG_ERR_UNSUPPORTED;
  }
  if (amax_p) zero_u32<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_p));
  if (empty) return fog_launch_status();
  FwdArgs a;
  a.Q = Q; a.K = K; a.V = V;
  a.sinv_q = sinv_q; a.sinv_k = sinv_k; a.sinv_v = sinv_v; a.scale_p = scale_p;
  a.O = reinterpret_cast<uint16_t*>(O_bf16); a.lse = lse; a.amax_p = reinterpret_cast<uint32_t*>(amax_p);
  a.softmax_scale = softmax_scale;
  a.BH = B * H; a.S = S; a.nqb = (S + BQ - 1) / BQ;
  a.G = H / H_kv;
  const int grid = a.BH * a.nqb;
  if (causal) attn_fwd_kernel<true><<<grid, kThreads, 0, s>>>(a);
  else        attn_fwd_kernel<false><<<grid, kThreads, 0, s>>>(a);
  return fog_launch_status();
}
