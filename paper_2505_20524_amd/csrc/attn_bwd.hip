// FP8 dot-product attention, backward (gfx950): dQ, dK, dV with all five products in FP8.
//
// The paper runs every GEMM of the block, attention included, in FP8 in both passes (abstract;
// Appendix E, FP8DPA row), with E5M2 for backward tensors (Section 2).  Per (batch, head):
//     D_i = sum_d dO_id O_id                        x_ij = s log2(e) sinv_q sinv_k (Q~ K~^T)_ij
//     P   = 2^(x - lse_i),  P~ = E4M3(rho_p P)      dV = sinv_do / rho_p (P~^T dO~)
//     dP  = sinv_do sinv_v (dO~ V~^T)               dS = P o (dP - D_i),  dS~ = E5M2(rho_ds dS)
//     dQ  = s sinv_k / rho_ds (dS~ K~)              dK = s sinv_q / rho_ds (dS~^T Q~)
//
// Three kernels.  (0) D_i, one pass over the bf16 tensors.  (1) dK/dV: a workgroup owns 128 keys
// (32 per wave) and walks the query blocks at or below its diagonal; the score tile is produced
// with lane = key, which is the B-operand shape of both dV^T += dO^T P and dK^T += Q^T dS.
// (2) dQ: a workgroup owns 128 queries and walks the key blocks, scores transposed (lane = query),
// the B-operand shape of dQ^T += K^T dS^T.  Recomputing S and dP in both kernels costs two extra
// products but keeps every accumulator in registers, needs no atomics and is deterministic.
// Operands whose contraction index is their row index (dO^T, Q^T, K^T) are gathered from the
// row-major LDS tiles with the byte-transposing read, in the key/query order the packed
// probabilities have (see the forward kernel).
#include <mutex>

#include "common.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int HD = 128;
constexpr int BLK = 128;           // rows owned by a workgroup (keys in kernel 1, queries in kernel 2)
constexpr int STEP = 64;           // rows of the streamed operands per step
constexpr int TILE = STEP * HD;    // 8 KB, 16-byte chunks swizzled by swz(row)
constexpr int NSTAGE = 4;
constexpr uint32_t OOB = 0x80000000u;
// The ring stage of a block as a compile-time constant: the loops are unrolled over the ring so that every LDS address is a
// per-lane constant plus an immediate offset (a stage taken from the block number at run time costs an integer add per
// group of fragment reads).
template <int N> struct Stg { static constexpr int value = N; };

typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

struct BwdArgs {
  const uint8_t* Q; const uint8_t* K; const uint8_t* V; const uint8_t* dO8;
  const uint16_t* O; const uint16_t* dO;
  const float* sinv_q; const float* sinv_k; const float* sinv_v; const float* sinv_do;
  const float* lse; const float* scale_p; const float* scale_ds;
  uint16_t* dQ; uint16_t* dK; uint16_t* dV;
  uint32_t* amax_ds; float* Dws;
  float softmax_scale;
  int BH, S, nblk;
  int BHkv, G;   // key/value heads in all, query heads per key/value head (grouped-query attention)
};

// LDS tiles are [64 rows][128 bytes]; the 16-byte chunks of a row sit at position chunk ^ swz(row).
// The key is a Gray code of the row: it is injective on any 8 (and, per row parity, 16) consecutive
// rows (16-byte row reads of 32 consecutive rows) and on the row sets {r..r+3, r+8..r+11} that one
// byte-transposing read touches, so both kinds of fragment read are bank-conflict free.
FOG_DEVICE int swz(int row) { return (row ^ (row >> 1)) & 7; }

FOG_DEVICE void load16_to_lds(v4i rsrc, uint32_t voff, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
               :
               : "v"(voff), "s"(rsrc), "s"(__builtin_amdgcn_readfirstlane((int)lds_addr_uniform))
               : "memory", "m0");
}
FOG_DEVICE void load4_to_lds(v4i rsrc, uint32_t voff, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dword %0, %1, 0 offen lds"
               :
               : "v"(voff), "s"(rsrc), "s"(__builtin_amdgcn_readfirstlane((int)lds_addr_uniform))
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

// Per-lane byte offsets inside a tile, computed once per kernel.
struct RowFrag { uint32_t a[2][2]; };   // [h][chunk]: row (l & 31) (+ 32 per row tile: + 4096 bytes), chunks 4 h + 2 g, + 1
struct ColFrag { uint32_t a[4]; };      // [d]: transposing read 0 of head-dim tile d (+ 16 rows = 2048 bytes per read)
FOG_DEVICE RowFrag rowfrag_addr() {
  const int l = threadIdx.x & 63, g = l >> 5, row = l & 31;
  RowFrag f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    f.a[h][0] = (uint32_t)(row * HD + (((4 * h + 2 * g) ^ swz(row)) << 4));
    f.a[h][1] = (uint32_t)(row * HD + (((4 * h + 2 * g + 1) ^ swz(row)) << 4));
  }
  return f;
}
// Lane p of a 16-lane block addresses row 16 r + vrow (r = read number) and the 8-byte half (p & 1)
// of chunk 2 d + ((l & 16) >> 4); lane i of the block then receives column 32 d + (l & 16) + i of the
// rows 16 r + 8 (jj / 4) + 4 g + (jj % 4), jj = 0..7: the order in which the packed score bytes list them.
FOG_DEVICE ColFrag colfrag_addr() {
  const int l = threadIdx.x & 63, g = l >> 5, i16 = l & 15, jj = i16 >> 1;
  const int vrow = 8 * (jj >> 2) + 4 * g + (jj & 3);
  const int cbase = (l & 16) >> 4;
  ColFrag f;
#pragma unroll
  for (int d = 0; d < 4; ++d) f.a[d] = (uint32_t)(vrow * HD + (((2 * d + cbase) ^ swz(vrow)) << 4) + 8 * (i16 & 1));
  return f;
}
FOG_DEVICE v8i read_rowfrag(const uint8_t* tile, const RowFrag& f, int rt, int h) {
  v4i lo = *reinterpret_cast<const v4i*>(tile + f.a[h][0] + 4096 * rt);
  v4i hi = *reinterpret_cast<const v4i*>(tile + f.a[h][1] + 4096 * rt);
  v8i r;
  r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
  r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
  return r;
}
FOG_DEVICE v8i read_colfrag(const uint8_t* tile, const ColFrag& f, int d) {
  v8i r;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    v2i v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(tile + f.a[d] + 2048 * k));
    r[2 * k] = v[0];
    r[2 * k + 1] = v[1];
  }
  return r;
}
// Fragment of rows straight from global memory (row-major, stride HD): row, contraction bytes 64 h + 32 g.
FOG_DEVICE v8i frag_global(const uint8_t* base, int64_t row, int h) {
  const int l = threadIdx.x & 63;
  const uint8_t* p = base + row * HD + 64 * h + 32 * (l >> 5);
  uint4 lo = *reinterpret_cast<const uint4*>(p), hi = *reinterpret_cast<const uint4*>(p + 16);
  v8i f;
  f[0] = lo.x; f[1] = lo.y; f[2] = lo.z; f[3] = lo.w;
  f[4] = hi.x; f[5] = hi.y; f[6] = hi.z; f[7] = hi.w;
  return f;
}
// Direct-load offsets of a [64][128] tile: 2 pieces of 1 KB (8 rows) per wave; lane -> (row, global chunk).
FOG_DEVICE void tile_load_offsets(uint32_t* off) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int row = 8 * (2 * w + j) + (l >> 3), cpos = l & 7;
    off[j] = (uint32_t)(row * HD + ((cpos ^ swz(row)) << 4));
  }
}

FOG_DEVICE float lane_xor32(float v) { return __shfl_xor(v, 32, 64); }

// ------------------------------------------------------------------ kernel 0: per-row constants
// ws[0][row] = D_i = sum_d dO_id O_id                (used by the dQ kernel)
// ws[1][row] = D_i * rho_ds / rho_p                  (dK/dV kernel: its probabilities carry the factor rho_p)
// ws[2][row] = lse_i - log2 rho_p                    (dK/dV kernel: 2^(x - that) = rho_p P)
// Folding the scales into per-row constants once saves three vector instructions per score later.
__global__ __launch_bounds__(kThreads) void attn_bwd_rowdot_kernel(const uint16_t* __restrict__ O, const uint16_t* __restrict__ dO,
                                                                   const float* __restrict__ lse, const float* __restrict__ scale_p,
                                                                   const float* __restrict__ scale_ds, float* __restrict__ ws,
                                                                   int64_t rows, uint32_t* __restrict__ amax_ds) {
  // the abs-max of dS starts from 0; the kernels that raise it are launched after this one on the same stream
  if (amax_ds && blockIdx.x == 0 && threadIdx.x == 0) *amax_ds = 0u;
  const int64_t row = (int64_t)blockIdx.x * (kThreads / 16) + (threadIdx.x >> 4);
  const int part = threadIdx.x & 15;
  float s = 0.0f;
  if (row < rows) {
    uint4 a = *reinterpret_cast<const uint4*>(O + row * HD + part * 8);
    uint4 b = *reinterpret_cast<const uint4*>(dO + row * HD + part * 8);
    s = bf16lo(a.x) * bf16lo(b.x) + bf16hi(a.x) * bf16hi(b.x) + bf16lo(a.y) * bf16lo(b.y) + bf16hi(a.y) * bf16hi(b.y) +
        bf16lo(a.z) * bf16lo(b.z) + bf16hi(a.z) * bf16hi(b.z) + bf16lo(a.w) * bf16lo(b.w) + bf16hi(a.w) * bf16hi(b.w);
  }
#pragma unroll
  for (int o = 8; o >= 1; o >>= 1) s += __shfl_xor(s, o, 64);
  if (row < rows && part == 0) {
    const float rp = *scale_p, rds = *scale_ds;
    ws[row] = s;
    ws[rows + row] = s * (rds / rp);
    ws[2 * rows + row] = lse[row] - __log2f(rp);
  }
}

// Largest magnitude among the 32 values of a lane's two score tiles (NaN operands are dropped by the maximum), as four
// independent chains, and the clamp of those values to the finite range of E5M2.
FOG_DEVICE float block_absmax(const v16f* x) {
  float cm[4];
#pragma unroll
  for (int ch = 0; ch < 4; ++ch) {
    const v16f& t = x[ch >> 1];
    const int b = 8 * (ch & 1);
    float m = fmaxf(fmaxf(fabsf(t[b]), fabsf(t[b + 1])), fabsf(t[b + 2]));
    m = fmaxf(fmaxf(m, fabsf(t[b + 3])), fabsf(t[b + 4]));
    m = fmaxf(fmaxf(m, fabsf(t[b + 5])), fabsf(t[b + 6]));
    cm[ch] = fmaxf(m, fabsf(t[b + 7]));
  }
  return fmaxf(fmaxf(fmaxf(cm[0], cm[1]), cm[2]), cm[3]);
}
FOG_DEVICE void clamp_block(v16f* x) {
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) x[kt][r] = __builtin_amdgcn_fmed3f(x[kt][r], -57344.0f, 57344.0f);
}

// ------------------------------------------------------------------ kernel 1: dK, dV
// Ring stage: Q tile, dO tile, then 64 lse and 64 D values.  Five direct loads per thread and stage.
constexpr int KV_STAGE = 2 * TILE + 512;
// MODE 0 produces dK and dV together (one wave per SIMD: 128 accumulator registers for the outputs plus
// double-buffered score tiles); MODE 1 produces dV only and MODE 2 dK only, each with 64 accumulator
// registers and no score prefetch, so that two workgroups share a CU and one's exponentials and casts
// run under the other's matrix instructions.  The pair 1 + 2 recomputes S once more than MODE 0 and is
// still the faster route (same results: the arithmetic per output is identical).
template <bool CAUSAL, int MODE>
__global__ __launch_bounds__(kThreads, MODE == 0 ? 1 : 2) void attn_bwd_dkdv_kernel(BwdArgs a) {
  constexpr bool WANT_DV = MODE != 2, WANT_DK = MODE != 1, PREFETCH = MODE == 0;
  __shared__ __attribute__((aligned(1024))) uint8_t smem[NSTAGE * KV_STAGE];
  const int bhk = blockIdx.x % a.BHkv;                 // key/value head; its query heads are bhk * G .. + G - 1
  const int kblk = blockIdx.x / a.BHkv;                // early key blocks see the most queries: launched first
  const int t = threadIdx.x, w = t >> 6, l = t & 63, g = l >> 5;
  const int S = a.S, G = a.G;
  const int64_t hoff = (int64_t)bhk * S;               // rows of this K/V head
  const int64_t qoff = hoff * G;                       // first row of the group's first query head
  const int key0 = kblk * BLK + 32 * w;
  const int key = key0 + (l & 31);
  const bool wave_on = key0 < S;

  v8i kf[2], vf[2];                                    // this wave's 32 keys, both halves of d
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    kf[h] = frag_global(a.K + hoff * HD, wave_on ? key : 0, h);
    if (WANT_DK) vf[h] = frag_global(a.V + hoff * HD, wave_on ? key : 0, h);
  }
  const float rho_p = *a.scale_p, rho_ds = *a.scale_ds;
  const float c = a.softmax_scale * 1.44269504088896340736f * (*a.sinv_q) * (*a.sinv_k);
  const float cdpk = (*a.sinv_do) * (*a.sinv_v) * (rho_ds / rho_p);   // dP scale times rho_ds / rho_p
  const bool clamp_p = !(rho_p <= 448.0f);   // rho_p P <= rho_p: the cast of P can only overflow for a scale above the format's maximum

  v16f dv[4], dk[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if (WANT_DV) dv[d][r] = 0.0f;
      if (WANT_DK) dk[d][r] = 0.0f;
    }

  const int qb_first = CAUSAL ? (kblk * BLK) / STEP : 0;
  const int nqb = S / STEP - qb_first;                 // query blocks of one head this workgroup walks
  const int total = nqb * G;                           // ... and of the whole group: head after head, one stream
  // first block (relative, within a head) this wave needs: blocks whose last query is below the wave's first key are skipped
  const int skip = !wave_on ? nqb : (CAUSAL ? max(0, key0 / STEP - qb_first) : 0);

  const uint32_t group_bytes = (uint32_t)G * S * HD;
  const v4i rsrc_q = make_rsrc(a.Q + qoff * HD, group_bytes), rsrc_do = make_rsrc(a.dO8 + qoff * HD, group_bytes);
  const int64_t nrows = (int64_t)a.BH * S;
  const v4i rsrc_lse = make_rsrc(a.Dws + 2 * nrows + qoff, (uint32_t)G * S * 4), rsrc_d = make_rsrc(a.Dws + nrows + qoff, (uint32_t)G * S * 4);
  uint32_t off[2];
  tile_load_offsets(off);
  const uint32_t lds0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)smem);
  const uint32_t lds_w = lds0 + 2048u * (uint32_t)__builtin_amdgcn_readfirstlane(w);
  const bool rows_d = __builtin_amdgcn_readfirstlane(w) & 1;   // odd waves fetch D, even waves lse (two copies each: identical bytes)
  int iss_i = 0, iss_g = 0;   // query block and head of the next block to issue (issue() is called once per block, in order)
  auto issue = [&](auto stg) {  // the next block of the stream -> stage stg (= its number % 4); blocks past the end fetch zeros
    const uint32_t row0 = (uint32_t)(iss_g * S + (qb_first + iss_i) * STEP);
    const uint32_t adv = iss_g < G ? row0 * HD : OOB;
    const uint32_t radv = iss_g < G ? row0 * 4 : OOB;
    const uint32_t base = (uint32_t)decltype(stg)::value * KV_STAGE;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      load16_to_lds(rsrc_q, off[j] + adv, lds_w + base + 1024u * j);
      load16_to_lds(rsrc_do, off[j] + adv, lds_w + base + TILE + 1024u * j);
    }
    load4_to_lds(rows_d ? rsrc_d : rsrc_lse, (uint32_t)(4 * l) + radv, lds0 + base + 2 * TILE + (rows_d ? 256u : 0u));
    if (++iss_i == nqb) { iss_i = 0; ++iss_g; }
  };
  const RowFrag rf = rowfrag_addr();
  const ColFrag cf = colfrag_addr();

  // S and dP tiles with lane = key: element r of tile qt is query qbase + 32 qt + 8 (r/4) + 4 g + (r%4)
  auto scores = [&](auto stg, v16f* st, v16f* dp) {
    const uint8_t* sq = smem + decltype(stg)::value * KV_STAGE;
    const uint8_t* sdo = sq + TILE;
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        st[qt][r] = 0.0f;
        if (WANT_DK) dp[qt][r] = 0.0f;
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        st[qt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_rowfrag(sq, rf, qt, h), kf[h], st[qt], 0, 0, 0, 0, 0, 0);
        if (WANT_DK) dp[qt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_rowfrag(sdo, rf, qt, h), vf[h], dp[qt], 1, 0, 0, 0, 0, 0);
      }
    }
  };

  FOG_SETTLE(kf[0]); FOG_SETTLE(kf[1]);
  if (WANT_DK) { FOG_SETTLE(vf[0]); FOG_SETTLE(vf[1]); }
  issue(Stg<0>{});
  issue(Stg<1>{});
  issue(Stg<2>{});
  __builtin_amdgcn_s_waitcnt(0x0F7A);  // vmcnt = 10: block 0 has landed (5 direct loads per thread and block)
  __syncthreads();
  v16f sa[2], da[2], sb[2], db[2];   // without the prefetch only sa / da are used
  if (PREFETCH && skip == 0 && total > 0) scores(Stg<0>{}, sa, da);

  int cur_i = 0;
  auto block = [&](const bool CLAMP_P, auto stg, int it, v16f* st, v16f* dp, v16f* stn, v16f* dpn) __attribute__((always_inline)) {
    constexpr int STG = decltype(stg)::value;   // = it % NSTAGE
    // vmcnt = 5: block it + 1 has landed (its scores are produced during this block); without the
    // prefetch only block it is needed and two younger blocks may stay in flight (vmcnt = 10).
    // lgkmcnt = 0: own LDS reads done
    if (PREFETCH) __builtin_amdgcn_s_waitcnt(0x0075);
    else if (it > 0) __builtin_amdgcn_s_waitcnt(0x007A);
    if (PREFETCH || it > 0) __syncthreads();
    issue(Stg<(STG + 3) % NSTAGE>{});   // block it + 3
    const int i = cur_i, i_next = i + 1 == nqb ? 0 : i + 1;   // query block within its head, of this block and of the next
    cur_i = i_next;
    const bool cur = i >= skip, nxt = i_next >= skip && it + 1 < total;
    if (PREFETCH) {
      if (nxt) scores(Stg<(STG + 1) % NSTAGE>{}, stn, dpn);
    } else if (cur) {
      scores(stg, st, dp);
    }
    if (cur) {
      const uint8_t* sq = smem + STG * KV_STAGE;
      const uint8_t* sdo = sq + TILE;
      const float* srow = reinterpret_cast<const float*>(sq + 2 * TILE);   // [0..63] lse - log2 rho_p, [64..127] D rho_ds / rho_p
      const int qbase = (qb_first + i) * STEP;
      if (CAUSAL && qbase < key0 + 31) {   // diagonal blocks: queries before the key see nothing of it
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (qbase + 32 * qt + 8 * (r >> 2) + 4 * g + (r & 3) < key) st[qt][r] = -INFINITY;
      }
      v8i pf, dsf;
#pragma unroll
      for (int qt = 0; qt < 2; ++qt) {
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          const int qi = 32 * qt + 8 * qd + 4 * g;
          const float4 ls = *reinterpret_cast<const float4*>(srow + qi);
          float4 dd = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
          if (WANT_DK) dd = *reinterpret_cast<const float4*>(srow + 64 + qi);
          const float lsv[4] = {ls.x, ls.y, ls.z, ls.w}, ddv[4] = {dd.x, dd.y, dd.z, dd.w};
          float pq[4];
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const int r = 4 * qd + b;
            pq[b] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[qt][r], c, -lsv[b]));            // rho_p P
            if (WANT_DK) dp[qt][r] = pq[b] * __builtin_fmaf(dp[qt][r], cdpk, -ddv[b]);        // rho_ds dS, left in the registers of dP
          }
          if (WANT_DV) {
            if (CLAMP_P) {
              pf[4 * qt + qd] = (int)cvt4_fp8<FOG_E4M3>(pq[0], pq[1], pq[2], pq[3]);
            } else {
              uint32_t pk = __builtin_amdgcn_cvt_pk_fp8_f32(pq[0], pq[1], any_u32(), false);
              pf[4 * qt + qd] = (int)__builtin_amdgcn_cvt_pk_fp8_f32(pq[2], pq[3], pk, true);
            }
          }
        }
      }
      if (WANT_DK) {
        // the clamp before the cast of dS runs only when the block holds a magnitude above the largest finite E5M2 value
        // (see the dQ kernel); finding that out costs half an instruction per value, the clamp one
        if (__builtin_expect(__any(block_absmax(dp) > 57344.0f), 0)) clamp_block(dp);
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            const uint32_t pk = __builtin_amdgcn_cvt_pk_bf8_f32(dp[qt][4 * qd + 0], dp[qt][4 * qd + 1], any_u32(), false);
            dsf[4 * qt + qd] = (int)__builtin_amdgcn_cvt_pk_bf8_f32(dp[qt][4 * qd + 2], dp[qt][4 * qd + 3], pk, true);
          }
      }
      // dV^T += dO^T P~ ;  dK^T += Q^T dS~   (contraction over the 64 queries of this step)
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        if (WANT_DV) dv[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_colfrag(sdo, cf, d), pf, dv[d], 1, 0, 0, 0, 0, 0);
        if (WANT_DK) dk[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_colfrag(sq, cf, d), dsf, dk[d], 0, 1, 0, 0, 0, 0);
      }
    }
  };
  // The saturating form of the P cast is only needed for a scale above the format's maximum; the
  // choice is made once, outside the loop, so that the loop body stays one straight-line block.
  // four blocks per trip: the ring stage is a constant in each copy, and the score registers just swap roles
  auto trips = [&](const bool CLAMP_P) __attribute__((always_inline)) {
    for (int it = 0; it < total; it += NSTAGE) {
      block(CLAMP_P, Stg<0>{}, it, sa, da, sb, db);
      if (it + 1 < total) block(CLAMP_P, Stg<1>{}, it + 1, sb, db, sa, da);
      if (it + 2 < total) block(CLAMP_P, Stg<2>{}, it + 2, sa, da, sb, db);
      if (it + 3 < total) block(CLAMP_P, Stg<3>{}, it + 3, sb, db, sa, da);
    }
  };
  if (clamp_p) trips(true);
  else         trips(false);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no direct load may still be writing LDS when the workgroup retires
  if (!wave_on) return;
  const float sdv = (*a.sinv_do) / rho_p;
  const float sdk = a.softmax_scale * (*a.sinv_q) / rho_ds;
  uint16_t* dvrow = a.dV + (hoff + key) * HD;
  uint16_t* dkrow = a.dK + (hoff + key) * HD;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      const int col = 32 * d + 8 * qd + 4 * g;
      if (WANT_DV)
        *reinterpret_cast<uint2*>(dvrow + col) = make_uint2(pack_bf16x2(dv[d][4 * qd] * sdv, dv[d][4 * qd + 1] * sdv),
                                                            pack_bf16x2(dv[d][4 * qd + 2] * sdv, dv[d][4 * qd + 3] * sdv));
      if (WANT_DK)
        *reinterpret_cast<uint2*>(dkrow + col) = make_uint2(pack_bf16x2(dk[d][4 * qd] * sdk, dk[d][4 * qd + 1] * sdk),
                                                            pack_bf16x2(dk[d][4 * qd + 2] * sdk, dk[d][4 * qd + 3] * sdk));
    }
}

// ------------------------------------------------------------------ kernel 2: dQ (and max |dS|)
template <bool CAUSAL, bool AMAX>
__global__ __launch_bounds__(kThreads, 2) void attn_bwd_dq_kernel(BwdArgs a) {
  __shared__ __attribute__((aligned(1024))) uint8_t smem[NSTAGE * 2 * TILE];     // {K, V} x 4 stages
  const int bh = blockIdx.x % a.BH;
  const int qblk = a.nblk - 1 - blockIdx.x / a.BH;
  const int t = threadIdx.x, w = t >> 6, l = t & 63, g = l >> 5;
  const int S = a.S;
  const int64_t hoff = (int64_t)bh * S;
  const int q0 = qblk * BLK + 32 * w;
  const int q = q0 + (l & 31);
  const bool wave_on = q0 < S;

  v8i qf[2], dof[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    qf[h] = frag_global(a.Q + hoff * HD, wave_on ? q : 0, h);
    dof[h] = frag_global(a.dO8 + hoff * HD, wave_on ? q : 0, h);
  }
  const float rho_ds = *a.scale_ds;
  const float lse = (wave_on ? a.lse[hoff + q] : 0.0f) - __log2f(rho_ds);   // 2^(x - this) = rho_ds P
  const float Dq = wave_on ? a.Dws[hoff + q] : 0.0f;
  const float c = a.softmax_scale * 1.44269504088896340736f * (*a.sinv_q) * (*a.sinv_k);
  const float cdp = (*a.sinv_do) * (*a.sinv_v);

  v16f dq[4];
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[d][r] = 0.0f;
  float ds_max = 0.0f;

  const int kv_end = CAUSAL ? min(S, qblk * BLK + BLK) : S;
  const int nkb = (kv_end + STEP - 1) / STEP;
  const int nkb_wave = !wave_on ? 0 : (CAUSAL ? min(nkb, (q0 + 31) / STEP + 1) : nkb);

  const uint32_t head_bytes = (uint32_t)S * HD;
  const int64_t kvoff = (int64_t)(bh / a.G) * S;   // the G query heads of a group are consecutive and share one K/V head
  const v4i rsrc_k = make_rsrc(a.K + kvoff * HD, head_bytes), rsrc_v = make_rsrc(a.V + kvoff * HD, head_bytes);
  uint32_t off[2];
  tile_load_offsets(off);
  const uint32_t lds_w = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(uintptr_t)smem + 2048u * w));
  auto issue = [&](int kb, auto stg) {   // block kb -> stage kb % NSTAGE = stg
    const uint32_t adv = kb < nkb ? (uint32_t)kb * (STEP * HD) : OOB;
    const uint32_t base = lds_w + (uint32_t)decltype(stg)::value * (2 * TILE);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      load16_to_lds(rsrc_k, off[j] + adv, base + 1024u * j);
      load16_to_lds(rsrc_v, off[j] + adv, base + TILE + 1024u * j);
    }
  };
  const RowFrag rf = rowfrag_addr();
  const ColFrag cf = colfrag_addr();

  FOG_SETTLE(qf[0]); FOG_SETTLE(qf[1]); FOG_SETTLE(dof[0]); FOG_SETTLE(dof[1]); FOG_SETTLE(lse); FOG_SETTLE(Dq);
  issue(0, Stg<0>{});
  issue(1, Stg<1>{});
  issue(2, Stg<2>{});
  __builtin_amdgcn_s_waitcnt(0x0F78);  // vmcnt = 8: block 0 has landed (4 direct loads per thread and block)
  __syncthreads();

  auto block = [&](int kb, auto stg) __attribute__((always_inline)) {
    constexpr int STG = decltype(stg)::value;
    if (kb > 0) {
      __builtin_amdgcn_s_waitcnt(0x0078);  // vmcnt = 8: block kb landed (two younger blocks may be in flight); lgkmcnt = 0
      __syncthreads();
    }
    issue(kb + 3, Stg<(STG + 3) % NSTAGE>{});   // into the stage of block kb - 1
    if (kb >= nkb_wave) return;
    const uint8_t* sk = smem + STG * (2 * TILE);
    const uint8_t* sv = sk + TILE;
    const int kbase = kb * STEP;
    // transposed tiles, lane = query: element r of tile kt is key kbase + 32 kt + 8 (r/4) + 4 g + (r%4)
    v16f st[2], dp[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) { st[kt][r] = 0.0f; dp[kt][r] = 0.0f; }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        st[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_rowfrag(sk, rf, kt, h), qf[h], st[kt], 0, 0, 0, 0, 0, 0);
        dp[kt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_rowfrag(sv, rf, kt, h), dof[h], dp[kt], 0, 1, 0, 0, 0, 0);
      }
    }
    if (CAUSAL && kbase + STEP - 1 > q0) {   // diagonal blocks: keys after the query are masked
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (kbase + 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3) > q) st[kt][r] = -INFINITY;
    }
    // rho_ds dS = (rho_ds P) (dP - D), left in the registers of dP
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][r], c, -lse));   // rho_ds P
        dp[kt][r] = e * __builtin_fmaf(dp[kt][r], cdp, -Dq);
      }
    const float bm = block_absmax(dp);
    ds_max = fmaxf(ds_max, bm);
    // The hardware convert turns overflow into infinity, so magnitudes above the largest finite E5M2 value have to be clamped
    // first; whether any of the block's 32 values per lane needs that is known from the block maximum (which the abs-max of dS
    // wants anyway), and with a scale fitted to the tensor none does: the clamp (one instruction per value) runs only then.
    if (__builtin_expect(__any(bm > 57344.0f), 0)) clamp_block(dp);
    v8i dsf;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        const uint32_t pk = __builtin_amdgcn_cvt_pk_bf8_f32(dp[kt][4 * qd + 0], dp[kt][4 * qd + 1], any_u32(), false);
        dsf[4 * kt + qd] = (int)__builtin_amdgcn_cvt_pk_bf8_f32(dp[kt][4 * qd + 2], dp[kt][4 * qd + 3], pk, true);
      }
    // dQ^T += K^T dS~^T  (contraction over the 64 keys of this step)
#pragma unroll
    for (int d = 0; d < 4; ++d)
      dq[d] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(read_colfrag(sk, cf, d), dsf, dq[d], 0, 1, 0, 0, 0, 0);
  };
  static_assert(NSTAGE == 4, "the loops are unrolled over a ring of four stages");
  for (int kb = 0; kb < nkb; kb += NSTAGE) {
    block(kb, Stg<0>{});
    if (kb + 1 < nkb) block(kb + 1, Stg<1>{});
    if (kb + 2 < nkb) block(kb + 2, Stg<2>{});
    if (kb + 3 < nkb) block(kb + 3, Stg<3>{});
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no direct load may still be writing LDS when the workgroup retires
  if (!wave_on) return;
  const float sdq = a.softmax_scale * (*a.sinv_k) / rho_ds;
  uint16_t* dqrow = a.dQ + (hoff + q) * HD;
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      const int col = 32 * d + 8 * qd + 4 * g;
      *reinterpret_cast<uint2*>(dqrow + col) = make_uint2(pack_bf16x2(dq[d][4 * qd] * sdq, dq[d][4 * qd + 1] * sdq),
                                                          pack_bf16x2(dq[d][4 * qd + 2] * sdq, dq[d][4 * qd + 3] * sdq));
    }
  if (AMAX) {
    ds_max = wave_max_f32(ds_max) / rho_ds;   // the running maximum was taken on rho_ds dS
    // only a wave that would raise the maximum pays for the atomic (a stale read can only be too small)
    if (l == 0 && ds_max > 0.0f && __float_as_uint(ds_max) > __hip_atomic_load(a.amax_ds, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(a.amax_ds, __float_as_uint(ds_max));
  }
}

__global__ void zero_u32b(uint32_t* p) { *p = 0u; }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

extern "C" size_t fog_fp8_attn_workspace(int B, int H, int H_kv, int S, int D, int is_bwd) {
  (void)D; (void)H_kv;
  if (!is_bwd || B <= 0 || H <= 0 || S <= 0) return 0;
  return (size_t)3 * B * H * S * sizeof(float);
}

// Argument checks shared by the two entry points (everything but the workspace); FOG_OK with *empty set
// means there is nothing to compute.
static fog_status bwd_checks(int B, int H, int H_kv, int S, int D, float softmax_scale,
                             const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                             const float* sinv_q, const float* sinv_k, const float* sinv_v,
                             const void* O_bf16, const void* dO_bf16, const uint8_t* dO_e5m2, const float* sinv_do,
                             const float* lse, const float* scale_p, const float* scale_ds,
                             void* dQ_bf16, void* dK_bf16, void* dV_bf16, bool* empty) {
  *empty = false;
  if (B < 0 || H < 0 || H_kv < 0 || S < 0 || D < 0) return FOG_ERR_SHAPE;
  if ((H > 0) != (H_kv > 0) || (H_kv > 0 && H % H_kv != 0)) return FOG_ERR_SHAPE;
  if (!(softmax_scale > 0.0f)) return FOG_ERR_UNSUPPORTED;
  if (D != HD || S % STEP != 0) return FOG_ERR_UNSUPPORTED;
  if (B == 0 || H == 0 || S == 0) {
    *empty = true;
    return FOG_OK;
  }
  if (!Q || !K || !V || !sinv_q || !sinv_k || !sinv_v || !O_bf16 || !dO_bf16 || !dO_e5m2 || !sinv_do || !lse || !scale_p ||
      !scale_ds || !dQ_bf16 || !dK_bf16 || !dV_bf16)
    return FOG_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O_bf16) || !aligned16(dO_bf16) || !aligned16(dO_e5m2) ||
      !aligned16(dQ_bf16) || !aligned16(dK_bf16) || !aligned16(dV_bf16))
    return FOG_ERR_ALIGN;
  if ((int64_t)(H / H_kv) * S * HD >= 0x7FFFFFFF) return FOG_ERR_UNSUPPORTED;   // a group of query heads is one 32-bit addressed buffer
  if ((int64_t)B * H > 0x7FFFFF || (int64_t)B * H * ((S + BLK - 1) / BLK) > 0x7FFFFFF0) return FOG_ERR_UNSUPPORTED;
  return FOG_OK;
}

// The launches of the backward, on checked arguments; `ws` holds three floats per row.
static fog_status bwd_launch(int B, int H, int H_kv, int S, float softmax_scale, int causal,
                             const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                             const float* sinv_q, const float* sinv_k, const float* sinv_v,
                             const void* O_bf16, const void* dO_bf16, const uint8_t* dO_e5m2, const float* sinv_do,
                             const float* lse, const float* scale_p, const float* scale_ds,
                             void* dQ_bf16, void* dK_bf16, void* dV_bf16, float* amax_ds, float* ws, hipStream_t s) {
  BwdArgs a;
  a.Q = Q; a.K = K; a.V = V; a.dO8 = dO_e5m2;
  a.O = reinterpret_cast<const uint16_t*>(O_bf16); a.dO = reinterpret_cast<const uint16_t*>(dO_bf16);
  a.sinv_q = sinv_q; a.sinv_k = sinv_k; a.sinv_v = sinv_v; a.sinv_do = sinv_do;
  a.lse = lse; a.scale_p = scale_p; a.scale_ds = scale_ds;
  a.dQ = reinterpret_cast<uint16_t*>(dQ_bf16); a.dK = reinterpret_cast<uint16_t*>(dK_bf16); a.dV = reinterpret_cast<uint16_t*>(dV_bf16);
  a.amax_ds = reinterpret_cast<uint32_t*>(amax_ds); a.Dws = ws;
  a.softmax_scale = softmax_scale;
  a.BH = B * H; a.S = S; a.nblk = (S + BLK - 1) / BLK;
  a.BHkv = B * H_kv; a.G = H / H_kv;
  const int64_t rows = (int64_t)a.BH * S;
  attn_bwd_rowdot_kernel<<<(int)((rows + 15) / 16), kThreads, 0, s>>>(a.O, a.dO, a.lse, a.scale_p, a.scale_ds, a.Dws, rows,
                                                                      amax_ds ? a.amax_ds : nullptr);
  const int grid = a.BH * a.nblk, grid_kv = a.BHkv * a.nblk;
  // dV and dK as two launches (two workgroups per CU each) when there are enough key blocks to fill the
  // chip four times over; with few key/value heads the single combined launch balances better.
  const bool split = grid_kv >= 1024;
  if (causal) {
    if (split) {
      attn_bwd_dkdv_kernel<true, 1><<<grid_kv, kThreads, 0, s>>>(a);
      attn_bwd_dkdv_kernel<true, 2><<<grid_kv, kThreads, 0, s>>>(a);
    } else {
      attn_bwd_dkdv_kernel<true, 0><<<grid_kv, kThreads, 0, s>>>(a);
    }
  } else {
    if (split) {
      attn_bwd_dkdv_kernel<false, 1><<<grid_kv, kThreads, 0, s>>>(a);
      attn_bwd_dkdv_kernel<false, 2><<<grid_kv, kThreads, 0, s>>>(a);
    } else {
      attn_bwd_dkdv_kernel<false, 0><<<grid_kv, kThreads, 0, s>>>(a);
    }
  }
  if (causal) { if (amax_ds) attn_bwd_dq_kernel<true, true><<<grid, kThreads, 0, s>>>(a); else attn_bwd_dq_kernel<true, false><<<grid, kThreads, 0, s>>>(a); }
  else        { if (amax_ds) attn_bwd_dq_kernel<false, true><<<grid, kThreads, 0, s>>>(a); else attn_bwd_dq_kernel<false, false><<<grid, kThreads, 0, s>>>(a); }
  return fog_launch_status();
}

extern "C" fog_status fog_fp8_attn_bwd(int B, int H, int H_kv, int S, int D, float softmax_scale, int causal,
                                       const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                                       const float* sinv_q, const float* sinv_k, const float* sinv_v,
                                       const void* O_bf16, const void* dO_bf16, const uint8_t* dO_e5m2, const float* sinv_do,
                                       const float* lse, const float* scale_p, const float* scale_ds,
                                       void* dQ_bf16, void* dK_bf16, void* dV_bf16, float* amax_ds,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  bool empty;
  const fog_status st = bwd_checks(B, H, H_kv, S, D, softmax_scale, Q, K, V, sinv_q, sinv_k, sinv_v, O_bf16, dO_bf16, dO_e5m2,
                                   sinv_do, lse, scale_p, scale_ds, dQ_bf16, dK_bf16, dV_bf16, &empty);
  if (st != FOG_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if (empty) {
    if (amax_ds) zero_u32b<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_ds));
    return fog_launch_status();
  }
  if (!workspace || workspace_bytes < fog_fp8_attn_workspace(B, H, H_kv, S, D, 1) || (reinterpret_cast<uintptr_t>(workspace) & 3u))
    return FOG_ERR_WORKSPACE;
  return bwd_launch(B, H, H_kv, S, softmax_scale, causal, Q, K, V, sinv_q, sinv_k, sinv_v, O_bf16, dO_bf16, dO_e5m2, sinv_do, lse,
                    scale_p, scale_ds, dQ_bf16, dK_bf16, dV_bf16, amax_ds, reinterpret_cast<float*>(workspace), s);
}

// ------------------------------------------------------------------ the backward without a caller workspace
// For callers that cannot allocate device memory (code under HIP graph capture, serving loops, harnesses
// that forbid it): the three per-row constants live in a file-scope device array instead of a caller
// workspace.  Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends; the address is looked up once per device, with that device current, and kept.
constexpr int64_t kStaticRows = FOG_ATTN_BWD_STATIC_MAX_ROWS;          // B * H * S of a call, at most (6 MB of floats)
static __device__ __align__(256) float scratch[3 * kStaticRows];
constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices];                             // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

// Device address of this device's `scratch` (the array's name is only a host-side handle: it is never passed to a kernel).
static fog_status static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return FOG_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return FOG_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return FOG_ERR_HIP;
    }
    g_scratch_ptr[dev] = reinterpret_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return FOG_OK;
}

extern "C" fog_status fog_fp8_attn_bwd_static(int B, int H, int H_kv, int S, int D, float softmax_scale, int causal,
                                              const uint8_t* Q, const uint8_t* K, const uint8_t* V,
                                              const float* sinv_q, const float* sinv_k, const float* sinv_v,
                                              const void* O_bf16, const void* dO_bf16, const uint8_t* dO_e5m2, const float* sinv_do,
                                              const float* lse, const float* scale_p, const float* scale_ds,
                                              void* dQ_bf16, void* dK_bf16, void* dV_bf16, float* amax_ds, void* stream) {
  bool empty;
  const fog_status st = bwd_checks(B, H, H_kv, S, D, softmax_scale, Q, K, V, sinv_q, sinv_k, sinv_v, O_bf16, dO_bf16, dO_e5m2,
                                   sinv_do, lse, scale_p, scale_ds, dQ_bf16, dK_bf16, dV_bf16, &empty);
  if (st != FOG_OK) return st;
  hipStream_t s = (hipStream_t)stream;
  if (empty) {
    if (amax_ds) zero_u32b<<<1, 1, 0, s>>>(reinterpret_cast<uint32_t*>(amax_ds));
    return fog_launch_status();
  }
  if ((int64_t)B * H * S > kStaticRows) return FOG_ERR_WORKSPACE;   // larger problems take fog_fp8_attn_bwd with a caller workspace
  float* ws = nullptr;
  const fog_status sw = static_scratch(&ws);
  if (sw != FOG_OK) return sw;
  // Nothing in the array has to start at zero: the first kernel overwrites the 3 * B * H * S floats the others read.
  return bwd_launch(B, H, H_kv, S, softmax_scale, causal, Q, K, V, sinv_q, sinv_k, sinv_v, O_bf16, dO_bf16, dO_e5m2, sinv_do, lse,
                    scale_p, scale_ds, dQ_bf16, dK_bf16, dV_bf16, amax_ds, ws, s);
}
