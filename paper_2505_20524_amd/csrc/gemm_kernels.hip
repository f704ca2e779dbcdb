// Scaled FP8 GEMM for gfx950:  C = sinvA * sinvB * (decode(A) x decode(B)),  binary32 accumulate, bf16 out
// (the end-to-end FP8 product of Appendix E of the paper), in the three layouts a linear layer
// needs: NT (forward), NN (data gradient), TN (weight gradient).
//
// Design: one workgroup of 4 waves owns a 256 x 256 tile of C and walks K in steps of 64 bytes, one
// v_mfma_f32_32x32x64_f8f6f4 deep.  Each wave owns a 128 x 128 quadrant = 4 x 4 MFMA tiles (256
// accumulator registers), so every 32-byte operand fragment read from LDS feeds four MFMAs.
//
// Memory pipeline: operand tiles go from global memory straight into LDS (buffer_load ... lds, no
// register staging).  The unit of loading is a PAIR of K-steps (128 contraction bytes): every load
// instruction then covers whole 128-byte lines of the operand (8 rows x 128 bytes, or 4 contraction
// rows x 256 bytes), which halves the number of requests the vector cache sends to L2 compared with
// 64-byte row pieces; that request stream, not HBM, is what limits this kernel.  LDS holds two pair
// stages of 64 KB (32 KB per operand).  While the MFMAs of one K-step run, the fragments of the next
// are read into registers (double buffered), and during the second K-step of a pair the stage of the
// previous pair, fully read by then, is refilled with the pair after next.  Out-of-range rows,
// columns and K tails are zero-filled by the buffer bounds check.
//
// Operand storage in LDS, chosen so that the direct loads (which write 64 lanes x 16 bytes
// contiguously) and the fragment reads are both bank-conflict free:
//   * "K-contiguous" operands (A of NT/NN, B of NT): [256 rows][128 bytes]; the eight 16-byte chunks
//     of a row are XOR-swizzled with (row >> 1) & 7 by choosing which global chunk each lane fetches;
//     a lane reads the 32 contraction bytes of its K-step with two 16-byte reads.
//   * "K-major" operands (B of NN, A and B of TN): [128 k][256 bytes], the sixteen chunks of a row
//     swizzled with k & 7; a lane gathers 8 contraction bytes of its own column with the
//     byte-transposing LDS read (ds_read_b64_tr_b8), four of them per 32-byte fragment.
// Both give byte j of a lane's fragment the contraction index 32 * (lane / 32) + j of the step,
// which is what the MFMA expects of both operands.
//
// The MFMA is issued with the B fragment as first operand so that a lane ends up with four
// consecutive output columns per register quad and can store 8 bytes of bf16 at a time.
//
// Contraction split.  A launch with fewer tiles than compute units leaves the rest of the chip idle
// (the weight gradient of a 2048 x 2048 projection over 16384 tokens is 64 tiles of K = 16384).  With a
// caller workspace such a product is cut along K into `splits` chunks: the unit of work becomes
// (tile, chunk), every unit leaves its binary32 accumulators in the workspace, and a second kernel adds
// the chunks of a tile in a fixed order, applies the scales and rounds once to bf16.  Deterministic (no
// atomics); the sums differ from the unsplit kernel's only in the order of binary32 additions.
#include "common.h"
#include "launch.h"
#include "../../include/fog_probe.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int PAIR_K = 2 * BK;               // contraction bytes per load unit
constexpr int OPERAND_BYTES = 256 * PAIR_K;  // 32 KB per operand and pair stage, both storage forms
// LDS map: the two pair stages of the A operand first (64 KB), then those of B (64 KB), so that
// "stage * 32 KB + K-step half + tile row offset" of any fragment read fits the 16-bit immediate
// of the LDS instructions and one address register per operand serves both stages.
constexpr int RING_A = 0, RING_B = 2 * OPERAND_BYTES;
constexpr int RING_BYTES = 4 * OPERAND_BYTES;  // 131072
constexpr int EPI_STRIDE = 64 + 16;           // epilogue staging: 32 rows x 32 bf16, padded rows
constexpr int EPI_BUF = 32 * EPI_STRIDE;      // one staged block
constexpr int EPI_BYTES = 2 * EPI_BUF;        // per wave: two blocks
constexpr int LDS_BYTES = RING_BYTES + 4 * EPI_BYTES;  // 151552
constexpr uint32_t OOB = 0x80000000u;        // a buffer offset past any operand (spans are < 2^31 bytes)

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  uint16_t* C;
  const float* sinv_a;
  const float* sinv_b;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int tiles_m, tiles_n;
  int vec_store;  // C rows allow 16-byte stores
  int wide_store; // interior tiles are stored as whole 128-byte lines (launches of several tiles per workgroup)
  uint32_t a_bytes, b_bytes;  // addressable span of each operand
  // contraction split (splits == 1: none): work item = chunk * tiles + tile, chunk c covers
  // contraction indices [c * k_chunk, min(K, (c + 1) * k_chunk)); partial holds splits * tiles blocks
  // of 256 x 256 floats in the register order of the accumulators
  int splits, k_chunk;
  float* partial;
};

typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

// 16 bytes per lane from buffer `rsrc` at byte offset `voff` (zero when out of range) to
// LDS[m0 + 16 * lane].  Issued as inline assembly so that the compiler's own wait-count
// insertion does not serialise the LDS reads of other stages behind these loads; completion is
// awaited explicitly with s_waitcnt vmcnt + barrier in the main loop.
FOG_DEVICE void load_to_lds(v4i rsrc, uint32_t voff, uint32_t lds_addr_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, 0 offen lds"
               :
               : "v"(voff), "s"(rsrc), "s"(lds_addr_uniform)
               : "memory", "m0");
}

// Raw buffer descriptor (stride 0): 48-bit base, byte count for the bounds check, dword-format flags.
FOG_DEVICE v4i make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t b = reinterpret_cast<uint64_t>(base);
  v4i r;
  r[0] = (int)(uint32_t)b;
  r[1] = (int)((uint32_t)(b >> 32) & 0xFFFFu);
  r[2] = (int)bytes;
  r[3] = 0x00020000;
  return r;
}

// Per-thread state of one operand's direct loads.  A wave fetches 8 pieces of 1 KB per pair of
// K-steps; piece j of wave w lands at byte 8192 w + 1024 j of the operand's pair stage.  The
// swizzle makes the offsets of even and of odd pieces two arithmetic progressions, so two
// offsets and a uniform stride describe all eight.
struct LoadPlan {
  uint32_t off[2];   // byte offset of pieces 0 and 1 of the NEXT pair to issue; piece j is at
                     // off[j & 1] + (j >> 1) * stride2; >= OOB when the piece's column chunk is outside the matrix
  int klim[2];       // the chunk of piece j of the pair that starts at contraction index k0 is inside
                     // the matrix iff k0 + kdelta * j < klim[j & 1]  (kdelta: 0 K-contiguous, 4 K-major)
  int jlim;          // pieces j >= jlim lie below the last row of a K-contiguous operand
  uint32_t stride2;  // uniform: 16 rows (K-contiguous) or 8 contraction rows (K-major)
  uint32_t step;     // uniform: offset increment per pair of K-steps
};

// K-contiguous operand: piece j covers tile rows 64 w + 8 j .. + 7; lane -> (row, LDS chunk position).
// The plans cover contraction indices kb .. kb + K - 1 of the operand (a chunk of a split product, or all of it).
FOG_DEVICE LoadPlan plan_kc(int64_t ld, int row0, int rows, int kb, int K) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r8 = l >> 3, pos = l & 7;
  LoadPlan p;
  p.step = PAIR_K;
  p.stride2 = (uint32_t)(16 * ld);
  const int first = row0 + 64 * w + r8;      // global row of piece 0
  const int rem = rows - first;
  p.jlim = rem > 0 ? (rem + 7) >> 3 : 0;
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    // row = 64 w + 8 j + r8: the swizzle key (row >> 1) & 7 is (r8 >> 1) ^ 4 (j & 1)
    const int c = pos ^ (r8 >> 1) ^ (4 * par);  // global chunk that lives at LDS position pos of this row
    p.klim[par] = K - 16 * c;
    p.off[par] = (uint32_t)((int64_t)(first + 8 * par) * ld + 16 * c + kb);
  }
  return p;
}
// K-major operand: piece j covers contraction rows 32 w + 4 j .. + 3 of the pair; lane -> (k, LDS chunk position).
FOG_DEVICE LoadPlan plan_km(int64_t ld, int col0, int cols, int kb, int K) {
  const int l = threadIdx.x & 63, w = threadIdx.x >> 6;
  LoadPlan p;
  p.step = (uint32_t)(PAIR_K * ld);
  p.stride2 = (uint32_t)(8 * ld);
  p.jlim = 8;
  const int k = 32 * w + (l >> 4);            // contraction row of piece 0 within the pair
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    // k + 4 j: the swizzle key (k + 4 j) & 7 is ((l >> 4) & 7) ^ 4 (j & 1)
    const int c = (l & 15) ^ (l >> 4) ^ (4 * par);
    p.klim[par] = K - k;
    p.off[par] = (col0 + 16 * c < cols) ? (uint32_t)((int64_t)(kb + k + 4 * par) * ld + col0 + 16 * c) : OOB;  // cols % 16 == 0
  }
  return p;
}
// Issue piece j of the pair that starts at contraction index k0.  Lanes whose chunk lies at or past
// K (K tail, or pairs past the end) or below the last row fetch zeros.  Offsets that start at OOB
// stay >= OOB (spans are < 2^31 bytes).  Branch-free.
template <bool KM>
FOG_DEVICE void issue_piece(const LoadPlan& p, int j, v4i rsrc, int k0, uint32_t lds_piece_addr) {
  const bool ok = (KM || j < p.jlim) && (k0 + (KM ? 4 * j : 0) < p.klim[j & 1]);
  load_to_lds(rsrc, ok ? p.off[j & 1] + (uint32_t)(j >> 1) * p.stride2 : OOB, lds_piece_addr);
}
FOG_DEVICE void advance(LoadPlan& p) {
  p.off[0] += p.step;
  p.off[1] += p.step;
}

// ---- LDS -> MFMA operand fragments (32 rows x 64 contraction bytes; 32 bytes per lane) ----
// Per-lane byte offsets inside an operand's pair stage, computed once; tile i / read r / K-step
// half / stage are added as compile-time constants so that they fold into the instructions'
// immediate offsets.
struct FragAddr {
  uint32_t a[4];
};
// K-contiguous: a[2 h], a[2 h + 1] = the two 16-byte chunks of row (l & 31) for the K-step half h;
// row tile i adds 4096 i.
FOG_DEVICE FragAddr fragaddr_kc(int row_base) {
  const int l = threadIdx.x & 63;
  const int row = row_base + (l & 31);   // row_base is a multiple of 32: the swizzle key is tile-independent
  const int s = (row >> 1) & 7;
  FragAddr f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int c = 4 * h + 2 * (l >> 5);
    f.a[2 * h] = row * PAIR_K + ((c ^ s) << 4);
    f.a[2 * h + 1] = row * PAIR_K + (((c + 1) ^ s) << 4);
  }
  return f;
}
// K-major: a[j] = address of this lane's 8-byte piece for column tile j, read 0 of the first K-step
// of the pair; read r adds 2048 r, the second K-step adds 16384.
// Within a block of 16 lanes the transposing read hands lane i the bytes (i & 7) of the rows addressed
// by lanes 2 jj + (i >> 3), jj = 0..7.  Lane p therefore points at contraction row kbase + p / 2 and at
// the 8-byte column group p % 2, which gives lane i column col + i.
FOG_DEVICE FragAddr fragaddr_km(int col_base) {
  const int l = threadIdx.x & 63;
  const int i = l & 15;
  const int k = 32 * (l >> 5) + (i >> 1);   // + 8 r (+ 64): the swizzle key k & 7 does not depend on r
  FragAddr f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int col = col_base + 32 * j + (l & 16) + 8 * (i & 1);
    f.a[j] = k * 256 + (((col >> 4) ^ (k & 7)) << 4) + (col & 8);
  }
  return f;
}
// Fragment of row / column tile i for the K-step half h of the pair stage at `stage`.
template <bool KM>
FOG_DEVICE v8i read_frag(const uint8_t* stage, const FragAddr& fa, int i, int h) {
  v8i f;
  if (KM) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      v2i v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(stage + fa.a[i] + 16384 * h + 2048 * r));
      f[2 * r] = v[0];
      f[2 * r + 1] = v[1];
    }
  } else {
    v4i lo = *reinterpret_cast<const v4i*>(stage + fa.a[2 * h] + 4096 * i);
    v4i hi = *reinterpret_cast<const v4i*>(stage + fa.a[2 * h + 1] + 4096 * i);
    f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3];
    f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
  }
  return f;
}

// Tile order.  Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Every XCD
// owns one contiguous run of logical tile numbers and its workgroups walk that run together, so that
// the tiles in flight on an XCD at any time are neighbours (groups of 4 tile rows, column by
// column) and share a few A and B panels.
struct TileWalk {
  int first, end, stride;  // logical tile numbers of this workgroup: first, first + stride, ... < end
};
FOG_DEVICE TileWalk tile_walk(int total) {
  const int per_xcd = (total + 7) >> 3;
  const int xcd = blockIdx.x & 7, idx = blockIdx.x >> 3, n_in_xcd = gridDim.x >> 3;
  TileWalk t;
  t.first = xcd * per_xcd + idx;
  t.end = min(total, (xcd + 1) * per_xcd);
  t.stride = n_in_xcd;
  return t;
}
FOG_DEVICE void tile_origin(int logical, int tiles_m, int tiles_n, int& m0, int& n0) {
  constexpr int GM = 4;   // 4 tile rows x 8 tile columns in flight per XCD: the A panels of a group (4 x 256 rows x K) about fit its 4 MB L2
  const int width = GM * tiles_n;
  const int group = logical / width;
  const int first_m = group * GM;
  const int gsz = (tiles_m - first_m) < GM ? (tiles_m - first_m) : GM;
  const int rem = logical - group * width;
  m0 = (first_m + rem % gsz) * BM;
  n0 = (rem / gsz) * BN;
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// Two floats -> packed bf16 with the hardware convert (round to nearest even).
FOG_DEVICE uint32_t cvt_pk_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// SPLIT: the work items are (tile, contraction chunk) pairs and the epilogue leaves the binary32
// accumulators in the workspace instead of writing C (see the header comment).
// PRODUCTS_ONLY (measurement helper fog_probe_gemm_products_only, never the product path): interior tiles skip
// their epilogue, so that the launch shows what the conversion, staging and stores of the finished tiles cost.
template <int LAYOUT, int FA, int FB, bool SPLIT, bool PRODUCTS_ONLY = false>
__global__ __launch_bounds__(kThreads) void fp8_gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
  constexpr bool A_KM = LAYOUT == FOG_TN;
  constexpr bool B_KM = LAYOUT != FOG_NT;

  const int ntiles = g.tiles_m * g.tiles_n;
  const TileWalk walk = tile_walk(SPLIT ? ntiles * g.splits : ntiles);
  if (walk.first >= walk.end) return;

  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int wm = (w >> 1) * 128, wn = (w & 1) * 128;

  const v4i rsrc_a = make_rsrc(g.A, g.a_bytes), rsrc_b = make_rsrc(g.B, g.b_bytes);
  // LDS byte address of this wave's first piece in stage 0 (wave-uniform, kept in a scalar register)
  const uint32_t lds_w = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)(uintptr_t)smem + 8192u * w));
  const FragAddr fa_addr = A_KM ? fragaddr_km(wm) : fragaddr_kc(wm);
  const FragAddr fb_addr = B_KM ? fragaddr_km(wn) : fragaddr_kc(wn);
  const uint8_t* ring_a = smem + RING_A;
  const uint8_t* ring_b = smem + RING_B;
  const float alpha = (*g.sinv_a) * (*g.sinv_b);

  v16f acc[4][4];   // written by the first K-step of every tile (zero accumulator input), never cleared
  v16f zero16;
#pragma unroll
  for (int r = 0; r < 16; ++r) zero16[r] = 0.0f;

  const int nk = ((SPLIT ? g.k_chunk : g.K) + BK - 1) / BK;   // every chunk of a split takes the steps of a full chunk
  const int nk4 = (nk + 3) & ~3;  // steps are handled four at a time (two pair stages); steps past K multiply zeros
  // work item -> tile, first contraction index, number of contraction indices
  auto item_range = [&](int item, int& logical, int& kb, int& klen) {
    if (SPLIT) {
      const int c = item / ntiles;
      logical = item - c * ntiles;
      kb = c * g.k_chunk;
      klen = min(g.K - kb, g.k_chunk);
    } else {
      logical = item; kb = 0; klen = g.K;
    }
  };

#define FOG_LOAD_A(j, k0, ST) issue_piece<A_KM>(pa, j, rsrc_a, k0, lds_w + RING_A + (ST) * OPERAND_BYTES + 1024u * (j))
#define FOG_LOAD_B(j, k0, ST) issue_piece<B_KM>(pb, j, rsrc_b, k0, lds_w + RING_B + (ST) * OPERAND_BYTES + 1024u * (j))
#define FOG_ISSUE_PAIR(k0, ST)                                \
  do {                                                        \
    _Pragma("unroll") for (int j = 0; j < 8; ++j) {           \
      FOG_LOAD_A(j, k0, ST);                                  \
      FOG_LOAD_B(j, k0, ST);                                  \
    }                                                         \
    advance(pa); advance(pb);                                 \
  } while (0)
#define FOG_RA(i, ST, H) read_frag<A_KM>(ring_a + (ST) * OPERAND_BYTES, fa_addr, i, H)
#define FOG_RB(j, ST, H) read_frag<B_KM>(ring_b + (ST) * OPERAND_BYTES, fb_addr, j, H)
#define FOG_MFMA(j, FAI_, FB_, i) \
  acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(FB_[j], FAI_, acc[i][j], FB, FA, 0, 0, 0, 0)
  // first K-step of a tile: the accumulator input is the constant 0, so the 256 accumulator registers
  // never have to be cleared between tiles
#define FOG_MFMA_Z(j, FAI_, FB_, i) \
  acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(FB_[j], FAI_, zero16, FB, FA, 0, 0, 0, 0)
#define FOG_FENCE() __builtin_amdgcn_sched_barrier(0)
  // One K-step = 16 MFMAs on the fragments fetched one step earlier, dealt out with the LDS reads
  // of the next step's fragments and (second step of a pair) the 16 direct loads of the pair after
  // next; the matrix core must not idle while the wave issues them, so the order is pinned.
  // Registers: the B fragments are double buffered (FB_CUR / FB_IN); the A fragments of rows 0..2
  // are refreshed in place as soon as their row of MFMAs has been issued, only row 3 has a second
  // copy (A3_CUR / A3_IN), so that every read is issued at least three MFMAs before the step ends.
  // L(n) is the n-th of 16 load slots (empty in the first step of a pair).
#define FOG_STEP_BODY(RST, RH, FB_IN, FB_CUR, A3_IN, A3_CUR, L, MF)                                   \
  do {                                                                                             \
    FOG_FENCE(); MF(0, fa[0], FB_CUR, 0); FOG_FENCE();                                       \
    L(0); FB_IN[0] = FOG_RB(0, RST, RH);                                                           \
    FOG_FENCE(); MF(1, fa[0], FB_CUR, 0); FOG_FENCE();                                       \
    L(1);                                                                                          \
    FOG_FENCE(); MF(2, fa[0], FB_CUR, 0); FOG_FENCE();                                       \
    L(2); FB_IN[1] = FOG_RB(1, RST, RH);                                                           \
    FOG_FENCE(); MF(3, fa[0], FB_CUR, 0); FOG_FENCE();                                       \
    L(3);                                                                                          \
    FOG_FENCE(); MF(0, fa[1], FB_CUR, 1); FOG_FENCE();                                       \
    L(4); fa[0] = FOG_RA(0, RST, RH);                                                              \
    FOG_FENCE(); MF(1, fa[1], FB_CUR, 1); FOG_FENCE();                                       \
    L(5); FB_IN[2] = FOG_RB(2, RST, RH);                                                           \
    FOG_FENCE(); MF(2, fa[1], FB_CUR, 1); FOG_FENCE();                                       \
    L(6);                                                                                          \
    FOG_FENCE(); MF(3, fa[1], FB_CUR, 1); FOG_FENCE();                                       \
    L(7); FB_IN[3] = FOG_RB(3, RST, RH);                                                           \
    FOG_FENCE(); MF(0, fa[2], FB_CUR, 2); FOG_FENCE();                                       \
    L(8); fa[1] = FOG_RA(1, RST, RH);                                                              \
    FOG_FENCE(); MF(1, fa[2], FB_CUR, 2); FOG_FENCE();                                       \
    L(9); A3_IN = FOG_RA(3, RST, RH);                                                              \
    FOG_FENCE(); MF(2, fa[2], FB_CUR, 2); FOG_FENCE();                                       \
    L(10);                                                                                         \
    FOG_FENCE(); MF(3, fa[2], FB_CUR, 2); FOG_FENCE();                                       \
    L(11);                                                                                         \
    FOG_FENCE(); MF(0, A3_CUR, FB_CUR, 3); FOG_FENCE();                                      \
    L(12); fa[2] = FOG_RA(2, RST, RH);                                                             \
    FOG_FENCE(); MF(1, A3_CUR, FB_CUR, 3); FOG_FENCE();                                      \
    L(13);                                                                                         \
    FOG_FENCE(); MF(2, A3_CUR, FB_CUR, 3); FOG_FENCE();                                      \
    L(14);                                                                                         \
    FOG_FENCE(); MF(3, A3_CUR, FB_CUR, 3); FOG_FENCE();                                      \
    L(15);                                                                                         \
    FOG_FENCE();                                                                                   \
  } while (0)
#define FOG_NO_LOAD(n) do { } while (0)
  // First K-step of the pair in stage ST: the second half of that stage is read; nothing is loaded
  // and nothing in LDS changes hands, so the waves do not synchronise (the compiler's own counters
  // make each wave wait for its fragment reads).
#define FOG_STEP_FIRST(ST, FB_IN, FB_CUR, A3_IN, A3_CUR) FOG_STEP_BODY(ST, 1, FB_IN, FB_CUR, A3_IN, A3_CUR, FOG_NO_LOAD, FOG_MFMA)
#define FOG_STEP_FIRST_Z(ST, FB_IN, FB_CUR, A3_IN, A3_CUR) FOG_STEP_BODY(ST, 1, FB_IN, FB_CUR, A3_IN, A3_CUR, FOG_NO_LOAD, FOG_MFMA_Z)
  // Second K-step of the pair in stage ST.  Wait until this thread's direct loads have landed and its
  // fragment reads have returned, then synchronise: the pair in the other stage is visible to every
  // wave and stage ST, read to the end during the previous step, is free.  Its refill (the pair that
  // starts at contraction index K0_) is issued over the step, one load per MFMA, while the first
  // half of the other stage is read.  Right after an epilogue the 32 output stores of the finished
  // tile are outstanding too and younger than the loads that matter (the counter is decremented in
  // issue order), so 32 operations may stay in flight: the stores drain while the next tile computes.
  // s_waitcnt immediates: lgkmcnt = 0, expcnt unbounded, vmcnt = 0 (0x0070) or 32 (0x8070).
#define FOG_STEP_SECOND(ST, K0_, FB_IN, FB_CUR, A3_IN, A3_CUR, LAX)                               \
  do {                                                                                             \
    const int k0_ = (K0_);                                                                         \
    if (LAX) __builtin_amdgcn_s_waitcnt(0x8070);                                                   \
    else     __builtin_amdgcn_s_waitcnt(0x0070);                                                   \
    __syncthreads();                                                                               \
    FOG_STEP_BODY(1 - (ST), 0, FB_IN, FB_CUR, A3_IN, A3_CUR, FOG_L##ST, FOG_MFMA);                           \
    advance(pa); advance(pb);                                                                      \
  } while (0)
#define FOG_L0(n) do { if ((n) < 8) FOG_LOAD_A((n), k0_, 0); else FOG_LOAD_B((n) - 8, k0_, 0); } while (0)
#define FOG_L1(n) do { if ((n) < 8) FOG_LOAD_A((n), k0_, 1); else FOG_LOAD_B((n) - 8, k0_, 1); } while (0)

  // The load stream runs ahead of the MFMAs across tile boundaries: during the last four steps of a
  // tile the first two pairs of the workgroup's next tile are already being fetched, so a new tile
  // starts with its data in LDS and its first fragments in registers, and the epilogue's stores
  // drain while the next tile computes.
  int m0, n0, logical, kb, klen;
  item_range(walk.first, logical, kb, klen);
  tile_origin(logical, g.tiles_m, g.tiles_n, m0, n0);
  LoadPlan pa = A_KM ? plan_km(g.lda, m0, g.M, kb, klen) : plan_kc(g.lda, m0, g.M, kb, klen);
  LoadPlan pb = B_KM ? plan_km(g.ldb, n0, g.N, kb, klen) : plan_kc(g.ldb, n0, g.N, kb, klen);
  v8i fa[4], fa3, xb[4], yb[4];   // A fragments (row 3 twice), B fragments twice
  FOG_ISSUE_PAIR(0, 0);
  FOG_ISSUE_PAIR(PAIR_K, 1);
  __builtin_amdgcn_s_waitcnt(0x4F70);  // vmcnt = 16: the first pair has landed
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    fa[i] = FOG_RA(i, 0, 0);
    xb[i] = FOG_RB(i, 0, 0);
  }

  uint8_t* epi = smem + RING_BYTES + w * EPI_BYTES;  // this wave's private staging area
  bool stores_pending = false;                        // uniform: an epilogue's stores may still be in flight
  for (int tile = walk.first; tile < walk.end; tile += walk.stride) {
    const int m_cur = m0, n_cur = n0;
    const int next = tile + walk.stride;
    // Four K-steps (two pairs) per trip; FIRST_ is the form of the trip's first step.
#define FOG_TRIP(FIRST_)                                                                             \
  do {                                                                                               \
    if (kt == nk4 - 4) {                                                                             \
      /* last four steps of this tile: the loads issued now belong to the next tile (all zero-fill  \
         if there is none, which keeps the outstanding-load count the waits assume) */              \
      if (next < walk.end) {                                                                         \
        item_range(next, logical, kb, klen);                                                         \
        tile_origin(logical, g.tiles_m, g.tiles_n, m0, n0);                                          \
        pa = A_KM ? plan_km(g.lda, m0, g.M, kb, klen) : plan_kc(g.lda, m0, g.M, kb, klen);           \
        pb = B_KM ? plan_km(g.ldb, n0, g.N, kb, klen) : plan_kc(g.ldb, n0, g.N, kb, klen);           \
      } else {                                                                                       \
        pa.off[0] = pa.off[1] = pb.off[0] = pb.off[1] = OOB;                                         \
      }                                                                                              \
    }                                                                                                \
    /* K-step number (within its tile) of the first pair issued below */                             \
    const int ki = kt == nk4 - 4 ? 0 : kt + 4;                                                       \
    FIRST_(0, yb, xb, fa3, fa[3]);                                                                   \
    FOG_STEP_SECOND(0, ki * BK, xb, yb, fa[3], fa3, stores_pending);                                 \
    FOG_STEP_FIRST(1, yb, xb, fa3, fa[3]);                                                           \
    FOG_STEP_SECOND(1, ki * BK + PAIR_K, xb, yb, fa[3], fa3, false);                                 \
    stores_pending = false;                                                                          \
  } while (0)
    int kt = 0;
    FOG_TRIP(FOG_STEP_FIRST_Z);          // the tile's first step starts the accumulators from zero
    for (kt = 4; kt < nk4; kt += 4) FOG_TRIP(FOG_STEP_FIRST);
#undef FOG_TRIP
    // fa, xb now hold step 0 of the next tile.
    // Epilogue.  With B as the first MFMA operand, lane l holds for tile (i, j), register r:
    //   row    m = m_cur + wm + 32 i + (l & 31)
    //   column n = n_cur + wn + 32 j + 8 (r / 4) + 4 (l / 32) + (r % 4)
    // Each 32 x 32 block is scaled, converted to bf16, parked in one of the wave's two LDS staging
    // buffers (alternating, so that the next block is converted while this one is written out) and
    // stored as 16-byte pieces, four lanes per 64-byte row segment: 32 coalesced stores per lane.  The stores are
    // non-temporal: a result of 100 to 235 MB cannot stay in the caches anyway, and as ordinary stores its dirty lines
    // were written back during whatever kernel came next (the abs-max pass of the next layer ran a third slower).
    if (SPLIT) {
      // The accumulators as they are: float4 number ((w * 16 + 4 i + j) * 4 + qd) * 64 + l of this item's block,
      // i.e. 1 KB per wave and store instruction.  Waited for at once (the next item's prefetch is waited for
      // with them, as on the edge-tile path below).
      float4* dst = reinterpret_cast<float4*>(g.partial) + (int64_t)tile * (BM * BN / 4) + (w * 16) * 256 + l;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int qd = 0; qd < 4; ++qd)
            dst[((4 * i + j) * 4 + qd) * 64] = make_float4(acc[i][j][4 * qd + 0], acc[i][j][4 * qd + 1], acc[i][j][4 * qd + 2], acc[i][j][4 * qd + 3]);
      __builtin_amdgcn_s_waitcnt(0x0F70);
      continue;
    }
    const bool fast = g.vec_store != 0 && m_cur + BM <= g.M && n_cur + BN <= g.N;
    if (PRODUCTS_ONLY && fast) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) asm volatile("" ::"v"(acc[i][j]));   // the products stay, their results go nowhere
      stores_pending = false;
      continue;
    }
    const int prow = l >> 2, piece = l & 3;   // this lane's row (+ 16 t) and 16-byte piece of a staged block
    if (fast && g.wide_store) {
      // Launches in which a workgroup computes several tiles: two neighbouring 32 x 32 blocks are staged together, so that a
      // store instruction covers 8 rows of 128 bytes (whole lines of C) instead of 16 rows of 64 bytes.  One staging buffer per
      // wave (LDS operations of a wave execute in order, so refilling it needs no wait); the longer dependency chain per block
      // is hidden by the next tile's products, which is why single-tile launches keep the narrow form below.
      constexpr int WIDE = 128 + 8;   // row stride of the staged 32 x 64 block: rows 34 banks apart
      const int row8 = l >> 3, piece8 = l & 7;
      uint16_t* cbase = g.C + (int64_t)(m_cur + wm + row8) * g.ldc + (n_cur + wn + 8 * piece8);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int jp = 0; jp < 2; ++jp) {
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const int j = 2 * jp + jj;
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
              const float v0 = acc[i][j][4 * qd + 0] * alpha, v1 = acc[i][j][4 * qd + 1] * alpha;
              const float v2 = acc[i][j][4 * qd + 2] * alpha, v3 = acc[i][j][4 * qd + 3] * alpha;
              *reinterpret_cast<uint2*>(epi + (l & 31) * WIDE + 64 * jj + 16 * qd + 8 * (l >> 5)) = make_uint2(cvt_pk_bf16(v0, v1), cvt_pk_bf16(v2, v3));
            }
          }
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint2 lo = *reinterpret_cast<const uint2*>(epi + (8 * t + row8) * WIDE + 16 * piece8);
            const uint2 hi = *reinterpret_cast<const uint2*>(epi + (8 * t + row8) * WIDE + 16 * piece8 + 8);
            st_nt16(cbase + (int64_t)(32 * i + 8 * t) * g.ldc + 64 * jp, make_uint4(lo.x, lo.y, hi.x, hi.y));
          }
        }
      }
    } else if (fast) {
      uint16_t* cbase = g.C + (int64_t)(m_cur + wm + prow) * g.ldc + (n_cur + wn + 8 * piece);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint8_t* buf = epi + ((i * 4 + j) & 1) * EPI_BUF;
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            const float v0 = acc[i][j][4 * qd + 0] * alpha, v1 = acc[i][j][4 * qd + 1] * alpha;
            const float v2 = acc[i][j][4 * qd + 2] * alpha, v3 = acc[i][j][4 * qd + 3] * alpha;
            *reinterpret_cast<uint2*>(buf + (l & 31) * EPI_STRIDE + 16 * qd + 8 * (l >> 5)) = make_uint2(cvt_pk_bf16(v0, v1), cvt_pk_bf16(v2, v3));
          }
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const uint4 v = *reinterpret_cast<const uint4*>(buf + (16 * t + prow) * EPI_STRIDE + 16 * piece);
            st_nt16(cbase + (int64_t)(32 * i + 16 * t) * g.ldc + 32 * j, v);
          }
        }
      }
    } else {
      // edge tiles and unaligned C: the same staging, element-wise guarded stores
#pragma unroll
      for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint8_t* buf = epi + ((i * 4 + j) & 1) * EPI_BUF;
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            const float v0 = acc[i][j][4 * qd + 0] * alpha, v1 = acc[i][j][4 * qd + 1] * alpha;
            const float v2 = acc[i][j][4 * qd + 2] * alpha, v3 = acc[i][j][4 * qd + 3] * alpha;
            *reinterpret_cast<uint2*>(buf + (l & 31) * EPI_STRIDE + 16 * qd + 8 * (l >> 5)) = make_uint2(cvt_pk_bf16(v0, v1), cvt_pk_bf16(v2, v3));
          }
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const uint4 v = *reinterpret_cast<const uint4*>(buf + (16 * t + prow) * EPI_STRIDE + 16 * piece);
            const int m = m_cur + wm + 32 * i + 16 * t + prow;
            const int n = n_cur + wn + 32 * j + 8 * piece;
            if (m < g.M) {
              uint16_t* dst = g.C + (int64_t)m * g.ldc + n;
              const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (n + e < g.N) dst[e] = (uint16_t)(wv[e >> 1] >> (16 * (e & 1)));
            }
          }
        }
      }
    }
    stores_pending = fast;  // the slow path is only taken by edge tiles; its stores are simply waited for
    if (!fast) __builtin_amdgcn_s_waitcnt(0x0F70);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): no direct load may still be writing LDS when the workgroup retires
#undef FOG_LOAD_A
#undef FOG_LOAD_B
#undef FOG_ISSUE_PAIR
#undef FOG_RA
#undef FOG_RB
#undef FOG_MFMA
#undef FOG_MFMA_Z
#undef FOG_STEP_FIRST_Z
#undef FOG_FENCE
#undef FOG_STEP_BODY
#undef FOG_NO_LOAD
#undef FOG_STEP_FIRST
#undef FOG_STEP_SECOND
#undef FOG_L0
#undef FOG_L1
}

// C = 0 for K == 0 (no contraction): bf16 zeros.
__global__ __launch_bounds__(256) void gemm_zero_kernel(uint16_t* C, int64_t ldc, int M, int N) {
  const int64_t total = (int64_t)M * N;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256)
    C[(i / N) * ldc + (i % N)] = 0;
}

// Number of compute units of the current device (the persistent grid size), queried once per process.
int compute_units() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cus = n;
  }
  return cus;
}

// Persistent grid for `total` work items: one workgroup per compute unit (a multiple of 8 so that every XCD
// gets the same number), fewer when there are fewer items.  The launch takes ceil(total / grid) rounds
// whatever happens; the smallest grid that still needs that many rounds leaves no workgroup idle in the last
// one and, on a power-limited part, lets the busy CUs clock higher (896 tiles: 224 workgroups x 4 rounds
// instead of 256 x 3.5).
int persistent_grid(int64_t total, int* rounds_out = nullptr) {
  int grid = (compute_units() / 8) * 8;
  if (grid < 8) grid = 8;
  const int64_t rounds = (total + grid - 1) / grid;
  const int64_t need = (((total + rounds - 1) / rounds + 7) / 8) * 8;
  if (grid > need) grid = (int)need;
  if (rounds_out) *rounds_out = (int)rounds;
  return grid;
}

// Split of the contraction (1 = none) for a product of `tiles` output tiles over K, from a cost model in
// shader cycles: a K-step costs about 1100 cycles, the bf16 epilogue of a tile about 9000 (all CUs write at
// once), the binary32 one twice that, and the reduce pass moves its bytes at about 2000 per cycle plus a
// launch.  A split is only taken when the model promises a clear gain (measured: the 64-tile weight gradient of
// a 2048 x 2048 projection over 16384 tokens 131 -> 72 us, the 128-tile data gradient 4096 x 2048 over 8192 81 ->
// 74 us; a 192-tile product, which the model rejects, loses when forced: 179 -> 227 us).
struct SplitPlan { int splits, k_chunk; };
SplitPlan choose_split(int64_t M, int64_t N, int64_t K, int64_t tiles) {
  SplitPlan best{1, (int)K};
  if (tiles >= compute_units() || K < 1024) return best;
  auto cost = [&](int splits, int64_t k_chunk) {
    int rounds = 0;
    persistent_grid(tiles * splits, &rounds);
    const int64_t steps = ((k_chunk + BK - 1) / BK + 3) & ~(int64_t)3;
    double c = (double)rounds * (steps * 1100.0 + (splits > 1 ? 18000.0 : 9000.0));
    if (splits > 1) c += ((double)tiles * splits * BM * BN * 4 + 2.0 * M * N) / 2000.0 + 6000.0;
    return c;
  };
#ifndef FOG_SPLIT_MIN_GAIN
#define FOG_SPLIT_MIN_GAIN 0.93   /* a split must promise this fraction of the unsplit time, or less */
#endif
  const double unsplit = cost(1, K);
  double best_cost = unsplit * FOG_SPLIT_MIN_GAIN;
  for (int want = 2; want <= 16; ++want) {
    const int64_t k_chunk = ((K + want - 1) / want + 255) / 256 * 256;
    if (k_chunk < 512) break;
    const int splits = (int)((K + k_chunk - 1) / k_chunk);
    if (splits < 2) continue;
    const double c = cost(splits, k_chunk);
    if (c < best_cost) { best_cost = c; best = SplitPlan{splits, (int)k_chunk}; }
  }
  return best;
}

// Second pass of a split product: a workgroup owns one 32 x 32 block of C (the 256 float4 that one wave
// wrote with four consecutive store instructions), adds the chunks in ascending order, scales, rounds to
// bf16 and writes the block through LDS as 16-byte row pieces.
__global__ __launch_bounds__(256) void gemm_split_reduce_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint8_t blk[32 * EPI_STRIDE];
  const int ntiles = g.tiles_m * g.tiles_n;
  const int logical = blockIdx.x >> 6, sub = blockIdx.x & 63;     // 64 blocks of 32 x 32 per tile: sub = w * 16 + 4 i + j
  const int t = threadIdx.x, l = t & 63, qd = t >> 6;
  const float4* src = reinterpret_cast<const float4*>(g.partial) + (int64_t)logical * (BM * BN / 4) + sub * 256 + t;
  float4 acc = src[0];
  for (int c = 1; c < g.splits; ++c) {
    const float4 v = src[(int64_t)c * ntiles * (BM * BN / 4)];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  const float alpha = (*g.sinv_a) * (*g.sinv_b);
  *reinterpret_cast<uint2*>(blk + (l & 31) * EPI_STRIDE + 16 * qd + 8 * (l >> 5)) =
      make_uint2(cvt_pk_bf16(acc.x * alpha, acc.y * alpha), cvt_pk_bf16(acc.z * alpha, acc.w * alpha));
  __syncthreads();
  int m0, n0;
  tile_origin(logical, g.tiles_m, g.tiles_n, m0, n0);
  const int w = sub >> 4, i = (sub >> 2) & 3, j = sub & 3;
  const int mb = m0 + (w >> 1) * 128 + 32 * i, nb = n0 + (w & 1) * 128 + 32 * j;   // origin of the block in C
  if (t < 128) {
    const int row = t >> 2, piece = t & 3;
    const int m = mb + row, n = nb + 8 * piece;
    if (m < g.M && n < g.N) {
      const uint4 v = *reinterpret_cast<const uint4*>(blk + row * EPI_STRIDE + 16 * piece);
      uint16_t* dst = g.C + (int64_t)m * g.ldc + n;
      if (g.vec_store && n + 8 <= g.N) {
        st_nt16(dst, v);
      } else {
        const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (n + e < g.N) dst[e] = (uint16_t)(wv[e >> 1] >> (16 * (e & 1)));
      }
    }
  }
}

template <int LAYOUT, int FA, int FB>
fog_status launch(const GemmArgs& g, hipStream_t s) {
  static bool configured = false;  // per instantiation pair; the attribute is sticky for the process
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(fp8_gemm_kernel<LAYOUT, FA, FB, false>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(fp8_gemm_kernel<LAYOUT, FA, FB, true>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
      return FOG_ERR_HIP;
    configured = true;
  }
  const int64_t tiles = (int64_t)g.tiles_m * g.tiles_n;
  if (g.splits > 1) {
    fp8_gemm_kernel<LAYOUT, FA, FB, true><<<persistent_grid(tiles * g.splits), kThreads, LDS_BYTES, s>>>(g);
    gemm_split_reduce_kernel<<<(int)(tiles * 64), 256, 0, s>>>(g);
  } else {
    fp8_gemm_kernel<LAYOUT, FA, FB, false><<<persistent_grid(tiles), kThreads, LDS_BYTES, s>>>(g);
  }
  return fog_launch_status();
}

template <int LAYOUT>
fog_status launch_fmt(const GemmArgs& g, int fa, int fb, hipStream_t s) {
  if (fa == FOG_E4M3) return fb == FOG_E4M3 ? launch<LAYOUT, 0, 0>(g, s) : launch<LAYOUT, 0, 1>(g, s);
  return fb == FOG_E4M3 ? launch<LAYOUT, 1, 0>(g, s) : launch<LAYOUT, 1, 1>(g, s);
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" size_t fog_fp8_gemm_workspace(fog_layout, int64_t M, int64_t N, int64_t K) {
  if (M <= 0 || N <= 0 || K <= 0 || M > 0x7FFFFF00 || N > 0x7FFFFF00 || K > 0x7FFFFF00) return 0;
  const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  const SplitPlan sp = choose_split(M, N, K, tiles);
  return sp.splits > 1 ? (size_t)sp.splits * tiles * BM * BN * sizeof(float) : 0;
}

extern "C" fog_status fog_fp8_gemm(fog_layout layout, int64_t M, int64_t N, int64_t K,
                                   const uint8_t* A, fog_fp8 fmtA, int64_t lda, const float* scale_inv_A,
                                   const uint8_t* B, fog_fp8 fmtB, int64_t ldb, const float* scale_inv_B,
                                   void* C_bf16, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
  if (M < 0 || N < 0 || K < 0) return FOG_ERR_SHAPE;
  if (layout != FOG_NT && layout != FOG_NN && layout != FOG_TN) return FOG_ERR_UNSUPPORTED;
  if ((fmtA != FOG_E4M3 && fmtA != FOG_E5M2) || (fmtB != FOG_E4M3 && fmtB != FOG_E5M2)) return FOG_ERR_UNSUPPORTED;
  if (M == 0 || N == 0) return FOG_OK;
  if (!C_bf16 || !scale_inv_A || !scale_inv_B) return FOG_ERR_NULL;
  if (K > 0 && (!A || !B)) return FOG_ERR_NULL;
  if (M > 0x7FFFFF00 || N > 0x7FFFFF00 || K > 0x7FFFFF00) return FOG_ERR_UNSUPPORTED;
  // row lengths of the stored operands
  const int64_t a_cols = layout == FOG_TN ? M : K;
  const int64_t b_cols = layout == FOG_NT ? K : N;
  if (K > 0 && (lda < a_cols || ldb < b_cols)) return FOG_ERR_SHAPE;
  if (ldc < N) return FOG_ERR_SHAPE;
  if (K > 0 && (a_cols % 16 != 0 || b_cols % 16 != 0)) return FOG_ERR_UNSUPPORTED;
  if (K > 0 && (!aligned(A, 16) || !aligned(B, 16) || lda % 16 != 0 || ldb % 16 != 0)) return FOG_ERR_ALIGN;
  if (!aligned(C_bf16, 2)) return FOG_ERR_ALIGN;
  GemmArgs g;
  g.A = A; g.B = B; g.C = reinterpret_cast<uint16_t*>(C_bf16);
  g.sinv_a = scale_inv_A; g.sinv_b = scale_inv_B;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.M = (int)M; g.N = (int)N; g.K = (int)K;
  g.tiles_m = (int)((M + BM - 1) / BM);
  g.tiles_n = (int)((N + BN - 1) / BN);
  if ((int64_t)g.tiles_m * g.tiles_n > 0x7FFFFFF0) return FOG_ERR_UNSUPPORTED;
  g.vec_store = aligned(C_bf16, 16) && ldc % 8 == 0;
  g.wide_store = (int64_t)g.tiles_m * g.tiles_n >= 2 * (int64_t)compute_units();
  // addressable span of each operand (last row may be shorter than the leading dimension)
  const int64_t a_rows = layout == FOG_TN ? K : M, b_rows = layout == FOG_NT ? N : K;
  const int64_t a_span = K > 0 ? (a_rows - 1) * lda + a_cols : 0, b_span = K > 0 ? (b_rows - 1) * ldb + b_cols : 0;
  if (a_span >= 0x7FFFFFFF || b_span >= 0x7FFFFFFF) return FOG_ERR_UNSUPPORTED;  // 32-bit buffer offsets
  g.a_bytes = (uint32_t)a_span; g.b_bytes = (uint32_t)b_span;
  g.splits = 1; g.k_chunk = (int)K; g.partial = nullptr;
  if (K > 0 && workspace && aligned(workspace, 16)) {
    // the split the workspace query promised, when the caller brought that much
    const SplitPlan sp = choose_split(M, N, K, (int64_t)g.tiles_m * g.tiles_n);
    if (sp.splits > 1 && workspace_bytes >= (size_t)sp.splits * g.tiles_m * g.tiles_n * BM * BN * sizeof(float)) {
      g.splits = sp.splits; g.k_chunk = sp.k_chunk; g.partial = reinterpret_cast<float*>(workspace);
    }
  }
  hipStream_t s = (hipStream_t)stream;
  if (K == 0) {
    int64_t blocks = (M * N + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    gemm_zero_kernel<<<(int)blocks, 256, 0, s>>>(g.C, ldc, g.M, g.N);
    return fog_launch_status();
  }
  switch (layout) {
    case FOG_NT: return launch_fmt<FOG_NT>(g, fmtA, fmtB, s);
    case FOG_NN: return launch_fmt<FOG_NN>(g, fmtA, fmtB, s);
    default: return launch_fmt<FOG_TN>(g, fmtA, fmtB, s);
  }
}

// Measurement helper (include/fog_probe.h): the NT product of E4M3 operands with the epilogue of every tile left out.
extern "C" fog_status fog_probe_gemm_products_only(int64_t M, int64_t N, int64_t K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                                                   const float* scale_inv_A, const float* scale_inv_B, void* C_bf16, int64_t ldc, void* stream) {
  if (M <= 0 || N <= 0 || K <= 0) return FOG_ERR_SHAPE;
  if (!A || !B || !C_bf16 || !scale_inv_A || !scale_inv_B) return FOG_ERR_NULL;
  if (M % BM != 0 || N % BN != 0 || K % 16 != 0 || M > 0x7FFFFF00 || N > 0x7FFFFF00 || K > 0x7FFFFF00) return FOG_ERR_UNSUPPORTED;
  if (lda < K || ldb < K || ldc < N) return FOG_ERR_SHAPE;
  if (!aligned(A, 16) || !aligned(B, 16) || lda % 16 != 0 || ldb % 16 != 0 || !aligned(C_bf16, 16) || ldc % 8 != 0) return FOG_ERR_ALIGN;
  GemmArgs g;
  g.A = A; g.B = B; g.C = reinterpret_cast<uint16_t*>(C_bf16);
  g.sinv_a = scale_inv_A; g.sinv_b = scale_inv_B;
  g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.M = (int)M; g.N = (int)N; g.K = (int)K;
  g.tiles_m = (int)(M / BM); g.tiles_n = (int)(N / BN);
  g.vec_store = 1;
  g.wide_store = 0;
  const int64_t a_span = (M - 1) * lda + K, b_span = (N - 1) * ldb + K;
  if (a_span >= 0x7FFFFFFF || b_span >= 0x7FFFFFFF) return FOG_ERR_UNSUPPORTED;
  g.a_bytes = (uint32_t)a_span; g.b_bytes = (uint32_t)b_span;
  g.splits = 1; g.k_chunk = (int)K; g.partial = nullptr;
  static bool configured = false;
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(fp8_gemm_kernel<FOG_NT, 0, 0, false, true>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
      return FOG_ERR_HIP;
    configured = true;
  }
  fp8_gemm_kernel<FOG_NT, 0, 0, false, true><<<persistent_grid((int64_t)g.tiles_m * g.tiles_n), kThreads, LDS_BYTES, (hipStream_t)stream>>>(g);
  return fog_launch_status();
}
