// Scaled FP8 GEMM for gfx950:  C = sinvA * sinvB * (decode(A) x decode(B)),  binary32 accumulate, bf16 out
// (the end-to-end FP8 product of Appendix E of the paper), in the three layouts a linear layer
// needs: NT (forward), NN (data gradient), TN (weight gradient).
//
// Design: one workgroup of 4 waves owns a 256 x 256 tile of C and walks K in steps of 128 bytes.
// Each wave owns a 128 x 128 quadrant = 4 x 4 MFMA tiles of v_mfma_f32_32x32x64_f8f6f4
// (256 accumulator registers), so every 32-byte operand fragment read from LDS feeds four MFMAs.
// Operand tiles are double buffered in LDS; the next K-step's global loads are issued before the
// current step's MFMAs and written to the other buffer afterwards (one barrier per step).
//
// Operand storage in LDS, chosen so that fragment reads are bank-conflict free:
//   * "K-contiguous" operands (A of NT/NN, B of NT): [256 rows][128 bytes], 16-byte chunks
//     XOR-swizzled with (row & 7); a lane reads its 32 contraction bytes with two 16-byte reads.
//   * "K-major" operands (B of NN, A and B of TN): [128 k][256 + 16 bytes]; a lane gathers 8
//     contraction bytes of its own column with the byte-transposing LDS read
//     (ds_read_b64_tr_b8), four of them per 32-byte fragment.
// Both give byte j of a lane's fragment the contraction index 32 * (lane / 32) + j within a
// 64-wide half step, which is what the MFMA expects of both operands.
//
// The MFMA is issued with the B fragment as first operand so that a lane ends up with four
// consecutive output columns per register quad and can store 8 bytes of bf16 at a time.
#include "common.h"
#include "launch.h"

namespace {

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int kThreads = 256;
constexpr int KC_BYTES = 256 * BK;          // K-contiguous operand tile
constexpr int KM_STRIDE = 256 + 16;         // K-major operand tile row stride
constexpr int KM_BYTES = BK * KM_STRIDE;
constexpr int OPERAND_BYTES = KM_BYTES;     // slot size (the larger of the two)
constexpr int STAGE_BYTES = 2 * OPERAND_BYTES;
constexpr int LDS_BYTES = 2 * STAGE_BYTES;  // 139264

struct GemmArgs {
  const uint8_t* A;
  const uint8_t* B;
  uint16_t* C;
  const float* sinv_a;
  const float* sinv_b;
  int64_t lda, ldb, ldc;
  int M, N, K;
  int tiles_m, tiles_n;
  int vec_store;  // C rows allow 8-byte stores
};

typedef __attribute__((address_space(3))) v2i* lds_v2i_ptr;

// ---- global -> registers, one K-step of one operand (8 x 16 bytes per thread) ----
// K-contiguous: tile rows are matrix rows [row0, row0+256), bytes [k0, k0+128).
FOG_DEVICE void gload_kc(const uint8_t* __restrict__ base, int64_t ld, int row0, int rows, int k0, int K, uint4* r) {
  const int t = threadIdx.x;
  const int cc = t & 7;
  const int k = k0 + cc * 16;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int row = row0 + (t >> 3) + 32 * i;
    row = row < rows ? row : rows - 1;  // clamp: rows past the edge are computed but never stored
    if (k < K)
      r[i] = *reinterpret_cast<const uint4*>(base + (int64_t)row * ld + k);
    else
      r[i] = make_uint4(0, 0, 0, 0);
  }
}
FOG_DEVICE void swrite_kc(uint8_t* lds, const uint4* r) {
  const int t = threadIdx.x;
  const int cc = t & 7;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = (t >> 3) + 32 * i;
    *reinterpret_cast<uint4*>(lds + row * BK + ((cc ^ (row & 7)) << 4)) = r[i];
  }
}
// K-major: tile rows are contraction indices [k0, k0+128), bytes are columns [col0, col0+256).
FOG_DEVICE void gload_km(const uint8_t* __restrict__ base, int64_t ld, int col0, int cols, int k0, int K, uint4* r) {
  const int t = threadIdx.x;
  const int cc = t & 15;
  const int c = col0 + cc * 16;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = k0 + (t >> 4) + 16 * i;
    if (k < K && c < cols)  // cols % 16 == 0: a chunk is inside or outside as a whole
      r[i] = *reinterpret_cast<const uint4*>(base + (int64_t)k * ld + c);
    else
      r[i] = make_uint4(0, 0, 0, 0);
  }
}
FOG_DEVICE void swrite_km(uint8_t* lds, const uint4* r) {
  const int t = threadIdx.x;
  const int cc = t & 15;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int k = (t >> 4) + 16 * i;
    *reinterpret_cast<uint4*>(lds + k * KM_STRIDE + cc * 16) = r[i];
  }
}

// ---- LDS -> MFMA operand fragment (32 rows x 64 contraction bytes; 32 bytes per lane) ----
FOG_DEVICE v8i frag_kc(const uint8_t* lds, int row_base, int h) {
  const int l = threadIdx.x & 63;
  const int row = row_base + (l & 31);
  const int chunk = 4 * h + 2 * (l >> 5);
  const uint8_t* p = lds + row * BK;
  v4i lo = *reinterpret_cast<const v4i*>(p + ((chunk ^ (row & 7)) << 4));
  v4i hi = *reinterpret_cast<const v4i*>(p + (((chunk + 1) ^ (row & 7)) << 4));
  v8i f;
  f[0] = lo[0]; f[1] = lo[1]; f[2] = lo[2]; f[3] = lo[3];
  f[4] = hi[0]; f[5] = hi[1]; f[6] = hi[2]; f[7] = hi[3];
  return f;
}
FOG_DEVICE v8i frag_km(const uint8_t* lds, int col_base, int h) {
  const int l = threadIdx.x & 63;
  const int i = l & 15;
  // Within a block of 16 lanes the transposing read hands lane i the bytes (i & 7) of the rows
  // addressed by lanes 2j + (i >> 3), j = 0..7.  Lane p therefore points at contraction row
  // kbase + p / 2 and at the 8-byte column group p % 2, which gives lane i column col + i.
  const int col = col_base + (l & 16) + 8 * (i & 1);
  const int kb = 64 * h + 32 * (l >> 5) + (i >> 1);
  v8i f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    v2i v = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(lds + (kb + 8 * r) * KM_STRIDE + col));
    f[2 * r] = v[0];
    f[2 * r + 1] = v[1];
  }
  return f;
}

template <int LAYOUT, int FA, int FB>
__global__ __launch_bounds__(kThreads) void fp8_gemm_kernel(GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr bool A_KM = LAYOUT == FOG_TN;
  constexpr bool B_KM = LAYOUT != FOG_NT;

  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Give every XCD one
  // contiguous run of tiles, walked in groups of 8 tile rows, so that the tiles resident on an
  // XCD at any time share a few A and B panels.
  const int total = g.tiles_m * g.tiles_n;
  const int per_xcd = (total + 7) >> 3;
  const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (logical >= total) return;
  constexpr int GM = 8;
  const int width = GM * g.tiles_n;
  const int group = logical / width;
  const int first_m = group * GM;
  const int gsz = (g.tiles_m - first_m) < GM ? (g.tiles_m - first_m) : GM;
  const int rem = logical - group * width;
  const int tm = first_m + rem % gsz;
  const int tn = rem / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  const int wm = (w >> 1) * 128, wn = (w & 1) * 128;

  v16f acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int nk = (g.K + BK - 1) / BK;
  uint4 ra[8], rb[8];

  auto gload = [&](int kt) {
    if (A_KM) gload_km(g.A, g.lda, m0, g.M, kt * BK, g.K, ra); else gload_kc(g.A, g.lda, m0, g.M, kt * BK, g.K, ra);
    if (B_KM) gload_km(g.B, g.ldb, n0, g.N, kt * BK, g.K, rb); else gload_kc(g.B, g.ldb, n0, g.N, kt * BK, g.K, rb);
  };
  auto swrite = [&](int stage) {
    uint8_t* sa = smem + stage * STAGE_BYTES;
    uint8_t* sb = sa + OPERAND_BYTES;
    if (A_KM) swrite_km(sa, ra); else swrite_kc(sa, ra);
    if (B_KM) swrite_km(sb, rb); else swrite_kc(sb, rb);
  };

  if (nk > 0) {
    gload(0);
    swrite(0);
  }
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) gload(kt + 1);
    const uint8_t* sa = smem + cur * STAGE_BYTES;
    const uint8_t* sb = sa + OPERAND_BYTES;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      v8i fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = A_KM ? frag_km(sa, wm + 32 * i, h) : frag_kc(sa, wm + 32 * i, h);
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[j] = B_KM ? frag_km(sb, wn + 32 * j, h) : frag_kc(sb, wn + 32 * j, h);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], acc[i][j], FB, FA, 0, 0, 0, 0);
    }
    if (kt + 1 < nk) swrite(cur ^ 1);
    __syncthreads();
  }

  // Epilogue.  With B as the first MFMA operand, lane l holds for tile (i, j), register r:
  //   row    m = m0 + wm + 32 i + (l & 31)
  //   column n = n0 + wn + 32 j + 8 (r / 4) + 4 (l / 32) + (r % 4)
  const float alpha = (*g.sinv_a) * (*g.sinv_b);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + wm + 32 * i + (l & 31);
    if (m >= g.M) continue;
    uint16_t* crow = g.C + (int64_t)m * g.ldc;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        const int n = n0 + wn + 32 * j + 8 * qd + 4 * (l >> 5);
        const float v0 = acc[i][j][4 * qd + 0] * alpha, v1 = acc[i][j][4 * qd + 1] * alpha;
        const float v2 = acc[i][j][4 * qd + 2] * alpha, v3 = acc[i][j][4 * qd + 3] * alpha;
        if (g.vec_store && n + 3 < g.N) {
          uint2 o = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
          *reinterpret_cast<uint2*>(crow + n) = o;
        } else {
          if (n + 0 < g.N) crow[n + 0] = (uint16_t)f32_to_bf16(v0);
          if (n + 1 < g.N) crow[n + 1] = (uint16_t)f32_to_bf16(v1);
          if (n + 2 < g.N) crow[n + 2] = (uint16_t)f32_to_bf16(v2);
          if (n + 3 < g.N) crow[n + 3] = (uint16_t)f32_to_bf16(v3);
        }
      }
    }
  }
}

template <int LAYOUT, int FA, int FB>
fog_status launch(const GemmArgs& g, hipStream_t s) {
  auto kern = fp8_gemm_kernel<LAYOUT, FA, FB>;
  static bool configured = false;  // per instantiation; the attribute is sticky for the process
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES) != hipSuccess)
      return FOG_ERR_HIP;
    configured = true;
  }
  const int total = g.tiles_m * g.tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  kern<<<grid, kThreads, LDS_BYTES, s>>>(g);
  return fog_launch_status();
}

template <int LAYOUT>
fog_status launch_fmt(const GemmArgs& g, int fa, int fb, hipStream_t s) {
  if (fa == FOG_E4M3) return fb == FOG_E4M3 ? launch<LAYOUT, 0, 0>(g, s) : launch<LAYOUT, 0, 1>(g, s);
  return fb == FOG_E4M3 ? launch<LAYOUT, 1, 0>(g, s) : launch<LAYOUT, 1, 1>(g, s);
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" size_t fog_fp8_gemm_workspace(fog_layout, int64_t, int64_t, int64_t) { return 0; }

extern "C" fog_status fog_fp8_gemm(fog_layout layout, int64_t M, int64_t N, int64_t K,
                                   const uint8_t* A, fog_fp8 fmtA, int64_t lda, const float* scale_inv_A,
                                   const uint8_t* B, fog_fp8 fmtB, int64_t ldb, const float* scale_inv_B,
                                   void* C_bf16, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
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
  g.vec_store = aligned(C_bf16, 8) && ldc % 4 == 0;
  hipStream_t s = (hipStream_t)stream;
  switch (layout) {
    case FOG_NT: return launch_fmt<FOG_NT>(g, fmtA, fmtB, s);
    case FOG_NN: return launch_fmt<FOG_NN>(g, fmtA, fmtB, s);
    default: return launch_fmt<FOG_TN>(g, fmtA, fmtB, s);
  }
}
