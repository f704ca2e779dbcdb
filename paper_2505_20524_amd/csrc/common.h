// Device-side helpers shared by the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/fog.h"

typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

#define FOG_DEVICE static __device__ __forceinline__

// bf16 bit pattern (low 16 bits) -> float, exact.
FOG_DEVICE float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
FOG_DEVICE float bf16hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// float -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN).
FOG_DEVICE uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
FOG_DEVICE uint32_t pack_bf16x2(float lo, float hi) { return f32_to_bf16(lo) | (f32_to_bf16(hi) << 16); }

// A register whose contents do not matter.  The packed FP8 converts write one half of their destination and keep the
// other; a dword that both halves of are about to be written needs no initial value, and a literal 0 would cost a move.
FOG_DEVICE uint32_t any_u32() {
  uint32_t r;
  asm volatile("" : "=v"(r));
  return r;
}

// Saturating round-to-nearest-even cast of four floats to one dword of FP8 codes (byte i <- v_i).
// The hardware convert rounds to nearest even but turns overflow into NaN / infinity, so the
// magnitude is clamped to the largest finite value first.
template <int FMT>
FOG_DEVICE uint32_t cvt4_fp8(float a, float b, float c, float d) {
  uint32_t r = any_u32();
  if (FMT == FOG_E4M3) {
    const float mx = 448.0f;
    a = __builtin_amdgcn_fmed3f(a, -mx, mx); b = __builtin_amdgcn_fmed3f(b, -mx, mx);
    c = __builtin_amdgcn_fmed3f(c, -mx, mx); d = __builtin_amdgcn_fmed3f(d, -mx, mx);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, r, false);
    r = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, r, true);
  } else {
    const float mx = 57344.0f;
    a = __builtin_amdgcn_fmed3f(a, -mx, mx); b = __builtin_amdgcn_fmed3f(b, -mx, mx);
    c = __builtin_amdgcn_fmed3f(c, -mx, mx); d = __builtin_amdgcn_fmed3f(d, -mx, mx);
    r = __builtin_amdgcn_cvt_pk_bf8_f32(a, b, r, false);
    r = __builtin_amdgcn_cvt_pk_bf8_f32(c, d, r, true);
  }
  return r;
}

// The same cast for tensors that may hold NaN (the bulk casts): the clamp above returns the smallest of
// its operands for a NaN input, i.e. the largest finite code with a minus sign, so NaN inputs are patched
// afterwards to the NaN code 0x7F with the input's sign.  Infinities saturate through the clamp.  The test
// costs two unordered compares per four values; the patch runs only in waves that hold a NaN.
template <int FMT>
FOG_DEVICE uint32_t cvt4_fp8_nan(float a, float b, float c, float d, bool* saw_nan = nullptr) {
  uint32_t r = cvt4_fp8<FMT>(a, b, c, d);
  if (__builtin_expect(__builtin_isunordered(a, b) || __builtin_isunordered(c, d), 0)) {
    if (saw_nan) *saw_nan = true;
    if (a != a) r = (r & 0xFFFFFF00u) | 0x0000007Fu | ((__float_as_uint(a) >> 24) & 0x00000080u);
    if (b != b) r = (r & 0xFFFF00FFu) | 0x00007F00u | ((__float_as_uint(b) >> 16) & 0x00008000u);
    if (c != c) r = (r & 0xFF00FFFFu) | 0x007F0000u | ((__float_as_uint(c) >> 8) & 0x00800000u);
    if (d != d) r = (r & 0x00FFFFFFu) | 0x7F000000u | (__float_as_uint(d) & 0x80000000u);
  }
  return r;
}

// Bit pattern of a thread's running abs-max (a non-negative float, kept with fmaxf, which drops NaN
// operands) for the integer reductions that follow: a thread that saw a NaN contributes the NaN pattern,
// which orders above every finite value and infinity, so a diverged tensor shows in the abs-max.
FOG_DEVICE uint32_t amax_bits(float m, bool saw_nan) { return saw_nan ? 0x7FC00000u : __float_as_uint(m); }

// Wave-wide (64 lanes) reductions through cross-lane shuffles.
FOG_DEVICE uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    uint32_t t = (uint32_t)__shfl_xor((int)v, o, 64);
    v = v > t ? v : t;
  }
  return v;
}
FOG_DEVICE float wave_max_f32(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
FOG_DEVICE float wave_sum_f32(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// max over the magnitudes of the two bf16 halves of each dword, kept as packed u16 pairs.
FOG_DEVICE uint32_t pkmax_abs_bf16(uint32_t acc, uint32_t w) {
  us2 a = __builtin_bit_cast(us2, acc);
  us2 b = __builtin_bit_cast(us2, w & 0x7FFF7FFFu);
  us2 m = __builtin_elementwise_max(a, b);
  return __builtin_bit_cast(uint32_t, m);
}

// Streaming (non-temporal) 16- and 8-byte global accesses: data touched once should not evict
// what other kernels keep in cache.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
FOG_DEVICE uint4 ld_nt16(const void* p) {
  u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(v[0], v[1], v[2], v[3]);
}
FOG_DEVICE void st_nt16(void* p, uint4 v) {
  u32x4 w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(p));
}
FOG_DEVICE void st_nt8(void* p, uint2 v) {
  u32x2 w = {v.x, v.y};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x2*>(p));
}

// Makes the compiler treat `v` as used here.  Kernels that stream tiles into LDS with direct loads
// issued from inline assembly wait for those loads with explicit s_waitcnt immediates; the
// compiler does not see them, so any ordinary global load still "outstanding" in its bookkeeping
// when the loop starts would make it put s_waitcnt vmcnt(0) inside the loop (where the value is
// first used), which also waits for the whole prefetch stream.  Using every such value once
// before the first direct load moves that wait in front of the loop.
#define FOG_SETTLE(v) asm volatile("" ::"v"(v))
