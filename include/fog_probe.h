/*
 * fog_probe.h -- measurement helpers of the benchmark, exported by the same library as the hot path
 * (include/fog.h) but NOT part of it: nothing here is called by the kernels or by a training step.
 * They measure what the GPU itself sustains, so that a kernel's fraction of the published peak can be
 * read against the fraction a register-resident loop reaches on the same operand bits.
 */
#ifndef FOG_PROBE_H_
#define FOG_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#include "fog.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Register-resident FP8 matrix-instruction loop: every wave of a grid that fills the chip (one workgroup of
 * four waves per compute unit) issues `iters` rounds of 16 independent v_mfma_f32_32x32x64_f8f6f4 (E4M3 x E4M3)
 * on operand fragments it loaded once from `operand_bytes`; nothing but the matrix cores and the register
 * file is used inside the loop.  The instruction issues every 64 cycles whatever the operands are, so the
 * rate that comes out is the clock the part sustains under that load: the operand BIT PATTERNS set the
 * power drawn and with it the clock.
 *   operand_bytes : DEVICE pointer, 65536 bytes of FP8 codes (the caller chooses the pattern: one constant,
 *                   codes of small magnitude, uniformly random bytes, ...), 16-byte aligned.
 *   iters         : rounds per wave (each 16 instructions = 16 * 131072 flop per wave).
 *   tflops        : HOST pointer, receives the achieved TFLOP/s (HIP events around the launch; the call
 *                   synchronises the stream).
 *   mfma_clock_ghz: HOST pointer or NULL, receives 64 cycles * instructions per wave / elapsed time: the clock
 *                   at which the matrix cores ran if they never idled.
 *   sink          : DEVICE pointer, 4 bytes per thread of the grid (compute units * 256 threads), receives a
 *                   checksum so that the loop cannot be optimised away.
 * Errors: NULL, SHAPE (iters < 1), ALIGN, HIP.
 */
fog_status fog_probe_mfma_rate(const uint8_t* operand_bytes, int iters, float* sink, size_t sink_bytes,
                               double* tflops, double* mfma_clock_ghz, void* stream);

/*
 * The instruction mix of the attention forward's inner loop with NO memory traffic at all: per key block and wave,
 * four score products (v_mfma_f32_32x32x64_f8f6f4 on register-resident fragments), the softmax arithmetic on the
 * lane's 32 scores (max, fused multiply-add, exp2, row-sum add, two packed FP8 converts per four values) and four
 * P V products.  Timed three ways on a grid of compute units * waves_per_simd workgroups of four waves:
 *   what = 0 : everything;   what = 1 : the eight matrix instructions only;   what = 2 : the softmax arithmetic only.
 *   what = 3 : everything, with the four P V products of the PREVIOUS block dealt out between the four groups of eight scores
 *              of this block's softmax (one matrix instruction, then eight scores' worth of vector work, order pinned): what an
 *              interleave inside the wave gains over taking the phases in turn.
 * If the matrix cores and the vector ALU overlapped perfectly, time(0) would be max(time(1), time(2)); what the part
 * does with this mix is an upper bound for any attention kernel built from these instructions.
 *   ns_per_block : HOST pointer, receives nanoseconds per key block and wave, divided by waves_per_simd (the time a SIMD
 *                  spends per wave-block).   sink : as in fog_probe_mfma_rate, compute units * waves_per_simd * 256 floats.
 * Errors: NULL, SHAPE (iters < 1, waves_per_simd outside 1..3, what outside 0..3), WORKSPACE (sink too small), HIP.
 */
fog_status fog_probe_attention_loop(int what, int waves_per_simd, int iters, float* sink, size_t sink_bytes,
                                    double* ns_per_block, void* stream);

/*
 * What a matrix instruction costs the vector ALU of its own wave.  One wave per SIMD; per trip eight independent
 * v_mfma_f32_32x32x64_f8f6f4, each followed, in pinned program order, by `vector_ops` vector operations on registers
 * of their own:
 *   op = 0 : v_fma_f32;  1 : v_exp_f32;  2 : v_cvt_pk_fp8_f32;
 *   op = 3 : a quarter of a softmax group (fma, exp, add, and a max3 or a packed convert in turn): 4 per matrix
 *            instruction is the ratio of the attention forward at head dimension 128.
 * with_mfma = 0 times the vector operations alone.  The result is shader cycles (the wave's cycle counter, averaged
 * over the workgroups) per slot = one matrix instruction plus its vector operations: 64 while the vector work hides
 * under the matrix instruction, then a line whose intercept is what the matrix instruction takes from the vector ALU.
 *   vector_ops : 0, 4, 8, 16 or 32.      cycles_per_slot : HOST pointer.
 *   sink : DEVICE pointer, 8-byte aligned, compute units * 256 floats + compute units * 8 bytes.
 * Errors: NULL, SHAPE, ALIGN, WORKSPACE, HIP.  Synchronises the stream.
 */
fog_status fog_probe_mfma_coissue(int op, int vector_ops, int with_mfma, int iters, float* sink, size_t sink_bytes,
                                  double* cycles_per_slot, void* stream);

/*
 * Whether the vector work of one wave runs under the matrix instructions of ANOTHER wave on the same SIMD.  Workgroups of
 * eight waves, one per compute unit: waves 0-3 issue nothing but independent v_mfma_f32_32x32x64_f8f6f4 (iters_matrix
 * trips of eight), waves 4-7, which share their SIMDs, nothing but the vector operations of fog_probe_mfma_coissue
 * (iters_vector trips of eight groups of `vector_ops` operations).  Each role counts its own shader cycles:
 *   matrix_cycles_per_instruction : 64 when the matrix wave is not held up;
 *   vector_cycles_per_group       : to be compared with the same call with iters_matrix = 0 (the vector waves alone).
 * With trip counts chosen so that one role outlasts the other, the shorter role is measured entirely under the longer one.
 *   op : as in fog_probe_mfma_coissue.   vector_ops : 8 or 32.   Both results are HOST pointers.
 *   sink : DEVICE pointer, 8-byte aligned, compute units * 512 floats + compute units * 16 bytes.
 * Errors: NULL, SHAPE, ALIGN, WORKSPACE, HIP.  Synchronises the stream.
 */
fog_status fog_probe_mfma_cross_wave(int op, int vector_ops, int iters_matrix, int iters_vector, float* sink, size_t sink_bytes,
                                     double* matrix_cycles_per_instruction, double* vector_cycles_per_group, void* stream);

/*
 * The NT product of fog_fp8_gemm (E4M3 x E4M3) with the epilogue of every tile left out: the same kernel, the same
 * operand loads and matrix instructions, but no tile is scaled, converted, staged or stored (C stays untouched).
 * Timed next to fog_fp8_gemm on the same operands it shows what the epilogues cost a launch, which is what a kernel
 * that hid them completely under the next tile's products could gain.  Asynchronous on `stream`, like fog_fp8_gemm.
 *   M, N multiples of 256, K of 16; pointers as for fog_fp8_gemm with C 16-byte aligned and ldc a multiple of 8.
 * Errors: SHAPE, NULL, UNSUPPORTED (sizes the fast path does not cover), ALIGN, HIP.
 */
fog_status fog_probe_gemm_products_only(int64_t M, int64_t N, int64_t K, const uint8_t* A, int64_t lda, const uint8_t* B, int64_t ldb,
                                        const float* scale_inv_A, const float* scale_inv_B, void* C_bf16, int64_t ldc, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FOG_PROBE_H_ */
