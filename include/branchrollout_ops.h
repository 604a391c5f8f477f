/*
 * libbranchrollout -- op-level entry points of the velocity network, for checking
 * single kernels against a reference and for timing them in isolation.  They are
 * not part of the rollout API; conventions as in branchrollout.h.
 */
#ifndef BRANCHROLLOUT_OPS_H
#define BRANCHROLLOUT_OPS_H

#include "branchrollout.h"

#ifdef __cplusplus
extern "C" {
#endif

/* C[m, n] = epilogue(sum_k A[m, k] W[n, k] + bias[n]); A dev [M, lda], W dev [N, ldw]
 * in `dtype` (BR_F32 / BR_BF16), bias dev [N] fp32.
 *   epilogue 0: out[m, n] = acc                  out in `dtype`  [M, ldo]
 *            1: out[m, n] = gelu_tanh(acc)       out in `dtype`
 *            2: out[m, n] += gate[cond[m / L]][n] * acc    out fp32 in place;
 *               gate row r at mods + r*mods_stride + gate_off, cond dev [M / L]
 *            4: out[m, n] = acc                  out fp32
 * BR_BF16 needs K % 64 == 0, lda % 8 == 0, ldw % 8 == 0; N % 4 == 0 always.
 * variant: bf16 kernel (-1 = automatic; 4 / 5 / 6 = 256x256 / 128x128 / 256x128 tile per workgroup,
 * 7 = persistent 256x256 streaming kernel, needs K % 128 == 0; bits 4..11 = column-group width of
 * the tile walk, 0 = the kernel's own choice; for the persistent kernel bits 12..19 / 20..23 = start
 * delay step, in half microseconds, of workgroups that have / do not have a tile less than the longest
 * tile list on their compute die: group g = (workgroup index on the die) / 4 % 8 starts g steps late;
 * bits 20..23 hold the second of the two; bits 24..30 = rows of a row block of the tile walk in units
 * of 8 tile rows, 0 = the kernel's own choice). */
br_status br_op_gemm(int32_t dtype, int32_t epilogue, const void* A, int32_t lda, const void* W,
                     int32_t ldw, int32_t M, int32_t N, int32_t K, const float* bias, void* out,
                     int32_t ldo, const float* mods, int32_t mods_stride, int32_t gate_off,
                     const int32_t* cond, int32_t L, int32_t variant, void* stream);

/* out[b, l, h*DH + d] = softmax_j(q_l . k_j / sqrt(DH)) v_j for every sample b and
 * head h; qkv dev [B, L, 3*NH*DH] (q | k | v), out dev [B, L, NH*DH], both `dtype`.
 * BR_BF16: DH 64 or 128, qkv 16-byte aligned, L*3*NH*DH*2 below 4 GiB (BR_ESHAPE otherwise).
 * q_prescaled = 1 (BR_BF16 only, BR_EINVAL otherwise): the q third holds q * log2(e) / sqrt(DH)
 * instead of q -- the layout the network's QKV projection writes, which spares the kernel one
 * multiplication per score; the result is the same function of the unscaled q. */
br_status br_op_attention(int32_t dtype, const void* qkv, void* out, int32_t B, int32_t L,
                          int32_t NH, int32_t DH, int32_t q_prescaled, void* stream);

/* out[r, :] = LayerNorm(x[src(r), :]) * (1 + scale) + shift, eps 1e-6, no affine;
 * r = b*rows_per_sample + tok, src(r) = b*L_in + tok; shift / scale are the rows
 * mods + cond[b]*mods_stride + {shift_off, scale_off}.  x dev fp32, out dev `dtype`. */
br_status br_op_ln_modulate(int32_t dtype, const float* x, void* out, int32_t n_rows,
                            int32_t rows_per_sample, int32_t L_in, int32_t H, const float* mods,
                            int32_t mods_stride, int32_t shift_off, int32_t scale_off,
                            const int32_t* cond, void* stream);

/* Per-launch timing of the main kernels with HIP events recorded on the launch
 * stream around each launch (off by default; single-threaded use).  While enabled
 * every instrumented launch adds one record; br_profile_read waits for the
 * recorded events, sums work (flops for GEMM and attention, bytes for the others)
 * and milliseconds per kernel id, clears the records and returns up to max_ids
 * entries.  Ids: GEMM = epilogue*8 + tile variant; attention = 100 + head dim;
 * 200 SDE step, 201 log-prob re-evaluation, 300 LayerNorm-modulate, 301 adaLN modulation GEMV
 * (bytes = the weights it streams). */
br_status br_profile_enable(int32_t on);
br_status br_profile_read(int32_t max_ids, int32_t* ids, double* work, double* ms,
                          int64_t* launches, int32_t* n_ids);

#ifdef __cplusplus
}
#endif
#endif
