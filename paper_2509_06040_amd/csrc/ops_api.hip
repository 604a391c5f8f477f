// Op-level C-ABI entry points (single kernels of the velocity network).
#include "../../include/branchrollout_ops.h"
#include "common.h"
#include "dit.h"

using namespace br;

extern "C" br_status br_op_gemm(int32_t dtype, int32_t epilogue, const void* A, int32_t lda, const void* W, int32_t ldw,
                                int32_t M, int32_t N, int32_t K, const float* bias, void* out, int32_t ldo,
                                const float* mods, int32_t mods_stride, int32_t gate_off, const int32_t* cond,
                                int32_t L, int32_t variant, void* stream) {
  BR_REQUIRE(A && W && bias && out, BR_EINVAL, "br_op_gemm: NULL argument");
  BR_REQUIRE(dtype == BR_F32 || dtype == BR_BF16, BR_EINVAL, "br_op_gemm: unknown dtype");
  BR_REQUIRE(M >= 0 && N >= 4 && K >= 1 && lda >= K && ldw >= K && ldo >= N && N % 4 == 0 && ldo % 4 == 0, BR_EINVAL,
             "br_op_gemm: bad sizes");
  BR_REQUIRE(epilogue == EPI_BIAS || epilogue == EPI_BIAS_GELU || epilogue == EPI_BIAS_GATE_RES ||
                 epilogue == EPI_BIAS_F32, BR_EINVAL, "br_op_gemm: unsupported epilogue");
  EpiArgs ea{};
  ea.bias = bias;
  ea.out = out;
  ea.ldo = ldo;
  if (epilogue == EPI_BIAS_GATE_RES) {
    BR_REQUIRE(mods && cond && L >= 1 && M % L == 0, BR_EINVAL, "br_op_gemm: gate arguments missing");
    ea.mods = mods;
    ea.A = mods_stride;
    ea.gate_off = gate_off;
    ea.condmap = cond;
    ea.L = L;
  }
  if (M == 0) return BR_OK;
  if (dtype == BR_BF16)
    return launch_gemm_bf16(epilogue, (const bf16*)A, lda, (const bf16*)W, ldw, M, N, K, ea, variant,
                            (hipStream_t)stream);
  return launch_gemm(dtype, epilogue, A, lda, W, ldw, M, N, K, ea, (hipStream_t)stream);
}

extern "C" br_status br_op_attention(int32_t dtype, const void* qkv, void* out, int32_t B, int32_t L, int32_t NH,
                                     int32_t DH, int32_t q_prescaled, void* stream) {
  BR_REQUIRE(qkv && out, BR_EINVAL, "br_op_attention: NULL argument");
  BR_REQUIRE(dtype == BR_F32 || dtype == BR_BF16, BR_EINVAL, "br_op_attention: unknown dtype");
  BR_REQUIRE(B >= 1 && L >= 1 && NH >= 1, BR_EINVAL, "br_op_attention: bad sizes");
  BR_REQUIRE(q_prescaled == 0 || (q_prescaled == 1 && dtype == BR_BF16), BR_EINVAL,
             "br_op_attention: q_prescaled is 0, or 1 with BR_BF16");
  return launch_attention(dtype, qkv, out, B, L, NH, DH, q_prescaled, (hipStream_t)stream);
}

extern "C" br_status br_op_ln_modulate(int32_t dtype, const float* x, void* out, int32_t n_rows,
                                       int32_t rows_per_sample, int32_t L_in, int32_t H, const float* mods,
                                       int32_t mods_stride, int32_t shift_off, int32_t scale_off, const int32_t* cond,
                                       void* stream) {
  BR_REQUIRE(x && out && mods && cond, BR_EINVAL, "br_op_ln_modulate: NULL argument");
  BR_REQUIRE(dtype == BR_F32 || dtype == BR_BF16, BR_EINVAL, "br_op_ln_modulate: unknown dtype");
  BR_REQUIRE(n_rows >= 0 && rows_per_sample >= 1 && L_in >= rows_per_sample && H >= 4 && H % 4 == 0, BR_EINVAL,
             "br_op_ln_modulate: bad sizes");
  return launch_ln_modulate(dtype, x, out, n_rows, rows_per_sample, L_in, H, mods, mods_stride, shift_off, scale_off,
                            cond, (hipStream_t)stream);
}
