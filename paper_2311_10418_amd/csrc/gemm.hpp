// GEMM launcher shared by the C-ABI entry point and the stage driver.
#pragma once
#include "common.hpp"

struct GemmEpi {
    const void* bias;          // [N] or NULL
    const void* R;             // residual / saved pre-activation, [M,N]
    const void* R2;            // second saved tensor (gated MLP backward)
    void* C2;                  // second output
    const int32_t* row_valid;  // rows with a negative entry are written as zeros (RESID epilogue)
    int accumulate;            // ACC32: add to C instead of overwriting
    // DGELU epilogue, direct-to-LDS NT kernel only (see gemm_colsum_fused): partial column sums of the OUTPUT (before
    // its rounding to bf16), float32 [gemm_colsum_rows(M)][N], every entry written; NULL = not wanted
    float* colsum;
};

// true if launch_gemm with these arguments and p.colsum set fills p.colsum (otherwise it ignores the field)
bool gemm_colsum_fused(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K, const void* A, const void* B,
                       const void* C, int32_t epilogue);
inline size_t gemm_colsum_rows(int32_t M) { return (size_t)((M + 255) / 256) * 2; }

ds_status launch_gemm(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K, const void* A, const void* B,
                      void* C, int32_t epilogue, const GemmEpi& p, bool force_generic, float* split_ws,
                      size_t split_ws_floats, hipStream_t st);
