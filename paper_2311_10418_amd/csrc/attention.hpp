// Arguments shared by the attention kernels (generic and MFMA).
#pragma once
#include "common.hpp"

struct AttnArgs {
    int32_t dtype, n_seq, n_heads, head_dim, mask;   // mask: 0 none, 1 causal
    const int32_t *q_row, *q_len, *k_row, *k_len;    // DEVICE, per sequence
    int32_t max_q_len, max_k_len;
    const void *q, *k, *v;
    long long ldq, ldk, ldv;
    void* o;                                          // forward output / backward input
    const void* d_o;
    long long ldo;
    float* lse;
    float* delta;
    long long lse_stride;
    void *dq, *dk, *dv;
    float scale;
    // MFMA path: scratch for feature-major copies (V^T forward; Q^T, dO^T, K^T backward); the
    // sequence tables must list sequences in ascending row order
    void* scratch;
    size_t scratch_bytes;
    int32_t q_total_rows, k_total_rows;               // rows of the query-side / key-side streams
    const void *qT, *kT, *vT, *doT;                   // filled by the launchers
    long long ldTq, ldTk;
};

long long attn_ld_t(int total_rows, int n_seq);
size_t attn_scratch_bytes(int n_heads, int head_dim, int q_total_rows, int k_total_rows, int n_seq);

ds_status attn_fwd_generic(const AttnArgs& a, hipStream_t st);
ds_status attn_bwd_generic(const AttnArgs& a, hipStream_t st);
ds_status attn_delta(const AttnArgs& a, hipStream_t st);
// MFMA (bf16, head_dim 64 or 128) paths; return DS_EINVAL when the shape is not supported.
bool attn_mfma_supported(const AttnArgs& a);
ds_status attn_fwd_mfma(const AttnArgs& a, hipStream_t st);
ds_status attn_bwd_mfma(const AttnArgs& a, hipStream_t st);

ds_status launch_attention_fwd(const AttnArgs& a, bool force_generic, hipStream_t st);
ds_status launch_attention_bwd(const AttnArgs& a, bool force_generic, hipStream_t st);
