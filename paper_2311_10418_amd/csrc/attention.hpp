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
    // MFMA path: scratch holds the work lists (see attn_scratch_bytes); filled in by attn_prepare_lists
    void* scratch;
    size_t scratch_bytes;
    int32_t q_total_rows, k_total_rows;               // rows of the query-side / key-side streams
    int32_t lists_ready;                              // the scratch already holds this call's work lists
    int32_t lists_want_both;                          // build the key-side list too even if this call only needs the query side
    const int32_t* n_items;                           // DEVICE [2]: query-side, key-side item counts
    const int2 *items_q, *items_k;                    // DEVICE (sequence, 128-row block), longest first
    int32_t max_items_q, max_items_k;                 // host upper bounds = grid sizes
    // DEVICE [n_heads][q_total_rows][8] bf16 each: {hi, lo, 0 x 6} splits of lse/scale and of delta, written by the
    // dQ kernel, fetched by the dK/dV kernel straight into LDS
    void *aug_lse, *aug_delta;
};

size_t attn_scratch_bytes(int n_heads, int head_dim, int q_total_rows, int k_total_rows, int n_seq);
ds_status attn_prepare_lists(AttnArgs& a, bool need_key_side, hipStream_t st);

ds_status attn_fwd_generic(const AttnArgs& a, hipStream_t st);
ds_status attn_bwd_generic(const AttnArgs& a, hipStream_t st);
ds_status attn_delta(const AttnArgs& a, hipStream_t st);
// MFMA (bf16, head_dim 64 or 128) paths; return DS_EINVAL when the shape is not supported.
bool attn_mfma_supported(const AttnArgs& a);
ds_status attn_fwd_mfma(const AttnArgs& a, hipStream_t st);
ds_status attn_bwd_mfma(const AttnArgs& a, hipStream_t st);

ds_status launch_attention_fwd(const AttnArgs& a, bool force_generic, hipStream_t st);
ds_status launch_attention_bwd(const AttnArgs& a, bool force_generic, hipStream_t st);
