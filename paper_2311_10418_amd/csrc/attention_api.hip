// C-ABI entry points and dispatch for variable-length attention.
#include "attention.hpp"
#include <cmath>

static ds_status check(const AttnArgs& a) {
    if (a.n_seq <= 0 || a.n_heads <= 0 || a.head_dim <= 0 || a.head_dim > 128 || a.head_dim % 8) return DS_EINVAL;
    if (a.dtype != DS_DTYPE_F32 && a.dtype != DS_DTYPE_BF16) return DS_EINVAL;
    if (a.mask != 0 && a.mask != 1) return DS_EINVAL;
    if (!a.q_row || !a.q_len || !a.k_row || !a.k_len || !a.q || !a.k || !a.v || !a.o || !a.lse) return DS_EINVAL;
    if (a.max_q_len <= 0 || a.max_k_len <= 0) return DS_EINVAL;
    if (a.n_seq > 65535 || a.n_heads > 65535) return DS_EINVAL;
    return DS_OK;
}

ds_status launch_attention_fwd(const AttnArgs& a, bool force_generic, hipStream_t st) {
    ds_status s = check(a);
    if (s != DS_OK) return s;
    if (!force_generic && attn_mfma_supported(a)) return attn_fwd_mfma(a, st);
    return attn_fwd_generic(a, st);
}

ds_status launch_attention_bwd(const AttnArgs& a, bool force_generic, hipStream_t st) {
    ds_status s = check(a);
    if (s != DS_OK) return s;
    if (!a.d_o || !a.delta || !a.dq || !a.dk || !a.dv) return DS_EINVAL;
    if (!force_generic && attn_mfma_supported(a)) return attn_bwd_mfma(a, st);      // computes delta itself
    s = attn_delta(a, st);
    if (s != DS_OK) return s;
    return attn_bwd_generic(a, st);
}

extern "C" ds_status ds_attention_fwd(int32_t dtype, int32_t n_seq, int32_t n_heads, int32_t head_dim, int32_t mask,
                                      const int32_t* q_row, const int32_t* q_len, const int32_t* k_row,
                                      const int32_t* k_len, int32_t max_q_len, int32_t max_k_len, const void* q,
                                      int32_t ldq, const void* k, int32_t ldk, const void* v, int32_t ldv, void* o,
                                      int32_t ldo, float* lse, int32_t lse_stride, int32_t k_total_rows, void* scratch,
                                      int64_t scratch_bytes, int32_t force_generic, void* hip_stream) {
    AttnArgs a{};
    a.dtype = dtype; a.n_seq = n_seq; a.n_heads = n_heads; a.head_dim = head_dim; a.mask = mask;
    a.q_row = q_row; a.q_len = q_len; a.k_row = k_row; a.k_len = k_len;
    a.max_q_len = max_q_len; a.max_k_len = max_k_len;
    a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldk = ldk; a.ldv = ldv;
    a.o = o; a.ldo = ldo; a.lse = lse; a.lse_stride = lse_stride;
    a.scratch = scratch; a.scratch_bytes = scratch_bytes > 0 ? (size_t)scratch_bytes : 0;
    a.q_total_rows = lse_stride; a.k_total_rows = k_total_rows;
    a.scale = head_dim > 0 ? 1.0f / std::sqrt((float)head_dim) : 0.f;
    return launch_attention_fwd(a, force_generic != 0, (hipStream_t)hip_stream);
}

extern "C" ds_status ds_attention_bwd(int32_t dtype, int32_t n_seq, int32_t n_heads, int32_t head_dim, int32_t mask,
                                      const int32_t* q_row, const int32_t* q_len, const int32_t* k_row,
                                      const int32_t* k_len, int32_t max_q_len, int32_t max_k_len, const void* q,
                                      int32_t ldq, const void* k, int32_t ldk, const void* v, int32_t ldv, const void* o,
                                      const void* d_o, int32_t ldo, const float* lse, float* delta, int32_t lse_stride,
                                      void* dq, void* dk, void* dv, int32_t k_total_rows, void* scratch,
                                      int64_t scratch_bytes, int32_t force_generic, void* hip_stream) {
    AttnArgs a{};
    a.dtype = dtype; a.n_seq = n_seq; a.n_heads = n_heads; a.head_dim = head_dim; a.mask = mask;
    a.q_row = q_row; a.q_len = q_len; a.k_row = k_row; a.k_len = k_len;
    a.max_q_len = max_q_len; a.max_k_len = max_k_len;
    a.q = q; a.k = k; a.v = v; a.ldq = ldq; a.ldk = ldk; a.ldv = ldv;
    a.o = const_cast<void*>(o); a.d_o = d_o; a.ldo = ldo; a.lse = const_cast<float*>(lse); a.delta = delta;
    a.lse_stride = lse_stride; a.dq = dq; a.dk = dk; a.dv = dv;
    a.scratch = scratch; a.scratch_bytes = scratch_bytes > 0 ? (size_t)scratch_bytes : 0;
    a.q_total_rows = lse_stride; a.k_total_rows = k_total_rows;
    a.scale = head_dim > 0 ? 1.0f / std::sqrt((float)head_dim) : 0.f;
    return launch_attention_bwd(a, force_generic != 0, (hipStream_t)hip_stream);
}

extern "C" int64_t ds_attention_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t q_total_rows, int32_t k_total_rows,
                                              int32_t n_seq) {
    if (n_heads <= 0 || head_dim <= 0 || q_total_rows <= 0 || k_total_rows <= 0 || n_seq <= 0) return 0;
    return (int64_t)attn_scratch_bytes(n_heads, head_dim, q_total_rows, k_total_rows, n_seq);
}
