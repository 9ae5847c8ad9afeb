// The stage driver: owns the device workspace, binds a layout (uploads its tables once), and
// enqueues forward then backward of every layer over the whole layout.
//
// All micro-batches of the layout live in one padded token stream, so every row-wise operator
// (norms, projections, MLP, their gradients) is ONE launch over all micro-batches, and the
// weight-gradient GEMMs contract over the tokens of all micro-batches at once, which is the
// paper's gradient accumulation across micro-batches (section "Background", pipeline-parallel
// paragraph).  Only attention looks at sequence boundaries, through the layout's sequence
// table.  Padding rows: inputs are masked to zero on entry, residual epilogues write zeros to
// padding rows, attention never touches them, and zero rows stay zero through the backward
// pass, so padding contributes nothing to any weight gradient.
#include "attention.hpp"
#include "gemm.hpp"
#include "layout.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <vector>



namespace {

__global__ __launch_bounds__(256) void zero_pad_rows_kernel(int rows, int row_bytes16, uint4* __restrict__ buf,
                                                            const int32_t* __restrict__ row_valid) {
    // one wavefront per row; only padding rows are written
    const int w = (blockIdx.x * blockDim.x + threadIdx.x) >> 6, lane = threadIdx.x & 63;
    const int nw = (gridDim.x * blockDim.x) >> 6;
    for (int r = w; r < rows; r += nw) {
        if (row_valid[r] >= 0) continue;
        uint4* p = buf + (size_t)r * row_bytes16;
        for (int c = lane; c < row_bytes16; c += 64) p[c] = make_uint4(0u, 0u, 0u, 0u);
    }
}

struct Arena {
    char* base = nullptr;
    size_t size = 0, used = 0;
    void* take(size_t bytes) {
        const size_t a = (used + 255) & ~size_t(255);
        if (a + bytes > size) return nullptr;
        used = a + bytes;
        return base + a;
    }
};

struct StreamTables {          // device tables of one token stream
    int32_t* row_valid = nullptr;   // [max_rows]  sorted sequence position, or -1 for padding
    int32_t* seq_row = nullptr;     // [max_seqs]
    int32_t* seq_len = nullptr;     // [max_seqs]
};

struct LayerBufs {
    void *u1, *qkv, *o, *x1, *u2, *z, *a, *xout;
    float *stats1, *stats2, *lse;
    void *wqkv_t, *wo_t, *w1_t, *w2_t;      // [out][in] copies of the layer's matrices (bf16 fast path)
};

}  // namespace

struct ds_stage {
    ds_stage_config cfg{};
    size_t es = 4;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    Arena arena;
    StreamTables tab;
    int32_t* h_tables = nullptr;       // pinned staging for table uploads
    size_t h_tables_ints = 0;
    hipEvent_t upload_done = nullptr;
    uint64_t bound_uid = 0;
    int32_t bound_rows = 0, bound_seqs = 0, bound_max_len = 0;
    bool bound_has_pad = false;
    std::vector<LayerBufs> layers;
    void *x0 = nullptr, *dyA = nullptr, *dyB = nullptr, *dz = nullptr, *du = nullptr, *dx1 = nullptr, *d_o = nullptr,
         *dqkv = nullptr;
    float *delta = nullptr, *partial = nullptr, *split_ws = nullptr;
    void *xt = nullptr, *dyt = nullptr;     // token-major -> feature-major copies for the weight-gradient GEMMs
    void* attn_scratch = nullptr;           // feature-major copies for the attention kernels
    size_t attn_scratch_bytes = 0;
    bool nt_mode = false;
    size_t split_ws_floats = 0;
    int32_t launches = 0;
    // optional per-kernel-group timing
    bool prof_on = false;
    std::vector<hipEvent_t> ev_pool;
    std::vector<int> ev_cat;
    int ev_used = 0;
};

namespace {

ds_status bind_layout(ds_stage* s, const ds_layout* lo, hipStream_t st) {
    if (lo->uid == s->bound_uid) return DS_OK;
    if (lo->has_tgt != (s->cfg.model == DS_MODEL_T5)) return DS_ELAYOUT;
    if (lo->total_rows > s->cfg.max_rows || lo->n_seq > s->cfg.max_seqs) return DS_ELAYOUT;
    // a previous upload may still be reading the staging buffer
    DS_HIP_CHECK(hipEventSynchronize(s->upload_done));
    const int R = lo->total_rows, S = lo->n_seq;
    int32_t* rv = s->h_tables;
    int32_t* sr = rv + s->cfg.max_rows;
    int32_t* sl = sr + s->cfg.max_seqs;
    std::fill(rv, rv + R, -1);
    int max_len = 0;
    for (int i = 0; i < S; ++i) {
        sr[i] = lo->seq_row[i];
        sl[i] = lo->seq_len[i];
        max_len = std::max(max_len, lo->seq_len[i]);
        for (int r = 0; r < lo->seq_len[i]; ++r) rv[lo->seq_row[i] + r] = i;
    }
    DS_HIP_CHECK(hipMemcpyAsync(s->tab.row_valid, rv, sizeof(int32_t) * R, hipMemcpyHostToDevice, st));
    DS_HIP_CHECK(hipMemcpyAsync(s->tab.seq_row, sr, sizeof(int32_t) * S, hipMemcpyHostToDevice, st));
    DS_HIP_CHECK(hipMemcpyAsync(s->tab.seq_len, sl, sizeof(int32_t) * S, hipMemcpyHostToDevice, st));
    DS_HIP_CHECK(hipEventRecord(s->upload_done, st));
    s->bound_uid = lo->uid;
    s->bound_rows = R;
    s->bound_seqs = S;
    s->bound_max_len = max_len;
    s->bound_has_pad = lo->total_tokens != (int64_t)lo->total_rows;
    return DS_OK;
}

ds_status zero_pad_rows(ds_stage* s, void* buf, int cols, hipStream_t st) {
    if (!s->bound_has_pad) return DS_OK;
    const int R = s->bound_rows;
    const int row16 = (int)((size_t)cols * s->es / 16);
    int blocks = (R + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(zero_pad_rows_kernel, dim3(blocks), dim3(256), 0, st, R, row16, (uint4*)buf, s->tab.row_valid);
    DS_LAUNCH_CHECK();
    s->launches++;
    return DS_OK;
}

#define DS_TRY(expr)                    \
    do {                                \
        ds_status st__ = (expr);        \
        if (st__ != DS_OK) return st__; \
    } while (0)

ds_status gemm(ds_stage* s, int ta, int tb, int M, int N, int K, const void* A, const void* B, void* C, int epi,
               const void* bias, const void* R, const void* R2, void* C2, bool mask_rows, int accumulate, hipStream_t st) {
    GemmEpi p{bias, R, R2, C2, mask_rows && s->bound_has_pad ? s->tab.row_valid : nullptr, accumulate};
    s->launches++;
    return launch_gemm(s->cfg.dtype, ta, tb, M, N, K, A, B, C, epi, p, false, s->split_ws, s->split_ws_floats, st);
}

AttnArgs self_attn_args(ds_stage* s, const void* qkv, int mask) {
    const int d = s->cfg.d_model, h = s->cfg.n_heads, hd = d / h;
    AttnArgs a{};
    a.dtype = s->cfg.dtype;
    a.n_seq = s->bound_seqs;
    a.n_heads = h;
    a.head_dim = hd;
    a.mask = mask;
    a.q_row = a.k_row = s->tab.seq_row;
    a.q_len = a.k_len = s->tab.seq_len;
    a.max_q_len = a.max_k_len = s->bound_max_len;
    const char* base = (const char*)qkv;
    a.q = base;
    a.k = base + (size_t)d * s->es;
    a.v = base + (size_t)2 * d * s->es;
    a.ldq = a.ldk = a.ldv = 3 * d;
    a.ldo = d;
    a.lse_stride = s->bound_rows;
    a.scale = 1.0f / std::sqrt((float)hd);
    a.scratch = s->attn_scratch;
    a.scratch_bytes = s->attn_scratch_bytes;
    a.q_total_rows = a.k_total_rows = s->bound_rows;
    return a;
}

// Runs fn, bracketed by a pair of HIP events on the stream when profiling is on.
template <class F>
ds_status timed(ds_stage* s, int cat, hipStream_t st, F&& fn) {
    if (!s->prof_on || s->ev_used + 2 > (int)s->ev_pool.size()) return fn();
    hipEvent_t e0 = s->ev_pool[s->ev_used], e1 = s->ev_pool[s->ev_used + 1];
    DS_HIP_CHECK(hipEventRecord(e0, st));
    const ds_status r = fn();
    DS_HIP_CHECK(hipEventRecord(e1, st));
    s->ev_cat[s->ev_used / 2] = cat;
    s->ev_used += 2;
    return r;
}

ds_status gpt_fwd_bwd(ds_stage* s, const ds_gpt_layer* w, const ds_stage_io* io, const ds_gpt_layer* g, int accumulate,
                      hipStream_t st) {
    const int R = s->bound_rows, d = s->cfg.d_model, F = s->cfg.d_ff, L = s->cfg.n_layers;
    const int dt = s->cfg.dtype;
    const bool pad = s->bound_has_pad;
    auto G = [&](int cat, int ta, int tb, int M, int N, int K, const void* A, const void* B, void* C, int epi,
                 const void* bias, const void* Rr, void* C2, bool mask, int acc) {
        return timed(s, cat, st, [&] { return gemm(s, ta, tb, M, N, K, A, B, C, epi, bias, Rr, nullptr, C2, mask, acc, st); });
    };
    // bf16 fast path: every GEMM runs as C = A B^T with both operands contiguous along the contraction
    // (the direct-to-LDS kernel).  Forward uses [out][in] copies of the weights made at the top of the
    // call; a weight gradient dW[in][out] = X^T dY uses feature-major copies of X and dY whose token
    // dimension is zero-padded to a multiple of 64.
    const bool nt = s->nt_mode;
    const int Rp = (R + 63) & ~63;
    auto FWD = [&](int N, int K, const void* X, const void* W, const void* Wt, void* C, int epi, const void* bias,
                   const void* Rr, void* C2, bool mask) {
        if (nt) return G(DS_PROF_GEMM_FWD, 0, 1, R, N, K, X, Wt, C, epi, bias, Rr, C2, mask, 0);
        return G(DS_PROF_GEMM_FWD, 0, 0, R, N, K, X, W, C, epi, bias, Rr, C2, mask, 0);
    };
    auto WGRAD = [&](int Kin, int Nout, const void* X, const void* dY, void* dW) {
        if (!nt) return G(DS_PROF_GEMM_WGRAD, 1, 0, Kin, Nout, R, X, dY, dW, DS_EPI_ACC32, nullptr, nullptr, nullptr, false, accumulate);
        return timed(s, DS_PROF_GEMM_WGRAD, st, [&] {
            DS_TRY(launch_transpose_bf16(R, Kin, Rp, X, s->xt, st));
            DS_TRY(launch_transpose_bf16(R, Nout, Rp, dY, s->dyt, st));
            s->launches += 2;
            return gemm(s, 0, 1, Kin, Nout, Rp, s->xt, s->dyt, dW, DS_EPI_ACC32, nullptr, nullptr, nullptr, nullptr, false, accumulate, st);
        });
    };
    if (nt) {
        DS_TRY(timed(s, DS_PROF_GEMM_FWD, st, [&] {
            for (int l = 0; l < L; ++l) {
                LayerBufs& b = s->layers[l];
                DS_TRY(launch_transpose_bf16(d, 3 * d, d, w[l].w_qkv, b.wqkv_t, st));
                DS_TRY(launch_transpose_bf16(d, d, d, w[l].w_o, b.wo_t, st));
                DS_TRY(launch_transpose_bf16(d, F, d, w[l].w_1, b.w1_t, st));
                DS_TRY(launch_transpose_bf16(F, d, F, w[l].w_2, b.w2_t, st));
                s->launches += 4;
            }
            return DS_OK;
        }));
    }
    auto colsum = [&](int n, const void* x, void* out) {
        s->launches += 2;
        return timed(s, DS_PROF_COLSUM, st, [&] { return ds_colsum(dt, R, n, x, (float*)out, s->partial, accumulate, st); });
    };

    // ---------------- forward (ForwardPass of every micro-batch)
    const void* x_in = io->act_in;
    if (pad) {
        DS_TRY(timed(s, DS_PROF_OTHER, st, [&] { return launch_mask_rows(dt, R, d, io->act_in, s->x0, s->tab.row_valid, st); }));
        s->launches++;
        x_in = s->x0;
    }
    for (int l = 0; l < L; ++l) {
        LayerBufs& b = s->layers[l];
        void* x_out = (l == L - 1) ? io->act_out : b.xout;
        DS_TRY(timed(s, DS_PROF_NORM, st, [&] { return ds_norm_fwd(dt, 0, R, d, x_in, w[l].ln1_g, w[l].ln1_b, b.u1, b.stats1, st); }));
        DS_TRY(FWD(3 * d, d, b.u1, w[l].w_qkv, b.wqkv_t, b.qkv, DS_EPI_NONE, w[l].b_qkv, nullptr, nullptr, false));
        AttnArgs a = self_attn_args(s, b.qkv, 1);
        a.o = b.o;
        a.lse = b.lse;
        DS_TRY(timed(s, DS_PROF_ATTN_FWD, st, [&] { return launch_attention_fwd(a, false, st); }));
        DS_TRY(timed(s, DS_PROF_OTHER, st, [&] { return zero_pad_rows(s, b.o, d, st); }));
        DS_TRY(FWD(d, d, b.o, w[l].w_o, b.wo_t, b.x1, DS_EPI_RESID, w[l].b_o, x_in, nullptr, true));
        DS_TRY(timed(s, DS_PROF_NORM, st, [&] { return ds_norm_fwd(dt, 0, R, d, b.x1, w[l].ln2_g, w[l].ln2_b, b.u2, b.stats2, st); }));
        DS_TRY(FWD(F, d, b.u2, w[l].w_1, b.w1_t, b.z, DS_EPI_GELU, w[l].b_1, nullptr, b.a, false));
        DS_TRY(FWD(d, F, b.a, w[l].w_2, b.w2_t, x_out, DS_EPI_RESID, w[l].b_2, b.x1, nullptr, true));
        s->launches += 3;
        x_in = x_out;
    }

    // ---------------- backward (BackwardPass of every micro-batch; weight gradients summed over all of them)
    const void* dy = io->grad_out;
    if (pad) {
        DS_TRY(timed(s, DS_PROF_OTHER, st, [&] { return launch_mask_rows(dt, R, d, io->grad_out, s->dyA, s->tab.row_valid, st); }));
        s->launches++;
        dy = s->dyA;
    }
    void* pp[2] = {s->dyB, s->dyA};
    int flip = 0;
    for (int l = L - 1; l >= 0; --l) {
        LayerBufs& b = s->layers[l];
        const void* xl_in = (l == 0) ? (pad ? s->x0 : io->act_in) : s->layers[l - 1].xout;
        void* dx_in = (l == 0) ? io->grad_in : pp[flip];
        // MLP
        DS_TRY(WGRAD(F, d, b.a, dy, g[l].w_2));
        DS_TRY(colsum(d, dy, g[l].b_2));
        DS_TRY(G(DS_PROF_GEMM_DGRAD, 0, 1, R, F, d, dy, w[l].w_2, s->dz, DS_EPI_DGELU, nullptr, b.z, nullptr, false, 0));
        DS_TRY(WGRAD(d, F, b.u2, s->dz, g[l].w_1));
        DS_TRY(colsum(F, s->dz, g[l].b_1));
        DS_TRY(G(DS_PROF_GEMM_DGRAD, 0, 1, R, d, F, s->dz, w[l].w_1, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr, false, 0));
        DS_TRY(timed(s, DS_PROF_NORM, st, [&] {
            return ds_norm_bwd(dt, 0, R, d, s->du, b.x1, w[l].ln2_g, b.stats2, dy, s->dx1, (float*)g[l].ln2_g,
                               (float*)g[l].ln2_b, s->partial, accumulate, st);
        }));
        // attention
        DS_TRY(WGRAD(d, d, b.o, s->dx1, g[l].w_o));
        DS_TRY(colsum(d, s->dx1, g[l].b_o));
        DS_TRY(G(DS_PROF_GEMM_DGRAD, 0, 1, R, d, d, s->dx1, w[l].w_o, s->d_o, DS_EPI_NONE, nullptr, nullptr, nullptr, false, 0));
        AttnArgs a = self_attn_args(s, b.qkv, 1);
        a.o = b.o;
        a.d_o = s->d_o;
        a.lse = b.lse;
        a.delta = s->delta;
        char* dq = (char*)s->dqkv;
        a.dq = dq;
        a.dk = dq + (size_t)d * s->es;
        a.dv = dq + (size_t)2 * d * s->es;
        DS_TRY(timed(s, DS_PROF_ATTN_BWD, st, [&] { return launch_attention_bwd(a, false, st); }));
        DS_TRY(timed(s, DS_PROF_OTHER, st, [&] { return zero_pad_rows(s, s->dqkv, 3 * d, st); }));
        DS_TRY(WGRAD(d, 3 * d, b.u1, s->dqkv, g[l].w_qkv));
        DS_TRY(colsum(3 * d, s->dqkv, g[l].b_qkv));
        DS_TRY(G(DS_PROF_GEMM_DGRAD, 0, 1, R, d, 3 * d, s->dqkv, w[l].w_qkv, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr, false, 0));
        DS_TRY(timed(s, DS_PROF_NORM, st, [&] {
            return ds_norm_bwd(dt, 0, R, d, s->du, xl_in, w[l].ln1_g, b.stats1, s->dx1, dx_in, (float*)g[l].ln1_g,
                               (float*)g[l].ln1_b, s->partial, accumulate, st);
        }));
        s->launches += 2 * 3 + 3;
        dy = dx_in;
        flip ^= 1;
    }
    return DS_OK;
}

}  // namespace

extern "C" ds_status ds_stage_create(const ds_stage_config* cfg, ds_stage** out) {
    if (!cfg || !out) return DS_EINVAL;
    *out = nullptr;
    if (cfg->model != DS_MODEL_GPT && cfg->model != DS_MODEL_T5) return DS_EINVAL;
    if (cfg->dtype != DS_DTYPE_F32 && cfg->dtype != DS_DTYPE_BF16) return DS_EINVAL;
    if (cfg->n_layers <= 0 || cfg->d_model <= 0 || cfg->n_heads <= 0 || cfg->d_ff <= 0) return DS_EINVAL;
    if (cfg->d_model % cfg->n_heads || cfg->d_model % 8 || cfg->d_ff % 8 || cfg->d_model > 4096) return DS_EINVAL;
    const int hd = cfg->d_model / cfg->n_heads;
    if (hd > 128 || hd % 8) return DS_EINVAL;
    if (cfg->max_rows <= 0 || cfg->max_seqs <= 0) return DS_EINVAL;
    if (cfg->model == DS_MODEL_T5) return DS_EINVAL;   // encoder-decoder stage: not built yet
    if (cfg->model == DS_MODEL_GPT && (cfg->n_dec_layers != 0 || cfg->max_rows_tgt != 0)) return DS_EINVAL;

    ds_stage* s = new (std::nothrow) ds_stage();
    if (!s) return DS_ENOMEM;
    s->cfg = *cfg;
    s->es = dtype_size(cfg->dtype);
    const size_t R = (size_t)cfg->max_rows, d = cfg->d_model, F = cfg->d_ff, h = cfg->n_heads, L = cfg->n_layers;
    const size_t es = s->es;
    auto al = [](size_t b) { return (b + 255) & ~size_t(255); };
    size_t need = 0;
    const size_t per_layer = al(R * d * es) * 5 + al(R * 3 * d * es) + al(R * F * es) * 2 + al(R * 2 * 4) * 2 + al(R * h * 4);
    need += per_layer * L;
    need += al(R * d * es) * 6 + al(R * F * es) + al(R * 3 * d * es);       // x0 dyA dyB du dx1 d_o, dz, dqkv
    need += al(R * h * 4);                                                  // delta
    const size_t partial_floats = std::max<size_t>((size_t)ds_norm_bwd_scratch_floats(1, (int)d), (size_t)2048 * 1024);
    need += al(partial_floats * 4);
    s->split_ws_floats = 3 * std::max(d * 3 * d, d * F);
    need += al(s->split_ws_floats * 4);
    need += al(R * 4) + 2 * al((size_t)cfg->max_seqs * 4);
    need += 4096;
    s->nt_mode = cfg->dtype == DS_DTYPE_BF16 && d % 256 == 0 && F % 256 == 0;
    const size_t Rp = (R + 63) & ~size_t(63);
    if (cfg->dtype == DS_DTYPE_BF16 && (hd == 64 || hd == 128)) {
        s->attn_scratch_bytes = attn_scratch_bytes(cfg->n_heads, hd, cfg->max_rows, cfg->max_rows, cfg->max_seqs);
        need += al(s->attn_scratch_bytes);
    }
    if (s->nt_mode) {
        need += L * (al(3 * d * d * es) + al(d * d * es) + 2 * al(d * F * es));
        need += al(std::max(d, F) * Rp * es) + al(std::max(3 * d, F) * Rp * es);
    }

    if (hipMalloc(&s->ws, need) != hipSuccess) {
        (void)hipGetLastError();
        delete s;
        return DS_ENOMEM;
    }
    s->ws_bytes = need;
    s->arena.base = (char*)s->ws;
    s->arena.size = need;
    bool ok = true;
    auto take = [&](size_t bytes) {
        void* p = s->arena.take(bytes);
        if (!p) ok = false;
        return p;
    };
    s->layers.resize(L);
    for (size_t l = 0; l < L; ++l) {
        LayerBufs& b = s->layers[l];
        b.u1 = take(R * d * es);
        b.qkv = take(R * 3 * d * es);
        b.o = take(R * d * es);
        b.x1 = take(R * d * es);
        b.u2 = take(R * d * es);
        b.z = take(R * F * es);
        b.a = take(R * F * es);
        b.xout = take(R * d * es);
        b.stats1 = (float*)take(R * 2 * 4);
        b.stats2 = (float*)take(R * 2 * 4);
        b.lse = (float*)take(R * h * 4);
        b.wqkv_t = b.wo_t = b.w1_t = b.w2_t = nullptr;
        if (s->nt_mode) {
            b.wqkv_t = take(3 * d * d * es);
            b.wo_t = take(d * d * es);
            b.w1_t = take(d * F * es);
            b.w2_t = take(d * F * es);
        }
    }
    if (s->attn_scratch_bytes) s->attn_scratch = take(s->attn_scratch_bytes);
    if (s->nt_mode) {
        s->xt = take(std::max(d, F) * Rp * es);
        s->dyt = take(std::max(3 * d, F) * Rp * es);
    }
    s->x0 = take(R * d * es);
    s->dyA = take(R * d * es);
    s->dyB = take(R * d * es);
    s->du = take(R * d * es);
    s->dx1 = take(R * d * es);
    s->d_o = take(R * d * es);
    s->dz = take(R * F * es);
    s->dqkv = take(R * 3 * d * es);
    s->delta = (float*)take(R * h * 4);
    s->partial = (float*)take(partial_floats * 4);
    s->split_ws = (float*)take(s->split_ws_floats * 4);
    s->tab.row_valid = (int32_t*)take(R * 4);
    s->tab.seq_row = (int32_t*)take((size_t)cfg->max_seqs * 4);
    s->tab.seq_len = (int32_t*)take((size_t)cfg->max_seqs * 4);
    s->h_tables_ints = R + 2 * (size_t)cfg->max_seqs;
    if (!ok || hipHostMalloc((void**)&s->h_tables, s->h_tables_ints * 4, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&s->upload_done, hipEventDisableTiming) != hipSuccess) {
        (void)hipGetLastError();
        ds_stage_destroy(s);
        return ok ? DS_EHIP : DS_ENOMEM;
    }
    *out = s;
    return DS_OK;
}

extern "C" void ds_stage_destroy(ds_stage* s) {
    if (!s) return;
    for (hipEvent_t e : s->ev_pool) (void)hipEventDestroy(e);
    if (s->upload_done) (void)hipEventDestroy(s->upload_done);
    if (s->h_tables) (void)hipHostFree(s->h_tables);
    if (s->ws) (void)hipFree(s->ws);
    delete s;
}

extern "C" ds_status ds_stage_profile_enable(ds_stage* s, int32_t enable) {
    if (!s) return DS_EINVAL;
    if (enable && s->ev_pool.empty()) {
        const int pairs = 2048;
        s->ev_pool.reserve(2 * pairs);
        for (int i = 0; i < 2 * pairs; ++i) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return DS_EHIP;
            s->ev_pool.push_back(e);
        }
        s->ev_cat.assign(pairs, 0);
    }
    s->prof_on = enable != 0;
    s->ev_used = 0;
    return DS_OK;
}

extern "C" ds_status ds_stage_profile_read(ds_stage* s, float* ms, int32_t* count) {
    if (!s || !ms || !count) return DS_EINVAL;
    for (int c = 0; c < DS_PROF_COUNT; ++c) { ms[c] = 0.f; count[c] = 0; }
    for (int i = 0; i + 1 < s->ev_used; i += 2) {
        DS_HIP_CHECK(hipEventSynchronize(s->ev_pool[i + 1]));
        float t = 0.f;
        DS_HIP_CHECK(hipEventElapsedTime(&t, s->ev_pool[i], s->ev_pool[i + 1]));
        ms[s->ev_cat[i / 2]] += t;
        count[s->ev_cat[i / 2]]++;
    }
    s->ev_used = 0;
    return DS_OK;
}

extern "C" int64_t ds_stage_workspace_bytes(const ds_stage* s) { return s ? (int64_t)s->ws_bytes : 0; }
extern "C" int32_t ds_stage_last_launch_count(const ds_stage* s) { return s ? s->launches : 0; }

extern "C" ds_status stage_fwd_bwd(ds_stage* s, const ds_layout* lo, const void* weights, const void* weights_dec,
                                   const ds_stage_io* io, void* grads, void* grads_dec, int32_t accumulate,
                                   void* hip_stream) {
    if (!s || !lo || !weights || !io || !grads) return DS_EINVAL;
    if (!io->act_in || !io->grad_out || !io->act_out || !io->grad_in) return DS_EINVAL;
    (void)weights_dec;
    (void)grads_dec;
    hipStream_t st = (hipStream_t)hip_stream;
    ds_status r = bind_layout(s, lo, st);
    if (r != DS_OK) return r;
    s->launches = 0;
    if (s->cfg.model == DS_MODEL_GPT)
        return gpt_fwd_bwd(s, (const ds_gpt_layer*)weights, io, (const ds_gpt_layer*)grads, accumulate ? 1 : 0, st);
    return DS_EINVAL;
}

// ---------------------------------------------------------------------------- pack / unpack
// canonical: sequences back to back in ORIGINAL sample order.  Builds the row map on the host,
// uploads it, runs one gather / scatter kernel.  Helper outside any timed region: it allocates
// and synchronises.
static ds_status pack_common(const ds_layout* lo, int which, int dtype, int d, const void* src, void* dst, bool to_stream,
                             hipStream_t st) {
    if (!lo || !src || !dst || d <= 0 || d % 8) return DS_EINVAL;
    if (dtype != DS_DTYPE_F32 && dtype != DS_DTYPE_BF16) return DS_EINVAL;
    if (which != 0 && which != 1) return DS_EINVAL;
    if (which == 1 && !lo->has_tgt) return DS_ELAYOUT;
    const std::vector<int32_t>& seq_row = which ? lo->seq_row_tgt : lo->seq_row;
    const std::vector<int32_t>& seq_len = which ? lo->seq_len_tgt : lo->seq_len;
    const int rows = which ? lo->total_rows_tgt : lo->total_rows;
    // canonical offset of each original sample
    std::vector<int64_t> canon(lo->n_seq + 1, 0);
    {
        std::vector<int32_t> len_orig(lo->n_seq);
        for (int sidx = 0; sidx < lo->n_seq; ++sidx) len_orig[lo->perm[sidx]] = seq_len[sidx];
        for (int i = 0; i < lo->n_seq; ++i) canon[i + 1] = canon[i] + len_orig[i];
    }
    std::vector<int32_t> map(rows, -1);
    for (int sidx = 0; sidx < lo->n_seq; ++sidx)
        for (int r = 0; r < seq_len[sidx]; ++r) map[seq_row[sidx] + r] = (int32_t)(canon[lo->perm[sidx]] + r);
    int32_t* dmap = nullptr;
    DS_HIP_CHECK(hipMalloc((void**)&dmap, sizeof(int32_t) * (size_t)rows));
    ds_status r = DS_OK;
    if (hipMemcpyAsync(dmap, map.data(), sizeof(int32_t) * (size_t)rows, hipMemcpyHostToDevice, st) != hipSuccess) r = DS_EHIP;
    if (r == DS_OK)
        r = to_stream ? launch_gather_rows(dtype, rows, d, src, dst, dmap, st)
                      : launch_scatter_rows(dtype, rows, d, src, dst, dmap, st);
    if (hipStreamSynchronize(st) != hipSuccess && r == DS_OK) r = DS_EHIP;
    (void)hipFree(dmap);
    return r;
}

extern "C" ds_status ds_pack(const ds_layout* lo, int32_t which, int32_t dtype, int32_t d, const void* canonical,
                             void* stream_rows, void* hip_stream) {
    return pack_common(lo, which, dtype, d, canonical, stream_rows, true, (hipStream_t)hip_stream);
}

extern "C" ds_status ds_unpack(const ds_layout* lo, int32_t which, int32_t dtype, int32_t d, const void* stream_rows,
                               void* canonical, void* hip_stream) {
    return pack_common(lo, which, dtype, d, stream_rows, canonical, false, (hipStream_t)hip_stream);
}

extern "C" const char* ds_version(void) { return "dynastage 0.1 gfx950"; }
