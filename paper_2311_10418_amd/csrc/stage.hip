// The stage driver: owns the device workspace, binds a layout (uploads its tables once), and
// enqueues forward then backward of every layer over the whole layout.
//
// All micro-batches of the layout live in one padded token stream (two for an encoder-decoder
// stage), so every row-wise operator (norms, projections, MLP, their gradients) is ONE launch over
// all micro-batches, and the weight-gradient GEMMs contract over the tokens of all micro-batches at
// once, which is the paper's gradient accumulation across micro-batches (section "Background",
// pipeline-parallel paragraph).  Only attention looks at sequence boundaries, through the layout's
// sequence tables.  Padding rows: inputs are masked to zero on entry, residual epilogues write zeros
// to padding rows, attention never touches them (its output buffers' padding rows are zero-filled),
// and zero rows stay zero through the backward pass, so padding contributes nothing to any weight
// gradient.
//
// bf16 fast path ("nt mode"): forward and input-gradient GEMMs run as C = A B^T with both operands contiguous
// along the contraction (forward uses [out][in] copies of the weights, made at the top of the call unless the
// caller has promised unchanged weights); a weight gradient dW[in][out] = X^T dY reads X and dY token-major as
// they are (the kernel's TN form turns the tiles in LDS), so no transposed copy of an activation exists.
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

// Bump allocator over the workspace.  With base == nullptr it only measures.
struct Arena {
    char* base = nullptr;
    size_t used = 0;
    void* take(size_t bytes) {
        const size_t a = (used + 255) & ~size_t(255);
        used = a + bytes;
        return base ? base + a : nullptr;
    }
};

struct Stream {                     // one padded token stream of the bound layout + its device tables
    int32_t* row_valid = nullptr;   // [max_rows]  sorted sequence position, or -1 for padding
    int32_t* seq_row = nullptr;     // [max_seqs]
    int32_t* seq_len = nullptr;     // [max_seqs]
    int R = 0, max_len = 0;
    bool has_pad = false;
};

struct GptBufs {
    void *u1, *qkv, *o, *x1, *u2, *z, *a, *xout;
    float *stats1, *stats2, *lse;
    void *wqkv_t, *wo_t, *w1_t, *w2_t;          // [out][in] copies of the layer's matrices (nt mode)
};

struct T5Bufs {                                  // encoder layer; a decoder layer also uses the cross-attention part
    void *u1, *qkv, *o, *x1, *u2, *zg, *zu, *a, *xout;
    float *stats1, *stats2, *lse;
    void *uc, *qc, *kvc, *oc, *x2;
    float *statsc, *lsec;
    void *wqkv_t, *wo_t, *wg_t, *wu_t, *w2_t, *wcq_t, *wckv_t, *wco_t;
};

}  // namespace

struct ds_stage {
    ds_stage_config cfg{};
    size_t es = 4;
    void* ws = nullptr;
    size_t ws_bytes = 0;
    Arena arena;
    Stream main, tgt;
    int32_t n_seq = 0;
    int32_t* h_tables = nullptr;       // pinned staging for table uploads
    hipEvent_t upload_done = nullptr;
    uint64_t bound_uid = 0;
    std::vector<GptBufs> gpt;
    std::vector<T5Bufs> enc, dec;
    // backward temporaries (sized for the longer stream)
    void *x0 = nullptr, *y0 = nullptr, *dyA = nullptr, *dyB = nullptr, *dz = nullptr, *dz2 = nullptr, *du = nullptr,
         *dx1 = nullptr, *dx2 = nullptr, *d_o = nullptr, *dqkv = nullptr, *dqc = nullptr, *dkvc = nullptr, *de = nullptr,
         *deB = nullptr;
    float *delta = nullptr, *partial = nullptr, *split_ws = nullptr;
    // Bias-gradient column sums (decoder-only stage) run on a stream of their own beside the GEMMs that follow their
    // producer: nothing on the main stream reads what they write, so they only have to be back before the tensor they
    // read is overwritten (joined at the end of every layer's backward pass).  Same priority as the caller's stream.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    float* partial_side = nullptr;     // their partial sums (the main stream's `partial` belongs to the norm kernels)
    bool side_pending = false;
    float* colsum_rows = nullptr;      // partial column sums written by the GELU-backward GEMM epilogue (decoder-only stage)
    // scratch of the matrix-core attention kernels (work lists, backward statistics): one per kind of attention the
    // model runs (decoder-only: causal self-attention; encoder-decoder: encoder self-, decoder self-, cross-attention)
    void* attn_scratch[3] = {nullptr, nullptr, nullptr};
    size_t attn_scratch_bytes = 0;
    bool nt_mode = false;
    // the attention work lists in a scratch depend only on the layout and on which streams / mask they were built
    // for: they are kept across layers and calls while both stay the same
    uint64_t lists_uid[3] = {0, 0, 0};
    int lists_kind[3] = {-1, -1, -1};
    size_t split_ws_floats = 0;
    int32_t launches = 0;
    // transposed weight copies: whose weights they were made from, and whether the caller promised those stay as they are
    bool weights_unchanged = false;
    std::vector<char> wt_key;          // the layer structs (device pointers) the copies were made from; empty = no copies
    // optional per-kernel-group timing
    bool prof_on = false;
    std::vector<hipEvent_t> ev_pool;
    std::vector<int> ev_cat;
    int ev_used = 0;
};

namespace {

#define DS_TRY(expr)                    \
    do {                                \
        ds_status st__ = (expr);        \
        if (st__ != DS_OK) return st__; \
    } while (0)

// Lays out (or, with a null arena base, measures) every workspace buffer.
void carve(ds_stage* s) {
    const ds_stage_config& c = s->cfg;
    Arena& ar = s->arena;
    ar.used = 0;
    const size_t es = s->es, d = c.d_model, F = c.d_ff, h = c.n_heads;
    const size_t R = c.max_rows, Rt = c.model == DS_MODEL_T5 ? c.max_rows_tgt : 0, Rm = std::max(R, Rt);
    const size_t S = c.max_seqs;
    const bool nt = s->nt_mode;
    auto f32 = [&](size_t n) { return (float*)ar.take(n * 4); };
    // Full recomputation: only a layer's output (the next layer's input) is kept per layer; what a layer saves for its
    // backward lives in ONE set of buffers per kind of layer, refilled by re-running the layer's forward right before
    // its backward.
    const bool share = c.recompute == DS_RECOMPUTE_FULL;
    if (c.model == DS_MODEL_GPT) {
        s->gpt.resize(c.n_layers);
        for (size_t li = 0; li < s->gpt.size(); ++li) {
            GptBufs& b = s->gpt[li];
            if (share && li > 0) {
                b = s->gpt[0];
            } else {
                b.u1 = ar.take(R * d * es); b.qkv = ar.take(R * 3 * d * es); b.o = ar.take(R * d * es);
                b.x1 = ar.take(R * d * es); b.u2 = ar.take(R * d * es); b.z = ar.take(R * F * es);
                b.a = ar.take(R * F * es);
                b.stats1 = f32(2 * R); b.stats2 = f32(2 * R); b.lse = f32(R * h);
            }
            b.xout = ar.take(R * d * es);
            b.wqkv_t = b.wo_t = b.w1_t = b.w2_t = nullptr;
            if (nt) {
                b.wqkv_t = ar.take(3 * d * d * es); b.wo_t = ar.take(d * d * es);
                b.w1_t = ar.take(d * F * es); b.w2_t = ar.take(d * F * es);
            }
        }
    } else {
        auto layer = [&](T5Bufs& b, const T5Bufs* shared, size_t rows, bool is_dec) {
            if (shared) {
                b = *shared;
            } else {
                b.u1 = ar.take(rows * d * es); b.qkv = ar.take(rows * 3 * d * es); b.o = ar.take(rows * d * es);
                b.x1 = ar.take(rows * d * es); b.u2 = ar.take(rows * d * es); b.zg = ar.take(rows * F * es);
                b.zu = ar.take(rows * F * es); b.a = ar.take(rows * F * es);
                b.stats1 = f32(2 * rows); b.stats2 = f32(2 * rows); b.lse = f32(rows * h);
                b.uc = b.qc = b.kvc = b.oc = b.x2 = nullptr;
                b.statsc = b.lsec = nullptr;
                if (is_dec) {
                    b.uc = ar.take(rows * d * es); b.qc = ar.take(rows * d * es); b.kvc = ar.take(R * 2 * d * es);
                    b.oc = ar.take(rows * d * es); b.x2 = ar.take(rows * d * es);
                    b.statsc = f32(2 * rows); b.lsec = f32(rows * h);
                }
            }
            b.xout = ar.take(rows * d * es);
            b.wqkv_t = b.wo_t = b.wg_t = b.wu_t = b.w2_t = b.wcq_t = b.wckv_t = b.wco_t = nullptr;
            if (nt) {
                b.wqkv_t = ar.take(3 * d * d * es); b.wo_t = ar.take(d * d * es);
                b.wg_t = ar.take(d * F * es); b.wu_t = ar.take(d * F * es); b.w2_t = ar.take(d * F * es);
                if (is_dec) {
                    b.wcq_t = ar.take(d * d * es); b.wckv_t = ar.take(2 * d * d * es); b.wco_t = ar.take(d * d * es);
                }
            }
        };
        s->enc.resize(c.n_layers);
        s->dec.resize(c.n_dec_layers);
        for (size_t li = 0; li < s->enc.size(); ++li) layer(s->enc[li], share && li > 0 ? &s->enc[0] : nullptr, R, false);
        for (size_t li = 0; li < s->dec.size(); ++li) layer(s->dec[li], share && li > 0 ? &s->dec[0] : nullptr, Rt, true);
    }
    s->x0 = ar.take(R * d * es);
    s->dyA = ar.take(Rm * d * es); s->dyB = ar.take(Rm * d * es);
    s->du = ar.take(Rm * d * es); s->dx1 = ar.take(Rm * d * es); s->d_o = ar.take(Rm * d * es);
    s->dz = ar.take(Rm * F * es); s->dqkv = ar.take(Rm * 3 * d * es);
    s->delta = f32(Rm * h);
    if (c.model == DS_MODEL_T5) {
        s->y0 = ar.take(Rt * d * es);
        s->dz2 = ar.take(Rm * F * es); s->dx2 = ar.take(Rt * d * es);
        s->dqc = ar.take(Rt * d * es); s->dkvc = ar.take(R * 2 * d * es);
        s->de = ar.take(R * d * es); s->deB = ar.take(R * d * es);
    }
    const size_t partial_floats = std::max<size_t>((size_t)ds_norm_bwd_scratch_floats(1, (int)d), (size_t)2048 * 1024);
    s->partial = f32(partial_floats);
    s->partial_side = c.model == DS_MODEL_GPT ? f32((size_t)2048 * 1024) : nullptr;
    s->colsum_rows = (c.model == DS_MODEL_GPT && s->nt_mode) ? f32(gemm_colsum_rows((int32_t)R) * F) : nullptr;
    s->split_ws_floats = 4 * std::max(d * 3 * d, d * F);
    s->split_ws = f32(s->split_ws_floats);
    s->main.row_valid = (int32_t*)ar.take(R * 4);
    s->main.seq_row = (int32_t*)ar.take(S * 4);
    s->main.seq_len = (int32_t*)ar.take(S * 4);
    if (Rt) {
        s->tgt.row_valid = (int32_t*)ar.take(Rt * 4);
        s->tgt.seq_row = (int32_t*)ar.take(S * 4);
        s->tgt.seq_len = (int32_t*)ar.take(S * 4);
    }
    const int hd = c.d_model / c.n_heads;
    s->attn_scratch_bytes = 0;
    for (int k = 0; k < 3; ++k) s->attn_scratch[k] = nullptr;
    if (c.dtype == DS_DTYPE_BF16 && (hd == 64 || hd == 128)) {
        s->attn_scratch_bytes = attn_scratch_bytes(c.n_heads, hd, (int)Rm, (int)Rm, (int)S);
        for (int k = 0; k < (c.model == DS_MODEL_T5 ? 3 : 1); ++k) s->attn_scratch[k] = ar.take(s->attn_scratch_bytes);
    }
    ar.take(4096);
}

ds_status upload_stream(ds_stage* s, Stream& sm, int32_t* host, int max_rows, int R, int S, const std::vector<int32_t>& row,
                        const std::vector<int32_t>& len, int64_t tokens, hipStream_t st) {
    int32_t* rv = host;
    int32_t* sr = rv + max_rows;
    int32_t* sl = sr + s->cfg.max_seqs;
    std::fill(rv, rv + R, -1);
    int max_len = 0;
    for (int i = 0; i < S; ++i) {
        sr[i] = row[i];
        sl[i] = len[i];
        max_len = std::max(max_len, len[i]);
        for (int r = 0; r < len[i]; ++r) rv[row[i] + r] = i;
    }
    DS_HIP_CHECK(hipMemcpyAsync(sm.row_valid, rv, sizeof(int32_t) * R, hipMemcpyHostToDevice, st));
    DS_HIP_CHECK(hipMemcpyAsync(sm.seq_row, sr, sizeof(int32_t) * S, hipMemcpyHostToDevice, st));
    DS_HIP_CHECK(hipMemcpyAsync(sm.seq_len, sl, sizeof(int32_t) * S, hipMemcpyHostToDevice, st));
    sm.R = R;
    sm.max_len = max_len;
    sm.has_pad = tokens != (int64_t)R;
    return DS_OK;
}

ds_status bind_layout(ds_stage* s, const ds_layout* lo, hipStream_t st) {
    if (lo->uid == s->bound_uid) return DS_OK;
    const bool t5 = s->cfg.model == DS_MODEL_T5;
    if (lo->has_tgt != t5) return DS_ELAYOUT;
    if (lo->total_rows > s->cfg.max_rows || lo->n_seq > s->cfg.max_seqs) return DS_ELAYOUT;
    if (t5 && lo->total_rows_tgt > s->cfg.max_rows_tgt) return DS_ELAYOUT;
    // a previous upload may still be reading the staging buffer
    DS_HIP_CHECK(hipEventSynchronize(s->upload_done));
    s->bound_uid = 0;
    DS_TRY(upload_stream(s, s->main, s->h_tables, s->cfg.max_rows, lo->total_rows, lo->n_seq, lo->seq_row, lo->seq_len,
                         lo->total_tokens, st));
    if (t5)
        DS_TRY(upload_stream(s, s->tgt, s->h_tables + s->cfg.max_rows + 2 * (size_t)s->cfg.max_seqs, s->cfg.max_rows_tgt,
                             lo->total_rows_tgt, lo->n_seq, lo->seq_row_tgt, lo->seq_len_tgt, lo->total_tokens_tgt, st));
    DS_HIP_CHECK(hipEventRecord(s->upload_done, st));
    s->n_seq = lo->n_seq;
    s->bound_uid = lo->uid;
    return DS_OK;
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

// The operators both model kinds are built from, each one launch (group) over a whole stream.
struct Ops {
    ds_stage* s;
    hipStream_t st;
    int accumulate;
    int dt, d, F;
    bool nt;
    int cur_kind = -1, cur_slot = 0;    // of the attention arguments built last

    ds_status gemm_raw(int cat, int ta, int tb, int M, int N, int K, const void* A, const void* B, void* C, int epi,
                       const void* bias, const void* R, const void* R2, void* C2, const int32_t* row_valid, int acc,
                       float* colsum_rows = nullptr) {
        return timed(s, cat, st, [&] {
            GemmEpi p{bias, R, R2, C2, row_valid, acc, colsum_rows};
            s->launches++;
            return launch_gemm(dt, ta, tb, M, N, K, A, B, C, epi, p, false, s->split_ws, s->split_ws_floats, st);
        });
    }
    // Y[rows,N] = X[rows,K] W[K,N] (+ epilogue); Wt = the [N][K] copy used in nt mode
    ds_status fwd(const Stream& sm, int N, int K, const void* X, const void* W, const void* Wt, void* C, int epi,
                  const void* bias, const void* R, void* C2, bool mask) {
        const int32_t* rv = mask && sm.has_pad ? sm.row_valid : nullptr;
        if (nt) return gemm_raw(DS_PROF_GEMM_FWD, 0, 1, sm.R, N, K, X, Wt, C, epi, bias, R, nullptr, C2, rv, 0);
        return gemm_raw(DS_PROF_GEMM_FWD, 0, 0, sm.R, N, K, X, W, C, epi, bias, R, nullptr, C2, rv, 0);
    }
    // dX[rows,K] = dY[rows,N] W[K,N]^T (+ epilogue)
    ds_status dgrad(const Stream& sm, int K, int N, const void* dY, const void* W, void* C, int epi, const void* R,
                    const void* R2, void* C2) {
        return gemm_raw(DS_PROF_GEMM_DGRAD, 0, 1, sm.R, K, N, dY, W, C, epi, nullptr, R, R2, C2, nullptr, 0);
    }
    // dZ[rows,K] = (dY W^T) * G with G = GELU'(Z) as the forward pass stored it, and bias_grad[K] (+)= column sums of dZ.
    // Where the GEMM kernel can, the sums come out of its epilogue (one partial row per 128 rows, then a small
    // reduction); otherwise from a pass over dZ.
    ds_status dgrad_gelu_bias(const Stream& sm, int K, int N, const void* dY, const void* W, void* dZ, const void* G,
                              void* bias_grad) {
        if (s->colsum_rows && gemm_colsum_fused(dt, 0, 1, sm.R, K, N, dY, W, dZ, DS_EPI_MULR)) {
            DS_TRY(gemm_raw(DS_PROF_GEMM_DGRAD, 0, 1, sm.R, K, N, dY, W, dZ, DS_EPI_MULR, nullptr, G, nullptr, nullptr, nullptr, 0,
                            s->colsum_rows));
            s->launches++;
            return timed(s, DS_PROF_COLSUM, st, [&] {
                return launch_reduce_partials((int32_t)gemm_colsum_rows(sm.R), K, s->colsum_rows, (float*)bias_grad, accumulate, st);
            });
        }
        DS_TRY(dgrad(sm, K, N, dY, W, dZ, DS_EPI_MULR, G, nullptr, nullptr));
        return colsum(sm, K, dZ, bias_grad);
    }
    // dW[K,N] (+)= X[rows,K]^T dY[rows,N]
    ds_status wgrad(const Stream& sm, int K, int N, const void* X, const void* dY, void* dW) {
        return gemm_raw(DS_PROF_GEMM_WGRAD, 1, 0, K, N, sm.R, X, dY, dW, DS_EPI_ACC32, nullptr, nullptr, nullptr, nullptr,
                        nullptr, accumulate);
    }
    ds_status weight_t(int K, int N, const void* W, void* Wt) {      // [K][N] -> [N][K]
        s->launches++;
        return launch_transpose_bf16(K, N, K, W, Wt, st);
    }
    ds_status colsum(const Stream& sm, int n, const void* x, void* out) {
        s->launches += 2;
        return timed(s, DS_PROF_COLSUM, st, [&] { return ds_colsum(dt, sm.R, n, x, (float*)out, s->partial, accumulate, st); });
    }
    // The same on the side stream: starts once everything enqueued so far on the main stream is done, runs beside
    // what is enqueued after it.  x must stay as it is, and out untouched, until join_side().
    ds_status colsum_side(const Stream& sm, int n, const void* x, void* out) {
        if (!s->side) return colsum(sm, n, x, out);
        s->launches += 2;
        DS_HIP_CHECK(hipEventRecord(s->ev_fork, st));
        DS_HIP_CHECK(hipStreamWaitEvent(s->side, s->ev_fork, 0));
        s->side_pending = true;
        return timed(s, DS_PROF_COLSUM, s->side, [&] {
            return ds_colsum(dt, sm.R, n, x, (float*)out, s->partial_side, accumulate, s->side);
        });
    }
    ds_status join_side() {
        if (!s->side_pending) return DS_OK;
        DS_HIP_CHECK(hipEventRecord(s->ev_join, s->side));
        DS_HIP_CHECK(hipStreamWaitEvent(st, s->ev_join, 0));
        s->side_pending = false;
        return DS_OK;
    }
    ds_status norm_fwd(const Stream& sm, int rms, const void* x, const void* g, const void* b, void* y, float* stats) {
        s->launches++;
        return timed(s, DS_PROF_NORM, st, [&] { return ds_norm_fwd(dt, rms, sm.R, d, x, g, b, y, stats, st); });
    }
    ds_status norm_bwd(const Stream& sm, int rms, const void* dy, const void* x, const void* g, const float* stats,
                       const void* resid, void* dx, void* dg, void* db) {
        s->launches += 2;
        return timed(s, DS_PROF_NORM, st, [&] {
            return ds_norm_bwd(dt, rms, sm.R, d, dy, x, g, stats, resid, dx, (float*)dg, (float*)db, s->partial, accumulate, st);
        });
    }
    ds_status mask_rows(const Stream& sm, const void* in, void* out) {
        s->launches++;
        return timed(s, DS_PROF_OTHER, st, [&] { return launch_mask_rows(dt, sm.R, d, in, out, sm.row_valid, st); });
    }
    ds_status zero_pad(const Stream& sm, void* buf, int cols) {
        if (!sm.has_pad) return DS_OK;
        return timed(s, DS_PROF_OTHER, st, [&] {
            const int row16 = (int)((size_t)cols * s->es / 16);
            int blocks = (sm.R + 3) / 4;
            if (blocks > 4096) blocks = 4096;
            hipLaunchKernelGGL(zero_pad_rows_kernel, dim3(blocks), dim3(256), 0, st, sm.R, row16, (uint4*)buf, sm.row_valid);
            DS_LAUNCH_CHECK();
            s->launches++;
            return DS_OK;
        });
    }
    AttnArgs attn_args(const Stream& q, const Stream& k, int mask) {
        const int h = s->cfg.n_heads, hd = d / h;
        AttnArgs a{};
        a.dtype = dt;
        a.n_seq = s->n_seq;
        a.n_heads = h;
        a.head_dim = hd;
        a.mask = mask;
        a.q_row = q.seq_row; a.q_len = q.seq_len;
        a.k_row = k.seq_row; a.k_len = k.seq_len;
        a.max_q_len = q.max_len; a.max_k_len = k.max_len;
        a.ldo = d;
        a.lse_stride = q.R;
        a.scale = 1.0f / std::sqrt((float)hd);
        a.q_total_rows = q.R;
        a.k_total_rows = k.R;
        cur_kind = (&q == &s->tgt ? 1 : 0) | (&k == &s->tgt ? 2 : 0) | (mask ? 4 : 0);
        // scratch 0: self-attention over the main stream, 1: self-attention over the target stream, 2: cross-attention
        cur_slot = s->cfg.model != DS_MODEL_T5 ? 0 : (&q != &s->tgt ? 0 : (&k == &s->tgt ? 1 : 2));
        a.scratch = s->attn_scratch[cur_slot];
        a.scratch_bytes = s->attn_scratch_bytes;
        a.lists_want_both = 1;
        a.lists_ready = (s->lists_uid[cur_slot] != 0 && s->lists_uid[cur_slot] == s->bound_uid &&
                         s->lists_kind[cur_slot] == cur_kind) ? 1 : 0;
        return a;
    }
    // after a launch that went through the matrix-core kernels: the scratch now holds both lists of this kind
    void lists_built(const AttnArgs& a) {
        if (attn_mfma_supported(a)) {
            s->lists_uid[cur_slot] = s->bound_uid;
            s->lists_kind[cur_slot] = cur_kind;
        }
    }
    // self-attention over a packed [rows, 3d] tensor
    ds_status self_fwd(const Stream& sm, int mask, const void* qkv, void* o, float* lse) {
        AttnArgs a = attn_args(sm, sm, mask);
        const char* base = (const char*)qkv;
        a.q = base; a.k = base + (size_t)d * s->es; a.v = base + (size_t)2 * d * s->es;
        a.ldq = a.ldk = a.ldv = 3 * d;
        a.o = o; a.lse = lse;
        s->launches += a.lists_ready ? 1 : 3;
        DS_TRY(timed(s, DS_PROF_ATTN_FWD, st, [&] { return launch_attention_fwd(a, false, st); }));
        lists_built(a);
        return zero_pad(sm, o, d);
    }
    ds_status self_bwd(const Stream& sm, int mask, const void* qkv, const void* o, const void* d_o, const float* lse, void* dqkv) {
        AttnArgs a = attn_args(sm, sm, mask);
        const char* base = (const char*)qkv;
        a.q = base; a.k = base + (size_t)d * s->es; a.v = base + (size_t)2 * d * s->es;
        a.ldq = a.ldk = a.ldv = 3 * d;
        a.o = const_cast<void*>(o); a.d_o = d_o; a.lse = const_cast<float*>(lse); a.delta = s->delta;
        char* g = (char*)dqkv;
        a.dq = g; a.dk = g + (size_t)d * s->es; a.dv = g + (size_t)2 * d * s->es;
        s->launches += a.lists_ready ? 2 : 4;
        DS_TRY(timed(s, DS_PROF_ATTN_BWD, st, [&] { return launch_attention_bwd(a, false, st); }));
        lists_built(a);
        return zero_pad(sm, dqkv, 3 * d);
    }
};

// ------------------------------------------------------------------------------------ GPT
ds_status gpt_fwd_bwd(ds_stage* s, const ds_gpt_layer* w, const ds_stage_io* io, const ds_gpt_layer* g, int accumulate,
                      hipStream_t st) {
    const int d = s->cfg.d_model, F = s->cfg.d_ff, L = s->cfg.n_layers;
    const Stream& sm = s->main;
    Ops op{s, st, accumulate, s->cfg.dtype, d, F, s->nt_mode};
    const size_t key_bytes = sizeof(ds_gpt_layer) * (size_t)L;
    const bool copies_valid = s->weights_unchanged && s->wt_key.size() == key_bytes && std::memcmp(s->wt_key.data(), w, key_bytes) == 0;
    if (op.nt && !copies_valid) {
        s->wt_key.clear();
        DS_TRY(timed(s, DS_PROF_TRANSPOSE, st, [&] {
            for (int l = 0; l < L; ++l) {
                GptBufs& b = s->gpt[l];
                DS_TRY(op.weight_t(d, 3 * d, w[l].w_qkv, b.wqkv_t));
                DS_TRY(op.weight_t(d, d, w[l].w_o, b.wo_t));
                DS_TRY(op.weight_t(d, F, w[l].w_1, b.w1_t));
                DS_TRY(op.weight_t(F, d, w[l].w_2, b.w2_t));
            }
            return DS_OK;
        }));
        s->wt_key.assign((const char*)w, (const char*)w + key_bytes);
    }

    // ---------------- forward (ForwardPass of every micro-batch)
    const void* x_in = io->act_in;
    if (sm.has_pad) {
        DS_TRY(op.mask_rows(sm, io->act_in, s->x0));
        x_in = s->x0;
    }
    const void* x0 = x_in;
    // forward of layer l from its input; x_out = NULL: only what the layer's backward reads (recomputation)
    auto layer_fwd = [&](int l, const void* xl, void* x_out) -> ds_status {
        GptBufs& b = s->gpt[l];
        DS_TRY(op.norm_fwd(sm, 0, xl, w[l].ln1_g, w[l].ln1_b, b.u1, b.stats1));
        DS_TRY(op.fwd(sm, 3 * d, d, b.u1, w[l].w_qkv, b.wqkv_t, b.qkv, DS_EPI_NONE, w[l].b_qkv, nullptr, nullptr, false));
        DS_TRY(op.self_fwd(sm, 1, b.qkv, b.o, b.lse));
        DS_TRY(op.fwd(sm, d, d, b.o, w[l].w_o, b.wo_t, b.x1, DS_EPI_RESID, w[l].b_o, xl, nullptr, true));
        DS_TRY(op.norm_fwd(sm, 0, b.x1, w[l].ln2_g, w[l].ln2_b, b.u2, b.stats2));
        DS_TRY(op.fwd(sm, F, d, b.u2, w[l].w_1, b.w1_t, b.z, DS_EPI_GELU_D, w[l].b_1, nullptr, b.a, false));   // b.z := GELU'(z)
        if (!x_out) return DS_OK;
        return op.fwd(sm, d, F, b.a, w[l].w_2, b.w2_t, x_out, DS_EPI_RESID, w[l].b_2, b.x1, nullptr, true);
    };
    for (int l = 0; l < L; ++l) {
        void* x_out = (l == L - 1) ? io->act_out : s->gpt[l].xout;
        DS_TRY(layer_fwd(l, x_in, x_out));
        x_in = x_out;
    }
    const bool recompute = s->cfg.recompute == DS_RECOMPUTE_FULL;

    // ---------------- backward (BackwardPass of every micro-batch; weight gradients summed over all of them)
    const void* dy = io->grad_out;
    if (sm.has_pad) {
        DS_TRY(op.mask_rows(sm, io->grad_out, s->dyA));
        dy = s->dyA;
    }
    void* pp[2] = {s->dyB, s->dyA};
    int flip = 0;
    for (int l = L - 1; l >= 0; --l) {
        GptBufs& b = s->gpt[l];
        const void* xl_in = (l == 0) ? x0 : s->gpt[l - 1].xout;
        void* dx_in = (l == 0) ? io->grad_in : pp[flip];
        // the shared buffers still hold the last layer's forward; every other layer's is run again
        if (recompute && l != L - 1) DS_TRY(layer_fwd(l, xl_in, nullptr));
        // MLP
        DS_TRY(op.colsum_side(sm, d, dy, g[l].b_2));        // (each column sum right behind its producer, beside the next GEMM)
        DS_TRY(op.wgrad(sm, F, d, b.a, dy, g[l].w_2));
        DS_TRY(op.dgrad_gelu_bias(sm, F, d, dy, w[l].w_2, s->dz, b.z, g[l].b_1));
        DS_TRY(op.wgrad(sm, d, F, b.u2, s->dz, g[l].w_1));
        DS_TRY(op.dgrad(sm, d, F, s->dz, w[l].w_1, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr));
        DS_TRY(op.norm_bwd(sm, 0, s->du, b.x1, w[l].ln2_g, b.stats2, dy, s->dx1, g[l].ln2_g, g[l].ln2_b));
        // attention
        DS_TRY(op.colsum_side(sm, d, s->dx1, g[l].b_o));
        DS_TRY(op.wgrad(sm, d, d, b.o, s->dx1, g[l].w_o));
        DS_TRY(op.dgrad(sm, d, d, s->dx1, w[l].w_o, s->d_o, DS_EPI_NONE, nullptr, nullptr, nullptr));
        DS_TRY(op.self_bwd(sm, 1, b.qkv, b.o, s->d_o, b.lse, s->dqkv));
        DS_TRY(op.colsum_side(sm, 3 * d, s->dqkv, g[l].b_qkv));
        DS_TRY(op.wgrad(sm, d, 3 * d, b.u1, s->dqkv, g[l].w_qkv));
        DS_TRY(op.dgrad(sm, d, 3 * d, s->dqkv, w[l].w_qkv, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr));
        DS_TRY(op.norm_bwd(sm, 0, s->du, xl_in, w[l].ln1_g, b.stats1, s->dx1, dx_in, g[l].ln1_g, g[l].ln1_b));
        // the next layer overwrites dx1 and dqkv, which the column sums on the side stream may still be reading
        DS_TRY(op.join_side());
        dy = dx_in;
        flip ^= 1;
    }
    return DS_OK;
}

// ------------------------------------------------------------------------------------ T5
// Self-attention sub-block forward: x1 = x + Attn(RMS1(x)) Wo
ds_status t5_self_fwd(Ops& op, const Stream& sm, int mask, const void* x, T5Bufs& b, const void* ln1_g, const void* w_qkv,
                      const void* w_o) {
    const int d = op.d;
    DS_TRY(op.norm_fwd(sm, 1, x, ln1_g, nullptr, b.u1, b.stats1));
    DS_TRY(op.fwd(sm, 3 * d, d, b.u1, w_qkv, b.wqkv_t, b.qkv, DS_EPI_NONE, nullptr, nullptr, nullptr, false));
    DS_TRY(op.self_fwd(sm, mask, b.qkv, b.o, b.lse));
    return op.fwd(sm, d, d, b.o, w_o, b.wo_t, b.x1, DS_EPI_RESID, nullptr, x, nullptr, true);
}
// Gated-GELU MLP forward: out = xin + (GELU(u Wg) * (u Wu)) W2,  u = RMS2(xin)
// (out = NULL: only what the backward reads, for recomputation)
ds_status t5_mlp_fwd(Ops& op, const Stream& sm, const void* xin, void* out, T5Bufs& b, const void* ln2_g, const void* w_g,
                     const void* w_u, const void* w_2) {
    const int d = op.d, F = op.F;
    DS_TRY(op.norm_fwd(sm, 1, xin, ln2_g, nullptr, b.u2, b.stats2));
    DS_TRY(op.fwd(sm, F, d, b.u2, w_g, b.wg_t, b.zg, DS_EPI_NONE, nullptr, nullptr, nullptr, false));
    DS_TRY(op.fwd(sm, F, d, b.u2, w_u, b.wu_t, b.zu, DS_EPI_GATE, nullptr, b.zg, b.a, false));
    if (!out) return DS_OK;
    return op.fwd(sm, d, F, b.a, w_2, b.w2_t, out, DS_EPI_RESID, nullptr, xin, nullptr, true);
}
// MLP backward: dy = gradient of the MLP output; writes dy + RMS2-backward(...) (the gradient of xin) into dxin
ds_status t5_mlp_bwd(Ops& op, const Stream& sm, const void* dy, const void* xin, void* dxin, T5Bufs& b, const void* ln2_g,
                     const void* w_g, const void* w_u, const void* w_2, void* g_ln2, void* g_wg, void* g_wu, void* g_w2) {
    ds_stage* s = op.s;
    const int d = op.d, F = op.F;
    DS_TRY(op.wgrad(sm, F, d, b.a, dy, g_w2));
    DS_TRY(op.dgrad(sm, F, d, dy, w_2, s->dz, DS_EPI_DGATE, b.zg, b.zu, s->dz2));      // dz = d zg, dz2 = d zu
    DS_TRY(op.wgrad(sm, d, F, b.u2, s->dz, g_wg));
    DS_TRY(op.wgrad(sm, d, F, b.u2, s->dz2, g_wu));
    DS_TRY(op.dgrad(sm, d, F, s->dz, w_g, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr));
    DS_TRY(op.dgrad(sm, d, F, s->dz2, w_u, s->d_o, DS_EPI_RESID, s->du, nullptr, nullptr));   // d_o = du + dzu Wu^T
    return op.norm_bwd(sm, 1, s->d_o, xin, ln2_g, b.stats2, dy, dxin, g_ln2, nullptr);
}
// Self-attention sub-block backward: dy = gradient of x1; writes the gradient of x into dx
ds_status t5_self_bwd(Ops& op, const Stream& sm, int mask, const void* dy, const void* x, void* dx, T5Bufs& b,
                      const void* ln1_g, const void* w_qkv, const void* w_o, void* g_ln1, void* g_wqkv, void* g_wo) {
    ds_stage* s = op.s;
    const int d = op.d;
    DS_TRY(op.wgrad(sm, d, d, b.o, dy, g_wo));
    DS_TRY(op.dgrad(sm, d, d, dy, w_o, s->d_o, DS_EPI_NONE, nullptr, nullptr, nullptr));
    DS_TRY(op.self_bwd(sm, mask, b.qkv, b.o, s->d_o, b.lse, s->dqkv));
    DS_TRY(op.wgrad(sm, d, 3 * d, b.u1, s->dqkv, g_wqkv));
    DS_TRY(op.dgrad(sm, d, 3 * d, s->dqkv, w_qkv, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr));
    return op.norm_bwd(sm, 1, s->du, x, ln1_g, b.stats1, dy, dx, g_ln1, nullptr);
}

ds_status t5_fwd_bwd(ds_stage* s, const ds_t5_enc_layer* we, const ds_t5_dec_layer* wd, const ds_stage_io* io,
                     const ds_t5_enc_layer* ge, const ds_t5_dec_layer* gd, int accumulate, hipStream_t st) {
    const int d = s->cfg.d_model, F = s->cfg.d_ff, Le = s->cfg.n_layers, Ld = s->cfg.n_dec_layers;
    const Stream& E = s->main;
    const Stream& D = s->tgt;
    Ops op{s, st, accumulate, s->cfg.dtype, d, F, s->nt_mode};
    const size_t key_e = sizeof(ds_t5_enc_layer) * (size_t)Le, key_d = sizeof(ds_t5_dec_layer) * (size_t)Ld;
    const bool copies_valid = s->weights_unchanged && s->wt_key.size() == key_e + key_d &&
                              std::memcmp(s->wt_key.data(), we, key_e) == 0 && std::memcmp(s->wt_key.data() + key_e, wd, key_d) == 0;
    if (op.nt && !copies_valid) {
        s->wt_key.clear();
        DS_TRY(timed(s, DS_PROF_TRANSPOSE, st, [&] {
            for (int l = 0; l < Le; ++l) {
                T5Bufs& b = s->enc[l];
                DS_TRY(op.weight_t(d, 3 * d, we[l].w_qkv, b.wqkv_t));
                DS_TRY(op.weight_t(d, d, we[l].w_o, b.wo_t));
                DS_TRY(op.weight_t(d, F, we[l].w_g, b.wg_t));
                DS_TRY(op.weight_t(d, F, we[l].w_u, b.wu_t));
                DS_TRY(op.weight_t(F, d, we[l].w_2, b.w2_t));
            }
            for (int l = 0; l < Ld; ++l) {
                T5Bufs& b = s->dec[l];
                DS_TRY(op.weight_t(d, 3 * d, wd[l].w_qkv, b.wqkv_t));
                DS_TRY(op.weight_t(d, d, wd[l].w_o, b.wo_t));
                DS_TRY(op.weight_t(d, d, wd[l].w_cq, b.wcq_t));
                DS_TRY(op.weight_t(d, 2 * d, wd[l].w_ckv, b.wckv_t));
                DS_TRY(op.weight_t(d, d, wd[l].w_co, b.wco_t));
                DS_TRY(op.weight_t(d, F, wd[l].w_g, b.wg_t));
                DS_TRY(op.weight_t(d, F, wd[l].w_u, b.wu_t));
                DS_TRY(op.weight_t(F, d, wd[l].w_2, b.w2_t));
            }
            return DS_OK;
        }));
        s->wt_key.assign((const char*)we, (const char*)we + key_e);
        s->wt_key.insert(s->wt_key.end(), (const char*)wd, (const char*)wd + key_d);
    }

    // ---------------- forward: encoder layers over the input stream
    const void* x_in = io->act_in;
    if (E.has_pad) {
        DS_TRY(op.mask_rows(E, io->act_in, s->x0));
        x_in = s->x0;
    }
    const void* x0 = x_in;
    const bool recompute = s->cfg.recompute == DS_RECOMPUTE_FULL;
    // forward of encoder layer l from its input; with_out = false: only what its backward reads (recomputation)
    auto enc_layer_fwd = [&](int l, const void* xl, bool with_out) -> ds_status {
        T5Bufs& b = s->enc[l];
        DS_TRY(t5_self_fwd(op, E, 0, xl, b, we[l].ln1_g, we[l].w_qkv, we[l].w_o));
        return t5_mlp_fwd(op, E, b.x1, with_out ? b.xout : nullptr, b, we[l].ln2_g, we[l].w_g, we[l].w_u, we[l].w_2);
    };
    for (int l = 0; l < Le; ++l) {
        DS_TRY(enc_layer_fwd(l, x_in, true));
        x_in = s->enc[l].xout;
    }
    const void* enc_out = x_in;

    // ---------------- forward: decoder layers over the target stream
    const void* y_in = io->act_in_tgt;
    if (D.has_pad) {
        DS_TRY(op.mask_rows(D, io->act_in_tgt, s->y0));
        y_in = s->y0;
    }
    const void* y0 = y_in;
    // forward of decoder layer l from its input; y_out = NULL: only what its backward reads (recomputation)
    auto dec_layer_fwd = [&](int l, const void* yl, void* y_out) -> ds_status {
        T5Bufs& b = s->dec[l];
        DS_TRY(t5_self_fwd(op, D, 1, yl, b, wd[l].ln1_g, wd[l].w_qkv, wd[l].w_o));
        // cross-attention: queries from the decoder stream, keys / values from the encoder output
        DS_TRY(op.norm_fwd(D, 1, b.x1, wd[l].lnc_g, nullptr, b.uc, b.statsc));
        DS_TRY(op.fwd(D, d, d, b.uc, wd[l].w_cq, b.wcq_t, b.qc, DS_EPI_NONE, nullptr, nullptr, nullptr, false));
        DS_TRY(op.fwd(E, 2 * d, d, enc_out, wd[l].w_ckv, b.wckv_t, b.kvc, DS_EPI_NONE, nullptr, nullptr, nullptr, false));
        {
            AttnArgs a = op.attn_args(D, E, 0);
            a.q = b.qc; a.ldq = d;
            a.k = b.kvc; a.v = (const char*)b.kvc + (size_t)d * s->es; a.ldk = a.ldv = 2 * d;
            a.o = b.oc; a.lse = b.lsec;
            s->launches += 2;
            DS_TRY(timed(s, DS_PROF_ATTN_FWD, st, [&] { return launch_attention_fwd(a, false, st); }));
            op.lists_built(a);
            DS_TRY(op.zero_pad(D, b.oc, d));
        }
        DS_TRY(op.fwd(D, d, d, b.oc, wd[l].w_co, b.wco_t, b.x2, DS_EPI_RESID, nullptr, b.x1, nullptr, true));
        return t5_mlp_fwd(op, D, b.x2, y_out, b, wd[l].ln2_g, wd[l].w_g, wd[l].w_u, wd[l].w_2);
    };
    for (int l = 0; l < Ld; ++l) {
        void* y_out = (l == Ld - 1) ? io->act_out : s->dec[l].xout;
        DS_TRY(dec_layer_fwd(l, y_in, y_out));
        y_in = y_out;
    }

    // ---------------- backward: decoder layers (last to first); de accumulates the gradient of the encoder output
    const void* dy = io->grad_out;
    if (D.has_pad) {
        DS_TRY(op.mask_rows(D, io->grad_out, s->dyA));
        dy = s->dyA;
    }
    void* pp[2] = {s->dyB, s->dyA};
    int flip = 0;
    bool de_set = false;
    void* de_cur = s->de;
    void* de_alt = s->deB;
    for (int l = Ld - 1; l >= 0; --l) {
        T5Bufs& b = s->dec[l];
        const void* yl_in = (l == 0) ? y0 : s->dec[l - 1].xout;
        void* dy_in = (l == 0) ? io->grad_in_tgt : pp[flip];
        if (recompute && l != Ld - 1) DS_TRY(dec_layer_fwd(l, yl_in, nullptr));
        // MLP: gradient of x2 into dx2
        DS_TRY(t5_mlp_bwd(op, D, dy, b.x2, s->dx2, b, wd[l].ln2_g, wd[l].w_g, wd[l].w_u, wd[l].w_2, gd[l].ln2_g, gd[l].w_g,
                          gd[l].w_u, gd[l].w_2));
        // cross-attention: gradient of x1 into dx1, of the encoder output into de
        DS_TRY(op.wgrad(D, d, d, b.oc, s->dx2, gd[l].w_co));
        DS_TRY(op.dgrad(D, d, d, s->dx2, wd[l].w_co, s->d_o, DS_EPI_NONE, nullptr, nullptr, nullptr));
        {
            AttnArgs a = op.attn_args(D, E, 0);
            a.q = b.qc; a.ldq = d;
            a.k = b.kvc; a.v = (const char*)b.kvc + (size_t)d * s->es; a.ldk = a.ldv = 2 * d;
            a.o = b.oc; a.d_o = s->d_o; a.lse = b.lsec; a.delta = s->delta;
            a.dq = s->dqc; a.dk = s->dkvc; a.dv = (char*)s->dkvc + (size_t)d * s->es;
            s->launches += 4;
            DS_TRY(timed(s, DS_PROF_ATTN_BWD, st, [&] { return launch_attention_bwd(a, false, st); }));
            op.lists_built(a);
            DS_TRY(op.zero_pad(D, s->dqc, d));
            DS_TRY(op.zero_pad(E, s->dkvc, 2 * d));
        }
        DS_TRY(op.wgrad(D, d, d, b.uc, s->dqc, gd[l].w_cq));
        DS_TRY(op.wgrad(E, d, 2 * d, enc_out, s->dkvc, gd[l].w_ckv));
        if (!de_set) {
            DS_TRY(op.dgrad(E, d, 2 * d, s->dkvc, wd[l].w_ckv, de_cur, DS_EPI_NONE, nullptr, nullptr, nullptr));
            de_set = true;
        } else {
            DS_TRY(op.dgrad(E, d, 2 * d, s->dkvc, wd[l].w_ckv, de_alt, DS_EPI_RESID, de_cur, nullptr, nullptr));
            std::swap(de_cur, de_alt);
        }
        DS_TRY(op.dgrad(D, d, d, s->dqc, wd[l].w_cq, s->du, DS_EPI_NONE, nullptr, nullptr, nullptr));
        DS_TRY(op.norm_bwd(D, 1, s->du, b.x1, wd[l].lnc_g, b.statsc, s->dx2, s->dx1, gd[l].lnc_g, nullptr));
        // causal self-attention: gradient of the layer input
        DS_TRY(t5_self_bwd(op, D, 1, s->dx1, yl_in, dy_in, b, wd[l].ln1_g, wd[l].w_qkv, wd[l].w_o, gd[l].ln1_g, gd[l].w_qkv,
                           gd[l].w_o));
        dy = dy_in;
        flip ^= 1;
    }

    // ---------------- backward: encoder layers.  The ping-pong buffers are free again.
    const void* dx = de_cur;
    flip = 0;
    for (int l = Le - 1; l >= 0; --l) {
        T5Bufs& b = s->enc[l];
        const void* xl_in = (l == 0) ? x0 : s->enc[l - 1].xout;
        void* dx_in = (l == 0) ? io->grad_in : pp[flip];
        if (recompute && l != Le - 1) DS_TRY(enc_layer_fwd(l, xl_in, false));
        DS_TRY(t5_mlp_bwd(op, E, dx, b.x1, s->dx1, b, we[l].ln2_g, we[l].w_g, we[l].w_u, we[l].w_2, ge[l].ln2_g, ge[l].w_g,
                          ge[l].w_u, ge[l].w_2));
        DS_TRY(t5_self_bwd(op, E, 0, s->dx1, xl_in, dx_in, b, we[l].ln1_g, we[l].w_qkv, we[l].w_o, ge[l].ln1_g, ge[l].w_qkv,
                           ge[l].w_o));
        dx = dx_in;
        flip ^= 1;
    }
    return DS_OK;
}

}  // namespace

namespace {
ds_status check_config(const ds_stage_config* cfg) {
    if (cfg->model != DS_MODEL_GPT && cfg->model != DS_MODEL_T5) return DS_EINVAL;
    if (cfg->dtype != DS_DTYPE_F32 && cfg->dtype != DS_DTYPE_BF16) return DS_EINVAL;
    if (cfg->n_layers <= 0 || cfg->d_model <= 0 || cfg->n_heads <= 0 || cfg->d_ff <= 0) return DS_EINVAL;
    if (cfg->d_model % cfg->n_heads || cfg->d_model % 8 || cfg->d_ff % 8 || cfg->d_model > 4096) return DS_EINVAL;
    const int hd = cfg->d_model / cfg->n_heads;
    if (hd > 128 || hd % 8) return DS_EINVAL;
    if (cfg->max_rows <= 0 || cfg->max_seqs <= 0) return DS_EINVAL;
    if (cfg->model == DS_MODEL_GPT && (cfg->n_dec_layers != 0 || cfg->max_rows_tgt != 0)) return DS_EINVAL;
    if (cfg->model == DS_MODEL_T5 && (cfg->n_dec_layers <= 0 || cfg->max_rows_tgt <= 0)) return DS_EINVAL;
    if (cfg->recompute != DS_RECOMPUTE_NONE && cfg->recompute != DS_RECOMPUTE_FULL) return DS_EINVAL;
    return DS_OK;
}
// a stage object with its workspace measured (arena.used) but not allocated
ds_status measure(const ds_stage_config* cfg, ds_stage** out) {
    ds_stage* s = new (std::nothrow) ds_stage();
    if (!s) return DS_ENOMEM;
    s->cfg = *cfg;
    s->es = dtype_size(cfg->dtype);
    s->nt_mode = cfg->dtype == DS_DTYPE_BF16 && cfg->d_model % 256 == 0 && cfg->d_ff % 256 == 0;
    try {
        carve(s);                                   // measuring pass
    } catch (const std::bad_alloc&) {
        delete s;
        return DS_ENOMEM;
    }
    *out = s;
    return DS_OK;
}
}  // namespace

extern "C" int64_t ds_stage_workspace_need(const ds_stage_config* cfg) {
    ds_stage* s = nullptr;
    if (!cfg || check_config(cfg) != DS_OK || measure(cfg, &s) != DS_OK) return -1;
    const int64_t need = (int64_t)s->arena.used;
    delete s;
    return need;
}

extern "C" ds_status ds_stage_create(const ds_stage_config* cfg, ds_stage** out) {
    if (!cfg || !out) return DS_EINVAL;
    *out = nullptr;
    DS_TRY(check_config(cfg));
    ds_stage* s = nullptr;
    DS_TRY(measure(cfg, &s));
    const size_t need = s->arena.used;
    if (hipMalloc(&s->ws, need) != hipSuccess) {
        (void)hipGetLastError();
        delete s;
        return DS_ENOMEM;
    }
    s->ws_bytes = need;
    s->arena.base = (char*)s->ws;
    carve(s);
    const size_t ints = (size_t)cfg->max_rows + (size_t)cfg->max_rows_tgt + 4 * (size_t)cfg->max_seqs;
    bool ok = hipHostMalloc((void**)&s->h_tables, ints * 4, hipHostMallocDefault) == hipSuccess &&
              hipEventCreateWithFlags(&s->upload_done, hipEventDisableTiming) == hipSuccess;
    if (ok && cfg->model == DS_MODEL_GPT)
        ok = hipStreamCreateWithFlags(&s->side, hipStreamNonBlocking) == hipSuccess &&
             hipEventCreateWithFlags(&s->ev_fork, hipEventDisableTiming) == hipSuccess &&
             hipEventCreateWithFlags(&s->ev_join, hipEventDisableTiming) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        ds_stage_destroy(s);
        return DS_EHIP;
    }
    *out = s;
    return DS_OK;
}

extern "C" void ds_stage_destroy(ds_stage* s) {
    if (!s) return;
    for (hipEvent_t e : s->ev_pool) (void)hipEventDestroy(e);
    if (s->upload_done) (void)hipEventDestroy(s->upload_done);
    if (s->ev_fork) (void)hipEventDestroy(s->ev_fork);
    if (s->ev_join) (void)hipEventDestroy(s->ev_join);
    if (s->side) (void)hipStreamDestroy(s->side);
    if (s->h_tables) (void)hipHostFree(s->h_tables);
    if (s->ws) (void)hipFree(s->ws);
    delete s;
}

extern "C" ds_status ds_stage_weights_unchanged(ds_stage* s, int32_t unchanged) {
    if (!s) return DS_EINVAL;
    s->weights_unchanged = unchanged != 0;
    return DS_OK;
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
    const bool t5 = s->cfg.model == DS_MODEL_T5;
    if (t5 && (!weights_dec || !grads_dec || !io->act_in_tgt || !io->grad_in_tgt)) return DS_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    ds_status r = bind_layout(s, lo, st);
    if (r != DS_OK) return r;
    s->launches = 0;
    if (!t5) return gpt_fwd_bwd(s, (const ds_gpt_layer*)weights, io, (const ds_gpt_layer*)grads, accumulate ? 1 : 0, st);
    return t5_fwd_bwd(s, (const ds_t5_enc_layer*)weights, (const ds_t5_dec_layer*)weights_dec, io,
                      (const ds_t5_enc_layer*)grads, (const ds_t5_dec_layer*)grads_dec, accumulate ? 1 : 0, st);
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
