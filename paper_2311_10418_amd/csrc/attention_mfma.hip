// bf16 variable-length attention on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16),
// head_dim 64 or 128, causal or unmasked (bidirectional / cross), forward and backward.
//
// Register layout (all three kernels).  A wavefront owns 32 "column" items (queries in forward and
// dQ, keys in dK/dV) and keeps them in the MFMA B operand, so that the score tile it computes is
// TRANSPOSED: lane l holds column l%32 and 16 of the 32 rows.  Everything that is per column
// (running max, running sum, log-sum-exp, delta, the rescale of the output accumulator) is then a
// per-lane scalar, and row reductions are in-lane plus one exchange between lanes l and l^32.  The
// probabilities leave the accumulator registers as the B operand of the second product without any
// data movement: accumulator registers 8u..8u+7 of a tile ARE a valid 16-deep B fragment provided
// the A operand lists the contraction index in the matching order,
//     slot j of lane-half g  <->  row 16t + 8*(j/4) + 4*g + j%4           (t = 16-row step).
//
// Memory layout.  The second product needs its A operand transposed (V^T, K^T, Q^T, dO^T).  A
// helper kernel (seq_transpose) writes feature-major copies of those tensors once per call, each
// sequence padded with zeros to a multiple of 64 tokens and the 64 tokens of a tile stored in the
// slot order above, so that one 16-byte LDS read yields a whole A fragment.  With that, EVERY tile
// an attention kernel consumes is a set of 16-byte-aligned contiguous row segments and goes
// global -> LDS directly (global_load_lds_dwordx4): no staging registers, double-buffered, the next
// 64-row block in flight while the current one feeds the MFMAs.  LDS tiles carry a 16-byte XOR
// swizzle (chosen per lane at load time) that makes the 16-byte fragment reads conflict-free on
// gfx950's 64-bank LDS.
//
// Backward is split into a dQ kernel and a dK/dV kernel so that every output element has one
// owner: no atomics, results are bit-reproducible.  Sequences are addressed through (row, length)
// tables, so padding rows cost nothing and packed layouts need no mask.
#include "attention.hpp"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// LDS swizzles.  gfx950 serves a 16-byte LDS read for 16 lanes per cycle (64 banks), so 16
// consecutive rows read at the same chunk index must fall into 16 different 16-byte units of a
// 256-byte window: 256-byte rows XOR the chunk with row%16, 128-byte rows with (row/2)%8.
template <int HD> __device__ __forceinline__ int off_rows(int row, int chunk) {      // [row][HD] tile
    return HD == 128 ? row * 256 + ((chunk ^ (row & 15)) << 4) : row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4);
}
__device__ __forceinline__ int off_tr(int d, int kg) {                                // [d][64 slots] tile
    return d * 128 + ((kg ^ ((d >> 1) & 7)) << 4);
}
__device__ __forceinline__ int slot_row(int t, int g, int j) { return 16 * t + 8 * (j >> 2) + 4 * g + (j & 3); }

__device__ __forceinline__ uint32_t pick4(const uint4& v, int w) {
    return w == 0 ? v.x : (w == 1 ? v.y : (w == 2 ? v.z : v.w));
}

// accumulator registers 8u..8u+7 of a 32x32 tile -> one bf16 B fragment
__device__ __forceinline__ bf16x8_t frag_from_acc(const f32x16_t& a, int u) {
    bf16x8_t f;
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = (bf16_t)a[8 * u + j];
    return f;
}

// store a transposed [HD x 32] accumulator block: lane column = row `row` of the output, 4 consecutive d per group
template <int HD>
__device__ __forceinline__ void store_cols(const f32x16_t (&acc)[HD / 32], float mul, bf16_t* __restrict__ out_row, int g) {
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4_t v;
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (bf16_t)(acc[dt][4 * q4 + j] * mul);
            *reinterpret_cast<bf16x4_t*>(out_row + dt * 32 + 8 * q4 + 4 * g) = v;
        }
}


typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// column of sequence s in a feature-major (transposed) copy; `row` is the sequence's first stream row
__device__ __forceinline__ long long tcol(int row, int s) { return (long long)((row + 63) & ~63) + 128LL * s; }

// ------------------------------------------------------------------------------------ seq_transpose
// out[c][tcol(s) + 64*tile + p] = in[row_s + 64*tile + slot_row(p)][c]  (zero beyond the sequence's
// length, up to the end of its last 64-token tile), for c in [0, C).  One work-group: 64 tokens x
// 256 features; each lane loads 8 token rows x 16 bytes, transposes 8x8 in registers, stores 8
// feature rows x 16 bytes; loads and stores form 128-byte contiguous segments.
__global__ __launch_bounds__(256) void seq_transpose_kernel(int C, const int32_t* __restrict__ seq_row,
                                                            const int32_t* __restrict__ seq_len,
                                                            const bf16_t* __restrict__ in, long long ld_in,
                                                            bf16_t* __restrict__ out, long long ld_out) {
    const int s = blockIdx.z, tile = blockIdx.y;
    const int len = seq_len[s];
    if (tile * 64 >= len) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bx = lane & 7, by = lane >> 3;
    const int c0 = blockIdx.x * 256 + wave * 64 + bx * 8;
    if (c0 >= C) return;
    const int row0 = seq_row[s];
    const int t = by >> 1, g = by & 1;
    uint32_t v[8][4];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int q = tile * 64 + slot_row(t, g, j);
        uint4 x = make_uint4(0u, 0u, 0u, 0u);
        if (q < len) x = *reinterpret_cast<const uint4*>(in + (long long)(row0 + q) * ld_in + c0);
        v[j][0] = x.x; v[j][1] = x.y; v[j][2] = x.z; v[j][3] = x.w;
    }
    bf16_t* o = out + tcol(row0, s) + tile * 64 + by * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
        const int w = i >> 1;
        uint4 r;
        r.x = __builtin_amdgcn_perm(v[1][w], v[0][w], sel);
        r.y = __builtin_amdgcn_perm(v[3][w], v[2][w], sel);
        r.z = __builtin_amdgcn_perm(v[5][w], v[4][w], sel);
        r.w = __builtin_amdgcn_perm(v[7][w], v[6][w], sel);
        *reinterpret_cast<uint4*>(o + (long long)(c0 + i) * ld_out) = r;
    }
}

// ------------------------------------------------------------------------------------ direct-to-LDS tile loads
// Token-major tile: 64 rows (row0.., clamped to the last valid row) x HD columns of a row-major tensor.
template <int HD>
__device__ __forceinline__ void issue_rows(char* __restrict__ lds, const bf16_t* __restrict__ base, long long ld, int row0,
                                           int n_valid, int wave, int lane) {
    constexpr int PER_WAVE = HD / 32;                 // wavefront instructions (1 KB each) per wavefront
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int u = (wave * PER_WAVE + i) * 64 + lane;
        int row, chunk;
        if (HD == 128) { row = u >> 4; chunk = (u & 15) ^ (row & 15); }
        else           { row = u >> 3; chunk = (u & 7) ^ ((row >> 1) & 7); }
        int r = row0 + row;
        r = r < n_valid ? r : n_valid - 1;
        __builtin_amdgcn_global_load_lds((gptr_t)(base + (long long)r * ld + chunk * 8),
                                         (lptr_t)(lds + (wave * PER_WAVE + i) * 1024), 16, 0, 0);
    }
}
// Feature-major tile: HD rows x 64 tokens (already padded and slot-ordered by seq_transpose).
template <int HD>
__device__ __forceinline__ void issue_cols(char* __restrict__ lds, const bf16_t* __restrict__ base_t, long long ld_t,
                                           long long col0, int wave, int lane) {
    constexpr int PER_WAVE = HD / 32;
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int u = (wave * PER_WAVE + i) * 64 + lane;
        const int d = u >> 3;
        const int chunk = (u & 7) ^ ((d >> 1) & 7);
        __builtin_amdgcn_global_load_lds((gptr_t)(base_t + (long long)d * ld_t + col0 + chunk * 8),
                                         (lptr_t)(lds + (wave * PER_WAVE + i) * 1024), 16, 0, 0);
    }
}

// wait for this wavefront's outstanding direct loads, then for everybody's
__device__ __forceinline__ void wait_tiles_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
    __builtin_amdgcn_s_barrier();
}

// ------------------------------------------------------------------------------------ forward
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TILE = 64 * HD * 2;                  // bytes of one K tile == one V^T tile
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int s = a.n_seq - 1 - blockIdx.z, h = blockIdx.y;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const int q0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * 128;
    if (q0 >= ql) return;
    const int krow = a.k_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + (long long)a.q_row[s] * a.ldq + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + (long long)krow * a.ldk + h * HD;
    const bf16_t* Vt = (const bf16_t*)a.vT + (long long)h * HD * a.ldTk;
    const long long kcol = tcol(krow, s);
    const int qw0 = q0 + wave * 32;
    const int qi = qw0 + col;
    const int qi_c = qi < ql ? qi : ql - 1;

    bf16x8_t qf[HD / 16];
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks)
        qf[ks] = *reinterpret_cast<const bf16x8_t*>(Q + (long long)qi_c * a.ldq + ks * 16 + g * 8);

    f32x16_t oacc[HD / 32];
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const float c = a.scale * kLog2e;

    const int kv_end = CAUSAL ? min(kl, q0 + 128) : kl;
    const int wave_last = CAUSAL ? min(kl - 1, qw0 + 31) : kl - 1;     // last key this wavefront can see
    const int nb = (kv_end + 63) / 64;
    issue_rows<HD>(smem, K, a.ldk, 0, kl, wave, lane);
    issue_cols<HD>(smem + TILE, Vt, a.ldTk, kcol, wave, lane);
    for (int b = 0; b < nb; ++b) {
        const int kv0 = b * 64;
        char* sK = smem + (b & 1) * (2 * TILE);
        char* sVt = sK + TILE;
        wait_tiles_and_sync();                          // block b has landed; the other stage is free
        if (b + 1 < nb) {
            char* nK = smem + ((b + 1) & 1) * (2 * TILE);
            issue_rows<HD>(nK, K, a.ldk, kv0 + 64, kl, wave, lane);
            issue_cols<HD>(nK + TILE, Vt, a.ldTk, kcol + kv0 + 64, wave, lane);
        }
        if (kv0 > wave_last || qw0 >= ql) continue;

        f32x16_t sacc[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[kt][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sK + off_rows<HD>(kt * 32 + col, ks * 2 + g));
                sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[kt], 0, 0, 0);
            }
        const bool need_mask = (kv0 + 64 > kl) || (CAUSAL && kv0 + 63 > qw0);
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float v = sacc[kt][e] * c;
                if (need_mask) {
                    const int key = kv0 + kt * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (key >= kl || (CAUSAL && key > qi)) v = -INFINITY;
                }
                sacc[kt][e] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        float rs = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(sacc[kt][e] - m_new);
                sacc[kt][e] = p;
                rs += p;
            }
        lsum = lsum * alpha + rs;
        m = m_new;
#pragma unroll
        for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[dt][e] *= alpha;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bf16x8_t pf = frag_from_acc(sacc[t >> 1], t & 1);
#pragma unroll
            for (int dt = 0; dt < HD / 32; ++dt) {
                const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(sVt + off_tr(dt * 32 + col, 2 * t + g));
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[dt], 0, 0, 0);
            }
        }
    }
    lsum += __shfl_xor(lsum, 32, 64);
    if (qi < ql) {
        const long long row = (long long)a.q_row[s] + qi;
        store_cols<HD>(oacc, 1.0f / lsum, (bf16_t*)a.o + row * a.ldo + h * HD, g);
        if (g == 0) a.lse[(size_t)h * a.lse_stride + row] = (m + __builtin_amdgcn_logf(lsum)) * kLn2;
    }
}

// ------------------------------------------------------------------------------------ backward: dQ
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TILE = 64 * HD * 2;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int s = a.n_seq - 1 - blockIdx.z, h = blockIdx.y;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const int q0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * 128;
    if (q0 >= ql) return;
    const long long qrow0 = a.q_row[s];
    const int krow = a.k_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* dO = (const bf16_t*)a.d_o + qrow0 * a.ldo + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + (long long)krow * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + (long long)krow * a.ldv + h * HD;
    const bf16_t* Kt = (const bf16_t*)a.kT + (long long)h * HD * a.ldTk;
    const long long kcol = tcol(krow, s);
    const int qw0 = q0 + wave * 32;
    const int qi = qw0 + col;
    const int qi_c = qi < ql ? qi : ql - 1;

    bf16x8_t qf[HD / 16], dof[HD / 16];
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) {
        qf[ks] = *reinterpret_cast<const bf16x8_t*>(Q + (long long)qi_c * a.ldq + ks * 16 + g * 8);
        dof[ks] = *reinterpret_cast<const bf16x8_t*>(dO + (long long)qi_c * a.ldo + ks * 16 + g * 8);
    }
    const float lse2 = a.lse[(size_t)h * a.lse_stride + qrow0 + qi_c] * kLog2e;
    const float delta = a.delta[(size_t)h * a.lse_stride + qrow0 + qi_c];
    const float c = a.scale * kLog2e;

    f32x16_t gacc[HD / 32];
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) gacc[dt][e] = 0.f;

    const int kv_end = CAUSAL ? min(kl, q0 + 128) : kl;
    const int wave_last = CAUSAL ? min(kl - 1, qw0 + 31) : kl - 1;
    const int nb = (kv_end + 63) / 64;
    issue_rows<HD>(smem, K, a.ldk, 0, kl, wave, lane);
    issue_rows<HD>(smem + TILE, V, a.ldv, 0, kl, wave, lane);
    issue_cols<HD>(smem + 2 * TILE, Kt, a.ldTk, kcol, wave, lane);
    for (int b = 0; b < nb; ++b) {
        const int kv0 = b * 64;
        char* sK = smem + (b & 1) * (3 * TILE);
        char* sV = sK + TILE;
        char* sKt = sV + TILE;
        wait_tiles_and_sync();
        if (b + 1 < nb) {
            char* n = smem + ((b + 1) & 1) * (3 * TILE);
            issue_rows<HD>(n, K, a.ldk, kv0 + 64, kl, wave, lane);
            issue_rows<HD>(n + TILE, V, a.ldv, kv0 + 64, kl, wave, lane);
            issue_cols<HD>(n + 2 * TILE, Kt, a.ldTk, kcol + kv0 + 64, wave, lane);
        }
        if (kv0 > wave_last || qw0 >= ql) continue;

        f32x16_t sacc[2], pacc[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) { sacc[kt][e] = 0.f; pacc[kt][e] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(sK + off_rows<HD>(kt * 32 + col, ks * 2 + g));
                sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sacc[kt], 0, 0, 0);
                const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(sV + off_rows<HD>(kt * 32 + col, ks * 2 + g));
                pacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[ks], pacc[kt], 0, 0, 0);
            }
        const bool need_mask = (kv0 + 64 > kl) || (CAUSAL && kv0 + 63 > qw0);
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float p = __builtin_amdgcn_exp2f(sacc[kt][e] * c - lse2);
                if (need_mask) {
                    const int key = kv0 + kt * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (key >= kl || (CAUSAL && key > qi)) p = 0.f;
                }
                sacc[kt][e] = p * (pacc[kt][e] - delta);          // dS^T
            }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bf16x8_t dsf = frag_from_acc(sacc[t >> 1], t & 1);
#pragma unroll
            for (int dt = 0; dt < HD / 32; ++dt) {
                const bf16x8_t kt_f = *reinterpret_cast<const bf16x8_t*>(sKt + off_tr(dt * 32 + col, 2 * t + g));
                gacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_f, dsf, gacc[dt], 0, 0, 0);
            }
        }
    }
    if (qi < ql) store_cols<HD>(gacc, a.scale, (bf16_t*)a.dq + (qrow0 + qi) * a.ldq + h * HD, g);
}

// ------------------------------------------------------------------------------------ backward: dK, dV
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(AttnArgs a) {
    // dynamic LDS, two stages of: Q, dO ([64][HD]), Q^T, dO^T ([HD][64 slots]); then 2 x (64 lse + 64 delta)
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TILE = 64 * HD * 2;
    float* s_stat = reinterpret_cast<float*>(smem + 8 * TILE);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int s = a.n_seq - 1 - blockIdx.z, h = blockIdx.y;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const int k0 = blockIdx.x * 128;
    if (k0 >= kl) return;
    const int qrow = a.q_row[s];
    const long long qrow0 = qrow, krow0 = a.k_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* dO = (const bf16_t*)a.d_o + qrow0 * a.ldo + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + krow0 * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + krow0 * a.ldv + h * HD;
    const bf16_t* Qt = (const bf16_t*)a.qT + (long long)h * HD * a.ldTq;
    const bf16_t* dOt = (const bf16_t*)a.doT + (long long)h * HD * a.ldTq;
    const long long qcol = tcol(qrow, s);
    const int kw0 = k0 + wave * 32;
    const int ki = kw0 + col;
    const int ki_c = ki < kl ? ki : kl - 1;

    bf16x8_t kf[HD / 16], vf[HD / 16];
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) {
        kf[ks] = *reinterpret_cast<const bf16x8_t*>(K + (long long)ki_c * a.ldk + ks * 16 + g * 8);
        vf[ks] = *reinterpret_cast<const bf16x8_t*>(V + (long long)ki_c * a.ldv + ks * 16 + g * 8);
    }
    const float c = a.scale * kLog2e;
    f32x16_t dkacc[HD / 32], dvacc[HD / 32];
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) { dkacc[dt][e] = 0.f; dvacc[dt][e] = 0.f; }

    const int q_begin = CAUSAL ? (k0 / 64) * 64 : 0;
    const int nb = (ql - q_begin + 63) / 64;
    const float* lse_row = a.lse + (size_t)h * a.lse_stride + qrow0;
    const float* delta_row = a.delta + (size_t)h * a.lse_stride + qrow0;
    auto issue_block = [&](int b) {
        const int q0 = q_begin + b * 64;
        char* n = smem + (b & 1) * (4 * TILE);
        issue_rows<HD>(n, Q, a.ldq, q0, ql, wave, lane);
        issue_rows<HD>(n + TILE, dO, a.ldo, q0, ql, wave, lane);
        issue_cols<HD>(n + 2 * TILE, Qt, a.ldTq, qcol + q0, wave, lane);
        issue_cols<HD>(n + 3 * TILE, dOt, a.ldTq, qcol + q0, wave, lane);
    };
    auto load_stats = [&](int b, float& l, float& dl) {
        if (tid < 64) {
            int r = q_begin + b * 64 + tid;
            r = r < ql ? r : ql - 1;
            l = lse_row[r] * kLog2e;
            dl = delta_row[r];
        }
    };
    float st_l = 0.f, st_d = 0.f;
    issue_block(0);
    load_stats(0, st_l, st_d);
    for (int b = 0; b < nb; ++b) {
        const int q0 = q_begin + b * 64;
        char* sQ = smem + (b & 1) * (4 * TILE);
        char* sdO = sQ + TILE;
        char* sQt = sdO + TILE;
        char* sdOt = sQt + TILE;
        float* s_lse = s_stat + (b & 1) * 128;
        float* s_delta = s_lse + 64;
        __builtin_amdgcn_s_waitcnt(0x0F70);             // vmcnt(0): this block's tiles and statistics have landed
        if (tid < 64) { s_lse[tid] = st_l; s_delta[tid] = st_d; }
        __builtin_amdgcn_s_waitcnt(0xC07F);             // lgkmcnt(0): the statistics are in LDS
        __builtin_amdgcn_s_barrier();
        if (b + 1 < nb) {
            issue_block(b + 1);
            load_stats(b + 1, st_l, st_d);
        }
        if (kw0 >= kl || (CAUSAL && q0 + 63 < kw0)) continue;

        f32x16_t sacc[2], pacc[2];
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int e = 0; e < 16; ++e) { sacc[qt][e] = 0.f; pacc[qt][e] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks)
#pragma unroll
            for (int qt = 0; qt < 2; ++qt) {
                const bf16x8_t qf = *reinterpret_cast<const bf16x8_t*>(sQ + off_rows<HD>(qt * 32 + col, ks * 2 + g));
                sacc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[ks], sacc[qt], 0, 0, 0);
                const bf16x8_t dof = *reinterpret_cast<const bf16x8_t*>(sdO + off_rows<HD>(qt * 32 + col, ks * 2 + g));
                pacc[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dof, vf[ks], pacc[qt], 0, 0, 0);
            }
        const bool need_mask = (q0 + 64 > ql) || (CAUSAL && q0 < kw0 + 31);
#pragma unroll
        for (int qt = 0; qt < 2; ++qt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int qloc = qt * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                float p = __builtin_amdgcn_exp2f(sacc[qt][e] * c - s_lse[qloc]);
                if (need_mask) {
                    const int q = q0 + qloc;
                    if (q >= ql || (CAUSAL && q < ki)) p = 0.f;
                }
                sacc[qt][e] = p;                                       // P
                pacc[qt][e] = p * (pacc[qt][e] - s_delta[qloc]);       // dS
            }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bf16x8_t pf = frag_from_acc(sacc[t >> 1], t & 1);
            const bf16x8_t dsf = frag_from_acc(pacc[t >> 1], t & 1);
#pragma unroll
            for (int dt = 0; dt < HD / 32; ++dt) {
                const bf16x8_t dot_f = *reinterpret_cast<const bf16x8_t*>(sdOt + off_tr(dt * 32 + col, 2 * t + g));
                dvacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot_f, pf, dvacc[dt], 0, 0, 0);
                const bf16x8_t qt_f = *reinterpret_cast<const bf16x8_t*>(sQt + off_tr(dt * 32 + col, 2 * t + g));
                dkacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt_f, dsf, dkacc[dt], 0, 0, 0);
            }
        }
    }
    if (ki < kl) {
        store_cols<HD>(dkacc, a.scale, (bf16_t*)a.dk + (krow0 + ki) * a.ldk + h * HD, g);
        store_cols<HD>(dvacc, 1.0f, (bf16_t*)a.dv + (krow0 + ki) * a.ldv + h * HD, g);
    }
}

ds_status seq_transpose(int C, int n_seq, int max_len, const int32_t* row, const int32_t* len, const void* in, long long ld_in,
                        void* out, long long ld_out, hipStream_t st) {
    dim3 grid((C + 255) / 256, (max_len + 63) / 64, n_seq);
    hipLaunchKernelGGL(seq_transpose_kernel, grid, dim3(256), 0, st, C, row, len, (const bf16_t*)in, ld_in, (bf16_t*)out, ld_out);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

template <class Kern>
ds_status set_smem(Kern kern, int bytes, bool& done) {
    if (!done) {
        DS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
        done = true;
    }
    return DS_OK;
}

template <int HD, bool CAUSAL>
ds_status fwd_launch(const AttnArgs& a, hipStream_t st) {
    static bool attr = false;
    auto kern = attn_fwd_mfma_kernel<HD, CAUSAL>;
    const int smem = 4 * (64 * HD * 2);
    ds_status r = set_smem(kern, smem, attr);
    if (r != DS_OK) return r;
    dim3 grid((a.max_q_len + 127) / 128, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

template <int HD, bool CAUSAL>
ds_status bwd_launch(const AttnArgs& a, hipStream_t st) {
    static bool attr_q = false, attr_kv = false;
    auto kq = attn_bwd_dq_mfma_kernel<HD, CAUSAL>;
    auto kkv = attn_bwd_dkv_mfma_kernel<HD, CAUSAL>;
    const int smem_q = 6 * (64 * HD * 2);
    const int smem_kv = 8 * (64 * HD * 2) + 256 * 4;
    ds_status r = set_smem(kq, smem_q, attr_q);
    if (r != DS_OK) return r;
    r = set_smem(kkv, smem_kv, attr_kv);
    if (r != DS_OK) return r;
    dim3 gq((a.max_q_len + 127) / 128, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(kq, gq, dim3(256), smem_q, st, a);
    DS_LAUNCH_CHECK();
    dim3 gk((a.max_k_len + 127) / 128, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(kkv, gk, dim3(256), smem_kv, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

}  // namespace

// Leading dimension (in tokens) of a feature-major copy of a stream of `total_rows` rows holding n_seq sequences.
long long attn_ld_t(int total_rows, int n_seq) { return (long long)((total_rows + 63) & ~63) + 128LL * n_seq + 64; }

size_t attn_scratch_bytes(int n_heads, int head_dim, int q_total_rows, int k_total_rows, int n_seq) {
    const size_t d = (size_t)n_heads * head_dim;
    // forward needs V^T; backward needs Q^T, dO^T (query side) and K^T (key side)
    return 2 * d * (size_t)attn_ld_t(q_total_rows, n_seq) * 2 + d * (size_t)attn_ld_t(k_total_rows, n_seq) * 2 + 1024;
}

bool attn_mfma_supported(const AttnArgs& a) {
    if (a.dtype != DS_DTYPE_BF16) return false;
    if (a.head_dim != 64 && a.head_dim != 128) return false;
    if (a.ldq % 8 || a.ldk % 8 || a.ldv % 8 || a.ldo % 8) return false;
    auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    if (!al(a.q) || !al(a.k) || !al(a.v) || !al(a.o)) return false;
    if (a.d_o && (!al(a.d_o) || !al(a.dq) || !al(a.dk) || !al(a.dv))) return false;
    if (!a.scratch || !al(a.scratch)) return false;
    if (a.q_total_rows <= 0 || a.k_total_rows <= 0) return false;
    if (a.scratch_bytes < attn_scratch_bytes(a.n_heads, a.head_dim, a.q_total_rows, a.k_total_rows, a.n_seq)) return false;
    return true;
}

ds_status attn_fwd_mfma(const AttnArgs& a0, hipStream_t st) {
    AttnArgs a = a0;
    const int d = a.n_heads * a.head_dim;
    a.ldTk = attn_ld_t(a.k_total_rows, a.n_seq);
    a.vT = a.scratch;
    ds_status r = seq_transpose(d, a.n_seq, a.max_k_len, a.k_row, a.k_len, a.v, a.ldv, a.scratch, a.ldTk, st);
    if (r != DS_OK) return r;
    if (a.head_dim == 128) return a.mask ? fwd_launch<128, true>(a, st) : fwd_launch<128, false>(a, st);
    return a.mask ? fwd_launch<64, true>(a, st) : fwd_launch<64, false>(a, st);
}

ds_status attn_bwd_mfma(const AttnArgs& a0, hipStream_t st) {
    AttnArgs a = a0;
    const size_t d = (size_t)a.n_heads * a.head_dim;
    a.ldTq = attn_ld_t(a.q_total_rows, a.n_seq);
    a.ldTk = attn_ld_t(a.k_total_rows, a.n_seq);
    char* base = (char*)a.scratch;
    a.qT = base;
    a.doT = base + d * a.ldTq * 2;
    a.kT = base + 2 * d * a.ldTq * 2;
    ds_status r = seq_transpose((int)d, a.n_seq, a.max_q_len, a.q_row, a.q_len, a.q, a.ldq, (void*)a.qT, a.ldTq, st);
    if (r != DS_OK) return r;
    r = seq_transpose((int)d, a.n_seq, a.max_q_len, a.q_row, a.q_len, a.d_o, a.ldo, (void*)a.doT, a.ldTq, st);
    if (r != DS_OK) return r;
    r = seq_transpose((int)d, a.n_seq, a.max_k_len, a.k_row, a.k_len, a.k, a.ldk, (void*)a.kT, a.ldTk, st);
    if (r != DS_OK) return r;
    if (a.head_dim == 128) return a.mask ? bwd_launch<128, true>(a, st) : bwd_launch<128, false>(a, st);
    return a.mask ? bwd_launch<64, true>(a, st) : bwd_launch<64, false>(a, st);
}
