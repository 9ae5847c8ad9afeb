// bf16 variable-length attention on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16),
// head_dim 64 or 128, causal or unmasked (bidirectional / cross), forward and backward.
//
// Layout idea (all three kernels).  A wavefront owns 32 "column" items (queries in forward and
// dQ, keys in dK/dV) and keeps them in the MFMA B operand, so that the score tile it computes
// is TRANSPOSED: lane l holds column l%32 and 16 of the 32 rows.  Everything that is per
// column (running max, running sum, log-sum-exp, delta, the rescale of the output accumulator)
// is then a per-lane scalar, and row reductions are in-lane plus one exchange between lanes l
// and l^32.  The probabilities leave the accumulator registers as the B operand of the second
// product without any data movement: accumulator registers 8u..8u+7 of a tile ARE a valid
// 16-deep B fragment provided the A operand lists the contraction index in the matching order,
//     slot j of lane-half g  <->  row 16t + 8*(j/4) + 4*g + j%4           (t = 16-row step)
// so the transposed operand tiles (V^T, K^T, Q^T, dO^T) are written to LDS in that slot order
// by a loader that transposes 8x8 bf16 blocks in registers (v_perm_b32).
//
// K/V (forward, dQ) or Q/dO (dK/dV) tiles of 64 rows are staged in LDS with a 16-byte XOR
// swizzle: conflict-free 16-byte fragment reads.  Backward is split into a dQ kernel and a
// dK/dV kernel so that every output element has one owner: no atomics, results are
// bit-reproducible.  Sequences are addressed through the (row, length) tables, so padding rows
// cost nothing, and packed layouts (several sequences in one padded row) need no mask.
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

// 64 rows x HD columns, rows row0.. of a tensor with leading dimension ld, clamped to the last valid row.
template <int HD>
__device__ __forceinline__ void load_rows(char* __restrict__ lds, const bf16_t* __restrict__ base, long long ld, int row0,
                                          int n_valid, int tid) {
    constexpr int CH = HD / 8;
#pragma unroll
    for (int c = tid; c < 64 * CH; c += 256) {
        const int row = c / CH, chunk = c % CH;
        int r = row0 + row;
        r = r < n_valid ? r : n_valid - 1;
        *reinterpret_cast<uint4*>(lds + off_rows<HD>(row, chunk)) =
            *reinterpret_cast<const uint4*>(base + (long long)r * ld + chunk * 8);
    }
}

// The same 64 x HD block, transposed into [HD][64 slots] with the slot order of the header comment.
template <int HD>
__device__ __forceinline__ void load_rows_transposed(char* __restrict__ lds, const bf16_t* __restrict__ base, long long ld,
                                                     int row0, int n_valid, int tid) {
    constexpr int CH = HD / 8;
    for (int bi = tid; bi < 8 * CH; bi += 256) {
        const int kg = bi & 7, dc = bi >> 3;
        const int t = kg >> 1, g = kg & 1;
        uint4 r[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            int row = row0 + slot_row(t, g, j);
            row = row < n_valid ? row : n_valid - 1;
            r[j] = *reinterpret_cast<const uint4*>(base + (long long)row * ld + dc * 8);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint4 o;
            const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
            o.x = __builtin_amdgcn_perm(pick4(r[1], i >> 1), pick4(r[0], i >> 1), sel);
            o.y = __builtin_amdgcn_perm(pick4(r[3], i >> 1), pick4(r[2], i >> 1), sel);
            o.z = __builtin_amdgcn_perm(pick4(r[5], i >> 1), pick4(r[4], i >> 1), sel);
            o.w = __builtin_amdgcn_perm(pick4(r[7], i >> 1), pick4(r[6], i >> 1), sel);
            *reinterpret_cast<uint4*>(lds + off_tr(dc * 8 + i, kg)) = o;
        }
    }
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

// ------------------------------------------------------------------------------------ forward
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(AttnArgs a) {
    __shared__ __attribute__((aligned(16))) char sK[64 * HD * 2];
    __shared__ __attribute__((aligned(16))) char sVt[HD * 128];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int s = a.n_seq - 1 - blockIdx.z, h = blockIdx.y;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const int q0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * 128;
    if (q0 >= ql) return;
    const bf16_t* Q = (const bf16_t*)a.q + (long long)a.q_row[s] * a.ldq + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + (long long)a.k_row[s] * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + (long long)a.k_row[s] * a.ldv + h * HD;
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
    for (int kv0 = 0; kv0 < kv_end; kv0 += 64) {
        __syncthreads();
        load_rows<HD>(sK, K, a.ldk, kv0, kl, tid);
        load_rows_transposed<HD>(sVt, V, a.ldv, kv0, kl, tid);
        __syncthreads();
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
    __shared__ __attribute__((aligned(16))) char sK[64 * HD * 2];
    __shared__ __attribute__((aligned(16))) char sV[64 * HD * 2];
    __shared__ __attribute__((aligned(16))) char sKt[HD * 128];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int s = a.n_seq - 1 - blockIdx.z, h = blockIdx.y;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const int q0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * 128;
    if (q0 >= ql) return;
    const long long qrow0 = a.q_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* dO = (const bf16_t*)a.d_o + qrow0 * a.ldo + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + (long long)a.k_row[s] * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + (long long)a.k_row[s] * a.ldv + h * HD;
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
    for (int kv0 = 0; kv0 < kv_end; kv0 += 64) {
        __syncthreads();
        load_rows<HD>(sK, K, a.ldk, kv0, kl, tid);
        load_rows<HD>(sV, V, a.ldv, kv0, kl, tid);
        load_rows_transposed<HD>(sKt, K, a.ldk, kv0, kl, tid);
        __syncthreads();
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
    // dynamic LDS: Q, dO ([64][HD]), Q^T, dO^T ([HD][64 slots]), then 64 log-sum-exp and 64 delta values
    extern __shared__ __attribute__((aligned(16))) char dkv_smem[];
    char* sQ = dkv_smem;
    char* sdO = sQ + 64 * HD * 2;
    char* sQt = sdO + 64 * HD * 2;
    char* sdOt = sQt + HD * 128;
    float* s_lse = reinterpret_cast<float*>(sdOt + HD * 128);
    float* s_delta = s_lse + 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int s = a.n_seq - 1 - blockIdx.z, h = blockIdx.y;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const int k0 = blockIdx.x * 128;
    if (k0 >= kl) return;
    const long long qrow0 = a.q_row[s], krow0 = a.k_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* dO = (const bf16_t*)a.d_o + qrow0 * a.ldo + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + krow0 * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + krow0 * a.ldv + h * HD;
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
    for (int q0 = q_begin; q0 < ql; q0 += 64) {
        __syncthreads();
        load_rows<HD>(sQ, Q, a.ldq, q0, ql, tid);
        load_rows<HD>(sdO, dO, a.ldo, q0, ql, tid);
        load_rows_transposed<HD>(sQt, Q, a.ldq, q0, ql, tid);
        load_rows_transposed<HD>(sdOt, dO, a.ldo, q0, ql, tid);
        if (tid < 64) {
            int r = q0 + tid;
            r = r < ql ? r : ql - 1;
            s_lse[tid] = a.lse[(size_t)h * a.lse_stride + qrow0 + r] * kLog2e;
            s_delta[tid] = a.delta[(size_t)h * a.lse_stride + qrow0 + r];
        }
        __syncthreads();
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

template <int HD, bool CAUSAL>
ds_status fwd_launch(const AttnArgs& a, hipStream_t st) {
    dim3 grid((a.max_q_len + 127) / 128, a.n_heads, a.n_seq);
    hipLaunchKernelGGL((attn_fwd_mfma_kernel<HD, CAUSAL>), grid, dim3(256), 0, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

template <int HD, bool CAUSAL>
ds_status bwd_launch(const AttnArgs& a, hipStream_t st) {
    static bool attr_set = false;
    auto kern = attn_bwd_dkv_mfma_kernel<HD, CAUSAL>;
    const int smem = 2 * (64 * HD * 2) + 2 * (HD * 128) + 128 * 4;
    if (!attr_set) {
        DS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        attr_set = true;
    }
    dim3 gq((a.max_q_len + 127) / 128, a.n_heads, a.n_seq);
    hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<HD, CAUSAL>), gq, dim3(256), 0, st, a);
    DS_LAUNCH_CHECK();
    dim3 gk((a.max_k_len + 127) / 128, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(kern, gk, dim3(256), smem, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
    if (a.dtype != DS_DTYPE_BF16) return false;
    if (a.head_dim != 64 && a.head_dim != 128) return false;
    if (a.ldq % 8 || a.ldk % 8 || a.ldv % 8 || a.ldo % 8) return false;
    auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
    if (!al(a.q) || !al(a.k) || !al(a.v) || !al(a.o)) return false;
    if (a.d_o && (!al(a.d_o) || !al(a.dq) || !al(a.dk) || !al(a.dv))) return false;
    return true;
}

ds_status attn_fwd_mfma(const AttnArgs& a, hipStream_t st) {
    if (a.head_dim == 128) return a.mask ? fwd_launch<128, true>(a, st) : fwd_launch<128, false>(a, st);
    return a.mask ? fwd_launch<64, true>(a, st) : fwd_launch<64, false>(a, st);
}

ds_status attn_bwd_mfma(const AttnArgs& a, hipStream_t st) {
    if (a.head_dim == 128) return a.mask ? bwd_launch<128, true>(a, st) : bwd_launch<128, false>(a, st);
    return a.mask ? bwd_launch<64, true>(a, st) : bwd_launch<64, false>(a, st);
}
