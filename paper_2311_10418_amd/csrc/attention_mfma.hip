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
// Memory.  Every tile is a block of 64 token rows x head_dim and goes global -> LDS directly
// (global_load_lds_dwordx4): no staging registers, double-buffered, the next block in flight while
// the current one feeds the MFMAs.  The first product reads its A fragments along the rows
// (ds_read_b128).  The second product needs the same tile TRANSPOSED (V^T, K^T, Q^T, dO^T as the A
// operand: 8 tokens in slot order for one feature per lane); gfx950's LDS transpose read
// (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i%4 of the 8 bytes addressed by
// lanes i/4, 4+i/4, 8+i/4, 12+i/4) delivers exactly that from the token-major tile: two reads per
// fragment, 4 consecutive tokens each.  No transposed copies exist in HBM.  Tiles carry a 16-byte
// XOR swizzle (applied by choosing which global chunk each lane fetches) that keeps both access
// patterns free of bank conflicts on the 64-bank LDS.
//
// Scheduling.  A small kernel lists the (sequence, 128-row block) work items of a call, long sequences
// first and the blocks of one sequence together; the attention grids walk that list, heads fastest, so
// that the work-groups sharing a sequence's tiles run on one XCD at the same time (one fetch from HBM per
// tile instead of one per block) and no work-group is launched for nothing.
//
// VALU economy (the matrix pipe is only as fast as the scalar work between its instructions): the
// softmax scale rides in one FMA with the running max, the accumulator is rescaled only when some
// lane's max moved, delta = rowsum(dO * O) is computed in the dQ kernel's prologue, and the dK/dV
// kernel gets "score - lse/scale" and "dP - delta" straight from the matrix pipe by appending
// [hi, lo] bf16 splits of the statistics to the contraction against a constant [-1, -1].
//
// Backward is split into a dQ kernel and a dK/dV kernel so that every output element has one
// owner: no atomics, results are bit-reproducible.  Sequences are addressed through (row, length)
// tables, so padding rows cost nothing and packed layouts need no mask.
#include "attention.hpp"
#include <type_traits>

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// sched_barrier mask: vector ALU, scalar ALU and transcendental instructions may cross, LDS accesses and MFMAs may not
constexpr int kFence = 0x2 | 0x4 | 0x400;
// how many fragment reads (forward) / pairs of reads (dQ) run in front of the MFMAs that use them
constexpr int FWD_AHEAD = 4, PV_AHEAD = 4, DQ_AHEAD = 2;

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;

// LDS swizzle: the 16-byte chunk index of a row is XORed with swz(row).  Row-wise fragment reads
// (16 lanes = 16 consecutive rows, same chunk) need the 16 rows in 16 different 16-byte units of a
// 256-byte window; transpose reads (32 lanes = 4 consecutive rows x 64 bytes) need the 4 rows in 4
// different 64-byte units.  Both hold for these bijections of the low row bits.
template <int HD> __device__ __forceinline__ int swz(int row) {
    return HD == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}
template <int HD> __device__ __forceinline__ int off_rows(int row, int chunk) {      // [row][HD] tile, 16-byte chunk
    return row * (HD * 2) + ((chunk ^ swz<HD>(row)) << 4);
}

// max of three through v_max3_f32 directly: fmaxf() makes the compiler canonicalise every operand first (one extra
// multiply per score), which the hardware instruction does not need
__device__ __forceinline__ float max3f(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// {hi, lo} bf16 pair with hi + lo = v to ~2^-17 relative, packed into one dword
__device__ __forceinline__ uint32_t split_hi_lo(float v) {
    const bf16_t hi = (bf16_t)v;
    const bf16_t lo = (bf16_t)(v - (float)hi);
    return (uint32_t)__builtin_bit_cast(unsigned short, hi) | ((uint32_t)__builtin_bit_cast(unsigned short, lo) << 16);
}

// accumulator registers 8u..8u+7 of a 32x32 tile -> one bf16 B fragment
__device__ __forceinline__ bf16x8_t frag_from_acc(const f32x16_t& a, int u) {
    bf16x8_t f;
#pragma unroll
    for (int j = 0; j < 8; ++j) f[j] = (bf16_t)a[8 * u + j];
    return f;
}

// Per-lane byte offsets of the transposed A fragments of a token-major tile: fragment (t, dt) lists,
// for feature dt*32 + lane%32, the tokens 16t + 4g + {0..3} (low read) and 16t + 8 + 4g + {0..3} (high read).
template <int HD> struct TrOffsets {
    int lo[HD / 32], hi[HD / 32];
    __device__ __forceinline__ void init(int lane) {
        const int i = lane & 15, halfd = (lane >> 4) & 1, g = lane >> 5;
        const int r_lo = 4 * g + (i >> 2), r_hi = r_lo + 8;
        const int c2 = halfd * 2 + ((i >> 1) & 1), byte = (i & 1) * 8;
#pragma unroll
        for (int dt = 0; dt < HD / 32; ++dt) {
            lo[dt] = off_rows<HD>(r_lo, dt * 4 + c2) + byte;
            hi[dt] = off_rows<HD>(r_hi, dt * 4 + c2) + byte;
        }
    }
};
template <int HD>
__device__ __forceinline__ bf16x8_t read_tr(const char* tile, const TrOffsets<HD>& o, int t, int dt) {
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + t * (16 * HD * 2) + o.lo[dt]));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + t * (16 * HD * 2) + o.hi[dt]));
    const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
}

// Direct-to-LDS loader of 64-row tiles of one row-major tensor: each wavefront issues HD/32 transfers of
// 64 x 16 bytes per tile.  A transfer is addressed as a wavefront-uniform base (tensor + first row of the tile,
// scalar arithmetic) plus a 32-bit byte offset per lane; the offsets of a tile whose 64 rows all exist are fixed
// for the whole kernel, so stepping along the sequence costs no vector instruction.  Only the ragged last tile
// recomputes them (rows past the end are clamped to the last valid row; the consumers mask the duplicates).
template <int HD> struct TileLoader {
    static constexpr int PW = HD / 32;
    const char* base;
    long long ld2;                                      // row stride in bytes (64 rows of it fit in 31 bits)
    int n_valid, wave, lane;
    uint32_t off_full[PW];
    uint32_t off_group[PW];                             // the same offsets as lds_dma16_group wants them
    __device__ __forceinline__ static int row_of(int u) { return HD == 128 ? (u >> 4) : (u >> 3); }
    __device__ __forceinline__ static int chunk_of(int u) {
        return (HD == 128 ? (u & 15) : (u & 7)) ^ swz<HD>(row_of(u));
    }
    __device__ __forceinline__ void setup(const bf16_t* base_, long long ld_, int n_valid_, int wave_, int lane_) {
        base = (const char*)base_; ld2 = ld_ * 2; n_valid = n_valid_; wave = wave_; lane = lane_;
#pragma unroll
        for (int i = 0; i < PW; ++i) {
            const int u = (wave * PW + i) * 64 + lane;
            off_full[i] = (uint32_t)(row_of(u) * (int)ld2 + chunk_of(u) * 16);
            off_group[i] = dma_lane_offset<PW>(off_full[i], i);
        }
    }
    // rows r0 .. r0+63 -> the tile at LDS address lds_tile; 0 <= r0 < n_valid.  A tile whose 64 rows all exist goes as
    // one group of PW transfers under a single M0 with the fixed offsets; the ragged last tile clamps its rows.
    __device__ __forceinline__ void issue(uint32_t lds_tile, int r0) const {
        const char* b = base + (long long)r0 * ld2;
        if (r0 + 64 <= n_valid) {
            lds_dma16_group<PW>(dma_group_base<PW>(b), off_group, lds_tile + wave * (PW * 1024));
        } else {
            const int last = n_valid - 1 - r0;
            uint32_t off[PW];
#pragma unroll
            for (int i = 0; i < PW; ++i) {
                const int u = (wave * PW + i) * 64 + lane;
                const int rr = min(row_of(u), last);
                off[i] = dma_lane_offset<PW>((uint32_t)(rr * (int)ld2 + chunk_of(u) * 16), i);
            }
            lds_dma16_group<PW>(dma_group_base<PW>(b), off, lds_tile + wave * (PW * 1024));
        }
    }
};

// this wavefront's direct loads have landed, then everybody's; the stage read in the previous step is free
__device__ __forceinline__ void wait_tiles_and_sync() {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
    __builtin_amdgcn_s_barrier();
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

// ------------------------------------------------------------------------------------ work lists
// items[0 .. n): the (sequence, block) pairs of `block` rows each; n is written to *n_items.  One work-group.
// Order: sequences by descending trip count of their longest block (a block's trip count = the number of
// 64-row steps its work-group takes), the blocks of one sequence next to each other, longest first.  The
// grids walk the list with heads fastest and the hardware deals consecutive work-groups round-robin to the
// XCDs, so with a head count that is a multiple of the XCD count every block of one (sequence, head) runs on
// the same XCD at about the same time and streams the same K / V (or Q / dO) tiles: all but the first fetch
// of a tile hit in that XCD's L2.  Long sequences still start first and the list ends with the shortest, so
// the grid's tail stays fine-grained.
__global__ __launch_bounds__(1024) void attn_worklist_kernel(int n_seq, const int32_t* __restrict__ own_len,
                                                             const int32_t* __restrict__ other_len, int causal,
                                                             int key_side, int max_items, int2* __restrict__ items,
                                                             int32_t* __restrict__ n_items) {
    constexpr int NB = 1024;
    __shared__ int hist[NB];
    __shared__ int start[NB];
    const int tid = threadIdx.x;
    // trip count of the longest block of a sequence: the last query block (it sees every key up to its own
    // end), the first key block (every query from its own start on), any block when nothing is masked
    auto longest = [&](int own, int other) {
        int n;
        if (!key_side) n = ((causal ? min(other, ((own + 127) >> 7) * 128) : other) + 63) >> 6;
        else n = (other + 63) >> 6;
        return min(max(n, 0), NB - 1);
    };
    hist[tid] = 0;
    __syncthreads();
    for (int s = tid; s < n_seq; s += NB) {
        const int own = own_len[s];
        if (own > 0) atomicAdd(&hist[longest(own, other_len[s])], (own + 127) >> 7);
    }
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int b = NB - 1; b >= 0; --b) { start[b] = run; run += hist[b]; }
        n_items[0] = min(run, max_items);
    }
    __syncthreads();
    for (int s = tid; s < n_seq; s += NB) {
        const int own = own_len[s];
        if (own <= 0) continue;
        const int nblk = (own + 127) >> 7;
        const int base = atomicAdd(&start[longest(own, other_len[s])], nblk);
        for (int j = 0; j < nblk; ++j)
            if (base + j < max_items) items[base + j] = make_int2(s, (!key_side && causal) ? nblk - 1 - j : j);
    }
}

// ------------------------------------------------------------------------------------ forward
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TILE = 64 * HD * 2;                  // bytes of one K tile == one V tile
    const uint32_t lds0 = lds_address(smem);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, g = lane >> 5;
    const int item = blockIdx.x / a.n_heads, h = blockIdx.x - item * a.n_heads;
    if (item >= a.n_items[0]) return;
    const int2 it = a.items_q[item];
    const int s = it.x, q0 = it.y * 128;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const long long qrow0 = a.q_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + (long long)a.k_row[s] * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + (long long)a.k_row[s] * a.ldv + h * HD;
    const int qw0 = q0 + wave * 32;
    const int qi = qw0 + col;
    const int qi_c = qi < ql ? qi : ql - 1;

    bf16x8_t qf[HD / 16];
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks)
        qf[ks] = *reinterpret_cast<const bf16x8_t*>(Q + (long long)qi_c * a.ldq + ks * 16 + g * 8);

    TileLoader<HD> ldK, ldV;
    ldK.setup(K, a.ldk, kl, wave, lane);
    ldV.setup(V, a.ldv, kl, wave, lane);
    TrOffsets<HD> tro;
    tro.init(lane);
    const int rbase = col * (HD * 2);
    const int rsw = swz<HD>(col);

    f32x16_t oacc[HD / 32];
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[dt][e] = 0.f;
    float m = -INFINITY, lsum = 0.f;                   // running max (in the exp2 domain) and sum
    const float c = a.scale * kLog2e;

    const int kv_end = CAUSAL ? min(kl, q0 + 128) : kl;
    const int wave_last = CAUSAL ? min(kl - 1, qw0 + 31) : kl - 1;     // last key this wavefront can see
    const int nb = (kv_end + 63) / 64;
    if (nb > 0) {                                       // (a sequence without keys: zero output, nothing to fetch)
        ldK.issue(lds0, 0);
        ldV.issue(lds0 + TILE, 0);
    }
    for (int b = 0; b < nb; ++b) {
        const int kv0 = b * 64;
        char* sK = smem + (b & 1) * (2 * TILE);
        char* sV = sK + TILE;
        wait_tiles_and_sync();                          // block b has landed; the other stage is free
        // The transfers of block b+1.  A wavefront cannot issue anything else while a transfer of its own passes the
        // address stage of the texture path (measured with timestamps: one burst of 8 transfers with an M0 each held
        // a wavefront for about 600 cycles of a 4400-cycle step; grouped under one M0 per tile, 250), so a wavefront
        // that computes in this step hands out the two groups between the MFMAs of its first product; only a ragged
        // last block (its per-lane offsets are recomputed) and wavefronts without work issue them at once.
        const bool have_next = b + 1 < nb;
        const bool active = !(kv0 > wave_last || qw0 >= ql);
        const bool spread = have_next && active && kv0 + 128 <= kl;
        const uint32_t nK_lds = lds0 + ((b + 1) & 1) * (2 * TILE);
        if (have_next && !spread) {
            ldK.issue(nK_lds, kv0 + 64);
            ldV.issue(nK_lds + TILE, kv0 + 64);
        }
        if (!active) continue;

        f32x16_t sacc[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[kt][e] = 0.f;
        // first product, S^T = K Q^T: fragment reads FWD_AHEAD MFMAs in front of their use, the order pinned by fences
        // (see the dK/dV kernel); two copies, with and without the transfers, so that neither holds a branch
        auto first_product = [&](auto with_dma) {
            constexpr bool DMA = decltype(with_dma)::value;
            constexpr int NF = 2 * (HD / 16);
            bf16x8_t fk[NF];
            auto read_k = [&](int i) {
                const int ks = i >> 1, kt = i & 1;
                fk[i] = *reinterpret_cast<const bf16x8_t*>(sK + kt * (32 * HD * 2) + rbase + (((ks * 2 + g) ^ rsw) << 4));
            };
#pragma unroll
            for (int i = 0; i < FWD_AHEAD; ++i) read_k(i);
#pragma unroll
            for (int i = 0; i < NF; ++i) {
                if (i + FWD_AHEAD < NF) read_k(i + FWD_AHEAD);
                __builtin_amdgcn_sched_barrier(kFence);
                sacc[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[i], qf[i >> 1], sacc[i & 1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(kFence);
                if (DMA && i == NF / 4 - 1) {           // the next K tile after a quarter of the product ...
                    ldK.issue(nK_lds, kv0 + 64);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (DMA && i == 3 * NF / 4 - 1) {       // ... the next V tile after three quarters
                    ldV.issue(nK_lds + TILE, kv0 + 64);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        if (spread) first_product(std::true_type{});
        else first_product(std::false_type{});
        // the first V^T fragments of the second product are fetched now and land during the softmax
        constexpr int NV = 4 * (HD / 32);
        bf16x8_t fv[NV];
        auto read_v = [&](int i) { fv[i] = read_tr<HD>(sV, tro, i / (HD / 32), i % (HD / 32)); };
#pragma unroll
        for (int i = 0; i < PV_AHEAD; ++i) read_v(i);
        __builtin_amdgcn_sched_barrier(kFence);
        const bool need_mask = (kv0 + 64 > kl) || (CAUSAL && kv0 + 63 > qw0);
        if (need_mask) {
            // the volatile statement keeps the whole mask computation inside a real branch: hoisted or if-converted,
            // its ~130 compare / select instructions would run on every step, not just on the diagonal and the tail
            int kbase = kv0;
            asm volatile("" : "+s"(kbase));
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = kbase + kt * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (key >= kl || (CAUSAL && key > qi)) sacc[kt][e] = -INFINITY;
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; e += 2) mx = max3f(mx, sacc[kt][e], sacc[kt][e + 1]);
        const float m_new = max3f(m, mx * c, __shfl_xor(mx, 32, 64) * c);
        float rs = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt][e], c, -m_new));
                sacc[kt][e] = p;
                rs += p;
            }
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        lsum = lsum * alpha + rs;
        if (__builtin_amdgcn_ballot_w64(m_new > m) != 0) {      // some column's max moved: rescale the accumulator
#pragma unroll
            for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[dt][e] *= alpha;
        }
        m = m_new;
        // second product, O^T += V^T P^T: transpose reads PV_AHEAD MFMAs in front of their use
        bf16x8_t pf;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (i + PV_AHEAD < NV) read_v(i + PV_AHEAD);
            if (i % (HD / 32) == 0) pf = frag_from_acc(sacc[(i / (HD / 32)) >> 1], (i / (HD / 32)) & 1);
            __builtin_amdgcn_sched_barrier(kFence);
            oacc[i % (HD / 32)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[i], pf, oacc[i % (HD / 32)], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(kFence);
        }
    }
    lsum += __shfl_xor(lsum, 32, 64);
    if (qi < ql) {
        const long long row = qrow0 + qi;
        store_cols<HD>(oacc, lsum > 0.f ? 1.0f / lsum : 0.f, (bf16_t*)a.o + row * a.ldo + h * HD, g);
        if (g == 0) a.lse[(size_t)h * a.lse_stride + row] = (m + __builtin_amdgcn_logf(lsum)) * kLn2;
    }
}

// ------------------------------------------------------------------------------------ backward: dQ (and delta)
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TILE = 64 * HD * 2;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, g = lane >> 5;
    const int item = blockIdx.x / a.n_heads, h = blockIdx.x - item * a.n_heads;
    if (item >= a.n_items[0]) return;
    const int2 it = a.items_q[item];
    const int s = it.x, q0 = it.y * 128;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const long long qrow0 = a.q_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* dO = (const bf16_t*)a.d_o + qrow0 * a.ldo + h * HD;
    const bf16_t* O = (const bf16_t*)a.o + qrow0 * a.ldo + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + (long long)a.k_row[s] * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + (long long)a.k_row[s] * a.ldv + h * HD;
    const int qw0 = q0 + wave * 32;
    const int qi = qw0 + col;
    const int qi_c = qi < ql ? qi : ql - 1;

    const uint32_t lds0 = lds_address(smem);
    TileLoader<HD> ldK, ldV;
    ldK.setup(K, a.ldk, kl, wave, lane);
    ldV.setup(V, a.ldv, kl, wave, lane);
    if (kl > 0) {
        ldK.issue(lds0, 0);
        ldV.issue(lds0 + TILE, 0);
    }

    bf16x8_t qf[HD / 16], dof[HD / 16];
    float delta = 0.f;                                  // rowsum(dO * O) of this lane's query, this head
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) {
        qf[ks] = *reinterpret_cast<const bf16x8_t*>(Q + (long long)qi_c * a.ldq + ks * 16 + g * 8);
        dof[ks] = *reinterpret_cast<const bf16x8_t*>(dO + (long long)qi_c * a.ldo + ks * 16 + g * 8);
        const bf16x8_t of = *reinterpret_cast<const bf16x8_t*>(O + (long long)qi_c * a.ldo + ks * 16 + g * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) delta = __builtin_fmaf((float)of[j], (float)dof[ks][j], delta);
    }
    delta += __shfl_xor(delta, 32, 64);
    const float lse_q = a.lse[(size_t)h * a.lse_stride + qrow0 + qi_c];
    if (g == 0 && qi < ql) {
        // for the dK/dV kernel: delta itself, and the {hi, lo} bf16 splits of lse/scale and delta that it appends
        // to its contractions (hi + lo reproduces the value to ~2^-17 relative)
        const size_t at = (size_t)h * a.lse_stride + qrow0 + qi;
        a.delta[at] = delta;
        reinterpret_cast<uint4*>(a.aug_lse)[at] = make_uint4(split_hi_lo(lse_q * (1.0f / a.scale)), 0u, 0u, 0u);
        reinterpret_cast<uint4*>(a.aug_delta)[at] = make_uint4(split_hi_lo(delta), 0u, 0u, 0u);
    }
    const float lse2 = lse_q * kLog2e;
    const float c = a.scale * kLog2e;

    TrOffsets<HD> tro;
    tro.init(lane);
    const int rbase = col * (HD * 2);
    const int rsw = swz<HD>(col);

    f32x16_t gacc[HD / 32];
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) gacc[dt][e] = 0.f;

    const int kv_end = CAUSAL ? min(kl, q0 + 128) : kl;
    const int wave_last = CAUSAL ? min(kl - 1, qw0 + 31) : kl - 1;
    const int nb = (kv_end + 63) / 64;
    for (int b = 0; b < nb; ++b) {
        const int kv0 = b * 64;
        char* sK = smem + (b & 1) * (2 * TILE);
        char* sV = sK + TILE;
        wait_tiles_and_sync();
        if (b + 1 < nb) {
            const uint32_t n = lds0 + ((b + 1) & 1) * (2 * TILE);
            ldK.issue(n, kv0 + 64);
            ldV.issue(n + TILE, kv0 + 64);
        }
        if (kv0 > wave_last || qw0 >= ql) continue;
        const bool need_mask = (kv0 + 64 > kl) || (CAUSAL && kv0 + 63 > qw0);
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            if (kv0 + kt * 32 > wave_last) continue;                    // the half beyond the last key this wavefront sees
            f32x16_t sacc, pacc;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
            {
                constexpr int NF = HD / 16;
                bf16x8_t fk[NF], fv[NF];
                auto read_kv = [&](int ks) {
                    const int o = kt * (32 * HD * 2) + rbase + (((ks * 2 + g) ^ rsw) << 4);
                    fk[ks] = *reinterpret_cast<const bf16x8_t*>(sK + o);
                    fv[ks] = *reinterpret_cast<const bf16x8_t*>(sV + o);
                };
#pragma unroll
                for (int ks = 0; ks < DQ_AHEAD; ++ks) read_kv(ks);
#pragma unroll
                for (int ks = 0; ks < NF; ++ks) {
                    if (ks + DQ_AHEAD < NF) read_kv(ks + DQ_AHEAD);
                    __builtin_amdgcn_sched_barrier(kFence);
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk[ks], qf[ks], sacc, 0, 0, 0);
                    pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fv[ks], dof[ks], pacc, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(kFence);
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[e], c, -lse2));   // P^T
            if (need_mask) {
                // one real branch around the whole mask (see the forward kernel): tested per element, it would cut
                // the chain of exponentials into sixteen basic blocks
                int kbase = kv0 + kt * 32;
                asm volatile("" : "+s"(kbase));
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = kbase + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (key >= kl || (CAUSAL && key > qi)) sacc[e] = 0.f;
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[e] *= pacc[e] - delta;          // dS^T
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const bf16x8_t dsf = frag_from_acc(sacc, u);
#pragma unroll
                for (int dt = 0; dt < HD / 32; ++dt) {
                    const bf16x8_t kt_f = read_tr<HD>(sK, tro, 2 * kt + u, dt);
                    gacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt_f, dsf, gacc[dt], 0, 0, 0);
                }
            }
        }
    }
    if (qi < ql) store_cols<HD>(gacc, a.scale, (bf16_t*)a.dq + (qrow0 + qi) * a.ldq + h * HD, g);
}

// ------------------------------------------------------------------------------------ backward: dK, dV
// LDS, a ring of four stages of: Q tile, dO tile ([64][HD]) and the two statistics tiles ([64 rows][8] bf16:
// {hi, lo, 0 x 6} of lse/scale and of delta, as the dQ kernel left them).  Three blocks are in flight while one is
// consumed: with one wavefront per SIMD (about 370 registers) nothing else hides the latency of the transfers.
template <int HD, bool CAUSAL>
__global__ __launch_bounds__(256, HD == 64 ? 2 : 1) void attn_bwd_dkv_mfma_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int TILE = 64 * HD * 2;
    constexpr int STAGE = 2 * TILE + 2048;
    constexpr int NS = 4;                               // ring of stages: three blocks in flight while one is consumed
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, g = lane >> 5;
    const int item = blockIdx.x / a.n_heads, h = blockIdx.x - item * a.n_heads;
    if (item >= a.n_items[1]) return;
    const int2 it = a.items_k[item];
    const int s = it.x, k0 = it.y * 128;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const long long qrow0 = a.q_row[s], krow0 = a.k_row[s];
    const bf16_t* Q = (const bf16_t*)a.q + qrow0 * a.ldq + h * HD;
    const bf16_t* dO = (const bf16_t*)a.d_o + qrow0 * a.ldo + h * HD;
    const bf16_t* K = (const bf16_t*)a.k + krow0 * a.ldk + h * HD;
    const bf16_t* V = (const bf16_t*)a.v + krow0 * a.ldv + h * HD;
    const int kw0 = k0 + wave * 32;
    const int ki = kw0 + col;
    const int ki_c = ki < kl ? ki : kl - 1;

    const int q_begin = CAUSAL ? k0 : 0;
    const int nb = (ql - q_begin + 63) / 64;            // >= 1: a key block exists only below the query count when causal
    TileLoader<HD> ldQ, ldO;
    ldQ.setup(Q, a.ldq, ql, wave, lane);
    ldO.setup(dO, a.ldo, ql, wave, lane);
    const char* aug_src = reinterpret_cast<const char*>(wave == 0 ? a.aug_lse : a.aug_delta) +
                          ((size_t)h * a.lse_stride + qrow0) * 16;
    // block blk -> stage blk % 4: Q tile, dO tile, and (wavefronts 0 and 1) the two statistics tiles, all by direct
    // transfers; indices past the last block are clamped (redundant transfers into a free stage keep the count of
    // outstanding transfers the same at every step)
    const uint32_t lds0 = lds_address(smem);
    auto issue_block = [&](int blk) {
        const uint32_t n = lds0 + (blk & (NS - 1)) * STAGE;
        const int bc = blk < nb ? blk : nb - 1;
        const int q0 = q_begin + bc * 64;
        ldQ.issue(n, q0);
        ldO.issue(n + TILE, q0);
        if (wave < 2) {
            int r = q0 + lane;
            r = r < ql ? r : ql - 1;
            lds_dma16_at(aug_src + (size_t)r * 16, n + 2 * TILE + wave * 1024);
        }
    };
    if (nb > 0) {
        issue_block(0);
        issue_block(1);
        issue_block(2);
    }

    bf16x8_t kf[HD / 16], vf[HD / 16];
#pragma unroll
    for (int ks = 0; ks < HD / 16; ++ks) {
        kf[ks] = *reinterpret_cast<const bf16x8_t*>(K + (long long)ki_c * a.ldk + ks * 16 + g * 8);
        vf[ks] = *reinterpret_cast<const bf16x8_t*>(V + (long long)ki_c * a.ldv + ks * 16 + g * 8);
    }
    bf16x8_t neg_ones;                                  // contraction slots 0, 1 (lane half 0) pick -hi - lo
#pragma unroll
    for (int j = 0; j < 8; ++j) neg_ones[j] = (bf16_t)((g == 0 && j < 2) ? -1.0f : 0.0f);
    const float c = a.scale * kLog2e;

    TrOffsets<HD> tro;
    tro.init(lane);
    const int rbase = col * (HD * 2);
    const int rsw = swz<HD>(col);

    f32x16_t dkacc[HD / 32], dvacc[HD / 32];
#pragma unroll
    for (int dt = 0; dt < HD / 32; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) { dkacc[dt][e] = 0.f; dvacc[dt][e] = 0.f; }

    // the K / V fragments (ordinary loads) are complete before the loop: left to the compiler, its waits for them
    // would sit inside the loop as "nothing outstanding", which would also drain the transfers in flight
    __builtin_amdgcn_s_waitcnt(0x0F70);
    // One step = one 64-query block.  The step exists in two versions, with and without the mask, and the loop is
    // cut into three: the (at most two) blocks on the diagonal, the blocks in the middle, the ragged last block.  The
    // middle loop, where the time goes, is then straight code: a mask test inside it, even one that is never taken,
    // splits the live ranges of the 128 accumulator registers and costs hundreds of register copies per step.
    const bool wave_has_keys = kw0 < kl;
    auto step = [&](int b, auto masked_t) {
        constexpr bool MASKED = decltype(masked_t)::value;
        const int q0 = q_begin + b * 64;
        char* sQ = smem + (b & (NS - 1)) * STAGE;
        char* sdO = sQ + TILE;
        char* s_lse = sdO + TILE;
        char* s_delta = s_lse + 1024;
        // block b has landed for this wavefront (the two newest blocks may still be in flight), then for everybody;
        // the stage read in the previous step is free
        if (wave < 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * (2 * (HD / 32) + 1)));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * (2 * (HD / 32))));
        __builtin_amdgcn_s_barrier();
        issue_block(b + 3);
        if (!wave_has_keys) return;
        if (MASKED && CAUSAL && q0 + 63 < kw0) return;
        if constexpr (!MASKED) {
            // Middle blocks: the two 32-query halves software-pipelined.  The exp / product work of half 0 sits between
            // the MFMAs of half 1's first products, that of half 1 between the MFMAs of half 0's second products, so
            // that the one wavefront of this SIMD keeps the matrix pipe and the vector ALU busy at the same time.
            constexpr int NA = HD / 16 + 1, AHEAD = 3, ND = 2 * (HD / 32), AHEAD_D = 2;
            f32x16_t sa[2], pa[2];
            bf16x8_t fq[NA], fo[NA], td[ND], tq[ND], pf[2], dsf[2];
            auto read_a = [&](int qt, int i) {
                if (i < HD / 16) {
                    const int o = qt * (32 * HD * 2) + rbase + (((i * 2 + g) ^ rsw) << 4);
                    fq[i] = *reinterpret_cast<const bf16x8_t*>(sQ + o);
                    fo[i] = *reinterpret_cast<const bf16x8_t*>(sdO + o);
                } else {
                    fq[i] = *reinterpret_cast<const bf16x8_t*>(s_lse + (qt * 32 + col) * 16);
                    fo[i] = *reinterpret_cast<const bf16x8_t*>(s_delta + (qt * 32 + col) * 16);
                }
            };
            auto softmax2 = [&](int qt, int e0) {         // two elements of half qt: P and dS in place
#pragma unroll
                for (int e = e0; e < e0 + 2; ++e) {
                    const float p = __builtin_amdgcn_exp2f(sa[qt][e] * c);
                    sa[qt][e] = p;
                    pa[qt][e] = p * pa[qt][e];
                }
            };
            auto phase_a = [&](int qt, bool with_prev) {
#pragma unroll
                for (int e = 0; e < 16; ++e) { sa[qt][e] = 0.f; pa[qt][e] = 0.f; }
#pragma unroll
                for (int i = 0; i < AHEAD; ++i) read_a(qt, i);
#pragma unroll
                for (int i = 0; i < NA; ++i) {
                    if (i + AHEAD < NA) read_a(qt, i + AHEAD);
                    __builtin_amdgcn_sched_barrier(kFence);
                    sa[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[i], i < HD / 16 ? kf[i < HD / 16 ? i : 0] : neg_ones, sa[qt], 0, 0, 0);
                    pa[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[i], i < HD / 16 ? vf[i < HD / 16 ? i : 0] : neg_ones, pa[qt], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(kFence);
                    if (with_prev && i < NA - 1) {          // 16 / (NA - 1) elements of the other half per slice
#pragma unroll
                        for (int e = i * (16 / (NA - 1)); e < (i + 1) * (16 / (NA - 1)); e += 2) softmax2(qt ^ 1, e);
                    }
                }
            };
            auto phase_d = [&](int qt, bool with_next) {
#pragma unroll
                for (int u = 0; u < 2; ++u) { pf[u] = frag_from_acc(sa[qt], u); dsf[u] = frag_from_acc(pa[qt], u); }
                auto read_d = [&](int j) {
                    td[j] = read_tr<HD>(sdO, tro, 2 * qt + j / (HD / 32), j % (HD / 32));
                    tq[j] = read_tr<HD>(sQ, tro, 2 * qt + j / (HD / 32), j % (HD / 32));
                };
#pragma unroll
                for (int j = 0; j < AHEAD_D; ++j) read_d(j);
#pragma unroll
                for (int j = 0; j < ND; ++j) {
                    if (j + AHEAD_D < ND) read_d(j + AHEAD_D);
                    __builtin_amdgcn_sched_barrier(kFence);
                    dvacc[j % (HD / 32)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(td[j], pf[j / (HD / 32)], dvacc[j % (HD / 32)], 0, 0, 0);
                    dkacc[j % (HD / 32)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[j], dsf[j / (HD / 32)], dkacc[j % (HD / 32)], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(kFence);
                    if (with_next) {
#pragma unroll
                        for (int e = j * (16 / ND); e < (j + 1) * (16 / ND); e += 2) softmax2(qt ^ 1, e);
                    }
                }
            };
            phase_a(0, false);
            phase_a(1, true);          // + exp / products of half 0
            phase_d(0, true);          // + exp / products of half 1
            phase_d(1, false);
            return;
        }
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            if (MASKED && (q0 + qt * 32 >= ql || (CAUSAL && q0 + qt * 32 + 31 < kw0))) continue;   // no visible query
            f32x16_t sacc, pacc;
#pragma unroll
            for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
            // S^T and dP^T: NA = HD/16 + 1 contraction slices (the last one is the appended statistics), two MFMAs each.
            // The fragment reads run AHEAD slices in front of the MFMAs that use them (left alone, the compiler puts
            // every read right before its MFMA, in the same four registers, and each MFMA waits a full LDS round
            // trip); the fences keep LDS reads and MFMAs in this order, other instructions may move across.
            constexpr int NA = HD / 16 + 1, AHEAD = 3;
            bf16x8_t fq[NA], fo[NA];
            auto read_a = [&](int i) {
                if (i < HD / 16) {
                    const int o = qt * (32 * HD * 2) + rbase + (((i * 2 + g) ^ rsw) << 4);
                    fq[i] = *reinterpret_cast<const bf16x8_t*>(sQ + o);
                    fo[i] = *reinterpret_cast<const bf16x8_t*>(sdO + o);
                } else {
                    fq[i] = *reinterpret_cast<const bf16x8_t*>(s_lse + (qt * 32 + col) * 16);
                    fo[i] = *reinterpret_cast<const bf16x8_t*>(s_delta + (qt * 32 + col) * 16);
                }
            };
#pragma unroll
            for (int i = 0; i < AHEAD; ++i) read_a(i);
#pragma unroll
            for (int i = 0; i < NA; ++i) {
                if (i + AHEAD < NA) read_a(i + AHEAD);
                __builtin_amdgcn_sched_barrier(kFence);
                // (last slice: score - lse/scale and dP - delta through the constant [-1, -1] operand)
                sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[i], i < HD / 16 ? kf[i < HD / 16 ? i : 0] : neg_ones, sacc, 0, 0, 0);
                pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo[i], i < HD / 16 ? vf[i < HD / 16 ? i : 0] : neg_ones, pacc, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(kFence);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float p = __builtin_amdgcn_exp2f(sacc[e] * c);
                if (MASKED) {
                    const int q = q0 + qt * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
                    if (q >= ql || (CAUSAL && q < ki)) p = 0.f;
                }
                sacc[e] = p;                                           // P
                pacc[e] = p * pacc[e];                                 // dS
            }
            // dV += dO^T P^T and dK += Q^T dS^T: ND = 2 * HD/32 pairs of MFMAs, transpose reads AHEAD_D pairs in front
            constexpr int ND = 2 * (HD / 32), AHEAD_D = 2;
            bf16x8_t td[ND], tq[ND];
            auto read_d = [&](int j) {
                td[j] = read_tr<HD>(sdO, tro, 2 * qt + j / (HD / 32), j % (HD / 32));
                tq[j] = read_tr<HD>(sQ, tro, 2 * qt + j / (HD / 32), j % (HD / 32));
            };
            bf16x8_t pf[2], dsf[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) { pf[u] = frag_from_acc(sacc, u); dsf[u] = frag_from_acc(pacc, u); }
#pragma unroll
            for (int j = 0; j < AHEAD_D; ++j) read_d(j);
#pragma unroll
            for (int j = 0; j < ND; ++j) {
                if (j + AHEAD_D < ND) read_d(j + AHEAD_D);
                __builtin_amdgcn_sched_barrier(kFence);
                dvacc[j % (HD / 32)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(td[j], pf[j / (HD / 32)], dvacc[j % (HD / 32)], 0, 0, 0);
                dkacc[j % (HD / 32)] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tq[j], dsf[j / (HD / 32)], dkacc[j % (HD / 32)], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(kFence);
            }
        }
    };
    const int n_diag = CAUSAL ? min(2, nb) : 0;         // causal: queries k0 .. k0+127 meet this block's own keys
    const int n_full = (ql - q_begin) / 64;             // blocks b < n_full have all their 64 rows
    int b = 0;
    for (; b < n_diag; ++b) step(b, std::true_type{});
    for (; b < n_full; ++b) step(b, std::false_type{});
    for (; b < nb; ++b) step(b, std::true_type{});
    __builtin_amdgcn_s_waitcnt(0x0F70);                 // no transfer may still be writing LDS when the work-group ends
    if (ki < kl) {
        store_cols<HD>(dkacc, a.scale, (bf16_t*)a.dk + (krow0 + ki) * a.ldk + h * HD, g);
        store_cols<HD>(dvacc, 1.0f, (bf16_t*)a.dv + (krow0 + ki) * a.ldv + h * HD, g);
    }
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
    hipLaunchKernelGGL(kern, dim3((unsigned)a.max_items_q * a.n_heads), dim3(256), smem, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

template <int HD, bool CAUSAL>
ds_status bwd_launch(const AttnArgs& a, hipStream_t st) {
    static bool attr_q = false, attr_kv = false;
    auto kq = attn_bwd_dq_mfma_kernel<HD, CAUSAL>;
    auto kkv = attn_bwd_dkv_mfma_kernel<HD, CAUSAL>;
    const int smem_q = 4 * (64 * HD * 2);
    const int smem_kv = 4 * (2 * (64 * HD * 2) + 2048);
    ds_status r = set_smem(kq, smem_q, attr_q);
    if (r != DS_OK) return r;
    r = set_smem(kkv, smem_kv, attr_kv);
    if (r != DS_OK) return r;
    hipLaunchKernelGGL(kq, dim3((unsigned)a.max_items_q * a.n_heads), dim3(256), smem_q, st, a);
    DS_LAUNCH_CHECK();
    hipLaunchKernelGGL(kkv, dim3((unsigned)a.max_items_k * a.n_heads), dim3(256), smem_kv, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

int items_bound(int total_rows, int n_seq) { return total_rows / 128 + n_seq; }

}  // namespace

// Scratch: two counters, two work lists (query-side and key-side blocks), then the two statistics tensors the
// backward kernels hand over ([n_heads][q_total_rows] entries of 16 bytes each).
static size_t lists_bytes(int q_total_rows, int k_total_rows, int n_seq) {
    const size_t b = 256 + sizeof(int2) * ((size_t)items_bound(q_total_rows, n_seq) + (size_t)items_bound(k_total_rows, n_seq));
    return (b + 255) & ~(size_t)255;
}
size_t attn_scratch_bytes(int n_heads, int head_dim, int q_total_rows, int k_total_rows, int n_seq) {
    (void)head_dim;
    return lists_bytes(q_total_rows, k_total_rows, n_seq) + 2 * (size_t)n_heads * q_total_rows * 16;
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
    const long long ld_max = 1LL << 23;                // 64 rows of a tile stay within a 31-bit byte offset
    if (a.ldq >= ld_max || a.ldk >= ld_max || a.ldv >= ld_max || a.ldo >= ld_max) return false;
    if (a.scratch_bytes < attn_scratch_bytes(a.n_heads, a.head_dim, a.q_total_rows, a.k_total_rows, a.n_seq)) return false;
    if ((long long)items_bound(a.q_total_rows, a.n_seq) * a.n_heads > 0x7fffffffLL) return false;
    if ((long long)items_bound(a.k_total_rows, a.n_seq) * a.n_heads > 0x7fffffffLL) return false;
    return true;
}

// Lay the work lists out in the scratch buffer and, unless the caller says they are already there, build them.
ds_status attn_prepare_lists(AttnArgs& a, bool need_key_side, hipStream_t st) {
    char* base = (char*)a.scratch;
    a.n_items = (const int32_t*)base;
    a.max_items_q = items_bound(a.q_total_rows, a.n_seq);
    a.max_items_k = items_bound(a.k_total_rows, a.n_seq);
    a.items_q = (const int2*)(base + 256);
    a.items_k = a.items_q + a.max_items_q;
    a.aug_lse = base + lists_bytes(a.q_total_rows, a.k_total_rows, a.n_seq);
    a.aug_delta = (char*)a.aug_lse + (size_t)a.n_heads * a.q_total_rows * 16;
    if (a.lists_ready) return DS_OK;
    hipLaunchKernelGGL(attn_worklist_kernel, dim3(1), dim3(1024), 0, st, a.n_seq, a.q_len, a.k_len, a.mask, 0, a.max_items_q,
                       (int2*)a.items_q, (int32_t*)base);
    DS_LAUNCH_CHECK();
    if (need_key_side || a.lists_want_both) {
        hipLaunchKernelGGL(attn_worklist_kernel, dim3(1), dim3(1024), 0, st, a.n_seq, a.k_len, a.q_len, a.mask, 1, a.max_items_k,
                           (int2*)a.items_k, (int32_t*)base + 1);
        DS_LAUNCH_CHECK();
    }
    return DS_OK;
}

ds_status attn_fwd_mfma(const AttnArgs& a0, hipStream_t st) {
    AttnArgs a = a0;
    ds_status r = attn_prepare_lists(a, false, st);
    if (r != DS_OK) return r;
    if (a.head_dim == 128) return a.mask ? fwd_launch<128, true>(a, st) : fwd_launch<128, false>(a, st);
    return a.mask ? fwd_launch<64, true>(a, st) : fwd_launch<64, false>(a, st);
}

ds_status attn_bwd_mfma(const AttnArgs& a0, hipStream_t st) {
    AttnArgs a = a0;
    ds_status r = attn_prepare_lists(a, true, st);
    if (r != DS_OK) return r;
    if (a.head_dim == 128) return a.mask ? bwd_launch<128, true>(a, st) : bwd_launch<128, false>(a, st);
    return a.mask ? bwd_launch<64, true>(a, st) : bwd_launch<64, false>(a, st);
}
