// GEMMs of the stage: projections forward (NN), input gradients (NT) and weight gradients (TN,
// the contraction running over every token of every micro-batch, which is the gradient
// accumulation across micro-batches).
//
// Two kernels:
//   * gemm_bf16_nt_kernel — the one the stage runs on: bf16 in, fp32 accumulate on the CDNA4 matrix cores
//     (v_mfma_f32_16x16x32_bf16), operands straight from global memory into LDS, NT form (forward with [N][K]
//     weight copies, input gradients) and TN form (weight gradients); described where it is defined.
//   * gemm_generic_kernel — any dtype / shape / stride, plain FMA; the fp32 path and the fallback for the operand
//     forms and shapes the matrix-core kernel does not take (NN; TN with an epilogue other than fp32 accumulation;
//     N not a multiple of 256).
// Epilogues go back through LDS so that global stores (and the residual / activation reads) are 16 bytes per lane
// and row-contiguous.  Work-group ids are remapped so that each XCD (own L2) gets a contiguous run of tiles.
#include "gemm.hpp"

#include <atomic>
#include <mutex>


namespace {

// ---------------------------------------------------------------------------- epilogues
// Applied to 8 consecutive columns n..n+7 of row m; acc holds the fp32 accumulators.
// What an epilogue reads besides the accumulators, fetched ahead of time (8 elements of R, of R2, the row flag),
// so that a caller can issue these loads for several rows at once instead of one dependent round trip per row.
// Kept in storage precision (16 bytes per operand for bf16) so that a whole tile's worth fits in registers.
template <class T> struct EpiPre {
    T r[8], r2[8];
    int valid;
};
template <class T>
__device__ __forceinline__ void load8_raw(const T* src, T (&dst)[8]) {
    if (sizeof(T) == 2) {
        const uint4 v = *reinterpret_cast<const uint4*>(src);
        __builtin_memcpy(dst, &v, 16);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) dst[j] = src[j];
    }
}
template <class T, int EPI>
__device__ __forceinline__ void epilogue_prefetch(int m, int n, int N, const GemmEpi& p, EpiPre<T>& q) {
    const size_t off = (size_t)m * N + n;
    q.valid = 1;
    if (EPI == DS_EPI_RESID) {
        if (p.row_valid) q.valid = p.row_valid[m] >= 0;
        load8_raw(reinterpret_cast<const T*>(p.R) + off, q.r);
    } else if (EPI == DS_EPI_DGELU || EPI == DS_EPI_GATE || EPI == DS_EPI_MULR) {
        load8_raw(reinterpret_cast<const T*>(p.R) + off, q.r);
    } else if (EPI == DS_EPI_DGATE) {
        load8_raw(reinterpret_cast<const T*>(p.R) + off, q.r);
        load8_raw(reinterpret_cast<const T*>(p.R2) + off, q.r2);
    }
}
template <int EPI> constexpr bool epilogue_reads() {
    return EPI == DS_EPI_RESID || EPI == DS_EPI_DGELU || EPI == DS_EPI_GATE || EPI == DS_EPI_DGATE || EPI == DS_EPI_MULR;
}

template <class T, int EPI>
__device__ __forceinline__ void epilogue8(int m, int n, int N, float (&acc)[8], T* __restrict__ C, const GemmEpi& p,
                                          const EpiPre<T>* pre = nullptr) {
    const size_t off = (size_t)m * N + n;
    if (EPI == DS_EPI_ACC32) {
        float* c = reinterpret_cast<float*>(C) + off;
        if (p.accumulate) {
            float old[8];
            Vec8<float>::load(c, old);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += old[j];
        }
        Vec8<float>::store(c, acc);
        return;
    }
    if (p.bias) {
        float b[8];
        Vec8<T>::load(reinterpret_cast<const T*>(p.bias) + n, b);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += b[j];
    }
    if (EPI == DS_EPI_NONE) {
        Vec8<T>::store_nt(C + off, acc);
    } else if (EPI == DS_EPI_GELU) {
        // round the pre-activation to storage precision first, so that forward and backward see the same z
        float z[8], a[8];
        Vec8<T>::store_nt(C + off, acc);
#pragma unroll
        for (int j = 0; j < 8; ++j) { z[j] = to_f32(from_f32<T>(acc[j])); a[j] = gelu_f(z[j]); }
        Vec8<T>::store_nt(reinterpret_cast<T*>(p.C2) + off, a);
    } else if (EPI == DS_EPI_GELU_D) {
        // what the layer's backward needs of the pre-activation is GELU'(z) alone: it is computed here, where the
        // logistic term is at hand anyway, and stored in place of z; the backward epilogue is then one multiplication
        float dz[8], a[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) gelu_and_grad_f(acc[j], a[j], dz[j]);
        Vec8<T>::store_nt(C + off, dz);
        Vec8<T>::store_nt(reinterpret_cast<T*>(p.C2) + off, a);
    } else if (EPI == DS_EPI_MULR) {
        float r[8];
        if (pre) {
#pragma unroll
            for (int j = 0; j < 8; ++j) r[j] = to_f32(pre->r[j]);
        } else {
            Vec8<T>::load(reinterpret_cast<const T*>(p.R) + off, r);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= r[j];
        Vec8<T>::store_nt(C + off, acc);
    } else if (EPI == DS_EPI_RESID) {
        if (pre) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = pre->valid ? acc[j] + to_f32(pre->r[j]) : 0.f;
        } else if (p.row_valid && p.row_valid[m] < 0) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = 0.f;
        } else {
            float r[8];
            Vec8<T>::load(reinterpret_cast<const T*>(p.R) + off, r);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += r[j];
        }
        Vec8<T>::store_nt(C + off, acc);
    } else if (EPI == DS_EPI_DGELU) {
        float z[8];
        if (pre) {
#pragma unroll
            for (int j = 0; j < 8; ++j) z[j] = to_f32(pre->r[j]);
        } else {
            Vec8<T>::load(reinterpret_cast<const T*>(p.R) + off, z);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] *= gelu_grad_f(z[j]);
        Vec8<T>::store_nt(C + off, acc);
    } else if (EPI == DS_EPI_GATE) {
        // acc = u Wu (stored); C2 = GELU(R) * acc with R = u Wg
        float zg[8], a[8];
        Vec8<T>::store_nt(C + off, acc);
        if (pre) {
#pragma unroll
            for (int j = 0; j < 8; ++j) zg[j] = to_f32(pre->r[j]);
        } else {
            Vec8<T>::load(reinterpret_cast<const T*>(p.R) + off, zg);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] = gelu_f(zg[j]) * to_f32(from_f32<T>(acc[j]));
        Vec8<T>::store_nt(reinterpret_cast<T*>(p.C2) + off, a);
    } else if (EPI == DS_EPI_DGATE) {
        // acc = da; R = zg, R2 = zu; C = dzg = da * zu * GELU'(zg); C2 = dzu = da * GELU(zg)
        float zg[8], zu[8], o1[8], o2[8];
        if (pre) {
#pragma unroll
            for (int j = 0; j < 8; ++j) { zg[j] = to_f32(pre->r[j]); zu[j] = to_f32(pre->r2[j]); }
        } else {
            Vec8<T>::load(reinterpret_cast<const T*>(p.R) + off, zg);
            Vec8<T>::load(reinterpret_cast<const T*>(p.R2) + off, zu);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            o1[j] = acc[j] * zu[j] * gelu_grad_f(zg[j]);
            o2[j] = acc[j] * gelu_f(zg[j]);
        }
        Vec8<T>::store_nt(C + off, o1);
        Vec8<T>::store(reinterpret_cast<T*>(p.C2) + off, o2);
    }
}

// ---------------------------------------------------------------------------- generic kernel
// 64x64 tile, 256 threads, 4x4 outputs per thread, K step 16.  A(m,k) = A[m*sam + k*sak].
// Requires N % 8 == 0 (8-wide epilogue); M, K arbitrary.
template <class T, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(int M, int N, int K, const T* __restrict__ A, long long sam,
                                                           long long sak, const T* __restrict__ B, long long sbk,
                                                           long long sbn, T* __restrict__ C, GemmEpi p) {
    __shared__ float As[16][68];
    __shared__ float Bs[16][68];
    const int t = threadIdx.x;
    const int tx = t & 7, ty = t >> 3;            // tx: 8 column groups of 8, ty: 32 row pairs
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = t + 256 * i;
            {
                const int mm = sak == 1 ? idx >> 4 : idx & 63;
                const int kk = sak == 1 ? idx & 15 : idx >> 6;
                const int m = m0 + mm, k = k0 + kk;
                As[kk][mm] = (m < M && k < K) ? to_f32(A[m * sam + k * sak]) : 0.f;
            }
            {
                const int nn = sbk == 1 ? idx >> 4 : idx & 63;
                const int kk = sbk == 1 ? idx & 15 : idx >> 6;
                const int n = n0 + nn, k = k0 + kk;
                Bs[kk][nn] = (n < N && k < K) ? to_f32(B[k * sbk + n * sbn]) : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const float a0 = As[kk][ty * 2], a1 = As[kk][ty * 2 + 1];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float b = Bs[kk][tx * 8 + j];
                acc[0][j] += a0 * b;
                acc[1][j] += a1 * b;
            }
        }
        __syncthreads();
    }
    const int n = n0 + tx * 8;
    if (n < N) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = m0 + ty * 2 + i;
            if (m < M) epilogue8<T, EPI>(m, n, N, acc[i], C, p);
        }
    }
}

// macro tile of the matrix-core kernel
constexpr int BM = 256, BN = 256, BK = 64;

// ---------------------------------------------------------------------------- NT / TN kernel, direct to LDS
// NT form: C[M,N] = A[M,K] * B[N,K]^T, both operands k-contiguous (K % 64 == 0, N % 256 == 0).
// TN form: C[M,N] = A[K,M]^T * B[K,N], both operands with the contraction index as the row (weight gradients).
//
// 256x256 macro tile, 8 wavefronts (2 per SIMD) in a 2x4 arrangement, each owning a 128x64 accumulator block:
// 8 x 4 blocks of v_mfma_f32_16x16x32_bf16, 128 accumulator registers.  Operands go global -> LDS directly
// (global_load_lds_dwordx4): no staging registers, no LDS write instructions.  A wavefront instruction deposits
// 64 x 16 bytes at consecutive LDS addresses; the XOR swizzle that makes the fragment reads conflict-free is
// obtained by choosing WHICH global chunk each lane fetches.  NT: 64-deep K tiles (whole 128-byte lines per row),
// two 64 KB stages, one barrier per tile.  TN: 32 k-rows of 512 bytes per tile, ring of 4 stages of 32 KB, three
// tiles in flight while one is consumed, fragments through the LDS transpose read.  Tile indices past the end
// are clamped (a few redundant loads into a free stage) so that the wait counts are the same at every step.
//
// Why 8 wavefronts: measured on MI355X, one 4-wavefront work-group cannot pull more than about 40-50 GB/s from
// L2 however many loads it keeps in flight, which is what a 256x256x(bf16) tile needs at full MFMA rate; the rate
// scales with the number of wavefronts on the CU; and a single wavefront per SIMD cannot keep the matrix pipe
// busy with the 16x16x32 shape (it needs two issuing).
constexpr int NT_DK = 32, NT_NS = 4, NT_HALF = 256 * NT_DK * 2, NT_STAGE = 2 * NT_HALF;
constexpr int NT_WM = 2, NT_WN = 4;             // wavefront grid of a work-group: 2 x 4, each wavefront 128 x 64
// how a K tile's direct-load instructions are spread over the MFMA groups of the main loops (see the loops)
constexpr int NT_G0 = 1, NT_G1 = 1, NT_G2 = 0;       // (in transfer groups: the A part, the B part)
// tile number -> tile coordinates: groups of NT_GROUP tile rows, column-major inside a group
constexpr int NT_GROUP = 4;
__host__ __device__ __forceinline__ void nt_tile_coords(int logical, int tiles_m, int tiles_n, int& tile_m, int& tile_n) {
    const int group_sz = NT_GROUP * tiles_n;
    const int group = logical / group_sz;
    const int first_m = group * NT_GROUP;
    const int gs = (tiles_m - first_m) < NT_GROUP ? (tiles_m - first_m) : NT_GROUP;
    const int in_group = logical - group * group_sz;
    tile_m = first_m + in_group % gs;
    tile_n = in_group / gs;
}

// WM x WN wavefronts per work-group; each owns a (256/WM) x (256/WN) accumulator block.
//
// TN form (weight gradients): C[M,N] = A[K,M]^T * B[K,N], both operands row-major with the
// contraction index (tokens) as the ROW.  A K tile is then 32 rows of 512 contiguous bytes per
// operand, fetched as whole rows, and the MFMA fragments (8 consecutive k for one m or n per lane)
// come out of LDS through the transpose read ds_read_b64_tr_b16, 4 k-rows per read; both operands
// use the same k order, so the contraction is unchanged.  K may be ragged: rows past the end read
// zeros.  This form needs no transposed copies of the activations.
//
// PS (persistent form, NT only, no uniform split-K): the first ps_wgs work-groups, one per compute unit, stay resident
// and take the n_main unsplit tiles one after another; the tail pieces are ordinary work-groups behind them.  The
// tiles keep their XCD-contiguous numbering: work-group w serves the run of XCD w % 8, starts with tile w / 8 of that
// run and draws every further one from that XCD's counter (ps_ctr[xcd], one atomic per tile, issued a whole main
// loop before its result is needed), so a faster compute unit takes more tiles, as under the hardware dispatcher.
// What persistence buys: the first K tile of the NEXT tile is requested before the epilogue of the current one
// starts (into stage 0, while the epilogue stages through LDS above it), so neither the latency of that first fetch
// nor the end of one work-group and the start of the next leaves the matrix cores idle.  The last work-group to
// finish puts the counters back to zero (ps_ctr[8] counts the finished ones).
template <int EPI, int WM, int WN, bool TNF, bool PS>
__global__ __launch_bounds__(WM * WN * 64, 1) void gemm_bf16_nt_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                                       const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
                                                                       int tiles_m, int tiles_n, int splits,
                                                                       int n_main, int tail_splits,
                                                                       float* __restrict__ split_ws, GemmEpi p,
                                                                       int ps_wgs, int* __restrict__ ps_ctr) {
    static_assert(!(PS && TNF), "the persistent form exists for the NT kernel only");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int NW = WM * WN;                    // wavefronts
    constexpr int TM = 256 / WM / 32, TN = 256 / WN / 32;   // 32x32 MFMA tiles per wavefront
    static_assert(16 % NW == 0, "wavefront count must divide 16");
    constexpr int STG_LD = TN * 32 + 4;            // fp32 row stride of the epilogue staging block
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // ---- work-group id -> (tile, split).  Two regimes share the kernel:
    //  * uniform split-K (weight gradients): every tile is cut into `splits` K ranges, partial sums go to split_ws
    //    as [split][M][N];
    //  * tail split-K (everything else): the first n_main tiles, a whole number of rounds over the compute units,
    //    run unsplit; each of the remaining tiles is cut into tail_splits K ranges so that the last, partly filled
    //    round costs 1/tail_splits of a round; their partial sums go to split_ws as [tail tile][split][256][256].
    // Tiles are numbered so that each XCD works on contiguous runs, in groups of 8 tile rows (L2 reuse).
    const int n_tiles = tiles_m * tiles_n;
    int logical, split, nsplit;
    bool tail = false;
    const bool persistent = PS && (int)blockIdx.x < ps_wgs;
    int run_start = 0, run_cnt = 0;                 // persistent: this XCD's run of unsplit tiles
    if (persistent) {
        const int xcd = blockIdx.x & 7;
        const int per = n_main >> 3, rem = n_main & 7;
        run_start = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
        run_cnt = per + (xcd < rem ? 1 : 0);
        logical = run_start + (blockIdx.x >> 3);    // (the host launches this form only with n_main >= 2 ps_wgs)
        split = 0;
        nsplit = 1;
    } else {
        const int pid = PS ? (int)blockIdx.x - ps_wgs + n_main : (int)blockIdx.x;
        const int total = splits > 1 ? n_tiles * splits : n_main;
        if (pid < total) {
            const int xcd = pid & 7, local = pid >> 3;
            const int per = total >> 3, rem = total & 7;
            const int start = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
            logical = start + local;
            split = logical / n_tiles;
            logical -= split * n_tiles;
            nsplit = splits;
        } else {
            const int r = pid - total;
            logical = n_main + r / tail_splits;
            split = r % tail_splits;
            nsplit = tail_splits;
            tail = true;
        }
    }

    // K tiles: TN form 32 k-rows of 512 bytes, ring of 4 stages; NT form 64 k (one whole 128-byte line per row and
    // request, which is what the L2 serves at full rate), 2 stages
    constexpr int DK = TNF ? NT_DK : 64;
    constexpr int NS = TNF ? NT_NS : 2;
    constexpr int HALF = 256 * DK * 2, STAGE = 2 * HALF;
    constexpr int LPW = HALF / 1024 / NW;          // direct-load instructions per operand per wavefront per K tile
    static_assert(NS * STAGE == NT_NS * NT_STAGE, "both forms use the same 128 KB of LDS");
    const int nt_total = TNF ? (K + DK - 1) / DK : K / DK;
    const int per_split = (nt_total + nsplit - 1) / nsplit;
    const int t_begin = split * per_split;
    const int t_end = (t_begin + per_split) < nt_total ? (t_begin + per_split) : nt_total;

    // accumulators: TM16 x TN16 blocks of 16 x 16 (v_mfma_f32_16x16x32_bf16: at the chip's power limit this shape
    // sustains about a sixth more than 32x32x16 on random operands, at the same LDS traffic per flop)
    constexpr int TM16 = 2 * TM, TN16 = 2 * TN, HA = TM16 / 2;
    f32x4_t acc[TM16][TN16];

    // what the transfers of a tile need: its corner, the operand bases there and the per-lane offsets (set_tile)
    int tile_m = 0, tile_n = 0, m0 = 0, n0 = 0;
    const char* pa = nullptr;
    const char* pb = nullptr;
    uint32_t offAg[LPW], offBg[LPW];                                // per-lane offsets as a transfer group wants them
    auto set_tile = [&](int lg) {
        nt_tile_coords(lg, tiles_m, tiles_n, tile_m, tile_n);
        m0 = tile_m * BM;
        n0 = tile_n * BN;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int u = (wave * LPW + i) * 64 + lane;
            uint32_t oa, ob;
            if constexpr (!TNF) {                                    // 16-byte unit of the 256 x 8 tile (128-byte rows)
                const int row = u >> 3, slot = u & 7;
                const int chunk = slot ^ ((row >> 1) & 7);
                int ra_ = m0 + row;
                ra_ = ra_ < M ? ra_ : M - 1;                        // rows past the edge: clamped, never stored
                oa = (uint32_t)(((long long)(ra_ - m0) * K + chunk * 8) * 2);
                ob = (uint32_t)(((long long)row * K + chunk * 8) * 2);
                offAg[i] = dma_lane_offset<LPW>(oa, i);
                offBg[i] = dma_lane_offset<LPW>(ob, i);
            } else {                                                // 16-byte unit of the 32 k-row tile (512-byte rows)
                const int row = u >> 5, pos = u & 31;
                const int chunk = (((pos >> 1) ^ (row & 7)) << 1) | (pos & 1);
                oa = (uint32_t)(((long long)row * M + chunk * 8) * 2);
                ob = (uint32_t)(((long long)row * N + chunk * 8) * 2);
                offAg[i] = dma_lane_offset<2 * LPW>(oa, i);         // group of four: A, A, B, B
                offBg[i] = dma_lane_offset<2 * LPW>(ob, LPW + i);
            }
        }
        pa = reinterpret_cast<const char*>(A) + (TNF ? (long long)m0 * 2 : (long long)m0 * K * 2);
        pb = reinterpret_cast<const char*>(B) + (TNF ? (long long)n0 * 2 : (long long)n0 * K * 2);
    };
    set_tile(logical);
    bool primed = false;                            // persistent: the first K tile of this tile is already on its way
    constexpr int PS_SLOT = 65536 + NW * 32 * (TN * 32 + 4) * 4;    // LDS word through which wavefront 0 hands on the next tile
    constexpr int STG_OFF = PS ? 65536 : 0;         // epilogue staging: above stage 0, which already receives the next tile
    for (;;) {
        // the epilogue below belongs to the tile the main loop has just finished, not to the one set_tile has moved on to
        const int em0 = m0, en0 = n0, etile_m = tile_m, elogical = logical;
        int next_local = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < TM16; ++i)
#pragma unroll
            for (int j = 0; j < TN16; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

        if (t_begin < t_end) {
            const uint32_t lds0 = lds_address(smem);
            const int wave_u = __builtin_amdgcn_readfirstlane(wave);
            const long long tile_step_a = TNF ? (long long)DK * M * 2 : DK * 2;
            const long long tile_step_b = TNF ? (long long)DK * N * 2 : DK * 2;
            const int frag_row = lane & 15, frag_grp = lane >> 4;       // operand row / k group of this lane
            const int t_last = t_end - 1;
            // The transfers of a K tile, in the groups the main loops hand out between their MFMAs (a wavefront cannot issue
            // anything else while a transfer of its own passes the address stage of the texture path, so they are neither
            // issued in one burst after the barrier, which left the matrix cores idle for about a quarter of every tile,
            // nor one at a time with an M0 of their own: a write of M0 waits for the transfer before it).
            //   NT form: s = 0 / 1 = this wavefront's part of the A / B tile, LPW transfers under one M0; wavefront-uniform
            //     base in scalar registers + per-lane offsets that never change (stepping along K costs no vector
            //     instruction); LDS destinations are scalar integers, not generic pointers.
            //   TN form: s = 0 = both parts (A, A, B, B in one 4 KB block of LDS per wavefront), through two buffer
            //     descriptors whose lengths end at the last row of a ragged K: rows past the end read zeros, with no
            //     per-lane test.
            auto issue_one = [&](int tile, int stage, int s) {
                tile = tile < t_last ? tile : t_last;
                if constexpr (TNF) {
                    static_assert(!TNF || LPW == 2, "one group = two A and two B transfers");
                    const int k_left = K - tile * DK;
                    const uint32_t rows = (uint32_t)(k_left < DK ? k_left : DK);
                    const i32x4_t buf_a = make_raw_buffer(pa + tile * tile_step_a - 3072, rows * (uint32_t)M * 2u + 3072u);
                    const i32x4_t buf_b = make_raw_buffer(pb + tile * tile_step_b - 3072, rows * (uint32_t)N * 2u + 3072u);
                    lds_dma16_buffers_2x2(buf_a, offAg[0], offAg[1], buf_b, offBg[0], offBg[1],
                                          lds0 + stage * STAGE + wave_u * (2 * LPW * 1024));
                } else {
                    const uint32_t dst_g = lds0 + stage * STAGE + (s ? HALF : 0) + wave_u * (LPW * 1024);
                    if (s) lds_dma16_group<LPW>(dma_group_base<LPW>(pb + tile * tile_step_b), offBg, dst_g);
                    else lds_dma16_group<LPW>(dma_group_base<LPW>(pa + tile * tile_step_a), offAg, dst_g);
                }
            };
            auto issue = [&](int tile, int stage) {
#pragma unroll
                for (int s = 0; s < (TNF ? 1 : 2); ++s) issue_one(tile, stage, s);
            };
            // NT: 128-byte rows: 16 consecutive rows at one chunk index must hit 16 different 16-byte units of a 256-byte
            // window: rows 2q and 2q+1 differ by 128 bytes, the XOR with (row/2)%8 separates the 8 row pairs
            auto off64 = [](int row, int chunk) { return row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4); };
            // TN: 512-byte rows.  One operand fragment (16 features x 32 k) is two transpose reads, each 16 k-rows x 32
            // bytes: lane (i = lane%16, g = lane/16) addresses k-row 4g + i/4 (+16 for the second read) at features
            // (i%4)*4 of the 16-feature unit and receives feature i at k-rows 4g..4g+3.  The 32 lanes served together
            // touch 8 k-rows, so the 32-byte unit index is XORed with row%8.  Both operands use the same k order, so the
            // contraction is unchanged.
            const int tr_x = 4 * ((lane >> 4) & 1) + ((lane >> 2) & 3);
            // (LDS layout of a TN stage: per wavefront w one 4 KB block = k-rows 4w .. 4w+3 of the A tile, then of the B tile)
            const int tr_base = (lane >> 4) * 4096 + ((lane & 15) >> 2) * 512 + (lane & 3) * 8;
            auto read_tr = [&](const char* base, int unit) {
                typedef short s16x4_t __attribute__((ext_vector_type(4)));
                typedef short s16x8_t __attribute__((ext_vector_type(8)));
                typedef __attribute__((address_space(3))) s16x4_t* lds4_t;
                const char* q = base + tr_base + ((unit ^ tr_x) << 5);
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)q);
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(q + 4 * 4096));
                const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(bf16x8_t, v);
            };
            // fragments of 32-deep k step `ks` of a stage: HA of this wavefront's TM16 row units (half h), all TN16 column units
            auto load_a = [&](int stage, int ks, int h, bf16x8_t (&fa)[HA]) {
                const char* a_base = smem + stage * STAGE;
#pragma unroll
                for (int i = 0; i < HA; ++i) {
                    if constexpr (TNF) fa[i] = read_tr(a_base, wm * TM16 + h * HA + i);
                    else fa[i] = *reinterpret_cast<const bf16x8_t*>(a_base + off64(wm * (TM * 32) + (h * HA + i) * 16 + frag_row, ks * 4 + frag_grp));
                }
            };
            auto load_b = [&](int stage, int ks, bf16x8_t (&fb)[TN16]) {
                const char* b_base = smem + stage * STAGE + (TNF ? 2 * 1024 : HALF);
#pragma unroll
                for (int j = 0; j < TN16; ++j) {
                    if constexpr (TNF) fb[j] = read_tr(b_base, wn * TN16 + j);
                    else fb[j] = *reinterpret_cast<const bf16x8_t*>(b_base + off64(wn * (TN * 32) + j * 16 + frag_row, ks * 4 + frag_grp));
                }
            };
            // One half step: HA x TN16 MFMAs on row units h*HA.., with transfers [s0, s0 + cnt) of K tile `tile` handed
            // out evenly between them.  Operands swapped on purpose: the accumulator block is C^T (rows = n, columns =
            // m), so a lane holds 4 CONSECUTIVE n per block and the epilogue stages with 16-byte writes.
            auto mma_dma = [&](int h, const bf16x8_t (&fa)[HA], const bf16x8_t (&fb)[TN16], int tile, int stage, int s0, int cnt) {
                int done = 0;
#pragma unroll
                for (int i = 0; i < HA; ++i)
#pragma unroll
                    for (int jj = 0; jj < TN16; ++jj) {
                        // boustrophedon order: consecutive MFMAs share one operand and the other changes to its neighbour
                        // (measured: about 2 % more sustained MFMA rate at the power limit than row-major order)
                        const int j = (i & 1) ? TN16 - 1 - jj : jj;
                        const int q = i * TN16 + jj;
#ifdef X_QPOS
                        if (done < cnt && q == (2 * done + 1) * (HA * TN16) / (2 * cnt)) {
#else
                        if (done < cnt && q == done * (HA * TN16) / cnt) {
#endif
                            __builtin_amdgcn_sched_barrier(0);
                            issue_one(tile, stage, s0 + done);
                            __builtin_amdgcn_sched_barrier(0);
                            ++done;
                        }
                        acc[h * HA + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[h * HA + i][j], 0, 0, 0);
                    }
            };
            // Software pipeline: the fragments of the next half step are read from LDS while the MFMAs of the current
            // one run, ACROSS the tile boundary too, so that no wavefront waits on LDS latency right after the barrier
            // (all 8 wavefronts leave it together, so nobody would be left to cover for the others).
            bf16x8_t fax[HA], fay[HA], fbx[TN16], fby[TN16];
            // transfers per K tile and wavefront: NVM instructions, handed out in NTR groups (TN: one, NT: A part, B part)
            constexpr int NVM = 2 * LPW, NTR = TNF ? 1 : 2;
            if constexpr (TNF) {
                // one 32-deep k step per tile, two half steps; the transfers of tile tl+3 go out in the first one, before the
                // barrier of iteration tl
                issue(t_begin, 0);
                issue(t_begin + 1, 1);
                issue(t_begin + 2, 2);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * NVM));         // tile t_begin: at most the two newest tiles outstanding
                __builtin_amdgcn_s_barrier();
                load_b(0, 0, fbx);
                load_a(0, 0, 0, fax);
                auto tn_iter = [&](int tl, bf16x8_t (&fb_cur)[TN16], bf16x8_t (&fb_next)[TN16]) {
                    const int st_ = (tl - t_begin) & (NS - 1);
                    // stage (tl-1)%4 is free: every wavefront finished reading it before the barrier it has passed last
                    load_a(st_, 0, 1, fay);
                    __builtin_amdgcn_sched_barrier(0);
                    mma_dma(0, fax, fb_cur, tl + 3, (st_ + 3) & (NS - 1), 0, 1);
                    __builtin_amdgcn_sched_barrier(0);
                    // tile tl+1: this wavefront's part has landed (tile tl+2 and the new transfers outstanding), its LDS
                    // reads are done ...
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * NVM) & 0xF0FF);        // vmcnt(2 NVM) lgkmcnt(0)
                    __builtin_amdgcn_s_barrier();                       // ... and everyone's
                    load_b((st_ + 1) & (NS - 1), 0, fb_next);           // past the last tile: a stale but valid stage, unused
                    load_a((st_ + 1) & (NS - 1), 0, 0, fax);
                    __builtin_amdgcn_sched_barrier(0);
                    mma_dma(1, fay, fb_cur, tl + 3, (st_ + 3) & (NS - 1), 1, 0);
                    __builtin_amdgcn_sched_barrier(0);
                };
                int tl = t_begin;
                for (; tl + 1 < t_end; tl += 2) {
                    tn_iter(tl, fbx, fby);
                    tn_iter(tl + 1, fby, fbx);
                }
                if (tl < t_end) tn_iter(tl, fbx, fby);
            } else {
                // two 64 KB stages, two 32-deep k steps = four half steps per tile, one barrier per tile.  Transfers of
                // tile tl+1 ride on the four half steps between two barriers: NT_G0 on the one right after the barrier
                // (the last half step of tile tl-1), then NT_G1, NT_G2, the rest
                static_assert(NT_G0 + NT_G1 + NT_G2 <= NTR, "more transfers scheduled than a tile has");
                if (!primed) issue(t_begin, 0);
                if constexpr (PS) {
                    // the tile after this one: drawn now, needed after the main loop (first tiles of a run: one per work-group)
                    if (persistent && t == 0)
                        next_local = (ps_wgs >> 3) + __hip_atomic_fetch_add(ps_ctr + (blockIdx.x & 7), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                __builtin_amdgcn_s_waitcnt(0x0F70);                     // vmcnt(0) (persistent: the previous tile's stores too)
                __builtin_amdgcn_s_barrier();
#pragma unroll
                for (int s_ = 0; s_ < NT_G0; ++s_) issue_one(t_begin + 1, 1, s_);
                load_b(0, 0, fbx);
                load_a(0, 0, 0, fax);
                for (int tl = t_begin; tl < t_end; ++tl) {
                    const int st_ = (tl - t_begin) & 1;
                    load_a(st_, 0, 1, fay);
                    __builtin_amdgcn_sched_barrier(0);
                    mma_dma(0, fax, fbx, tl + 1, st_ ^ 1, NT_G0, NT_G1);
                    __builtin_amdgcn_sched_barrier(0);
                    load_b(st_, 1, fby);
                    load_a(st_, 1, 0, fax);
                    __builtin_amdgcn_sched_barrier(0);
                    mma_dma(1, fay, fbx, tl + 1, st_ ^ 1, NT_G0 + NT_G1, NT_G2);
                    __builtin_amdgcn_sched_barrier(0);
                    load_a(st_, 1, 1, fay);
                    __builtin_amdgcn_sched_barrier(0);
                    mma_dma(0, fax, fby, tl + 1, st_ ^ 1, NT_G0 + NT_G1 + NT_G2, NTR - NT_G0 - NT_G1 - NT_G2);
                    __builtin_amdgcn_sched_barrier(0);
                    __builtin_amdgcn_s_waitcnt(0x0070);                 // vmcnt(0) lgkmcnt(0): tile tl+1 landed, reads of tile tl done
                    __builtin_amdgcn_s_barrier();
                    // this stage is free from here on: tile tl+2 starts to arrive in it
                    load_b(st_ ^ 1, 0, fbx);                            // past the last tile: a reloaded copy of it, unused
                    load_a(st_ ^ 1, 0, 0, fax);
                    __builtin_amdgcn_sched_barrier(0);
                    mma_dma(1, fay, fby, tl + 2, st_, 0, NT_G0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // drain the redundant tail transfers before LDS is reused by the epilogue (explicit: the compiler does not
            // see transfers issued by lds_dma16)
            __builtin_amdgcn_s_waitcnt(0x0070);     // vmcnt(0) lgkmcnt(0)
            if constexpr (PS) {
                if (persistent && t == 0) *reinterpret_cast<volatile int*>(smem + PS_SLOT) = next_local;
            }
            __builtin_amdgcn_s_barrier();
        }
        int next_logical = -1;
        if constexpr (PS) {
            if (persistent) {
                const int nl = __builtin_amdgcn_readfirstlane(*reinterpret_cast<volatile int*>(smem + PS_SLOT));
                if (nl < run_cnt) {
                    // the next tile's first K tile goes out before this tile's epilogue: stage 0 is free, the staging block
                    // lies above it
                    next_logical = run_start + nl;
                    set_tile(next_logical);
                    const uint32_t lds0 = lds_address(smem);
                    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
#pragma unroll
                    for (int s_ = 0; s_ < 2; ++s_) {
                        const uint32_t dst_g = lds0 + (s_ ? HALF : 0) + wave_u * (LPW * 1024);
                        if (s_) lds_dma16_group<LPW>(dma_group_base<LPW>(pb + t_begin * (long long)(DK * 2)), offBg, dst_g);
                        else lds_dma16_group<LPW>(dma_group_base<LPW>(pa + t_begin * (long long)(DK * 2)), offAg, dst_g);
                    }
                    primed = true;
                }
            }
        }

        auto epilogue = [&]() {
        // ---- epilogue through LDS: per wavefront a [32][STG_LD] fp32 staging block
        float* stage = reinterpret_cast<float*>(smem + STG_OFF) + wave * (32 * STG_LD);
        constexpr int LPR = TN * 4;                    // lanes per staged row (8 columns each)
        const int rd_row = lane / LPR, rd_col = (lane % LPR) * 8;
        constexpr int NPSS = 32 / (64 / LPR);          // staged rows each lane finishes per pass
        const bool direct = !tail && splits == 1;      // this work-group applies the epilogue itself
        // what the epilogue reads from memory, for every row this lane will finish: all in flight before the first pass
        // (one pass ahead only for the two-operand gated form, which would not fit in registers otherwise)
        constexpr bool PRE_ALL = EPI != DS_EPI_DGATE;
        EpiPre<bf16_t> pre[TM][NPSS];
        auto prefetch_pass = [&](int i) {
#pragma unroll
            for (int pss = 0; pss < NPSS; ++pss) {
                const int m = em0 + wm * (TM * 32) + i * 32 + pss * (64 / LPR) + rd_row;
                if (m < M) epilogue_prefetch<bf16_t, EPI>(m, en0 + wn * (TN * 32) + rd_col, N, p, pre[i][pss]);
            }
        };
        if (epilogue_reads<EPI>() && direct && PRE_ALL) {
#pragma unroll
            for (int i = 0; i < TM; ++i) prefetch_pass(i);
        }
        if constexpr (EPI == DS_EPI_NONE) {
            // Plain output (+ bias): nothing is computed after the transposition, so the bias is added and the value
            // rounded to bf16 BEFORE staging: half the LDS traffic of the fp32 staging below, which bounds the epilogue.
            if (direct) {
                bf16_t* stage_h = reinterpret_cast<bf16_t*>(stage);
                constexpr int LD_H = TN * 32 + 8;                       // bf16 row stride (144 bytes: 8-byte writes of 16 rows spread over the banks)
                float bias4[TN16][4];
#pragma unroll
                for (int j = 0; j < TN16; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        bias4[j][e] = p.bias ? (float)reinterpret_cast<const bf16_t*>(p.bias)[en0 + wn * (TN * 32) + j * 16 + 4 * (lane >> 4) + e] : 0.f;
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    wave_lds_sync();
#pragma unroll
                    for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                        for (int j = 0; j < TN16; ++j) {
                            typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
                            const f32x4_t a4 = acc[2 * i + i2][j];
                            const bf16x4_t h4 = {(bf16_t)(a4[0] + bias4[j][0]), (bf16_t)(a4[1] + bias4[j][1]),
                                                 (bf16_t)(a4[2] + bias4[j][2]), (bf16_t)(a4[3] + bias4[j][3])};
                            *reinterpret_cast<bf16x4_t*>(stage_h + (i2 * 16 + (lane & 15)) * LD_H + j * 16 + 4 * (lane >> 4)) = h4;
                        }
                    wave_lds_sync();
#pragma unroll
                    for (int pss = 0; pss < NPSS; ++pss) {
                        const int row = pss * (64 / LPR) + rd_row;
                        const int m = em0 + wm * (TM * 32) + i * 32 + row;
                        const int n = en0 + wn * (TN * 32) + rd_col;
                        if (m < M) {
                            const bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(stage_h + row * LD_H + rd_col);
                            __builtin_nontemporal_store(v, reinterpret_cast<bf16x8_t*>(C + (size_t)m * N + n));
                        }
                    }
                }
                return;
            }
        }
        // column sums of what this lane writes (DGELU: the bias gradient of the layer below comes out of this kernel
        // instead of a pass over the stored tensor); every lane finishes TM * NPSS rows of the same 8 columns
        float csum[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) csum[j] = 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            if (epilogue_reads<EPI>() && direct && !PRE_ALL) prefetch_pass(i);
            wave_lds_sync();            // the staging block is private to the wavefront: no work-group barrier (which would
                                        // also wait for the global stores of the previous pass to be acknowledged)
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                for (int j = 0; j < TN16; ++j) {    // lane = row m (lane%16 of block 2i+i2); its 4 registers = columns 4*(lane/16) + 0..3
                    const f32x4_t a4 = acc[2 * i + i2][j];
                    *reinterpret_cast<float4*>(stage + (i2 * 16 + (lane & 15)) * STG_LD + j * 16 + 4 * (lane >> 4)) =
                        make_float4(a4[0], a4[1], a4[2], a4[3]);
                }
            wave_lds_sync();
#pragma unroll
            for (int pss = 0; pss < NPSS; ++pss) {
                const int row = pss * (64 / LPR) + rd_row;
                const int m = em0 + wm * (TM * 32) + i * 32 + row;
                const int n = en0 + wn * (TN * 32) + rd_col;
                if (m < M) {
                    float v[8];
                    const float4 x0 = *reinterpret_cast<const float4*>(stage + row * STG_LD + rd_col);
                    const float4 x1 = *reinterpret_cast<const float4*>(stage + row * STG_LD + rd_col + 4);
                    v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w; v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
                    if (tail) {
                        Vec8<float>::store(split_ws + ((size_t)((elogical - n_main) * tail_splits + split) * BM + (m - em0)) * BN + (n - en0), v);
                    } else if (splits > 1) {
                        Vec8<float>::store(split_ws + ((size_t)split * M + m) * N + n, v);
                    } else if (epilogue_reads<EPI>()) {
                        epilogue8<bf16_t, EPI>(m, n, N, v, C, p, &pre[i][pss]);
                        if constexpr (EPI == DS_EPI_DGELU || EPI == DS_EPI_MULR) {
#pragma unroll
                            for (int j = 0; j < 8; ++j) csum[j] += v[j];
                        }
                    } else {
                        epilogue8<bf16_t, EPI>(m, n, N, v, C, p);
                    }
                }
            }
        }
        if constexpr (EPI == DS_EPI_DGELU || EPI == DS_EPI_MULR) {
            if (direct && p.colsum) {
                // lanes l, l + LPR, l + 2 LPR, ... hold the same columns: fold them, then one row of partial sums per
                // (tile row, wavefront row), written whether or not the wavefront had a valid row
#pragma unroll
                for (int o = LPR; o < 64; o <<= 1)
#pragma unroll
                    for (int j = 0; j < 8; ++j) csum[j] += __shfl_xor(csum[j], o, 64);
                if (lane < LPR)
                    Vec8<float>::store(p.colsum + (size_t)(etile_m * WM + wm) * N + en0 + wn * (TN * 32) + rd_col, csum);
            }
        }
        };
        epilogue();
        if (next_logical < 0) break;
        logical = next_logical;
    }   // for (;;): persistent work-groups go on with their next tile
    if constexpr (PS) {
        if (persistent && t == 0) {
            // every persistent work-group ends with a draw beyond its run; the last one to finish clears the counters
            const int done = __hip_atomic_fetch_add(ps_ctr + 8, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (done == ps_wgs - 1) {
#pragma unroll
                for (int i = 0; i < 9; ++i) ps_ctr[i] = 0;
            }
        }
    }
}

// sum the tail tiles' split-K partials ([tile][split][256][256]) and apply the epilogue; one thread per 8 columns
template <int EPI>
__global__ __launch_bounds__(256) void tail_finish_kernel(int M, int N, int tiles_m, int tiles_n, int n_main, int tail_splits,
                                                          const float* __restrict__ ws, bf16_t* __restrict__ C, GemmEpi p) {
    const int tile = blockIdx.y;
    int tile_m, tile_n;
    nt_tile_coords(n_main + tile, tiles_m, tiles_n, tile_m, tile_n);
    const float* base = ws + (size_t)tile * tail_splits * (BM * BN);
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < BM * (BN / 8); i += gridDim.x * blockDim.x) {
        const int r = i / (BN / 8), c8 = (i % (BN / 8)) * 8;
        const int m = tile_m * BM + r, n = tile_n * BN + c8;
        if (m >= M) continue;
        float v[8];
        Vec8<float>::load(base + (size_t)r * BN + c8, v);
        for (int sp = 1; sp < tail_splits; ++sp) {
            float w[8];
            Vec8<float>::load(base + ((size_t)sp * BM + r) * BN + c8, w);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] += w[j];
        }
        epilogue8<bf16_t, EPI>(m, n, N, v, C, p);
    }
}

// The same with the column sums of the output (p.colsum): one block of 1024 threads per 128-row half of a tile, which
// writes the row of p.colsum the main kernel's work-groups would have written had they finished the tile themselves.
template <int EPI>
__global__ __launch_bounds__(1024) void tail_finish_sums_kernel(int M, int N, int tiles_m, int tiles_n, int n_main, int tail_splits,
                                                                const float* __restrict__ ws, bf16_t* __restrict__ C, GemmEpi p) {
    __shared__ float red[32][BN];
    const int tile = blockIdx.y;
    int tile_m, tile_n;
    nt_tile_coords(n_main + tile, tiles_m, tiles_n, tile_m, tile_n);
    const float* base = ws + (size_t)tile * tail_splits * (BM * BN);
    const int c8 = (threadIdx.x & 31) * 8, n = tile_n * BN + c8;
    float csum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) csum[j] = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {                   // 4 x 32 rows; independent iterations, their loads in flight together
        const int r = blockIdx.x * 128 + k * 32 + (threadIdx.x >> 5);
        const int m = tile_m * BM + r;
        if (m >= M) continue;
        float v[8];
        Vec8<float>::load(base + (size_t)r * BN + c8, v);
        for (int sp = 1; sp < tail_splits; ++sp) {
            float w[8];
            Vec8<float>::load(base + ((size_t)sp * BM + r) * BN + c8, w);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] += w[j];
        }
        epilogue8<bf16_t, EPI>(m, n, N, v, C, p);
#pragma unroll
        for (int j = 0; j < 8; ++j) csum[j] += v[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[threadIdx.x >> 5][c8 + j] = csum[j];
    __syncthreads();
    if (threadIdx.x < BN) {
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 32; ++k) t += red[k][threadIdx.x];
        p.colsum[(size_t)(tile_m * 2 + blockIdx.x) * N + tile_n * BN + threadIdx.x] = t;
    }
}

// sum the split-K partials and apply the epilogue; one thread per 8 columns
template <int EPI>
__global__ __launch_bounds__(256) void splitk_finish_kernel(int M, int N, int splits, const float* __restrict__ ws,
                                                            bf16_t* __restrict__ C, GemmEpi p) {
    const long long total = (long long)M * (N / 8);
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const int m = (int)(i / (N / 8));
        const int n = (int)(i - (long long)m * (N / 8)) * 8;
        float v[8];
        Vec8<float>::load(ws + (size_t)m * N + n, v);
        for (int s = 1; s < splits; ++s) {
            float w[8];
            Vec8<float>::load(ws + ((size_t)s * M + m) * N + n, w);
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] += w[j];
        }
        epilogue8<bf16_t, EPI>(m, n, N, v, C, p);
    }
}

template <class T, int EPI>
ds_status launch_generic(int ta, int tb, int M, int N, int K, const void* A, const void* B, void* C, const GemmEpi& p,
                         hipStream_t st) {
    const long long sam = ta ? 1 : K, sak = ta ? M : 1;
    const long long sbk = tb ? 1 : N, sbn = tb ? K : 1;
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL((gemm_generic_kernel<T, EPI>), grid, dim3(256), 0, st, M, N, K, (const T*)A, sam, sak, (const T*)B,
                       sbk, sbn, (T*)C, p);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

// number of K splits of a weight-gradient GEMM: the fewest that bring the work-group count closest to a whole
// number of rounds over the compute units (time ~ rounds x split length)
static int cu_count() {
    static int n_cu = 0;
    if (n_cu == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        n_cu = v;
    }
    return n_cu;
}
static int choose_splits(int tiles, int nt, int M, int N, size_t split_ws_floats) {
    const int n_cu = cu_count();
    int best = 1;
    double best_cost = 1e30;
    for (int sp = 1; sp <= 16; ++sp) {
        if (sp > 1 && (sp > nt / 16 || (size_t)sp * M * N > split_ws_floats)) break;
        const int per = (nt + sp - 1) / sp;
        if ((nt + per - 1) / per != sp) continue;               // every split must own at least one K tile
        const double rounds = (double)(((long long)tiles * sp + n_cu - 1) / n_cu);
        const double cost = rounds * per * (1.0 + 0.01 * sp);    // slight preference for fewer partial sums
        if (cost < best_cost - 1e-9) { best_cost = cost; best = sp; }
    }
    return best;
}

// Tile counters of the persistent form: 64 slots of [8 per-XCD counters, 1 count of finished work-groups], all zero
// between launches (the last work-group of a launch clears its slot).  Launches take the slots in turn, so two
// launches can only share one if more than 64 are in flight on a device at the same time.
constexpr int PS_SLOTS = 64;
__device__ int g_ps_ctr[PS_SLOTS][16];
constexpr bool NT_PERSISTENT = true;
static int* ps_counters() {
    static std::mutex mu;
    static int* base[64] = {};
    static std::atomic<unsigned> next{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (!base[dev]) {
            void* ptr = nullptr;
            if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_ps_ctr)) != hipSuccess) return nullptr;
            base[dev] = static_cast<int*>(ptr);
        }
    }
    return base[dev] + 16 * (next.fetch_add(1) % PS_SLOTS);
}

template <int EPI, bool TNF>
ds_status launch_nt(int M, int N, int K, const void* A, const void* B, void* C, const GemmEpi& p, float* split_ws,
                    size_t split_ws_floats, hipStream_t st) {
    static bool attr_set = false;
    constexpr int WM = NT_WM, WN = NT_WN;
    auto kern = gemm_bf16_nt_kernel<EPI, WM, WN, TNF, false>;
    constexpr int stg = WM * WN * 32 * ((256 / WN) + 4) * 4;
    const int smem = NT_NS * NT_STAGE > stg ? NT_NS * NT_STAGE : stg;
    if (!attr_set) {
        DS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, smem));
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const int nt = TNF ? (K + NT_DK - 1) / NT_DK : K / 64;      // K tiles as the kernel counts them
    const int tiles = tiles_m * tiles_n;
    int splits = 1;
    if (EPI == DS_EPI_ACC32 && split_ws) splits = choose_splits(tiles, nt, M, N, split_ws_floats);
    // tail split-K: the tiles beyond the last whole round over the compute units share that round; a launch with
    // fewer tiles than compute units (small micro-batches) is all tail, so that the K loop is spread over the chip
    int n_main = tiles, tail_splits = 1;
    if (splits == 1 && split_ws) {
        const int n_cu = cu_count();
        const int rem = tiles % n_cu;
        if (rem > 0) {
            int ts = n_cu / rem;
            if (ts > 32) ts = 32;
            if (ts > nt / 4) ts = nt / 4;
            while (ts > 1 && (size_t)rem * ts * (BM * BN) > split_ws_floats) --ts;
            if (ts > 1) {
                const int per = (nt + ts - 1) / ts;
                ts = (nt + per - 1) / per;                      // every split owns at least one K tile
            }
            if (ts > 1) { n_main = tiles - rem; tail_splits = ts; }
        }
    }
    const int total = splits > 1 ? tiles * splits : n_main + (tiles - n_main) * tail_splits;
    bool launched = false;
    if constexpr (!TNF && NT_PERSISTENT) {
        // persistent form: one resident work-group per compute unit for the unsplit tiles, when each has several to do
        const int n_cu = cu_count();
        if (splits == 1 && n_cu % 8 == 0 && n_main >= 2 * n_cu) {
            static bool ps_attr_set = false;
            auto kern_ps = gemm_bf16_nt_kernel<EPI, WM, WN, false, true>;
            constexpr int smem_ps = 65536 + stg + 64;              // stage 0 | epilogue staging | hand-over word
            static_assert(smem_ps >= NT_NS * NT_STAGE && smem_ps <= 160 * 1024, "LDS of the persistent form");
            if (!ps_attr_set) {
                DS_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern_ps), hipFuncAttributeMaxDynamicSharedMemorySize, smem_ps));
                ps_attr_set = true;
            }
            int* ctr = ps_counters();
            if (ctr) {
                hipLaunchKernelGGL(kern_ps, dim3(n_cu + (tiles - n_main) * tail_splits), dim3(WM * WN * 64), smem_ps, st, M, N, K,
                                   (const bf16_t*)A, (const bf16_t*)B, (bf16_t*)C, tiles_m, tiles_n, splits, n_main, tail_splits,
                                   split_ws, p, n_cu, ctr);
                launched = true;
            }
        }
    }
    if (!launched)
        hipLaunchKernelGGL(kern, dim3(total), dim3(WM * WN * 64), smem, st, M, N, K, (const bf16_t*)A, (const bf16_t*)B, (bf16_t*)C,
                           tiles_m, tiles_n, splits, n_main, tail_splits, split_ws, p, 0, (int*)nullptr);
    DS_LAUNCH_CHECK();
    if (splits > 1) {
        long long items = (long long)M * (N / 8);
        long long g = (items + 255) / 256;
        if (g > 8192) g = 8192;
        hipLaunchKernelGGL(splitk_finish_kernel<EPI>, dim3((int)g), dim3(256), 0, st, M, N, splits, split_ws, (bf16_t*)C, p);
        DS_LAUNCH_CHECK();
    } else if (tail_splits > 1) {
        bool with_sums = false;
        if constexpr (EPI == DS_EPI_DGELU || EPI == DS_EPI_MULR) {
            if (p.colsum) {
                with_sums = true;
                hipLaunchKernelGGL(tail_finish_sums_kernel<EPI>, dim3(2, tiles - n_main), dim3(1024), 0, st, M, N, tiles_m, tiles_n,
                                   n_main, tail_splits, split_ws, (bf16_t*)C, p);
            }
        }
        if (!with_sums)
            hipLaunchKernelGGL(tail_finish_kernel<EPI>, dim3(8, tiles - n_main), dim3(256), 0, st, M, N, tiles_m, tiles_n,
                               n_main, tail_splits, split_ws, (bf16_t*)C, p);
        DS_LAUNCH_CHECK();
    }
    return DS_OK;
}

template <int EPI>
ds_status dispatch_epi(int dtype, int ta, int tb, int M, int N, int K, const void* A, const void* B, void* C,
                       const GemmEpi& p, bool force_generic, float* split_ws, size_t split_ws_floats, hipStream_t st) {
    if (dtype == DS_DTYPE_BF16 && !force_generic) {
        const bool ok_n = N % BN == 0;
        const bool ok_a = ta ? (M % BM == 0) : (K % BK == 0);
        const bool ok_b = tb ? (K % BK == 0) : true;
        const bool aligned = ((uintptr_t)A % 16 == 0) && ((uintptr_t)B % 16 == 0) && ((uintptr_t)C % 16 == 0);
        if (ok_n && ok_a && ok_b && aligned && M >= 1 && K >= 1) {
            if (!ta && tb) return launch_nt<EPI, false>(M, N, K, A, B, C, p, split_ws, split_ws_floats, st);
            if constexpr (EPI == DS_EPI_ACC32)      // (the TN form addresses a K tile of each operand through a 32-bit buffer length)
                if (ta && !tb && M <= (1 << 25) && N <= (1 << 25)) return launch_nt<EPI, true>(M, N, K, A, B, C, p, split_ws, split_ws_floats, st);
        }
    }
    if (dtype == DS_DTYPE_BF16) return launch_generic<bf16_t, EPI>(ta, tb, M, N, K, A, B, C, p, st);
    return launch_generic<float, EPI>(ta, tb, M, N, K, A, B, C, p, st);
}

}  // namespace

bool gemm_colsum_fused(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K, const void* A, const void* B,
                       const void* C, int32_t epilogue) {
    // the conditions under which dispatch_epi takes launch_nt<DS_EPI_DGELU or DS_EPI_MULR, false>
    static_assert(NT_WM == 2, "two rows of partial column sums per tile row");
    if ((epilogue != DS_EPI_DGELU && epilogue != DS_EPI_MULR) || dtype != DS_DTYPE_BF16 || ta || !tb) return false;
    if (N % BN || K % BK || M < 1 || K < 1) return false;
    return ((uintptr_t)A % 16 == 0) && ((uintptr_t)B % 16 == 0) && ((uintptr_t)C % 16 == 0);
}

// Shared with the stage driver.
ds_status launch_gemm(int32_t dtype, int32_t ta, int32_t tb, int32_t M, int32_t N, int32_t K, const void* A, const void* B,
                      void* C, int32_t epilogue, const GemmEpi& p, bool force_generic, float* split_ws,
                      size_t split_ws_floats, hipStream_t st) {
    if (M <= 0 || N <= 0 || K <= 0 || !A || !B || !C) return DS_EINVAL;
    if (N % 8) return DS_EINVAL;
    if (dtype != DS_DTYPE_F32 && dtype != DS_DTYPE_BF16) return DS_EINVAL;
    switch (epilogue) {
    case DS_EPI_NONE: return dispatch_epi<DS_EPI_NONE>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_GELU:
        if (!p.C2) return DS_EINVAL;
        return dispatch_epi<DS_EPI_GELU>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_RESID:
        if (!p.R) return DS_EINVAL;
        return dispatch_epi<DS_EPI_RESID>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_GELU_D:
        if (!p.C2) return DS_EINVAL;
        return dispatch_epi<DS_EPI_GELU_D>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_MULR:
        if (!p.R) return DS_EINVAL;
        return dispatch_epi<DS_EPI_MULR>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_DGELU:
        if (!p.R) return DS_EINVAL;
        return dispatch_epi<DS_EPI_DGELU>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_ACC32: return dispatch_epi<DS_EPI_ACC32>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_GATE:
        if (!p.R || !p.C2) return DS_EINVAL;
        return dispatch_epi<DS_EPI_GATE>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    case DS_EPI_DGATE:
        if (!p.R || !p.R2 || !p.C2) return DS_EINVAL;
        return dispatch_epi<DS_EPI_DGATE>(dtype, ta, tb, M, N, K, A, B, C, p, force_generic, split_ws, split_ws_floats, st);
    }
    return DS_EINVAL;
}

extern "C" ds_status ds_gemm(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                             const void* A, const void* B, void* C, int32_t epilogue, const void* bias, const void* R,
                             const void* R2, void* C2, const int32_t* row_valid, int32_t accumulate,
                             int32_t force_generic, void* hip_stream) {
    GemmEpi p{bias, R, R2, C2, row_valid, accumulate};
    return launch_gemm(dtype, trans_a, trans_b, M, N, K, A, B, C, epilogue, p, force_generic != 0, nullptr, 0,
                       (hipStream_t)hip_stream);
}

extern "C" ds_status ds_gemm_ws(int32_t dtype, int32_t trans_a, int32_t trans_b, int32_t M, int32_t N, int32_t K,
                                const void* A, const void* B, void* C, int32_t epilogue, const void* bias, const void* R,
                                const void* R2, void* C2, const int32_t* row_valid, int32_t accumulate,
                                int32_t force_generic, float* workspace, int64_t workspace_floats, void* hip_stream) {
    if (workspace_floats < 0 || (workspace_floats > 0 && (!workspace || ((uintptr_t)workspace & 15)))) return DS_EINVAL;
    GemmEpi p{bias, R, R2, C2, row_valid, accumulate};
    return launch_gemm(dtype, trans_a, trans_b, M, N, K, A, B, C, epilogue, p, force_generic != 0,
                       workspace_floats > 0 ? workspace : nullptr, (size_t)workspace_floats, (hipStream_t)hip_stream);
}
