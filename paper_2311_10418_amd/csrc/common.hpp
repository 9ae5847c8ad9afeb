// Shared device/host helpers for the HIP translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include "../../include/dynastage.h"

typedef __bf16 bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

#define DS_HIP_CHECK(expr)                         \
    do {                                           \
        hipError_t e__ = (expr);                   \
        if (e__ != hipSuccess) return DS_EHIP;     \
    } while (0)

#define DS_LAUNCH_CHECK()                          \
    do {                                           \
        if (hipGetLastError() != hipSuccess) return DS_EHIP; \
    } while (0)

constexpr float kLnEps = 1e-5f;
constexpr float kRmsEps = 1e-6f;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

// 8 consecutive elements <-> 8 floats
template <class T> struct Vec8;
template <> struct Vec8<float> {
    static __device__ __forceinline__ void load(const float* p, float (&v)[8]) {
        const float4 a = *reinterpret_cast<const float4*>(p);
        const float4 b = *reinterpret_cast<const float4*>(p + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
    static __device__ __forceinline__ void store(float* p, const float (&v)[8]) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    // streaming store: the line is not kept in L2 (outputs far larger than the cache would only evict operands
    // that other work-groups are about to read again)
    static __device__ __forceinline__ void store_nt(float* p, const float (&v)[8]) {
        const f32x4_t a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
        __builtin_nontemporal_store(a, reinterpret_cast<f32x4_t*>(p));
        __builtin_nontemporal_store(b, reinterpret_cast<f32x4_t*>(p + 4));
    }
};
template <> struct Vec8<bf16_t> {
    static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
        const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(p);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
    }
    static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
        bf16x8_t a;
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = (bf16_t)v[i];
        *reinterpret_cast<bf16x8_t*>(p) = a;
    }
    static __device__ __forceinline__ void store_nt(bf16_t* p, const float (&v)[8]) {
        bf16x8_t a;
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = (bf16_t)v[i];
        __builtin_nontemporal_store(a, reinterpret_cast<bf16x8_t*>(p));
    }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
    return v;
}

// tanh-form GELU and its derivative (fp32), written through the logistic function: with u = c (z + a z^3),
// 0.5 (1 + tanh u) = s := 1 / (1 + e^(-2u)), so GELU(z) = z s and GELU'(z) = s (1 + z (1 - s) 2 u'), u' = c (1 + 3 a z^2).
// One hardware exp2 and one reciprocal per value (quarter-rate instructions) and 5 resp. 9 ordinary ones: these
// run in GEMM epilogues on every output element, where the matrix cores wait for the vector ALU.  Relative error
// ~1e-6, far inside the bf16 and fp32 bars.  e^(-2u) = +inf / 0 at the extremes give s = 0 / 1, as they should.
__device__ __forceinline__ float gelu_sigmoid(float z, float w) {      // w = z * z
    constexpr float k1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;          // -2 c log2(e)
    constexpr float k2 = k1 * 0.044715f;
    const float e = __builtin_amdgcn_exp2f(z * __builtin_fmaf(k2, w, k1));           // e^(-2u)
    return __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ float gelu_f(float z) { return z * gelu_sigmoid(z, z * z); }
__device__ __forceinline__ void gelu_and_grad_f(float z, float& gelu, float& grad) {   // both from one logistic term
    constexpr float c2 = 2.0f * 0.7978845608028654f, c6a = 3.0f * 0.044715f * c2;
    const float w = z * z;
    const float s = gelu_sigmoid(z, w);
    gelu = z * s;
    grad = s * __builtin_fmaf(z * __builtin_fmaf(c6a, w, c2), 1.0f - s, 1.0f);
}
__device__ __forceinline__ float gelu_grad_f(float z) {
    constexpr float c2 = 2.0f * 0.7978845608028654f, c6a = 3.0f * 0.044715f * c2;
    const float w = z * z;
    const float s = gelu_sigmoid(z, w);
    const float zdu = z * __builtin_fmaf(c6a, w, c2);                                // z * 2 u'
    return s * __builtin_fmaf(zdu, 1.0f - s, 1.0f);
}

// One direct global -> LDS transfer, 16 bytes per lane (global_load_lds_dwordx4): the wavefront's 64 chunks land at
// lds_addr + 16 * lane.  lds_addr must be wavefront-uniform.  Issued through inline assembly on purpose: the
// compiler orders every later LDS read it cannot disambiguate (all transpose reads) behind a FULL vector-memory
// wait when it sees such a transfer in flight, which would serialise the prefetch pipelines built on it.  Every
// consumer here synchronises explicitly instead (s_waitcnt vmcnt(n) for its own transfers, then s_barrier).
// Compiler-generated vmcnt waits for ordinary loads stay correct: unseen transfers only make them wait longer.
__device__ __forceinline__ void lds_dma16(const void* gptr, const void* lds_ptr) {
    const uint32_t lds_addr =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_ptr);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_addr) : "memory", "m0");
}

// Orders the LDS writes of a wavefront's lanes before later LDS reads by other lanes of the SAME wavefront.  LDS
// operations of one wavefront execute in order, so no instruction is needed: this only stops the compiler from
// moving accesses across the point.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// s_waitcnt immediate "at most n vector-memory operations outstanding" (gfx9 encoding: vmcnt in bits 3:0 and 15:14,
// expcnt 6:4 and lgkmcnt 11:8 left at their maxima, i.e. not waited for)
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }

// The same transfer addressed as a wavefront-uniform base (scalar registers) plus a 32-bit byte offset per lane:
// the per-lane part can then stay fixed over a whole K loop, and stepping to the next tile is scalar arithmetic.
__device__ __forceinline__ void lds_dma16_s(const void* base, uint32_t lane_off, const void* lds_ptr) {
    const uint32_t lds_addr =
        __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_ptr);
    const uint64_t b = (uint64_t)(uintptr_t)base;
    // (the builtin returns a signed int: without the casts the low half would be sign-extended over the high half)
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const uint64_t sb = ((uint64_t)hi << 32) | (uint64_t)lo;
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 : : "v"(lane_off), "s"(sb), "s"(lds_addr) : "memory", "m0");
}

// LDS byte address of a pointer into shared memory, as the integer that M0 and the LDS instructions use.  Taken once
// per kernel: stage and tile addresses are then scalar integer arithmetic (a generic pointer converted per transfer
// costs a null check, a 64-bit vector add and two lane reads each time).
__device__ __forceinline__ uint32_t lds_address(const void* lds_ptr) {
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)lds_ptr);
}

// lds_dma16 with the destination given as an LDS address (see lds_address) instead of a generic pointer.
__device__ __forceinline__ void lds_dma16_at(const void* gptr, uint32_t lds_addr) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(m0v) : "memory", "m0");
}

// N (1..4) direct transfers of 64 x 16 bytes each that share ONE value of M0: transfer i lands at lds_addr + 1024 i
// and reads base + lane_off[i] (base wavefront-uniform).  The LDS destination of a transfer is M0 + the instruction's
// immediate offset + 16 * lane, and the immediate is added to the global address as well, so the caller passes lane
// offsets that are already reduced by 1024 i (see dma_lane_offset).  Why one M0: a transfer reads M0 when it is
// executed, so every write of M0 waits until the transfer before it has passed the address stage; with one write per
// transfer a wavefront spent about 75 cycles per transfer unable to issue anything else.
template <int N>
__device__ __forceinline__ void lds_dma16_group(const void* base, const uint32_t (&lane_off)[N], uint32_t lds_addr) {
    static_assert(N >= 1 && N <= 4, "the immediate offset reaches 3 x 1024");
    const uint64_t b = (uint64_t)(uintptr_t)base;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    const uint64_t sb = ((uint64_t)hi << 32) | (uint64_t)lo;
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_addr);
    if constexpr (N == 1)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     : : "v"(lane_off[0]), "s"(sb), "s"(m0v) : "memory", "m0");
    else if constexpr (N == 2)
        asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:1024"
                     : : "v"(lane_off[0]), "v"(lane_off[1]), "s"(sb), "s"(m0v) : "memory", "m0");
    else if constexpr (N == 3)
        asm volatile("s_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %3\n\t"
                     "global_load_lds_dwordx4 %1, %3 offset:1024\n\tglobal_load_lds_dwordx4 %2, %3 offset:2048"
                     : : "v"(lane_off[0]), "v"(lane_off[1]), "v"(lane_off[2]), "s"(sb), "s"(m0v) : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %4\n\t"
                     "global_load_lds_dwordx4 %1, %4 offset:1024\n\tglobal_load_lds_dwordx4 %2, %4 offset:2048\n\t"
                     "global_load_lds_dwordx4 %3, %4 offset:3072"
                     : : "v"(lane_off[0]), "v"(lane_off[1]), "v"(lane_off[2]), "v"(lane_off[3]), "s"(sb), "s"(m0v)
                     : "memory", "m0");
}
// Lane offset to hand to lds_dma16_group for transfer i of N when the bytes wanted are base + want: the group is
// given base - 1024 (N - 1), and the instruction adds 1024 i back.
template <int N> __device__ __forceinline__ uint32_t dma_lane_offset(uint32_t want, int i) { return want + 1024u * (uint32_t)(N - 1 - i); }
template <int N> __device__ __forceinline__ const char* dma_group_base(const char* base) { return base - 1024 * (N - 1); }

// Raw buffer descriptor over [base, base + bytes) (stride 0, no swizzle): a buffer load whose byte offset is at or
// beyond `bytes` returns zeros instead of touching memory.  base and bytes wavefront-uniform.
typedef int32_t i32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ i32x4_t make_raw_buffer(const void* base, uint32_t bytes) {
    const uint64_t b = (uint64_t)(uintptr_t)base;
    i32x4_t d;
    d[0] = __builtin_amdgcn_readfirstlane((uint32_t)b);
    d[1] = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32) & 0xFFFFu);
    d[2] = __builtin_amdgcn_readfirstlane(bytes);
    d[3] = 0x00020000;
    return d;
}
// Four direct transfers of 64 x 16 bytes under one M0, two through each of two buffers: they land at lds_addr,
// + 1024, + 2048, + 3072.  As with lds_dma16_group the immediate offsets (0, 1024, 2048, 3072) are added to the
// memory offsets too, range check included: the caller builds the buffers 3072 bytes early and 3072 bytes longer
// and passes lane offsets a0 + 3072, a1 + 2048, b0 + 1024, b1.
__device__ __forceinline__ void lds_dma16_buffers_2x2(i32x4_t buf_a, uint32_t a0, uint32_t a1, i32x4_t buf_b, uint32_t b0,
                                                      uint32_t b1, uint32_t lds_addr) {
    const uint32_t m0v = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %6\n\ts_nop 0\n\t"
                 "buffer_load_dwordx4 %0, %4, 0 offen lds\n\t"
                 "buffer_load_dwordx4 %1, %4, 0 offen offset:1024 lds\n\t"
                 "buffer_load_dwordx4 %2, %5, 0 offen offset:2048 lds\n\t"
                 "buffer_load_dwordx4 %3, %5, 0 offen offset:3072 lds"
                 : : "v"(a0), "v"(a1), "v"(b0), "v"(b1), "s"(buf_a), "s"(buf_b), "s"(m0v) : "memory", "m0");
}

static inline size_t dtype_size(int32_t dtype) { return dtype == DS_DTYPE_BF16 ? 2 : 4; }

// ---- launchers shared between translation units (all enqueue on `st`, return ds_status)
ds_status launch_mask_rows(int32_t dtype, int32_t rows, int32_t d, const void* in, void* out,
                           const int32_t* row_valid, hipStream_t st);
ds_status launch_gather_rows(int32_t dtype, int32_t out_rows, int32_t d, const void* in, void* out,
                             const int32_t* src_row, hipStream_t st);
// out[c] = (accumulate ? out[c] : 0) + sum over p < n_partial of partial[p * n + c]   (float32, fixed summation order)
ds_status launch_reduce_partials(int32_t n_partial, int32_t n, const float* partial, float* out, int32_t accumulate,
                                 hipStream_t st);
// out[c][r] = in[r][c] (bf16); out leading dimension rows_pad, columns rows..rows_pad-1 zero-filled
ds_status launch_transpose_bf16(int32_t rows, int32_t cols, int32_t rows_pad, const void* in, void* out, hipStream_t st);
ds_status launch_scatter_rows(int32_t dtype, int32_t in_rows, int32_t d, const void* in, void* out,
                              const int32_t* dst_row, hipStream_t st);
