// HBM-bound kernels of the stage: row masking / gathering, LayerNorm and RMSNorm forward and
// backward, column sums (bias gradients).  One 64-lane wavefront owns one row; row reductions
// use wavefront shuffles; every global access is a 16-byte (bf16) or 32-byte (fp32) vector
// per lane, consecutive lanes touching consecutive addresses.
#include "common.hpp"

#include <mutex>

namespace {

constexpr int kPartialRows = 2048;   // upper bound on partial-sum rows written by column reductions

// Partial column sums of ds_colsum_static: 4 MiB of device memory per GPU for the life of the process.  In host code
// this name is only a handle for hipGetSymbolAddress; kernels get the per-device address it returns.
constexpr int kStaticFloats = 1 << 20;
constexpr int kStaticMaxCols = 65536;
constexpr int kMaxDevices = 64;
__device__ __align__(256) float g_colsum_scratch[kStaticFloats];
float* g_colsum_scratch_ptr[kMaxDevices];        // device address of the array on each GPU; null until first used there
std::mutex g_colsum_scratch_mutex;

// ------------------------------------------------------------------ row copy kernels
template <class T>
__global__ __launch_bounds__(256) void mask_rows_kernel(int rows, int d8, const T* __restrict__ in, T* __restrict__ out,
                                                        const int32_t* __restrict__ row_valid) {
    const long long total = (long long)rows * d8;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const int r = (int)(i / d8);
        float v[8];
        if (row_valid == nullptr || row_valid[r] >= 0) {
            Vec8<T>::load(in + i * 8, v);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = 0.f;
        }
        Vec8<T>::store(out + i * 8, v);
    }
}

template <class T>
__global__ __launch_bounds__(256) void gather_rows_kernel(int out_rows, int d8, const T* __restrict__ in, T* __restrict__ out,
                                                          const int32_t* __restrict__ src_row) {
    const long long total = (long long)out_rows * d8;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const int r = (int)(i / d8);
        const int c = (int)(i - (long long)r * d8);
        const int s = src_row[r];
        float v[8];
        if (s >= 0) {
            Vec8<T>::load(in + ((long long)s * d8 + c) * 8, v);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[j] = 0.f;
        }
        Vec8<T>::store(out + i * 8, v);
    }
}

template <class T>
__global__ __launch_bounds__(256) void scatter_rows_kernel(int in_rows, int d8, const T* __restrict__ in, T* __restrict__ out,
                                                           const int32_t* __restrict__ dst_row) {
    const long long total = (long long)in_rows * d8;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const int r = (int)(i / d8);
        const int c = (int)(i - (long long)r * d8);
        const int t = dst_row[r];
        if (t < 0) continue;
        float v[8];
        Vec8<T>::load(in + i * 8, v);
        Vec8<T>::store(out + ((long long)t * d8 + c) * 8, v);
    }
}

// ------------------------------------------------------------------ bf16 transpose
// out[c][r] = in[r][c] for r < rows, zero for rows <= r < rows_pad (out has leading dimension rows_pad).
// One wavefront per 64x64 tile as 8x8 blocks of 8x8 elements: each lane loads 8 rows of 16 bytes,
// transposes them in registers (v_perm_b32) and stores 8 rows of 16 bytes; lanes are arranged 8x8 so
// that both the loads and the stores form 128-byte contiguous segments.  No LDS.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(int rows, int cols, int rows_pad, const bf16_t* __restrict__ in,
                                                             bf16_t* __restrict__ out) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bx = lane & 7, by = lane >> 3;
    const int c0 = blockIdx.x * 64 + bx * 8;
    const int r0 = (blockIdx.y * 4 + wave) * 64 + by * 8;
    if (r0 >= rows_pad || c0 >= cols) return;
    uint32_t v[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int r = r0 + i;
        uint4 x = make_uint4(0u, 0u, 0u, 0u);
        if (r < rows) x = *reinterpret_cast<const uint4*>(in + (size_t)r * cols + c0);
        v[i][0] = x.x; v[i][1] = x.y; v[i][2] = x.z; v[i][3] = x.w;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {          // output row c0+i gathers element i of the 8 loaded rows
        const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
        const int w = i >> 1;
        uint4 o;
        o.x = __builtin_amdgcn_perm(v[1][w], v[0][w], sel);
        o.y = __builtin_amdgcn_perm(v[3][w], v[2][w], sel);
        o.z = __builtin_amdgcn_perm(v[5][w], v[4][w], sel);
        o.w = __builtin_amdgcn_perm(v[7][w], v[6][w], sel);
        *reinterpret_cast<uint4*>(out + (size_t)(c0 + i) * rows_pad + r0) = o;
    }
}

inline int grid_for(long long work_items, int block) {
    long long g = (work_items + block - 1) / block;
    if (g > 65536) g = 65536;
    if (g < 1) g = 1;
    return (int)g;
}

// ------------------------------------------------------------------ norm forward
// stats[0..rows) = mean (LayerNorm) or unused (RMS); stats[rows..2rows) = rstd.
template <class T, bool RMS, int NI>
__global__ __launch_bounds__(256) void norm_fwd_kernel(int rows, int d, const T* __restrict__ x, const T* __restrict__ g,
                                                       const T* __restrict__ b, T* __restrict__ y, float* __restrict__ stats) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= rows) return;
    const T* xr = x + (size_t)row * d;
    float v[NI][8];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
        if (col < d) {
            Vec8<T>::load(xr + col, v[i]);
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[i][j];
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[i][j] = 0.f;
        }
    }
    const float inv_d = 1.0f / (float)d;
    const float mean = RMS ? 0.f : wave_sum(s) * inv_d;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
        if (col < d) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float t = v[i][j] - mean;
                q += t * t;
            }
        }
    }
    q = wave_sum(q) * inv_d;
    const float rstd = 1.0f / sqrtf(q + (RMS ? kRmsEps : kLnEps));
    T* yr = y + (size_t)row * d;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
        if (col < d) {
            float gg[8], bb[8], o[8];
            Vec8<T>::load(g + col, gg);
            if (!RMS) Vec8<T>::load(b + col, bb);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float xh = (v[i][j] - mean) * rstd;
                o[j] = RMS ? xh * gg[j] : xh * gg[j] + bb[j];
            }
            Vec8<T>::store(yr + col, o);
        }
    }
    if (lane == 0) {
        stats[row] = mean;
        stats[rows + row] = rstd;
    }
}

// Wide rows (2048 < d <= 4096): one row per work-group of NW wavefronts, each owning d / NW of the columns.  With one
// wavefront per row a lane holds 64 values and the kernel runs at 4.4 TB/s (LayerNorm, d = 4096); at 32 values per
// lane twice as many wavefronts fit and the loads of more rows are in flight: 5.2 TB/s, RMSNorm 5.8.  The two row
// sums (mean, then centred variance: the same two-pass arithmetic as above) are exchanged through LDS (double-buffered
// by row parity should a work-group take more than one row: two barriers per row).
template <class T, bool RMS, int NI, int NW>
__global__ __launch_bounds__(64 * NW) void norm_fwd_multi_kernel(int rows, int d, const T* __restrict__ x, const T* __restrict__ g,
                                                                 const T* __restrict__ b, T* __restrict__ y, float* __restrict__ stats) {
    __shared__ float red_s[2][NW], red_q[2][NW];
    const int part = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int hd = d / NW, c0 = part * hd;
    const float inv_d = 1.0f / (float)d;
    int par = 0;
    for (int row = blockIdx.x; row < rows; row += gridDim.x, par ^= 1) {      // all wavefronts: the same rows
        const T* xr = x + (size_t)row * d + c0;
        float v[NI][8];
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < hd) {
                Vec8<T>::load(xr + col, v[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) s += v[i][j];
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[i][j] = 0.f;
            }
        }
        float mean = 0.f;
        if (!RMS) {
            s = wave_sum(s);
            if (lane == 0) red_s[par][part] = s;
            __syncthreads();
#pragma unroll
            for (int w = 0; w < NW; ++w) mean += red_s[par][w];                // the same order in every wavefront
            mean *= inv_d;
        }
        float q = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < hd) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float t = v[i][j] - mean;
                    q += t * t;
                }
            }
        }
        q = wave_sum(q);
        if (lane == 0) red_q[par][part] = q;
        __syncthreads();
        q = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) q += red_q[par][w];
        q *= inv_d;
        const float rstd = 1.0f / sqrtf(q + (RMS ? kRmsEps : kLnEps));
        T* yr = y + (size_t)row * d + c0;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < hd) {
                float gg[8], bb[8], o[8];
                Vec8<T>::load(g + c0 + col, gg);
                if (!RMS) Vec8<T>::load(b + c0 + col, bb);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float xh = (v[i][j] - mean) * rstd;
                    o[j] = RMS ? xh * gg[j] : xh * gg[j] + bb[j];
                }
                Vec8<T>::store(yr + col, o);
            }
        }
        if (threadIdx.x == 0) {
            stats[row] = mean;
            stats[rows + row] = rstd;
        }
    }
}

// ------------------------------------------------------------------ norm backward
// dx = resid + rstd * (dy*g - mean(dy*g) - xhat * mean(dy*g*xhat))    (RMS: no mean(dy*g) term)
// partial[w][0][:] = sum over the rows wave w handled of dy*xhat, partial[w][1][:] = sum of dy.
template <class T, bool RMS, int NI>
__global__ __launch_bounds__(256) void norm_bwd_kernel(int rows, int d, const T* __restrict__ dy, const T* __restrict__ x,
                                                       const T* __restrict__ g, const float* __restrict__ stats,
                                                       const T* __restrict__ resid, T* __restrict__ dx,
                                                       float* __restrict__ partial) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + wave;
    const int nw = gridDim.x * 4;
    float gg[NI][8], dg[NI][8], db[NI][8];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) { dg[i][j] = 0.f; db[i][j] = 0.f; gg[i][j] = 0.f; }
        if (col < d) Vec8<T>::load(g + col, gg[i]);
    }
    const float inv_d = 1.0f / (float)d;
    for (int row = gw; row < rows; row += nw) {
        const float mean = RMS ? 0.f : stats[row];
        const float rstd = stats[rows + row];
        const T* dyr = dy + (size_t)row * d;
        const T* xr = x + (size_t)row * d;
        float a[NI][8], xh[NI][8];
        float c1 = 0.f, c2 = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < d) {
                Vec8<T>::load(dyr + col, a[i]);
                Vec8<T>::load(xr + col, xh[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    xh[i][j] = (xh[i][j] - mean) * rstd;
                    dg[i][j] += a[i][j] * xh[i][j];
                    db[i][j] += a[i][j];
                    a[i][j] *= gg[i][j];
                    c1 += a[i][j];
                    c2 += a[i][j] * xh[i][j];
                }
            }
        }
        c1 = RMS ? 0.f : wave_sum(c1) * inv_d;
        c2 = wave_sum(c2) * inv_d;
        T* dxr = dx + (size_t)row * d;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < d) {
                float o[8];
                if (resid) {
                    Vec8<T>::load(resid + (size_t)row * d + col, o);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = 0.f;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] += rstd * (a[i][j] - c1 - xh[i][j] * c2);
                Vec8<T>::store(dxr + col, o);
            }
        }
    }
    float* p0 = partial + (size_t)gw * 2 * d;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
        if (col < d) {
            Vec8<float>::store(p0 + col, dg[i]);
            if (!RMS) Vec8<float>::store(p0 + d + col, db[i]);
        }
    }
}

// Wide rows (d > 1024): one row per group of NW = 2 or 4 wavefronts (one work-group), each owning d / NW of the
// columns, so that the per-lane state (gain, dgamma / dbeta sums, dy * g, xhat: 5 x 8 x NI floats) leaves room for
// four wavefronts per SIMD; with one wavefront per row of 4096 columns it needs more than 256 registers and the
// kernel runs at half the memory rate.  The partial row sums are exchanged through LDS (double-buffered by row
// parity: one barrier per row).  partial[group][0][:] / [1][:] as above; a group writes all slices of its partial row.
template <class T, bool RMS, int NI, int NW>
__global__ __launch_bounds__(64 * NW) void norm_bwd_multi_kernel(int rows, int d, const T* __restrict__ dy, const T* __restrict__ x,
                                                                 const T* __restrict__ g, const float* __restrict__ stats,
                                                                 const T* __restrict__ resid, T* __restrict__ dx,
                                                                 float* __restrict__ partial) {
    __shared__ float red[2][NW][2];
    const int part = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int hd = d / NW, c0 = part * hd;
    float gg[NI][8], dg[NI][8], db[NI][8];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) { dg[i][j] = 0.f; db[i][j] = 0.f; gg[i][j] = 0.f; }
        if (col < hd) Vec8<T>::load(g + c0 + col, gg[i]);
    }
    const float inv_d = 1.0f / (float)d;
    int par = 0;
    for (int row = blockIdx.x; row < rows; row += gridDim.x, par ^= 1) {      // all wavefronts: the same rows
        const float mean = RMS ? 0.f : stats[row];
        const float rstd = stats[rows + row];
        const T* dyr = dy + (size_t)row * d + c0;
        const T* xr = x + (size_t)row * d + c0;
        float a[NI][8], xh[NI][8];
        float c1 = 0.f, c2 = 0.f;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < hd) {
                Vec8<T>::load(dyr + col, a[i]);
                Vec8<T>::load(xr + col, xh[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    xh[i][j] = (xh[i][j] - mean) * rstd;
                    dg[i][j] += a[i][j] * xh[i][j];
                    db[i][j] += a[i][j];
                    a[i][j] *= gg[i][j];
                    c1 += a[i][j];
                    c2 += a[i][j] * xh[i][j];
                }
            }
        }
        c1 = wave_sum(c1);
        c2 = wave_sum(c2);
        if (lane == 0) { red[par][part][0] = c1; red[par][part][1] = c2; }
        __syncthreads();
        c1 = 0.f;
        c2 = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) { c1 += red[par][w][0]; c2 += red[par][w][1]; }    // the same order in every wavefront
        c1 = RMS ? 0.f : c1 * inv_d;
        c2 *= inv_d;
        T* dxr = dx + (size_t)row * d + c0;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int col = (lane + 64 * i) * 8;
            if (col < hd) {
                float o[8];
                if (resid) {
                    Vec8<T>::load(resid + (size_t)row * d + c0 + col, o);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] = 0.f;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] += rstd * (a[i][j] - c1 - xh[i][j] * c2);
                Vec8<T>::store(dxr + col, o);
            }
        }
    }
    float* p0 = partial + (size_t)blockIdx.x * 2 * d + c0;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int col = (lane + 64 * i) * 8;
        if (col < hd) {
            Vec8<float>::store(p0 + col, dg[i]);
            if (!RMS) Vec8<float>::store(p0 + d + col, db[i]);
        }
    }
}

// out[c] = (accumulate ? out[c] : 0) + sum_p partial[p * stride + c];  block = 32 columns x 8 row lanes
// blockIdx.y = 1 (when launched with two rows of blocks) reduces a second set of partials into out2.
__global__ __launch_bounds__(256) void reduce_partials_kernel(int n_partial, int n, size_t stride,
                                                              const float* __restrict__ partial,
                                                              float* __restrict__ out, int accumulate,
                                                              const float* __restrict__ partial2 = nullptr,
                                                              float* __restrict__ out2 = nullptr) {
    __shared__ float red[8][33];
    if (blockIdx.y == 1) {
        partial = partial2;
        out = out2;
    }
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int col = blockIdx.x * 32 + tx;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (col < n) {
        int p = ty;
        for (; p + 24 < n_partial; p += 32) {
            s0 += partial[(size_t)p * stride + col];
            s1 += partial[(size_t)(p + 8) * stride + col];
            s2 += partial[(size_t)(p + 16) * stride + col];
            s3 += partial[(size_t)(p + 24) * stride + col];
        }
        for (; p < n_partial; p += 8) s0 += partial[(size_t)p * stride + col];
    }
    red[ty][tx] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (ty == 0 && col < n) {
        float s = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) s += red[k][tx];
        out[col] = accumulate ? out[col] + s : s;
    }
}

// ------------------------------------------------------------------ column sums
// block (64, 4): thread (tx, ty) owns 8 columns, rows blockIdx.y*4+ty, stepping gridDim.y*4.
template <class T>
__global__ __launch_bounds__(256) void colsum_kernel(int rows, int n, const T* __restrict__ x, float* __restrict__ partial) {
    __shared__ float red[4][64][9];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int col = (blockIdx.x * 64 + tx) * 8;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    if (col < n) {
        for (int r = blockIdx.y * 4 + ty; r < rows; r += gridDim.y * 4) {
            float v[8];
            Vec8<T>::load(x + (size_t)r * n + col, v);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += v[j];
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) red[ty][tx][j] = acc[j];
    __syncthreads();
    if (ty == 0 && col < n) {
        float o[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = red[0][tx][j] + red[1][tx][j] + red[2][tx][j] + red[3][tx][j];
        Vec8<float>::store(partial + (size_t)blockIdx.y * n + col, o);
    }
}

template <class T, bool RMS>
ds_status norm_fwd_dispatch(int rows, int d, const T* x, const T* g, const T* b, T* y, float* stats, hipStream_t st) {
    const int ni = (d + 511) / 512;
    if (ni > 4 && d % 16 == 0) {                 // wide rows: two wavefronts per row (see norm_fwd_multi_kernel)
        // one work-group per row: measured best (a grid striding over the rows with 16 K or 4 K work-groups is 6 - 30 % slower)
        hipLaunchKernelGGL((norm_fwd_multi_kernel<T, RMS, 4, 2>), dim3(rows), dim3(128), 0, st, rows, d, x, g, b, y, stats);
        DS_LAUNCH_CHECK();
        return DS_OK;
    }
    dim3 grid((rows + 3) / 4), block(256);
    if (ni <= 1) hipLaunchKernelGGL((norm_fwd_kernel<T, RMS, 1>), grid, block, 0, st, rows, d, x, g, b, y, stats);
    else if (ni <= 2) hipLaunchKernelGGL((norm_fwd_kernel<T, RMS, 2>), grid, block, 0, st, rows, d, x, g, b, y, stats);
    else if (ni <= 4) hipLaunchKernelGGL((norm_fwd_kernel<T, RMS, 4>), grid, block, 0, st, rows, d, x, g, b, y, stats);
    else hipLaunchKernelGGL((norm_fwd_kernel<T, RMS, 8>), grid, block, 0, st, rows, d, x, g, b, y, stats);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

template <class T, bool RMS>
ds_status norm_bwd_dispatch(int rows, int d, const T* dy, const T* x, const T* g, const float* stats, const T* resid,
                            T* dx, float* dg, float* db, float* partial, int accumulate, hipStream_t st) {
    const int ni = (d + 511) / 512;
    if (ni > 2 && d % 32 == 0) {                 // wide rows: two or four wavefronts per row (see norm_bwd_multi_kernel)
        const int np = rows < kPartialRows ? rows : kPartialRows;
        if (ni > 4) hipLaunchKernelGGL((norm_bwd_multi_kernel<T, RMS, 2, 4>), dim3(np), dim3(256), 0, st, rows, d, dy, x, g, stats, resid, dx, partial);
        else hipLaunchKernelGGL((norm_bwd_multi_kernel<T, RMS, 2, 2>), dim3(np), dim3(128), 0, st, rows, d, dy, x, g, stats, resid, dx, partial);
        DS_LAUNCH_CHECK();
        // dgamma and, for LayerNorm, dbeta in one launch
        hipLaunchKernelGGL(reduce_partials_kernel, dim3((d + 31) / 32, RMS ? 1 : 2), dim3(256), 0, st, np, d, (size_t)2 * d, partial, dg,
                           accumulate, (const float*)(partial + d), db);
        DS_LAUNCH_CHECK();
        return DS_OK;
    }
    int nblk = (rows + 3) / 4;
    if (nblk > kPartialRows / 4) nblk = kPartialRows / 4;
    dim3 grid(nblk), block(256);
    if (ni <= 1) hipLaunchKernelGGL((norm_bwd_kernel<T, RMS, 1>), grid, block, 0, st, rows, d, dy, x, g, stats, resid, dx, partial);
    else if (ni <= 2) hipLaunchKernelGGL((norm_bwd_kernel<T, RMS, 2>), grid, block, 0, st, rows, d, dy, x, g, stats, resid, dx, partial);
    else if (ni <= 4) hipLaunchKernelGGL((norm_bwd_kernel<T, RMS, 4>), grid, block, 0, st, rows, d, dy, x, g, stats, resid, dx, partial);
    else hipLaunchKernelGGL((norm_bwd_kernel<T, RMS, 8>), grid, block, 0, st, rows, d, dy, x, g, stats, resid, dx, partial);
    DS_LAUNCH_CHECK();
    const int np = nblk * 4;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((d + 31) / 32, RMS ? 1 : 2), dim3(256), 0, st, np, d, (size_t)2 * d, partial, dg,
                       accumulate, (const float*)(partial + d), db);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

}  // namespace

ds_status launch_mask_rows(int32_t dtype, int32_t rows, int32_t d, const void* in, void* out,
                           const int32_t* row_valid, hipStream_t st) {
    if (rows <= 0) return DS_OK;
    if (d % 8) return DS_EINVAL;
    const long long items = (long long)rows * (d / 8);
    if (dtype == DS_DTYPE_BF16)
        hipLaunchKernelGGL(mask_rows_kernel<bf16_t>, dim3(grid_for(items, 256)), dim3(256), 0, st, rows, d / 8,
                           (const bf16_t*)in, (bf16_t*)out, row_valid);
    else
        hipLaunchKernelGGL(mask_rows_kernel<float>, dim3(grid_for(items, 256)), dim3(256), 0, st, rows, d / 8,
                           (const float*)in, (float*)out, row_valid);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

ds_status launch_gather_rows(int32_t dtype, int32_t out_rows, int32_t d, const void* in, void* out,
                             const int32_t* src_row, hipStream_t st) {
    if (out_rows <= 0) return DS_OK;
    if (d % 8) return DS_EINVAL;
    const long long items = (long long)out_rows * (d / 8);
    if (dtype == DS_DTYPE_BF16)
        hipLaunchKernelGGL(gather_rows_kernel<bf16_t>, dim3(grid_for(items, 256)), dim3(256), 0, st, out_rows, d / 8,
                           (const bf16_t*)in, (bf16_t*)out, src_row);
    else
        hipLaunchKernelGGL(gather_rows_kernel<float>, dim3(grid_for(items, 256)), dim3(256), 0, st, out_rows, d / 8,
                           (const float*)in, (float*)out, src_row);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

ds_status launch_scatter_rows(int32_t dtype, int32_t in_rows, int32_t d, const void* in, void* out,
                              const int32_t* dst_row, hipStream_t st) {
    if (in_rows <= 0) return DS_OK;
    if (d % 8) return DS_EINVAL;
    const long long items = (long long)in_rows * (d / 8);
    if (dtype == DS_DTYPE_BF16)
        hipLaunchKernelGGL(scatter_rows_kernel<bf16_t>, dim3(grid_for(items, 256)), dim3(256), 0, st, in_rows, d / 8,
                           (const bf16_t*)in, (bf16_t*)out, dst_row);
    else
        hipLaunchKernelGGL(scatter_rows_kernel<float>, dim3(grid_for(items, 256)), dim3(256), 0, st, in_rows, d / 8,
                           (const float*)in, (float*)out, dst_row);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

ds_status launch_transpose_bf16(int32_t rows, int32_t cols, int32_t rows_pad, const void* in, void* out, hipStream_t st) {
    if (rows <= 0 || cols <= 0 || cols % 8 || rows_pad < rows || rows_pad % 8 || !in || !out) return DS_EINVAL;
    dim3 grid((cols + 63) / 64, (rows_pad + 255) / 256);
    hipLaunchKernelGGL(transpose_bf16_kernel, grid, dim3(256), 0, st, rows, cols, rows_pad, (const bf16_t*)in, (bf16_t*)out);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

extern "C" int64_t ds_norm_bwd_scratch_floats(int32_t rows, int32_t d) {
    (void)rows;
    return (int64_t)kPartialRows * 2 * (d > 0 ? d : 0);
}

extern "C" ds_status ds_norm_fwd(int32_t dtype, int32_t rms, int32_t rows, int32_t d, const void* x, const void* g,
                                 const void* b, void* y, float* stats, void* hip_stream) {
    if (rows < 0 || d <= 0 || d % 8 || d > 4096 || !x || !g || !y || !stats || (!rms && !b)) return DS_EINVAL;
    if (dtype != DS_DTYPE_F32 && dtype != DS_DTYPE_BF16) return DS_EINVAL;
    if (rows == 0) return DS_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == DS_DTYPE_BF16) {
        if (rms) return norm_fwd_dispatch<bf16_t, true>(rows, d, (const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)y, stats, st);
        return norm_fwd_dispatch<bf16_t, false>(rows, d, (const bf16_t*)x, (const bf16_t*)g, (const bf16_t*)b, (bf16_t*)y, stats, st);
    }
    if (rms) return norm_fwd_dispatch<float, true>(rows, d, (const float*)x, (const float*)g, (const float*)b, (float*)y, stats, st);
    return norm_fwd_dispatch<float, false>(rows, d, (const float*)x, (const float*)g, (const float*)b, (float*)y, stats, st);
}

extern "C" ds_status ds_norm_bwd(int32_t dtype, int32_t rms, int32_t rows, int32_t d, const void* dy, const void* x,
                                 const void* g, const float* stats, const void* resid, void* dx, float* dg, float* db,
                                 float* partial, int32_t accumulate, void* hip_stream) {
    if (rows <= 0 || d <= 0 || d % 8 || d > 4096 || !dy || !x || !g || !stats || !dx || !dg || !partial || (!rms && !db))
        return DS_EINVAL;
    if (dtype != DS_DTYPE_F32 && dtype != DS_DTYPE_BF16) return DS_EINVAL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == DS_DTYPE_BF16) {
        if (rms) return norm_bwd_dispatch<bf16_t, true>(rows, d, (const bf16_t*)dy, (const bf16_t*)x, (const bf16_t*)g, stats, (const bf16_t*)resid, (bf16_t*)dx, dg, db, partial, accumulate, st);
        return norm_bwd_dispatch<bf16_t, false>(rows, d, (const bf16_t*)dy, (const bf16_t*)x, (const bf16_t*)g, stats, (const bf16_t*)resid, (bf16_t*)dx, dg, db, partial, accumulate, st);
    }
    if (rms) return norm_bwd_dispatch<float, true>(rows, d, (const float*)dy, (const float*)x, (const float*)g, stats, (const float*)resid, (float*)dx, dg, db, partial, accumulate, st);
    return norm_bwd_dispatch<float, false>(rows, d, (const float*)dy, (const float*)x, (const float*)g, stats, (const float*)resid, (float*)dx, dg, db, partial, accumulate, st);
}

ds_status launch_reduce_partials(int32_t n_partial, int32_t n, const float* partial, float* out, int32_t accumulate,
                                 hipStream_t st) {
    if (n_partial <= 0 || n <= 0 || !partial || !out) return DS_EINVAL;
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((n + 31) / 32), dim3(256), 0, st, n_partial, n, (size_t)n, partial, out, accumulate,
                       (const float*)nullptr, (float*)nullptr);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

// Column sums in two kernels: gy partial rows of n floats each (gy <= max_partial_rows), then their sum in a fixed order.
static ds_status colsum_launch(int32_t dtype, int32_t rows, int32_t n, const void* x, float* out, float* partial,
                               int max_partial_rows, int32_t accumulate, hipStream_t st) {
    const int gx = (n / 8 + 63) / 64;
    int gy = (rows + 3) / 4;
    int cap = kPartialRows / gx > 0 ? kPartialRows / gx : 1;
    if (cap > max_partial_rows) cap = max_partial_rows;
    if (gy > cap) gy = cap;
    if (dtype == DS_DTYPE_BF16)
        hipLaunchKernelGGL(colsum_kernel<bf16_t>, dim3(gx, gy), dim3(256), 0, st, rows, n, (const bf16_t*)x, partial);
    else
        hipLaunchKernelGGL(colsum_kernel<float>, dim3(gx, gy), dim3(256), 0, st, rows, n, (const float*)x, partial);
    DS_LAUNCH_CHECK();
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((n + 31) / 32), dim3(256), 0, st, gy, n, (size_t)n, partial, out, accumulate,
                       (const float*)nullptr, (float*)nullptr);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

extern "C" ds_status ds_colsum(int32_t dtype, int32_t rows, int32_t n, const void* x, float* out, float* partial,
                               int32_t accumulate, void* hip_stream) {
    if (rows <= 0 || n <= 0 || n % 8 || !x || !out || !partial) return DS_EINVAL;
    if (dtype != DS_DTYPE_F32 && dtype != DS_DTYPE_BF16) return DS_EINVAL;
    return colsum_launch(dtype, rows, n, x, out, partial, kPartialRows, accumulate, (hipStream_t)hip_stream);
}

extern "C" ds_status ds_colsum_static(int32_t dtype, int32_t rows, int32_t n, const void* x, float* out, int32_t accumulate,
                                      void* hip_stream) {
    if (rows <= 0 || n <= 0 || n % 8 || !x || !out) return DS_EINVAL;
    if (dtype != DS_DTYPE_F32 && dtype != DS_DTYPE_BF16) return DS_EINVAL;
    if (n > kStaticMaxCols) return DS_ELIMIT;
    int dev = -1;
    DS_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return DS_ELIMIT;
    float* scratch = nullptr;
    {
        // once per device, with that device current: every GPU holds its own copy of the array at its own address
        std::lock_guard<std::mutex> lock(g_colsum_scratch_mutex);
        if (!g_colsum_scratch_ptr[dev]) {
            void* p = nullptr;
            DS_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(g_colsum_scratch)));
            if (!p) return DS_EHIP;
            g_colsum_scratch_ptr[dev] = (float*)p;
        }
        scratch = g_colsum_scratch_ptr[dev];
    }
    // every partial row the second kernel reads is written in full by the first: nothing needs clearing between calls
    return colsum_launch(dtype, rows, n, x, out, scratch, kStaticFloats / n, accumulate, (hipStream_t)hip_stream);
}
