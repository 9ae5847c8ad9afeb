// Variable-length attention, generic kernels (any dtype, head_dim <= 128, multiple of 8): the
// fp32 path and the fallback for shapes the MFMA kernels do not take.  One 64-lane wavefront
// per query row (forward, dQ) or per key row (dK/dV); no work is spent on padding because the
// kernels walk the sequence table, never the padded tensor.
#include "attention.hpp"

namespace {

template <class T>
__device__ __forceinline__ float dot_row(const float* __restrict__ a /*LDS, hd floats*/, const T* __restrict__ b, int hd) {
    float s = 0.f;
    for (int d = 0; d < hd; d += 8) {
        float v[8];
        Vec8<T>::load(b + d, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) s += a[d + j] * v[j];
    }
    return s;
}

// ---------------------------------------------------------------- forward
template <class T>
__global__ __launch_bounds__(256) void attn_fwd_generic_kernel(AttnArgs a) {
    __shared__ float sq[4][128];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int qi = blockIdx.x * 4 + w, h = blockIdx.y, s = blockIdx.z;
    const int hd = a.head_dim;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const bool active = qi < ql;
    const T* q = (const T*)a.q;
    const T* k = (const T*)a.k;
    const T* v = (const T*)a.v;
    const long long qr = (long long)a.q_row[s] + qi;
    if (active) {
        for (int d = lane; d < hd; d += 64) sq[w][d] = to_f32(q[qr * a.ldq + h * hd + d]) * a.scale;
    }
    __syncthreads();
    if (!active) return;
    const int nk = a.mask ? min(kl, qi + 1) : kl;
    const long long kr0 = a.k_row[s];
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int j0 = 0; j0 < nk; j0 += 64) {
        const int j = j0 + lane;
        const bool valid = j < nk;
        float sc = -INFINITY;
        if (valid) sc = dot_row<T>(sq[w], k + (kr0 + j) * a.ldk + h * hd, hd);
        const float m_new = fmaxf(m, wave_max(sc));
        const float alpha = __expf(m - m_new);
        const float p = valid ? __expf(sc - m_new) : 0.f;
        l = l * alpha + wave_sum(p);
        o0 *= alpha;
        o1 *= alpha;
        const int cnt = min(64, nk - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = __shfl(p, jj, 64);
            const T* vr = v + (kr0 + j0 + jj) * a.ldv + h * hd;
            if (lane < hd) o0 += pj * to_f32(vr[lane]);
            if (lane + 64 < hd) o1 += pj * to_f32(vr[lane + 64]);
        }
        m = m_new;
    }
    const float inv = l > 0.f ? 1.0f / l : 0.f;         // (no keys: zero output)
    T* o = (T*)a.o;
    if (lane < hd) o[qr * a.ldo + h * hd + lane] = from_f32<T>(o0 * inv);
    if (lane + 64 < hd) o[qr * a.ldo + h * hd + lane + 64] = from_f32<T>(o1 * inv);
    if (lane == 0) a.lse[(size_t)h * a.lse_stride + qr] = m + __logf(l);
}

// ---------------------------------------------------------------- delta = rowsum(dO * O)
template <class T>
__global__ __launch_bounds__(256) void attn_delta_kernel(AttnArgs a) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int qi = blockIdx.x * 4 + w, h = blockIdx.y, s = blockIdx.z;
    if (qi >= a.q_len[s]) return;
    const int hd = a.head_dim;
    const long long qr = (long long)a.q_row[s] + qi;
    const T* o = (const T*)a.o + qr * a.ldo + h * hd;
    const T* d_o = (const T*)a.d_o + qr * a.ldo + h * hd;
    float acc = 0.f;
    for (int d = lane; d < hd; d += 64) acc += to_f32(o[d]) * to_f32(d_o[d]);
    acc = wave_sum(acc);
    if (lane == 0) a.delta[(size_t)h * a.lse_stride + qr] = acc;
}

// ---------------------------------------------------------------- dQ: one wavefront per query row
template <class T>
__global__ __launch_bounds__(256) void attn_bwd_dq_generic_kernel(AttnArgs a) {
    __shared__ float sq[4][128];
    __shared__ float sdo[4][128];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int qi = blockIdx.x * 4 + w, h = blockIdx.y, s = blockIdx.z;
    const int hd = a.head_dim;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const bool active = qi < ql;
    const T* q = (const T*)a.q;
    const T* k = (const T*)a.k;
    const T* v = (const T*)a.v;
    const T* d_o = (const T*)a.d_o;
    const long long qr = (long long)a.q_row[s] + qi;
    if (active) {
        for (int d = lane; d < hd; d += 64) {
            sq[w][d] = to_f32(q[qr * a.ldq + h * hd + d]) * a.scale;
            sdo[w][d] = to_f32(d_o[qr * a.ldo + h * hd + d]);
        }
    }
    __syncthreads();
    if (!active) return;
    const int nk = a.mask ? min(kl, qi + 1) : kl;
    const long long kr0 = a.k_row[s];
    const float lse = a.lse[(size_t)h * a.lse_stride + qr];
    const float delta = a.delta[(size_t)h * a.lse_stride + qr];
    float g0 = 0.f, g1 = 0.f;
    for (int j0 = 0; j0 < nk; j0 += 64) {
        const int j = j0 + lane;
        float ds = 0.f;
        if (j < nk) {
            const float sc = dot_row<T>(sq[w], k + (kr0 + j) * a.ldk + h * hd, hd);
            const float p = __expf(sc - lse);
            const float dp = dot_row<T>(sdo[w], v + (kr0 + j) * a.ldv + h * hd, hd);
            ds = p * (dp - delta);
        }
        const int cnt = min(64, nk - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float dj = __shfl(ds, jj, 64);
            const T* kr = k + (kr0 + j0 + jj) * a.ldk + h * hd;
            if (lane < hd) g0 += dj * to_f32(kr[lane]);
            if (lane + 64 < hd) g1 += dj * to_f32(kr[lane + 64]);
        }
    }
    T* dq = (T*)a.dq;
    if (lane < hd) dq[qr * a.ldq + h * hd + lane] = from_f32<T>(g0 * a.scale);
    if (lane + 64 < hd) dq[qr * a.ldq + h * hd + lane + 64] = from_f32<T>(g1 * a.scale);
}

// ---------------------------------------------------------------- dK, dV: one wavefront per key row
template <class T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_generic_kernel(AttnArgs a) {
    __shared__ float sk[4][128];
    __shared__ float sv[4][128];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int kj = blockIdx.x * 4 + w, h = blockIdx.y, s = blockIdx.z;
    const int hd = a.head_dim;
    const int ql = a.q_len[s], kl = a.k_len[s];
    const bool active = kj < kl;
    const T* q = (const T*)a.q;
    const T* k = (const T*)a.k;
    const T* v = (const T*)a.v;
    const T* d_o = (const T*)a.d_o;
    const long long kr = (long long)a.k_row[s] + kj;
    if (active) {
        for (int d = lane; d < hd; d += 64) {
            sk[w][d] = to_f32(k[kr * a.ldk + h * hd + d]) * a.scale;
            sv[w][d] = to_f32(v[kr * a.ldv + h * hd + d]);
        }
    }
    __syncthreads();
    if (!active) return;
    const int i_begin = a.mask ? kj : 0;           // causal: only queries at or after the key see it
    const long long qr0 = a.q_row[s];
    float gk0 = 0.f, gk1 = 0.f, gv0 = 0.f, gv1 = 0.f;
    for (int i0 = i_begin; i0 < ql; i0 += 64) {
        const int i = i0 + lane;
        float p = 0.f, ds = 0.f;
        if (i < ql) {
            const float sc = dot_row<T>(sk[w], q + (qr0 + i) * a.ldq + h * hd, hd);
            p = __expf(sc - a.lse[(size_t)h * a.lse_stride + qr0 + i]);
            const float dp = dot_row<T>(sv[w], d_o + (qr0 + i) * a.ldo + h * hd, hd);
            ds = p * (dp - a.delta[(size_t)h * a.lse_stride + qr0 + i]);
        }
        const int cnt = min(64, ql - i0);
        for (int ii = 0; ii < cnt; ++ii) {
            const float pi = __shfl(p, ii, 64);
            const float di = __shfl(ds, ii, 64);
            const T* qrow = q + (qr0 + i0 + ii) * a.ldq + h * hd;
            const T* dorow = d_o + (qr0 + i0 + ii) * a.ldo + h * hd;
            if (lane < hd) {
                gv0 += pi * to_f32(dorow[lane]);
                gk0 += di * to_f32(qrow[lane]);
            }
            if (lane + 64 < hd) {
                gv1 += pi * to_f32(dorow[lane + 64]);
                gk1 += di * to_f32(qrow[lane + 64]);
            }
        }
    }
    T* dk = (T*)a.dk;
    T* dv = (T*)a.dv;
    if (lane < hd) {
        dk[kr * a.ldk + h * hd + lane] = from_f32<T>(gk0 * a.scale);
        dv[kr * a.ldv + h * hd + lane] = from_f32<T>(gv0);
    }
    if (lane + 64 < hd) {
        dk[kr * a.ldk + h * hd + lane + 64] = from_f32<T>(gk1 * a.scale);
        dv[kr * a.ldv + h * hd + lane + 64] = from_f32<T>(gv1);
    }
}

}  // namespace

template <class T>
static ds_status fwd_generic_t(const AttnArgs& a, hipStream_t st) {
    dim3 grid((a.max_q_len + 3) / 4, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(attn_fwd_generic_kernel<T>, grid, dim3(256), 0, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

ds_status attn_fwd_generic(const AttnArgs& a, hipStream_t st) {
    return a.dtype == DS_DTYPE_BF16 ? fwd_generic_t<bf16_t>(a, st) : fwd_generic_t<float>(a, st);
}

ds_status attn_delta(const AttnArgs& a, hipStream_t st) {
    dim3 grid((a.max_q_len + 3) / 4, a.n_heads, a.n_seq);
    if (a.dtype == DS_DTYPE_BF16)
        hipLaunchKernelGGL(attn_delta_kernel<bf16_t>, grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(attn_delta_kernel<float>, grid, dim3(256), 0, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

template <class T>
static ds_status bwd_generic_t(const AttnArgs& a, hipStream_t st) {
    dim3 gq((a.max_q_len + 3) / 4, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(attn_bwd_dq_generic_kernel<T>, gq, dim3(256), 0, st, a);
    DS_LAUNCH_CHECK();
    dim3 gk((a.max_k_len + 3) / 4, a.n_heads, a.n_seq);
    hipLaunchKernelGGL(attn_bwd_dkv_generic_kernel<T>, gk, dim3(256), 0, st, a);
    DS_LAUNCH_CHECK();
    return DS_OK;
}

ds_status attn_bwd_generic(const AttnArgs& a, hipStream_t st) {
    return a.dtype == DS_DTYPE_BF16 ? bwd_generic_t<bf16_t>(a, st) : bwd_generic_t<float>(a, st);
}
