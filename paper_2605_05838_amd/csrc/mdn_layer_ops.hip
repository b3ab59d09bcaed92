// The elementwise operations around the momentum delta rule in the MDN layer (Sec. 3.3, architecture paragraph), and
// their adjoints.  Front end, per token and head, on the short-convolution outputs x_q, x_k, x_v:
//     q' = SiLU(x_q),  k' = SiLU(x_k),  v = SiLU(x_v);   q = L2Norm(q' - d_h k')  (output correction, before the
//     normalisation);   k = L2Norm(k');   L2Norm(x) = x / sqrt(sum x^2 + eps)
// Back end:  y = sigmoid(g) * w * o / sqrt(mean(o^2) + eps)   (head-wise RMS norm with one weight vector, output gate).
// One wave per (token, head) row, a lane holds d/64 elements; the row sums are wave reductions.  HBM-bound streaming
// (arithmetic in fp32, tensors in the storage dtype).  Parameter gradients (dd [H], dw [dv]) are summed per workgroup
// in LDS, then added with one floating-point atomic per entry and workgroup.
#include "../../include/mdn.h"
#include "mdn_device.h"

#include <hip/hip_runtime.h>

namespace mdn {

namespace {

constexpr int LT = 256; // 4 rows per workgroup

__device__ __forceinline__ float sigm(float x) { return 1.f / (1.f + __expf(-x)); }
__device__ __forceinline__ float silu(float x) { return x * sigm(x); }
__device__ __forceinline__ float dsilu(float x) {
    const float s = sigm(x);
    return s * (1.f + x * (1.f - s));
}

template <typename T, int D> struct Row { // the D/64 elements of a row that this lane holds
    static constexpr int E = D / 64;
    float v[E];
    __device__ __forceinline__ void load(const T *p, int lane) {
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = to_f32(p[lane * E + e]);
    }
    __device__ __forceinline__ void store(T *p, int lane) const {
#pragma unroll
        for (int e = 0; e < E; ++e) p[lane * E + e] = from_f32<T>(v[e]);
    }
};

struct LayerDims {
    long long rows; // B*T*H
    int H;
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(LT) void frontend_fwd_kernel(LayerDims d, const T *xq, const T *xk, const T *xv, const float *dh,
                                                           float eps, T *q, T *k, T *v) {
    const int lane = lane_id();
    for (long long row = (long long)blockIdx.x * 4 + wave_id(); row < d.rows; row += (long long)gridDim.x * 4) {
        const float dc = dh[row % d.H];
        Row<T, DK> a, b;
        Row<T, DV> c;
        a.load(xq + row * DK, lane);
        b.load(xk + row * DK, lane);
        c.load(xv + row * DV, lane);
        float sq = 0.f, sk = 0.f;
#pragma unroll
        for (int e = 0; e < Row<T, DK>::E; ++e) {
            b.v[e] = silu(b.v[e]);
            a.v[e] = silu(a.v[e]) - dc * b.v[e];
            sq += a.v[e] * a.v[e];
            sk += b.v[e] * b.v[e];
        }
        const float iq = rsqrtf(reduce64(sq) + eps), ik = rsqrtf(reduce64(sk) + eps);
#pragma unroll
        for (int e = 0; e < Row<T, DK>::E; ++e) {
            a.v[e] *= iq;
            b.v[e] *= ik;
        }
#pragma unroll
        for (int e = 0; e < Row<T, DV>::E; ++e) c.v[e] = silu(c.v[e]);
        a.store(q + row * DK, lane);
        b.store(k + row * DK, lane);
        c.store(v + row * DV, lane);
    }
}

template <typename T, int DK, int DV>
__global__ __launch_bounds__(LT) void frontend_bwd_kernel(LayerDims d, const T *xq, const T *xk, const T *xv, const float *dh,
                                                           float eps, const T *dq, const T *dk, const T *dv, T *dxq, T *dxk,
                                                           T *dxv, float *dd) {
    extern __shared__ float s_dd[]; // [H]
    for (int c = threadIdx.x; c < d.H; c += LT) s_dd[c] = 0.f;
    __syncthreads();
    const int lane = lane_id();
    for (long long row = (long long)blockIdx.x * 4 + wave_id(); row < d.rows; row += (long long)gridDim.x * 4) {
        const int h = (int)(row % d.H);
        const float dc = dh[h];
        Row<T, DK> a, b, ga, gb;
        Row<T, DV> c, gc;
        a.load(xq + row * DK, lane);
        b.load(xk + row * DK, lane);
        c.load(xv + row * DV, lane);
        ga.load(dq + row * DK, lane);
        gb.load(dk + row * DK, lane);
        gc.load(dv + row * DV, lane);
        float qc[Row<T, DK>::E], ks[Row<T, DK>::E], sq = 0.f, sk = 0.f;
#pragma unroll
        for (int e = 0; e < Row<T, DK>::E; ++e) {
            ks[e] = silu(b.v[e]);
            qc[e] = silu(a.v[e]) - dc * ks[e];
            sq += qc[e] * qc[e];
            sk += ks[e] * ks[e];
        }
        const float iq = rsqrtf(reduce64(sq) + eps), ik = rsqrtf(reduce64(sk) + eps);
        float dotq = 0.f, dotk = 0.f;
#pragma unroll
        for (int e = 0; e < Row<T, DK>::E; ++e) {
            dotq += qc[e] * iq * ga.v[e];
            dotk += ks[e] * ik * gb.v[e];
        }
        dotq = reduce64(dotq);
        dotk = reduce64(dotk);
        float ddp = 0.f;
#pragma unroll
        for (int e = 0; e < Row<T, DK>::E; ++e) {
            const float dqc = (ga.v[e] - qc[e] * iq * dotq) * iq; // through the L2 norm of q' - d k'
            const float dks = (gb.v[e] - ks[e] * ik * dotk) * ik - dc * dqc;
            ddp -= dqc * ks[e];
            a.v[e] = dqc * dsilu(a.v[e]);
            b.v[e] = dks * dsilu(b.v[e]);
        }
#pragma unroll
        for (int e = 0; e < Row<T, DV>::E; ++e) c.v[e] = gc.v[e] * dsilu(c.v[e]);
        a.store(dxq + row * DK, lane);
        b.store(dxk + row * DK, lane);
        c.store(dxv + row * DV, lane);
        if (dd) {
            ddp = reduce64(ddp);
            if (lane == 0) atomicAdd(&s_dd[h], ddp);
        }
    }
    __syncthreads();
    if (dd)
        for (int c = threadIdx.x; c < d.H; c += LT) atomicAdd(&dd[c], s_dd[c]);
}

template <typename T, int DV>
__global__ __launch_bounds__(LT) void epilogue_fwd_kernel(LayerDims d, const T *o, const T *g, const float *w, float eps, T *y) {
    const int lane = lane_id();
    for (long long row = (long long)blockIdx.x * 4 + wave_id(); row < d.rows; row += (long long)gridDim.x * 4) {
        Row<T, DV> a, b;
        a.load(o + row * DV, lane);
        b.load(g + row * DV, lane);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < Row<T, DV>::E; ++e) ss += a.v[e] * a.v[e];
        const float ir = rsqrtf(reduce64(ss) * (1.f / DV) + eps);
#pragma unroll
        for (int e = 0; e < Row<T, DV>::E; ++e) a.v[e] = sigm(b.v[e]) * w[lane * Row<T, DV>::E + e] * a.v[e] * ir;
        a.store(y + row * DV, lane);
    }
}

template <typename T, int DV>
__global__ __launch_bounds__(LT) void epilogue_bwd_kernel(LayerDims d, const T *o, const T *g, const float *w, float eps,
                                                           const T *dy, T *dout, T *dg, float *dw) {
    __shared__ float s_dw[DV];
    for (int c = threadIdx.x; c < DV; c += LT) s_dw[c] = 0.f;
    __syncthreads();
    const int lane = lane_id();
    constexpr int E = Row<T, DV>::E;
    float dwp[E];
#pragma unroll
    for (int e = 0; e < E; ++e) dwp[e] = 0.f;
    for (long long row = (long long)blockIdx.x * 4 + wave_id(); row < d.rows; row += (long long)gridDim.x * 4) {
        Row<T, DV> a, b, c;
        a.load(o + row * DV, lane);
        b.load(g + row * DV, lane);
        c.load(dy + row * DV, lane);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) ss += a.v[e] * a.v[e];
        const float ir = rsqrtf(reduce64(ss) * (1.f / DV) + eps);
        float n[E], dn[E], dot = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const float sg = sigm(b.v[e]), we = w[lane * E + e];
            n[e] = a.v[e] * ir;
            dn[e] = c.v[e] * sg * we;
            dot += n[e] * dn[e];
            dwp[e] += c.v[e] * sg * n[e];
            b.v[e] = c.v[e] * we * n[e] * sg * (1.f - sg);
        }
        dot = reduce64(dot) * (1.f / DV);
#pragma unroll
        for (int e = 0; e < E; ++e) a.v[e] = (dn[e] - n[e] * dot) * ir;
        a.store(dout + row * DV, lane);
        b.store(dg + row * DV, lane);
    }
    if (dw) {
#pragma unroll
        for (int e = 0; e < E; ++e) atomicAdd(&s_dw[lane * E + e], dwp[e]);
        __syncthreads();
        for (int c = threadIdx.x; c < DV; c += LT) atomicAdd(&dw[c], s_dw[c]);
    }
}

__global__ void layer_zero_kernel(float *p, int n) {
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x) p[c] = 0.f;
}

int check(const mdn_shape *s, LayerDims *d) {
    if (!s) return MDN_ERR_NULL;
    if (s->dtype != MDN_DTYPE_BF16 && s->dtype != MDN_DTYPE_F32) return MDN_ERR_DTYPE;
    if (s->B < 1 || s->T < 1 || s->H < 1 || s->H > 4096) return MDN_ERR_SHAPE;
    if (!((s->dk == 64 && s->dv == 64) || (s->dk == 128 && s->dv == 128))) return MDN_ERR_SHAPE;
    d->rows = (long long)s->B * s->T * s->H;
    d->H = s->H;
    return MDN_OK;
}

// workgroups of a row-streaming launch; kernels that end with atomic adds on a parameter gradient take a lower cap
// (every workgroup adds to the same few addresses: 8192 workgroups x 128 adds ran the back end's adjoint at 1.5 TB/s)
int grid_for(long long rows, int cap = 8192) {
    const long long b = (rows + 3) / 4;
    return (int)(b < cap ? b : cap);
}

int status() { return hipGetLastError() == hipSuccess ? MDN_OK : MDN_ERR_LAUNCH; }

// F(T tag, DK tag) for the four (storage type, head dimension) combinations
template <typename F> int dispatch(const mdn_shape *s, F &&f) {
    const bool f32 = s->dtype == MDN_DTYPE_F32;
    if (s->dk == 64) return f32 ? f(float{}, std::integral_constant<int, 64>{}) : f(bf16_t{}, std::integral_constant<int, 64>{});
    return f32 ? f(float{}, std::integral_constant<int, 128>{}) : f(bf16_t{}, std::integral_constant<int, 128>{});
}

} // namespace

} // namespace mdn

using namespace mdn;

extern "C" {

int mdn_frontend_fwd(const mdn_shape *shape, const void *x_q, const void *x_k, const void *x_v, const float *d, float eps,
                     void *q, void *k, void *v, void *stream) {
    LayerDims ld;
    const int rc = check(shape, &ld);
    if (rc) return rc;
    if (!x_q || !x_k || !x_v || !d || !q || !k || !v) return MDN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dispatch(shape, [&](auto t, auto dim) {
        typedef decltype(t) T;
        constexpr int D = decltype(dim)::value;
        hipLaunchKernelGGL((frontend_fwd_kernel<T, D, D>), dim3(grid_for(ld.rows)), dim3(LT), 0, s, ld,
                           static_cast<const T *>(x_q), static_cast<const T *>(x_k), static_cast<const T *>(x_v), d, eps,
                           static_cast<T *>(q), static_cast<T *>(k), static_cast<T *>(v));
        return status();
    });
}

int mdn_frontend_bwd(const mdn_shape *shape, const void *x_q, const void *x_k, const void *x_v, const float *d, float eps,
                     const void *dq, const void *dk, const void *dv, void *dx_q, void *dx_k, void *dx_v, float *dd,
                     void *stream) {
    LayerDims ld;
    const int rc = check(shape, &ld);
    if (rc) return rc;
    if (!x_q || !x_k || !x_v || !d || !dq || !dk || !dv || !dx_q || !dx_k || !dx_v) return MDN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dd) hipLaunchKernelGGL(layer_zero_kernel, dim3(1), dim3(256), 0, s, dd, ld.H);
    return dispatch(shape, [&](auto t, auto dim) {
        typedef decltype(t) T;
        constexpr int D = decltype(dim)::value;
        hipLaunchKernelGGL((frontend_bwd_kernel<T, D, D>), dim3(grid_for(ld.rows, 2048)), dim3(LT), ld.H * sizeof(float), s, ld,
                           static_cast<const T *>(x_q), static_cast<const T *>(x_k), static_cast<const T *>(x_v), d, eps,
                           static_cast<const T *>(dq), static_cast<const T *>(dk), static_cast<const T *>(dv),
                           static_cast<T *>(dx_q), static_cast<T *>(dx_k), static_cast<T *>(dx_v), dd);
        return status();
    });
}

int mdn_epilogue_fwd(const mdn_shape *shape, const void *o, const void *g, const float *w, float eps, void *y, void *stream) {
    LayerDims ld;
    const int rc = check(shape, &ld);
    if (rc) return rc;
    if (!o || !g || !w || !y) return MDN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dispatch(shape, [&](auto t, auto dim) {
        typedef decltype(t) T;
        constexpr int D = decltype(dim)::value;
        hipLaunchKernelGGL((epilogue_fwd_kernel<T, D>), dim3(grid_for(ld.rows)), dim3(LT), 0, s, ld, static_cast<const T *>(o),
                           static_cast<const T *>(g), w, eps, static_cast<T *>(y));
        return status();
    });
}

int mdn_epilogue_bwd(const mdn_shape *shape, const void *o, const void *g, const float *w, float eps, const void *dy,
                     void *d_o, void *dg, float *dw, void *stream) {
    LayerDims ld;
    const int rc = check(shape, &ld);
    if (rc) return rc;
    if (!o || !g || !w || !dy || !d_o || !dg) return MDN_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dw) hipLaunchKernelGGL(layer_zero_kernel, dim3(1), dim3(256), 0, s, dw, shape->dv);
    return dispatch(shape, [&](auto t, auto dim) {
        typedef decltype(t) T;
        constexpr int D = decltype(dim)::value;
        hipLaunchKernelGGL((epilogue_bwd_kernel<T, D>), dim3(grid_for(ld.rows, 1024)), dim3(LT), 0, s, ld, static_cast<const T *>(o),
                           static_cast<const T *>(g), w, eps, static_cast<const T *>(dy), static_cast<T *>(d_o),
                           static_cast<T *>(dg), dw);
        return status();
    });
}

} // extern "C"
