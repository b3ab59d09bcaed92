// Recurrent (decoding) form, Eq. Mt.recurrent / St.recurrent in the operation order of the
// recurrent listing of Appendix E:
//     e = v - S^T (alpha k);  M = mu M - eta k e^T;  S = alpha S - beta M;  o = scale S^T q
// HBM-bound on reading and writing the two fp32 states once per call; plain fp32 FMA, no MFMA
// (a GEMV and a rank-1 update per token).  Grid = batch*head x dv/32; a workgroup owns 32 state
// columns; thread (slice, column group) holds dk/32 rows x 4 consecutive columns of S and M in
// registers, so every state access is a 16-byte vector and every wave-level access covers whole
// 128-byte lines.  The two reductions over dk go over the 8 slices of a wave by shuffles, then over
// the 4 waves through LDS.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

constexpr int RCOLS = 32, RCG = RCOLS / 4, RSLICES = kThreads / RCG; // 8 column groups x 32 slices

// sum over the 8 slices of a wave (lane = slice_in_wave * 8 + column group)
__device__ __forceinline__ f32x4 reduce_slices(f32x4 v) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        v[x] += dpp_move<0x128>(v[x]); // lane ^ 8 (rotation by half a row)
        v[x] = add_xor32(add_xor16(v[x]));
    }
    return v;
}

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void recurrent_kernel(Dims d, RecurrentArgs a) {
    constexpr int ROWS = DK / RSLICES;
    static_assert(ROWS >= 1, "dk too small for the slice count");
    __shared__ __align__(16) float redE[4][RCOLS], redO[4][RCOLS];
    const int bh = blockIdx.x, b = bh / d.H, h = bh % d.H;
    const int cg = threadIdx.x % RCG, sl = threadIdx.x / RCG, w = wave_id();
    const int j = blockIdx.y * RCOLS + cg * 4, r0 = sl * ROWS;
    f32x4 S[ROWS], M[ROWS];
    float *Sg = a.S + ((size_t)bh * DK + r0) * DV + j, *Mg = a.M + ((size_t)bh * DK + r0) * DV + j;
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        S[i] = *reinterpret_cast<const f32x4 *>(Sg + (size_t)i * DV);
        M[i] = *reinterpret_cast<const f32x4 *>(Mg + (size_t)i * DV);
    }
    for (int t = 0; t < d.T; ++t) {
        const size_t g = ((size_t)b * d.T + t) * d.H + h;
        const T *kt = static_cast<const T *>(a.k) + g * DK + r0;
        const T *qt = static_cast<const T *>(a.q) + g * DK + r0;
        const float al = a.alpha[g], be = a.beta[g], mu = a.mu[g], et = a.eta ? a.eta[g] : 1.f;
        float kk[ROWS];
        f32x4 part = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            kk[i] = to_f32(kt[i]);
            part += (al * kk[i]) * S[i];
        }
        part = reduce_slices(part);
        if ((threadIdx.x & 63) < RCG) *reinterpret_cast<f32x4 *>(&redE[w][cg * 4]) = part;
        __syncthreads();
        f32x4 e = load4(static_cast<const T *>(a.v) + g * DV + j);
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) e -= *reinterpret_cast<const f32x4 *>(&redE[ww][cg * 4]);
        f32x4 po = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            M[i] = mu * M[i] - (et * kk[i]) * e;
            S[i] = al * S[i] - be * M[i];
            po += to_f32(qt[i]) * S[i];
        }
        po = reduce_slices(po);
        if ((threadIdx.x & 63) < RCG) *reinterpret_cast<f32x4 *>(&redO[w][cg * 4]) = po;
        __syncthreads();
        if (sl == 0) {
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) o += *reinterpret_cast<const f32x4 *>(&redO[ww][cg * 4]);
            store4(static_cast<T *>(a.o) + g * DV + j, d.scale * o);
        }
    }
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        *reinterpret_cast<f32x4 *>(Sg + (size_t)i * DV) = S[i];
        *reinterpret_cast<f32x4 *>(Mg + (size_t)i * DV) = M[i];
    }
}

template <typename T, int DK, int DV>
hipError_t launch_recurrent_t(const Dims &d, const RecurrentArgs &a, hipStream_t s) {
    dim3 grid(d.BH, DV / RCOLS), block(kThreads);
    hipLaunchKernelGGL((recurrent_kernel<T, DK, DV>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_recurrent(const Dims &d, const RecurrentArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64)
        return f32 ? launch_recurrent_t<float, 64, 64>(d, a, s) : launch_recurrent_t<bf16_t, 64, 64>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_recurrent_t<float, 128, 128>(d, a, s) : launch_recurrent_t<bf16_t, 128, 128>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
