// Recurrent (decoding) form, Eq. Mt.recurrent / St.recurrent in the operation order of the
// recurrent listing of Appendix E:
//     e = v - S^T (alpha k);  M = mu M - eta k e^T;  S = alpha S - beta M;  o = scale S^T q
// HBM-bound on reading and writing the two fp32 states once per call; plain fp32 FMA, no MFMA
// (a GEMV and a rank-1 update per token).  Grid = batch*head x dv/32; a workgroup owns 32 state
// columns, thread (slice, col) holds dk/8 rows of S and M for its column in registers.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

constexpr int RCOLS = 32, RSLICES = kThreads / RCOLS;

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void recurrent_kernel(Dims d, RecurrentArgs a) {
    constexpr int ROWS = DK / RSLICES;
    __shared__ float redE[RSLICES][RCOLS], redO[RSLICES][RCOLS];
    const int bh = blockIdx.x, b = bh / d.H, h = bh % d.H;
    const int col = threadIdx.x % RCOLS, sl = threadIdx.x / RCOLS;
    const int j = blockIdx.y * RCOLS + col, r0 = sl * ROWS;
    float S[ROWS], M[ROWS];
    float *Sg = a.S + ((size_t)bh * DK + r0) * DV + j, *Mg = a.M + ((size_t)bh * DK + r0) * DV + j;
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        S[i] = Sg[(size_t)i * DV];
        M[i] = Mg[(size_t)i * DV];
    }
    for (int t = 0; t < d.T; ++t) {
        const size_t g = ((size_t)b * d.T + t) * d.H + h;
        const T *kt = static_cast<const T *>(a.k) + g * DK + r0;
        const T *qt = static_cast<const T *>(a.q) + g * DK + r0;
        const float al = a.alpha[g], be = a.beta[g], mu = a.mu[g], et = a.eta ? a.eta[g] : 1.f;
        float kk[ROWS], part = 0.f;
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            kk[i] = to_f32(kt[i]);
            part += al * kk[i] * S[i];
        }
        redE[sl][col] = part;
        __syncthreads();
        float e = to_f32(static_cast<const T *>(a.v)[g * DV + j]);
#pragma unroll
        for (int s = 0; s < RSLICES; ++s) e -= redE[s][col];
        float po = 0.f;
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            M[i] = mu * M[i] - et * kk[i] * e;
            S[i] = al * S[i] - be * M[i];
            po += to_f32(qt[i]) * S[i];
        }
        redO[sl][col] = po;
        __syncthreads();
        if (sl == 0) {
            float o = 0.f;
#pragma unroll
            for (int s = 0; s < RSLICES; ++s) o += redO[s][col];
            static_cast<T *>(a.o)[g * DV + j] = from_f32<T>(d.scale * o);
        }
    }
#pragma unroll
    for (int i = 0; i < ROWS; ++i) {
        Sg[(size_t)i * DV] = S[i];
        Mg[(size_t)i * DV] = M[i];
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
