// Reverse inter-chunk scan: adjoint of the forward scan of Sec. 3.1 "Chunkwise Algorithm"
// (the paper keeps V~ for the backward pass, "Practical Considerations", but prints no backward
// equations; these follow from differentiating the chunk formulas).  With dS', dM' the adjoints
// of the chunk-END states, walking the chunks from last to first:
//     dV~ = Bm^T dO + (Gamma_C eta . K) dS' - (Rho_C eta . K) dM'
//     dS  = a_C dS' + (a . Q~)^T dO - Y^T dV~
//     dM  = m_C dM' - b_C dS' - (b . Q~)^T dO + Z^T dV~
// Same decomposition as the forward scan: one workgroup per (batch*head, DVB dv-columns), states in
// fp32 accumulators (wave w owns dk rows [w*dk/4, (w+1)*dk/4)), a storage-type copy transposed in
// LDS as B operand, the per-token scalings along the contraction index folded into the LDS copies
// of dO, so that the A operands are the raw Q^T, -Y^T, Z^T, Bm^T and K.
// It writes dV~ (transposed per chunk) and the chunk-end adjoint states for the chunk-parallel
// gradient kernel.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

template <typename T, int DK, int DV, int DVB>
__global__ __launch_bounds__(kThreads) void scan_bwd_kernel(Dims d, ScanBwdArgs a) {
    typedef Op<T> O;
    constexpr int NT = DVB / 16, MT = DK / 64, G = DV / DVB;
    constexpr int LDST = 2 * DK + O::PAD, LDV = 64 + O::PAD;
    __shared__ __align__(16) T sD[DVB * LDST];  // [dv][dS'(dk) | dM'(dk)]
    __shared__ __align__(16) T sO0[DVB * LDV];  // dO^T
    __shared__ __align__(16) T sOa[DVB * LDV];  // (scale a . dO)^T
    __shared__ __align__(16) T sOb[DVB * LDV];  // (-scale b . dO)^T
    __shared__ __align__(16) T sDV[DVB * LDV];  // dV~^T

    int bh, blkv;
    xcd_map(blockIdx.x, G, bh, blkv);
    if (bh >= d.BH) return;
    const int b = bh / d.H, h = bh % d.H, dv0 = blkv * DVB;
    const int lane = lane_id(), w = wave_id(), r = lane & 15, kg = lane >> 4, i0 = w * 16;

    f32x4 accS[MT][NT], accM[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int row = (w * MT + mt) * 16 + kg * 4 + x, col = dv0 + nt * 16 + r;
                const size_t g = ((size_t)bh * DK + row) * DV + col;
                accS[mt][nt][x] = a.dS_final ? a.dS_final[g] : 0.f;
                accM[mt][nt][x] = a.dM_final ? a.dM_final[g] : 0.f;
            }

    const size_t rsk = (size_t)d.H * DK, rsv = (size_t)d.H * DV;
    for (int n = d.N - 1; n >= 0; --n) {
        const size_t blk = (size_t)bh * d.N + n;
        const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
        const float *coef = a.coef + blk * (kCoefRows * 64);

        // adjoints of this chunk's END states: operand copy to LDS, storage copy to HBM
        {
            T *ds = static_cast<T *>(a.dstates) + blk * (2 * DK * DV);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int row = (w * MT + mt) * 16 + kg * 4 + x, col = nt * 16 + r;
                        const T s = from_f32<T>(accS[mt][nt][x]), m = from_f32<T>(accM[mt][nt][x]);
                        sD[col * LDST + row] = s;
                        sD[col * LDST + DK + row] = m;
                        ds[row * DV + dv0 + col] = s;
                        ds[DK * DV + row * DV + dv0 + col] = m;
                    }
        }
        // dO slice of this chunk, transposed, in three scalings
        {
            const T *og = static_cast<const T *>(a.dO) + tok0 * DV + dv0;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + kg * 4 + x;
                const float sa = d.scale * coef[COEF_A * 64 + i], sb = d.scale * coef[COEF_B * 64 + i];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int col = nt * 16 + r;
                    const T raw = og[(size_t)i * rsv + col];
                    const float v = to_f32(raw);
                    sO0[col * LDV + i] = raw;
                    sOa[col * LDV + i] = from_f32<T>(sa * v);
                    sOb[col * LDV + i] = from_f32<T>(-sb * v);
                }
            }
        }
        __syncthreads();

        // ---------------- stage 1: dV~ for tokens j = i0..i0+15
        {
            f32x4 accD[NT], x1[NT], x2[NT];
            zero_acc(accD);
            zero_acc(x1);
            zero_acc(x2);
            mma_rows<T, NT, 64>(accD, static_cast<const T *>(a.BmT) + blk * 4096 + i0 * 64, 64, sO0, LDV);
            const T *kp = static_cast<const T *>(a.k) + (tok0 + (size_t)(i0 + r) * d.H) * DK + kg * O::EPL;
            const T *sp = sD + r * LDST + kg * O::EPL;
#pragma unroll
            for (int k0 = 0; k0 < DK; k0 += O::KSTEP) {
                const typename O::Frag fk = O::load(kp + k0);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    x1[nt] = O::mma(fk, O::load(sp + nt * 16 * LDST + k0), x1[nt]);
                    x2[nt] = O::mma(fk, O::load(sp + nt * 16 * LDST + DK + k0), x2[nt]);
                }
            }
            T *dvt = static_cast<T *>(a.dVtT) + blk * (DV * 64) + (size_t)dv0 * 64;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int j = i0 + kg * 4 + x;
                const float gc = coef[COEF_GC * 64 + j], rc = coef[COEF_RC * 64 + j];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int col = nt * 16 + r;
                    const T v = from_f32<T>(accD[nt][x] + gc * x1[nt][x] - rc * x2[nt][x]);
                    sDV[col * LDV + j] = v;
                    dvt[col * 64 + j] = v;
                }
            }
        }
        __syncthreads();

        // ---------------- stage 2: adjoints of the chunk-START states
        {
            const float aC = coef[COEF_SCALAR * 64 + 0], bC = coef[COEF_SCALAR * 64 + 1],
                        mC = coef[COEF_SCALAR * 64 + 2];
            const T *QTg = static_cast<const T *>(a.QT) + blk * (DK * 64);
            const T *YTg = static_cast<const T *>(a.nYT) + blk * (DK * 64);
            const T *ZTg = static_cast<const T *>(a.ZT) + blk * (DK * 64);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const float s = accS[mt][nt][x], m = accM[mt][nt][x];
                        accS[mt][nt][x] = aC * s;
                        accM[mt][nt][x] = mC * m - bC * s;
                    }
                const int m0 = (w * MT + mt) * 16 * 64;
                mma_rows<T, NT, 64>(accS[mt], QTg + m0, 64, sOa, LDV);
                mma_rows<T, NT, 64>(accS[mt], YTg + m0, 64, sDV, LDV);
                mma_rows<T, NT, 64>(accM[mt], QTg + m0, 64, sOb, LDV);
                mma_rows<T, NT, 64>(accM[mt], ZTg + m0, 64, sDV, LDV);
            }
        }
        __syncthreads();
    }

#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int row = (w * MT + mt) * 16 + kg * 4 + x, col = dv0 + nt * 16 + r;
                const size_t g = ((size_t)bh * DK + row) * DV + col;
                if (a.dS0) a.dS0[g] = accS[mt][nt][x];
                if (a.dM0) a.dM0[g] = accM[mt][nt][x];
            }
}

constexpr int kDVB = 32;

template <typename T, int DK, int DV>
hipError_t launch_t(const Dims &d, const ScanBwdArgs &a, hipStream_t s) {
    constexpr int G = DV / kDVB;
    dim3 grid(((d.BH + 7) / 8) * 8 * G), block(kThreads);
    hipLaunchKernelGGL((scan_bwd_kernel<T, DK, DV, kDVB>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_scan_bwd(const Dims &d, const ScanBwdArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64) return f32 ? launch_t<float, 64, 64>(d, a, s) : launch_t<bf16_t, 64, 64>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_t<float, 128, 128>(d, a, s) : launch_t<bf16_t, 128, 128>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
