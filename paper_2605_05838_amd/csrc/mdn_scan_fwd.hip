// Sequential inter-chunk propagation of the state S and the momentum M (forward), Sec. 3.1
// "Chunkwise Algorithm":
//     V~  = U - Y S + Z M
//     O   = diag(a) Q~ S - diag(b) Q~ M + Bm V~
//     S'  = a_C S - b_C M + (diag(Gamma_C) K~)^T V~
//     M'  = m_C M - (diag(Rho_C) K~)^T V~
// Every dv column of S, M, V~, O evolves independently, so one workgroup owns DVB columns of one
// (batch, head) and walks the chunks in order: grid = batch*head x dv/DVB, all workgroups of one
// (batch, head) on the same XCD so that the chunk operands they share are served by one L2.
//
// Inside a workgroup (4 waves): S, M live in fp32 MFMA accumulators (wave w owns dk rows
// [w*dk/4, (w+1)*dk/4)); a storage-type copy sits in LDS, transposed ([dv][dk | dk]), as the B
// operand of the dk-contractions.  Stage 1 (wave w owns tokens 16w..16w+15) forms V~ and the two
// inter-chunk read-outs; V~ goes to LDS transposed ([dv][token]) in three scalings (raw, Gamma_C eta,
// -Rho_C eta) and is the B operand of the token-contractions of stage 2.  The row scalings along
// the contraction index are folded into those copies, so the A operands are the raw K^T, Q.
// Two barriers per chunk.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

template <typename T, int DK, int DVB> struct ScanSmem {
    static constexpr int LDS_ST = 2 * DK + Op<T>::PAD; // state copy: [DVB][S(dk) | M(dk)]
    static constexpr int LDV = 64 + Op<T>::PAD;        // V~ copies: [DVB][64 tokens]
};

// write the accumulator tiles of this wave's state rows into the LDS operand copy
template <typename T, int DK, int NT>
__device__ __forceinline__ void publish_state(T *sSt, int ldst, const f32x4 (&accS)[DK / 64][NT],
                                              const f32x4 (&accM)[DK / 64][NT]) {
    const int r = lane_id() & 15, kg = lane_id() >> 4, w = wave_id();
#pragma unroll
    for (int mt = 0; mt < DK / 64; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int row = (w * (DK / 64) + mt) * 16 + kg * 4 + x, col = nt * 16 + r;
                sSt[col * ldst + row] = from_f32<T>(accS[mt][nt][x]);
                sSt[col * ldst + DK + row] = from_f32<T>(accM[mt][nt][x]);
            }
}

// REBUILD = false: full forward scan.  REBUILD = true: state reconstruction from saved V~ only
// (the update lines), writing the chunk-start states.
template <typename T, int DK, int DV, int DVB, bool REBUILD>
__global__ __launch_bounds__(kThreads) void scan_fwd_kernel(Dims d, ScanFwdArgs a) {
    typedef Op<T> O;
    typedef ScanSmem<T, DK, DVB> SM;
    constexpr int NT = DVB / 16, MT = DK / 64, G = DV / DVB;
    __shared__ __align__(16) T sSt[DVB * SM::LDS_ST];
    __shared__ __align__(16) T sV0[DVB * SM::LDV];
    __shared__ __align__(16) T sVg[DVB * SM::LDV];
    __shared__ __align__(16) T sVr[DVB * SM::LDV];

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
                accS[mt][nt][x] = a.S0 ? a.S0[g] : 0.f;
                accM[mt][nt][x] = a.M0 ? a.M0[g] : 0.f;
            }
    if (!REBUILD) publish_state<T, DK, NT>(sSt, SM::LDS_ST, accS, accM);
    __syncthreads();

    const size_t rsk = (size_t)d.H * DK, rsv = (size_t)d.H * DV;
    for (int n = 0; n < d.N; ++n) {
        const size_t blk = (size_t)bh * d.N + n;
        const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
        const float *coef = a.coef + blk * (kCoefRows * 64);

        if (a.states_saved) {
            T *st = static_cast<T *>(a.states_saved) + blk * (2 * DK * DV);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int row = (w * MT + mt) * 16 + kg * 4 + x, col = dv0 + nt * 16 + r;
                        st[row * DV + col] = from_f32<T>(accS[mt][nt][x]);
                        st[DK * DV + row * DV + col] = from_f32<T>(accM[mt][nt][x]);
                    }
        }

        // ---------------- stage 1: V~ and the inter-chunk read-outs for tokens i0..i0+15
        f32x4 accO[NT];
        float vt[NT][4]; // V~ rounded to the storage type
        if (!REBUILD) {
            const T *Ug = static_cast<const T *>(a.U) + blk * (64 * DV) + dv0;
            const T *Yg = static_cast<const T *>(a.nY) + blk * (64 * DK) + i0 * DK;
            const T *Zg = static_cast<const T *>(a.Z) + blk * (64 * DK) + i0 * DK;
            const T *Qg = static_cast<const T *>(a.q) + (tok0 + (size_t)i0 * d.H) * DK;
            f32x4 accV[NT], accOS[NT], accOM[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    accV[nt][x] = to_f32(Ug[(i0 + kg * 4 + x) * DV + nt * 16 + r]);
            zero_acc(accOS);
            zero_acc(accOM);
            const T *yp = Yg + r * DK + kg * O::EPL, *zp = Zg + r * DK + kg * O::EPL;
            const T *qp = Qg + (size_t)r * rsk + kg * O::EPL;
            const T *sp = sSt + r * SM::LDS_ST + kg * O::EPL;
#pragma unroll
            for (int k0 = 0; k0 < DK; k0 += O::KSTEP) {
                const typename O::Frag fy = O::load(yp + k0), fz = O::load(zp + k0), fq = O::load(qp + k0);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const typename O::Frag fs = O::load(sp + nt * 16 * SM::LDS_ST + k0);
                    const typename O::Frag fm = O::load(sp + nt * 16 * SM::LDS_ST + DK + k0);
                    accV[nt] = O::mma(fy, fs, accV[nt]);
                    accV[nt] = O::mma(fz, fm, accV[nt]);
                    accOS[nt] = O::mma(fq, fs, accOS[nt]);
                    accOM[nt] = O::mma(fq, fm, accOM[nt]);
                }
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + kg * 4 + x;
                const float sa = d.scale * coef[COEF_A * 64 + i], sb = d.scale * coef[COEF_B * 64 + i];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    accO[nt][x] = sa * accOS[nt][x] - sb * accOM[nt][x];
                    vt[nt][x] = rounded<T>(accV[nt][x]);
                }
            }
            if (a.vt_saved) {
                T *vs = static_cast<T *>(a.vt_saved) + tok0 * DV + dv0;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        vs[(size_t)(i0 + kg * 4 + x) * rsv + nt * 16 + r] = from_f32<T>(vt[nt][x]);
            }
        } else {
            const T *vs = static_cast<const T *>(a.vt_saved) + tok0 * DV + dv0;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int x = 0; x < 4; ++x) vt[nt][x] = to_f32(vs[(size_t)(i0 + kg * 4 + x) * rsv + nt * 16 + r]);
        }
        // V~ to LDS, transposed, in the three scalings of stage 2
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int i = i0 + kg * 4 + x;
            const float gc = coef[COEF_GC * 64 + i], rc = coef[COEF_RC * 64 + i];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int col = nt * 16 + r;
                if (!REBUILD) sV0[col * SM::LDV + i] = from_f32<T>(vt[nt][x]);
                sVg[col * SM::LDV + i] = from_f32<T>(gc * vt[nt][x]);
                sVr[col * SM::LDV + i] = from_f32<T>(-rc * vt[nt][x]);
            }
        }
        __syncthreads();

        // ---------------- stage 2: intra-chunk output and the state update
        if (!REBUILD) {
            const T *Bg = static_cast<const T *>(a.Bm) + blk * 4096 + i0 * 64;
            mma_rows<T, NT, 64>(accO, Bg, 64, sV0, SM::LDV);
            T *og = static_cast<T *>(a.o) + tok0 * DV + dv0;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    og[(size_t)(i0 + kg * 4 + x) * rsv + nt * 16 + r] = from_f32<T>(accO[nt][x]);
        }
        {
            const float aC = coef[COEF_SCALAR * 64 + 0], bC = coef[COEF_SCALAR * 64 + 1],
                        mC = coef[COEF_SCALAR * 64 + 2];
            const T *KTg = static_cast<const T *>(a.KT) + blk * (DK * 64);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        accS[mt][nt][x] = aC * accS[mt][nt][x] - bC * accM[mt][nt][x];
                        accM[mt][nt][x] = mC * accM[mt][nt][x];
                    }
                const T *Ka = KTg + ((w * MT + mt) * 16) * 64;
                mma_rows<T, NT, 64>(accS[mt], Ka, 64, sVg, SM::LDV);
                mma_rows<T, NT, 64>(accM[mt], Ka, 64, sVr, SM::LDV);
            }
        }
        if (!REBUILD) publish_state<T, DK, NT>(sSt, SM::LDS_ST, accS, accM);
        __syncthreads();
    }

    if (!REBUILD) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int row = (w * MT + mt) * 16 + kg * 4 + x, col = dv0 + nt * 16 + r;
                    const size_t g = ((size_t)bh * DK + row) * DV + col;
                    if (a.S_final) a.S_final[g] = accS[mt][nt][x];
                    if (a.M_final) a.M_final[g] = accM[mt][nt][x];
                }
    }
}

constexpr int kDVB = 32;

template <typename T, int DK, int DV, bool REBUILD>
hipError_t launch_scan_t(const Dims &d, const ScanFwdArgs &a, hipStream_t s) {
    constexpr int G = DV / kDVB;
    dim3 grid(((d.BH + 7) / 8) * 8 * G), block(kThreads);
    hipLaunchKernelGGL((scan_fwd_kernel<T, DK, DV, kDVB, REBUILD>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

template <bool REBUILD> hipError_t dispatch_scan(const Dims &d, const ScanFwdArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64)
        return f32 ? launch_scan_t<float, 64, 64, REBUILD>(d, a, s) : launch_scan_t<bf16_t, 64, 64, REBUILD>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_scan_t<float, 128, 128, REBUILD>(d, a, s)
                   : launch_scan_t<bf16_t, 128, 128, REBUILD>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace

hipError_t launch_scan_fwd(const Dims &d, const ScanFwdArgs &a, hipStream_t s) { return dispatch_scan<false>(d, a, s); }

hipError_t launch_rebuild(const Dims &d, const RebuildArgs &r, hipStream_t s) {
    ScanFwdArgs a = {};
    a.coef = r.coef;
    a.KT = r.KT;
    a.vt_saved = const_cast<void *>(r.vt_saved);
    a.S0 = r.S0;
    a.M0 = r.M0;
    a.states_saved = r.states;
    return dispatch_scan<true>(d, a, s);
}

} // namespace mdn
