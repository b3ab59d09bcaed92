// Reverse inter-chunk scan: adjoint of the forward scan of Sec. 3.1 "Chunkwise Algorithm"
// (the paper keeps V~ for the backward pass, "Practical Considerations", but prints no backward
// equations; these follow from differentiating the chunk formulas).  With dS', dM' the adjoints
// of the chunk-END states, walking the chunks from last to first:
//     dV~ = Bm^T dO + (Gamma_C eta . K) dS' - (Rho_C eta . K) dM'
//     dS  = a_C dS' + (a . Q~)^T dO - Y^T dV~
//     dM  = m_C dM' - b_C dS' - (b . Q~)^T dO + Z^T dV~
// With Y = T diag(a^-) P, Z = T diag(b^-) P, P = alpha K (Sec. 3.1) and dV = T^T dV~ (needed anyway):
//     Y^T dV~ = K^T (a . dV)        (alpha_i a_{i-1} = a_i)
//     Z^T dV~ = K^T (pb . dV)       (pb_i = alpha_i b_{i-1})
// so the transposes of Y and Z are never stored or read: the raw K^T tile and two per-token scalings do.
// Same decomposition as the forward scan: one workgroup per (batch*head, DVB dv-columns); every
// product is formed transposed (dv = MFMA row index) so that an accumulator lane holds 4 consecutive
// dv of one token or one dk row (row 4 kg + x of MFMA tile mv stands for column dv0 + kg*4*MV + 4 mv + x, so that a
// lane's MV tiles are neighbours in HBM and go as one vector); dS'^T, dM'^T in fp32 accumulators (wave w owns dk columns
// [w*dk/4, (w+1)*dk/4)), a storage-type copy in LDS (rows dv, contraction index dk | dk: see ATile) as A operand; the per-token
// scalings along the contraction index folded into the LDS copies of dO^T, so that the B operands
// are raw rows of Q^T, K^T, Bm^T, T^T and K; all of a chunk's fragments, its dO tile and
// coefficients are fetched into registers one chunk ahead.
// dV = T^T dV~ is formed from the LDS copy of dV~, written out, and fed back (scaled) into the state update.
// The chunk-end adjoint states are written for the chunk-parallel gradient kernel.
#include "mdn_device.h"
#include "mdn_kernels.h"

#include <stdlib.h>

namespace mdn {

namespace {

template <typename T, int DK, int MV> struct RevOps {
    typedef Op<T> O;
    static constexpr int KS = DK / O::KSTEP, KS2 = 64 / O::KSTEP, ND = DK / 64;
    typename O::Frag k[KS];            // stage 1: K row (token i0 + r)
    typename O::Frag bmT[KS2];         // stage 1: Bm^T row i0 + r
    typename O::Frag tT[KS2];          // stage 2: T^T row i0 + r
    typename O::Frag qT[ND][KS2], kT[ND][KS2]; // stage 3: rows (dk) of Q^T, K^T for this wave's state columns
    // (kept exactly as loaded: arithmetic on a freshly loaded value would make the wave wait for it, and for
    //  every load issued before it, at fetch time instead of one chunk later)
    typename Raw4<T>::type dO[MV];     // dO[token i0 + r][4 consecutive dv], storage form
    f32x4 c0, c1;                      // the token's coefficient row (COEF_*)
};

// The operands of one chunk are requested in five portions (P = 0..4) spread over the work on the previous chunk: a
// wave that issues them all at once sits at the issue until the memory pipeline has taken them (the time
// to move a chunk's operands into the CU), with its matrix work waiting behind.
template <typename T, int DK, int DV, int DVB, int P>
__device__ __forceinline__ void fetch_part(RevOps<T, DK, DVB / 16> &c, const Dims &d, const ScanBwdArgs &a, int bh, int b,
                                           int h, int n, int dv0) {
    typedef Op<T> O;
    typedef RevOps<T, DK, DVB / 16> CO;
    const int lane = lane_id(), w = wave_id(), r = lane & 15, kg = lane >> 4, i = w * 16 + r;
    // every address is a wave-uniform 64-bit base (chunk, batch, head: scalar arithmetic) plus a 32-bit lane offset that
    // does not change from chunk to chunk (at32: one address register per access, no vector 64-bit adds)
    const size_t blk = (size_t)bh * d.N + n;
    const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h; // the chunk's first token of this head
    const unsigned itok = (unsigned)(i * d.H);                        // this lane's token, in token rows
    if (P == 0) {
        // (through the vector path on purpose: a scalar load would share its wait counter with the LDS reads and
        //  make the first of those wait for memory)
        const float *coef = a.coef + blk * (kCoefRows * 64);
        c.c0 = *reinterpret_cast<const f32x4 *>(at32(coef, (unsigned)(i * kCoefRows)));
        c.c1 = *reinterpret_cast<const f32x4 *>(at32(coef, (unsigned)(i * kCoefRows + 4)));
        load_cols_raw<DVB / 16>(at32(static_cast<const T *>(a.dO) + tok0 * DV + dv0, itok * DV + kg * (DVB / 4)), c.dO);
    }
    if (P == 1) {
        const T *kp = static_cast<const T *>(a.k) + tok0 * DK;
#pragma unroll
        for (int s = 0; s < CO::KS; ++s) c.k[s] = O::load(at32(kp, itok * DK + kg * O::EPL + s * O::KSTEP));
    }
    if (P == 2) {
        const T *bp = static_cast<const T *>(a.BmT) + blk * 4096, *tp = static_cast<const T *>(a.TmT) + blk * 4096;
#pragma unroll
        for (int s = 0; s < CO::KS2; ++s) {
            c.bmT[s] = O::load(at32(bp, (unsigned)kblk<T>(64, i, s * O::KSTEP + kg * O::EPL)));
            c.tT[s] = O::load(at32(tp, (unsigned)kblk<T>(64, i, s * O::KSTEP + kg * O::EPL)));
        }
    }
    if (P == 3 || P == 4) {
        const T *src = static_cast<const T *>(P == 3 ? a.QT : a.KT) + blk * (DK * 64);
#pragma unroll
        for (int nd = 0; nd < CO::ND; ++nd)
#pragma unroll
            for (int s = 0; s < CO::KS2; ++s) {
                const typename O::Frag f =
                    O::load(at32(src, (unsigned)kblk<T>(DK, (w * CO::ND + nd) * 16 + r, s * O::KSTEP + kg * O::EPL)));
                if (P == 3) c.qT[nd][s] = f;
                if (P == 4) c.kT[nd][s] = f;
            }
    }
    __builtin_amdgcn_sched_barrier(0); // the portion leaves here, not where the scheduler would gather the loads
}

template <typename T, int DK, int DV, int DVB>
__device__ __forceinline__ void fetch_chunk(RevOps<T, DK, DVB / 16> &c, const Dims &d, const ScanBwdArgs &a, int bh,
                                            int b, int h, int n, int dv0) {
    fetch_part<T, DK, DV, DVB, 0>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, 1>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, 2>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, 3>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, 4>(c, d, a, bh, b, h, n, dv0);
}

template <typename T, int DK, int DV, int DVB>
__global__ __launch_bounds__(kThreads) void scan_bwd_kernel(Dims d, ScanBwdArgs a) {
    typedef Op<T> O;
    typedef RevOps<T, DK, DVB / 16> CO;
    constexpr int MV = DVB / 16, ND = DK / 64, G = DV / DVB;
    // the A operands that the workgroup builds itself (rows = dv; see ATile for how they sit in LDS)
    typedef ATile<T, DVB, 2 * DK> TD; // contraction over dk: dS' | dM'
    typedef ATile<T, DVB, 64> TV;     // contraction over the chunk's tokens
    __shared__ __align__(16) T sD[TD::SIZE];  // [dv][dS'(dk) | dM'(dk)]
    __shared__ __align__(16) T sO0[TV::SIZE]; // dO^T
    __shared__ __align__(16) T sOa[TV::SIZE]; // (scale a . dO)^T
    __shared__ __align__(16) T sOb[TV::SIZE]; // (-scale b . dO)^T
    __shared__ __align__(16) T sDV[TV::SIZE]; // dV~^T
    __shared__ __align__(16) T sRa[TV::SIZE]; // (-a . dV)^T
    __shared__ __align__(16) T sRb[TV::SIZE]; // (pb . dV)^T

    int bh, blkv;
    xcd_map(blockIdx.x, G, bh, blkv);
    if (bh >= d.BH) return;
    const int b = bh / d.H, h = bh % d.H, dv0 = blkv * DVB;
    const int lane = lane_id(), w = wave_id(), r = lane & 15, kg = lane >> 4, i = w * 16 + r;

    // element x of tile (mv, nd): dS[dk = (w*ND + nd)*16 + r][dv = mv*16 + kg*4 + x]
    f32x4 accS[MV][ND], accM[MV][ND];
#pragma unroll
    for (int mv = 0; mv < MV; ++mv)
#pragma unroll
        for (int nd = 0; nd < ND; ++nd) {
            const size_t g = ((size_t)bh * DK + (w * ND + nd) * 16 + r) * DV + dv0 + kg * (4 * MV) + mv * 4;
            accS[mv][nd] = a.dS_final ? *reinterpret_cast<const f32x4 *>(a.dS_final + g) : f32x4{0.f, 0.f, 0.f, 0.f};
            accM[mv][nd] = a.dM_final ? *reinterpret_cast<const f32x4 *>(a.dM_final + g) : f32x4{0.f, 0.f, 0.f, 0.f};
        }

    // one chunk: the operands of chunk n are in `cur`; those of chunk n-1 go on their way into `nxt`
    auto step = [&](int n, const CO &cur, CO &nxt) {
        const size_t blk = (size_t)bh * d.N + n;
        const int nn = n > d.n0 ? n - 1 : d.n0;
        fetch_part<T, DK, DV, DVB, 0>(nxt, d, a, bh, b, h, nn, dv0);

        // adjoints of this chunk's END states: operand copy to LDS, storage copy to HBM.  (The stores cost this
        // kernel ~45 us whoever issues them and whenever: in one burst here, 208 us; spread over the step in 8
        // portions, 213 us.  All values are narrowed first, so that the stores leave back to back.)
        {
            typename Raw4<T>::type sv[2 * ND][MV];
            T *ds = static_cast<T *>(a.dstates) + blk * (2 * DK * DV);
#pragma unroll
            for (int mv = 0; mv < MV; ++mv)
#pragma unroll
                for (int nd = 0; nd < ND; ++nd) {
                    const int dk = (w * ND + nd) * 16 + r;
                    sv[2 * nd][mv] = narrow4<T>(accS[mv][nd]);
                    sv[2 * nd + 1][mv] = narrow4<T>(accM[mv][nd]);
                    TD::put4_raw(sD, mv * 16 + kg * 4, dk, sv[2 * nd][mv]);
                    TD::put4_raw(sD, mv * 16 + kg * 4, DK + dk, sv[2 * nd + 1][mv]);
                }
#pragma unroll
            for (int nd = 0; nd < ND; ++nd) {
                // (dv0 is a multiple of 16: the workgroup's first column block is part of the uniform base)
                const unsigned off = (unsigned)vblk(DK, (w * ND + nd) * 16 + r, kg * (4 * MV));
                store_cols_raw<MV>(at32(ds + vblk(DK, 0, dv0), off), sv[2 * nd]);
                store_cols_raw<MV>(at32(ds + DK * DV + vblk(DK, 0, dv0), off), sv[2 * nd + 1]);
            }
            if constexpr (sizeof(T) == 2) {
                if (a.dstates_lo) { // what the rounding above dropped, rounded again (see GradArgs)
                    T *dl = static_cast<T *>(a.dstates_lo) + blk * (2 * DK * DV);
#pragma unroll
                    for (int nd = 0; nd < ND; ++nd) {
                        typename Raw4<T>::type ls[MV], lm[MV];
#pragma unroll
                        for (int mv = 0; mv < MV; ++mv) {
                            ls[mv] = narrow4<T>(accS[mv][nd] - widen4_packed(sv[2 * nd][mv]));
                            lm[mv] = narrow4<T>(accM[mv][nd] - widen4_packed(sv[2 * nd + 1][mv]));
                        }
                        const unsigned off = (unsigned)vblk(DK, (w * ND + nd) * 16 + r, kg * (4 * MV));
                        store_cols_raw<MV>(at32(dl + vblk(DK, 0, dv0), off), ls);
                        store_cols_raw<MV>(at32(dl + DK * DV + vblk(DK, 0, dv0), off), lm);
                    }
                }
            }
        }
        fetch_part<T, DK, DV, DVB, 1>(nxt, d, a, bh, b, h, nn, dv0);
        // dO^T slice of this chunk in three scalings
#pragma unroll
        for (int mv = 0; mv < MV; ++mv) {
            const f32x4 dOw = widen4(cur.dO[mv]);
            const float sa = d.scale * cur.c0[COEF_A], sb = d.scale * cur.c0[COEF_B];
            TV::put4_raw(sO0, mv * 16 + kg * 4, i, cur.dO[mv]);
            TV::put4(sOa, mv * 16 + kg * 4, i, sa * dOw);
            TV::put4(sOb, mv * 16 + kg * 4, i, -sb * dOw);
        }
        __syncthreads();

        // ---------------- stage 1: dV~^T for token j = i
        {
            f32x4 accD[MV], x1[MV], x2[MV];
            zero_acc(accD);
            zero_acc(x1);
            zero_acc(x2);
#pragma unroll
            for (int s = 0; s < CO::KS2; ++s)
#pragma unroll
                for (int mv = 0; mv < MV; ++mv)
                    accD[mv] = O::mma(TV::frag(sO0, mv, s * O::KSTEP, r, kg), cur.bmT[s], accD[mv]);
            fetch_part<T, DK, DV, DVB, 2>(nxt, d, a, bh, b, h, nn, dv0);
#pragma unroll
            for (int s = 0; s < CO::KS; ++s)
#pragma unroll
                for (int mv = 0; mv < MV; ++mv) {
                    x1[mv] = O::mma(TD::frag(sD, mv, s * O::KSTEP, r, kg), cur.k[s], x1[mv]);
                    x2[mv] = O::mma(TD::frag(sD, mv, DK + s * O::KSTEP, r, kg), cur.k[s], x2[mv]);
                }
            fetch_part<T, DK, DV, DVB, 3>(nxt, d, a, bh, b, h, nn, dv0);
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) TV::put4(sDV, mv * 16 + kg * 4, i, accD[mv] + cur.c1[COEF_GC - 4] * x1[mv] - cur.c1[COEF_RC - 4] * x2[mv]);
        }
        __syncthreads();

        // ---------------- stage 2: dV = T^T dV~ for token j = i: out to HBM, and back to LDS in the two scalings
        //                  with which it enters the state adjoints
        {
            f32x4 dR[MV];
            zero_acc(dR);
#pragma unroll
            for (int s = 0; s < CO::KS2; ++s)
#pragma unroll
                for (int mv = 0; mv < MV; ++mv)
                    dR[mv] = O::mma(TV::frag(sDV, mv, s * O::KSTEP, r, kg), cur.tT[s], dR[mv]);
            fetch_part<T, DK, DV, DVB, 4>(nxt, d, a, bh, b, h, nn, dv0);
            const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
            store_cols<T, MV>(at32(static_cast<T *>(a.dv) + tok0 * DV + dv0, (unsigned)(i * d.H) * DV + kg * (4 * MV)), dR);
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) {
                TV::put4(sRa, mv * 16 + kg * 4, i, -cur.c0[COEF_A] * dR[mv]);
                TV::put4(sRb, mv * 16 + kg * 4, i, cur.c0[COEF_PB] * dR[mv]);
            }
        }
        __syncthreads();

        // ---------------- stage 3: the adjoints of the chunk-START states
        {
            const float aC = cur.c0[COEF_AC], bC = cur.c1[COEF_BC - 4], mC = cur.c1[COEF_MC - 4];
#pragma unroll
            for (int mv = 0; mv < MV; ++mv)
#pragma unroll
                for (int nd = 0; nd < ND; ++nd) {
                    const f32x4 s = accS[mv][nd], m = accM[mv][nd];
                    accS[mv][nd] = aC * s;
                    accM[mv][nd] = mC * m - bC * s;
                }
#pragma unroll
            for (int s = 0; s < CO::KS2; ++s)
#pragma unroll
                for (int mv = 0; mv < MV; ++mv) {
                    const typename O::Frag fa = TV::frag(sOa, mv, s * O::KSTEP, r, kg);
                    const typename O::Frag fb = TV::frag(sOb, mv, s * O::KSTEP, r, kg);
                    const typename O::Frag fra = TV::frag(sRa, mv, s * O::KSTEP, r, kg);
                    const typename O::Frag frb = TV::frag(sRb, mv, s * O::KSTEP, r, kg);
#pragma unroll
                    for (int nd = 0; nd < ND; ++nd) {
                        accS[mv][nd] = O::mma(fa, cur.qT[nd][s], accS[mv][nd]);
                        accS[mv][nd] = O::mma(fra, cur.kT[nd][s], accS[mv][nd]);
                        accM[mv][nd] = O::mma(fb, cur.qT[nd][s], accM[mv][nd]);
                        accM[mv][nd] = O::mma(frb, cur.kT[nd][s], accM[mv][nd]);
                    }
                }
        }
        __syncthreads();
    };
    // two operand sets used alternately: handing one set over to the other by assignment would touch
    // every register of the set that was just requested, i.e. wait for all of its loads
    {
        CO opsA, opsB;
        fetch_chunk<T, DK, DV, DVB>(opsA, d, a, bh, b, h, d.n1 - 1, dv0);
        int n = d.n1 - 1;
        for (; n >= d.n0 + 1; n -= 2) {
            step(n, opsA, opsB);
            step(n - 1, opsB, opsA);
        }
        if (n == d.n0) step(n, opsA, opsB);
    }

#pragma unroll
    for (int mv = 0; mv < MV; ++mv)
#pragma unroll
        for (int nd = 0; nd < ND; ++nd) {
            const size_t g = ((size_t)bh * DK + (w * ND + nd) * 16 + r) * DV + dv0 + kg * (4 * MV) + mv * 4;
            if (a.dS0) *reinterpret_cast<f32x4 *>(a.dS0 + g) = accS[mv][nd];
            if (a.dM0) *reinterpret_cast<f32x4 *>(a.dM0 + g) = accM[mv][nd];
        }
}

template <typename T, int DK, int DV, int DVB>
hipError_t launch_t(const Dims &d, const ScanBwdArgs &a, hipStream_t s) {
    constexpr int G = DV / DVB;
    dim3 grid(((d.BH + 7) / 8) * 8 * G), block(kThreads);
    static const size_t spread =
        lds_bytes_for_one_workgroup_per_cu(reinterpret_cast<const void *>(&scan_bwd_kernel<T, DK, DV, DVB>));
    const size_t dyn = (int)grid.x <= num_cus() ? spread : 0; // no more workgroups than CUs: one per CU
    hipLaunchKernelGGL((scan_bwd_kernel<T, DK, DV, DVB>), grid, block, dyn, s, d, a);
    return hipGetLastError();
}

template <typename T, int DK, int DV> hipError_t pick_dvb(const Dims &d, const ScanBwdArgs &a, hipStream_t s) {
    if (scan_dvb(d) == 16) return launch_t<T, DK, DV, 16>(d, a, s);
    return launch_t<T, DK, DV, 32>(d, a, s);
}

} // namespace

hipError_t launch_scan_bwd(const Dims &d, const ScanBwdArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (!a.coef || !a.k || !a.dO || !a.BmT || !a.TmT || !a.QT || !a.KT) return hipErrorInvalidValue;
    if (d.dk == 64 && d.dv == 64) return f32 ? pick_dvb<float, 64, 64>(d, a, s) : pick_dvb<bf16_t, 64, 64>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? pick_dvb<float, 128, 128>(d, a, s) : pick_dvb<bf16_t, 128, 128>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
