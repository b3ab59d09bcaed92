// Sequential inter-chunk propagation of the state S and the momentum M (forward), Sec. 3.1
// "Chunkwise Algorithm":
//     V~  = U - Y S + Z M                      with U = T V, Y = T diag(a^-) P, Z = T diag(b^-) P, P = alpha K
//         = T (V - a . (K S) + pb . (K M))     alpha_i a_{i-1} = a_i, pb_i = alpha_i b_{i-1}  (T pulled out:
//                                              U, Y, Z are never formed, the scan applies T itself)
//     O   = diag(a) Q~ S - diag(b) Q~ M + Bm V~
//     S'  = a_C S - b_C M + (diag(Gamma_C) K~)^T V~
//     M'  = m_C M - (diag(Rho_C) K~)^T V~
// Every dv column of S, M, V~, O evolves independently, so one workgroup owns DVB columns of one
// (batch, head) and walks the chunks in order: grid = batch*head x dv/DVB, all workgroups of one
// (batch, head) on the same XCD so that the chunk operands they share are served by one L2.
//
// Inside a workgroup (4 waves) every product is formed TRANSPOSED, with the dv index as the MFMA
// row index: an accumulator lane then holds 4 consecutive dv of one token (or of one dk row), which
// is 8 contiguous bytes of V, V~, O and of the saved states in HBM.  Row m = 4 kg + x of MFMA tile mv stands
// for column dv0 + kg*4*MV + 4 mv + x of the workgroup's DVB = 16 MV columns, so that the MV tiles of a lane
// are neighbours in HBM and go as one vector (16-bit storage, MV = 2: 16 bytes); inside LDS the tiles keep
// their own order (row mv*16 + m), which no one outside the workgroup sees.
//   S^T, M^T live in fp32 accumulators (wave w owns dk columns [w*dk/4, (w+1)*dk/4)); a storage-type
//   copy sits in LDS (rows dv, contraction index dk | dk: see ATile) and is the A operand of the dk-contractions of stage 1a
//   (wave w owns tokens 16w..16w+15): (K S)^T, (K M)^T and the two inter-chunk read-outs.
//   R^T = (V - a.(K S) + pb.(K M))^T goes to LDS (rows dv, contraction index token); stage 1b contracts it over ALL
//   tokens with the wave's rows of T: V~^T, which goes to LDS the same way in three scalings (raw, Gamma_C eta,
//   -Rho_C eta): the A operand of the token-contractions of stage 2 (intra-chunk output, state update).
//   Scalings along a contraction index are folded into those copies, so the B operands are raw rows of
//   K, Q, T, Bm, K^T straight from HBM.
// Three barriers per chunk.  Nothing a chunk reads from HBM depends on the state, so all of a chunk's
// fragments, its V tile and its coefficients are requested one whole chunk ahead; the serial chain then
// only waits on LDS and MFMA latency.
#include "mdn_device.h"
#include "mdn_kernels.h"

#include <stdlib.h>

namespace mdn {

namespace {

static_assert(kCoefRows == kCoefBlockCols, "device-side and host-side view of the coefficient block");

// Operands of one chunk held by one lane.
template <typename T, int DK, int MV> struct ChunkOps {
    typedef Op<T> O;
    static constexpr int KS = DK / O::KSTEP, KS2 = 64 / O::KSTEP, ND = DK / 64;
    typename O::Frag kr[KS];              // stage 1: rows (token i0 + r) of K (32-bit storage)
    typename O::Frag q[KS];               // stage 1: rows of Q
    typename O::Frag tm[KS2];             // stage 1: row i0 + r of T = (I + A)^-1
    typename O::Frag bm[KS2];             // stage 2: Bm row i0 + r
    typename O::Frag kt[ND][KS2];         // stage 2: K^T rows (dk) of this wave's state columns (32-bit storage)
    // (everything here is kept exactly as loaded: arithmetic on a freshly loaded value would make the wave wait
    //  for it, and for every load issued before it, at fetch time instead of one chunk later)
    typename Raw4<T>::type u[MV];         // V[token i0 + r][4 MV consecutive dv] (V~ in reconstruction), storage form
    f32x4 c0, c1;                         // the token's coefficient row (COEF_*)
};

// The operands of one chunk are requested in portions (P = 0..4) spread over the work on the previous
// chunk: a wave that issues them all at once sits at the issue until the memory pipeline has taken them
// (the time to move a chunk's operands into the CU), with its matrix work waiting behind.
template <typename T, int DK, int DV, int DVB, bool REBUILD, int P, bool KTILE>
__device__ __forceinline__ void fetch_part(ChunkOps<T, DK, DVB / 16> &c, const Dims &d, const ScanFwdArgs &a, int bh,
                                           int b, int h, int n, int dv0) {
    typedef Op<T> O;
    typedef ChunkOps<T, DK, DVB / 16> CO;
    const int lane = lane_id(), w = wave_id() & 3, r = lane & 15, kg = lane >> 4, i = w * 16 + r;
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
        // the forward reads V, the reconstruction the saved V~
        const T *vs = static_cast<const T *>(REBUILD ? a.vt_saved : a.v) + tok0 * DV + dv0;
        load_cols_raw<DVB / 16>(at32(vs, itok * DV + kg * (DVB / 4)), c.u);
    }
    if (P == 1 && !REBUILD) {
        const T *Qg = static_cast<const T *>(a.q) + tok0 * DK;
#pragma unroll
        for (int s = 0; s < CO::KS; ++s) c.q[s] = O::load(at32(Qg, itok * DK + kg * O::EPL + s * O::KSTEP));
    }
    if (P == 2 && !KTILE) {
        const T *KTg = static_cast<const T *>(a.KT) + blk * (DK * 64);
#pragma unroll
        for (int nd = 0; nd < CO::ND; ++nd)
#pragma unroll
            for (int s = 0; s < CO::KS2; ++s)
                c.kt[nd][s] = O::load(at32(KTg, (unsigned)kblk<T>(DK, (w * CO::ND + nd) * 16 + r, s * O::KSTEP + kg * O::EPL)));
    }
    if (P == 3 && !REBUILD) {
        const T *Bg = static_cast<const T *>(a.Bm) + blk * 4096, *Tg = static_cast<const T *>(a.Tm) + blk * 4096;
#pragma unroll
        for (int s = 0; s < CO::KS2; ++s) {
            c.tm[s] = O::load(at32(Tg, (unsigned)kblk<T>(64, i, s * O::KSTEP + kg * O::EPL)));
            c.bm[s] = O::load(at32(Bg, (unsigned)kblk<T>(64, i, s * O::KSTEP + kg * O::EPL)));
        }
    }
    if (P == 4 && !REBUILD && !KTILE) {
        const T *Kg = static_cast<const T *>(a.k) + tok0 * DK;
#pragma unroll
        for (int s = 0; s < CO::KS; ++s) c.kr[s] = O::load(at32(Kg, itok * DK + kg * O::EPL + s * O::KSTEP));
    }
    __builtin_amdgcn_sched_barrier(0); // the portion leaves here, not where the scheduler would gather the loads
}

template <typename T, int DK, int DV, int DVB, bool REBUILD, bool KTILE>
__device__ __forceinline__ void fetch_chunk(ChunkOps<T, DK, DVB / 16> &c, const Dims &d, const ScanFwdArgs &a,
                                            int bh, int b, int h, int n, int dv0) {
    fetch_part<T, DK, DV, DVB, REBUILD, 0, KTILE>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, REBUILD, 4, KTILE>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, REBUILD, 1, KTILE>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, REBUILD, 3, KTILE>(c, d, a, bh, b, h, n, dv0);
    fetch_part<T, DK, DV, DVB, REBUILD, 2, KTILE>(c, d, a, bh, b, h, n, dv0);
}

// accumulator element x of tile (mv, nd) of wave w is S[dk = (w*ND + nd)*16 + r][dv = mv*16 + kg*4 + x]
template <typename T, int DK, int MV>
__device__ __forceinline__ void publish_state(T *sSt, const f32x4 (&accS)[MV][DK / 64], const f32x4 (&accM)[MV][DK / 64]) {
    typedef ATile<T, MV * 16, 2 * DK> TS;
    const int r = lane_id() & 15, kg = lane_id() >> 4, w = wave_id();
#pragma unroll
    for (int mv = 0; mv < MV; ++mv)
#pragma unroll
        for (int nd = 0; nd < DK / 64; ++nd) {
            const int dk = (w * (DK / 64) + nd) * 16 + r;
            TS::put4(sSt, mv * 16 + kg * 4, dk, accS[mv][nd]);
            TS::put4(sSt, mv * 16 + kg * 4, DK + dk, accM[mv][nd]);
        }
}

// REBUILD = false: full forward scan.  REBUILD = true: state reconstruction from saved V~ only
// (the update lines), writing the chunk-start states.
template <typename T, int DK, int DV, int DVB, bool REBUILD>
__global__ __launch_bounds__(kThreads) void scan_fwd_kernel(Dims d, ScanFwdArgs a) {
    typedef Op<T> O;
    typedef ChunkOps<T, DK, DVB / 16> CO;
    constexpr int MV = DVB / 16, ND = DK / 64, G = DV / DVB;
    // the A operands that the workgroup builds itself (rows = dv; see ATile for how they sit in LDS)
    typedef ATile<T, DVB, 2 * DK> TS; // state copy, contraction over dk: S | M
    typedef ATile<T, DVB, 64> TV;     // contraction over the chunk's tokens
    __shared__ __align__(16) T sSt[TS::SIZE];
    __shared__ __align__(16) T sRt[REBUILD ? 8 : TV::SIZE]; // R^T = (V - a.(K S) + pb.(K M))^T, all 64 tokens
    __shared__ __align__(16) T sV0[TV::SIZE];
    __shared__ __align__(16) T sVg[TV::SIZE];
    __shared__ __align__(16) T sVr[TV::SIZE];
    // 16-bit storage, full scan: the chunk's k rows come into LDS once (three chunks in flight) and serve both as
    // rows (stage 1) and, through transposing reads, as K^T (stage 2): as fast as reading both from HBM into
    // registers, and K^T need not exist for it.  (The reconstruction, which needs K^T alone, is faster with the K^T
    // tile from HBM: 128 against 148 us; so is the reverse scan with K, K^T, Q^T from HBM: 203 against 224 us with
    // k and q tiles in LDS.)  32-bit storage reads the rows and the K^T tile from HBM.
    constexpr bool KTILE = sizeof(T) == 2 && !REBUILD;
    __shared__ __align__(16) T sKr[KTILE ? 3 * 64 * DK : 8];

    int bh, blkv;
    xcd_map(blockIdx.x, G, bh, blkv);
    if (bh >= d.BH) return;
    const int b = bh / d.H, h = bh % d.H, dv0 = blkv * DVB;
    const int lane = lane_id(), w = wave_id(), r = lane & 15, kg = lane >> 4, i = w * 16 + r;

    // k rows of chunk n into ring slot `slot`
    auto request_k = [&](int n, int slot) {
        if constexpr (KTILE) {
            const T *kg0 = static_cast<const T *>(a.k) + (((size_t)b * d.T + (size_t)n * 64) * d.H + h) * DK;
            dma_token_tile<T, DK, 4>(sKr + slot * (64 * DK), kg0, (unsigned)(d.H * DK), __builtin_amdgcn_readfirstlane(w), lane);
        }
    };
    request_k(d.n0, 0);
    request_k(d.n0 + 1 < d.n1 ? d.n0 + 1 : d.n0, 1);

    f32x4 accS[MV][ND], accM[MV][ND];
#pragma unroll
    for (int mv = 0; mv < MV; ++mv)
#pragma unroll
        for (int nd = 0; nd < ND; ++nd) {
            const size_t g = ((size_t)bh * DK + (w * ND + nd) * 16 + r) * DV + dv0 + kg * (4 * MV) + mv * 4;
            accS[mv][nd] = a.S0 ? *reinterpret_cast<const f32x4 *>(a.S0 + g) : f32x4{0.f, 0.f, 0.f, 0.f};
            accM[mv][nd] = a.M0 ? *reinterpret_cast<const f32x4 *>(a.M0 + g) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
    if (!REBUILD) publish_state<T, DK, MV>(sSt, accS, accM);
    if (KTILE) __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): this wave's part of the first two k tiles has landed
    __syncthreads();

    // The chunk-start states leave for HBM out of a storage-type copy in registers.  Forward scan: narrowed ONCE at
    // the end of the step that produced them, for the LDS copy and for HBM alike (one burst; the stores cost this
    // kernel ~75 us whichever wave issues them and whenever).  Reconstruction, which does little else than store:
    // in 8 portions spread over the step (109 against 127 us in one burst).
    constexpr int NS = 2 * ND; // vector stores per lane: S and M, ND rows, MV * 4 consecutive columns each
    constexpr bool LO = sizeof(T) == 2;
    typename Raw4<T>::type sv[NS][MV];
    typename Raw4<T>::type sl[LO ? NS : 1][MV];
    // sv: the states in storage form; sl: what that rounding dropped, rounded again (16-bit storage, on request: the
    // reconstruction of a backward call that brings state adjoints in, and the forward of a packed batch of prompts,
    // whose sequences' final states start from these chunk-start states)
    auto narrow_states = [&]() {
#pragma unroll
        for (int nd = 0; nd < ND; ++nd)
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) {
                sv[2 * nd][mv] = narrow4<T>(accS[mv][nd]);
                sv[2 * nd + 1][mv] = narrow4<T>(accM[mv][nd]);
            }
        if constexpr (LO) {
            if (a.states_lo) {
#pragma unroll
                for (int nd = 0; nd < ND; ++nd)
#pragma unroll
                    for (int mv = 0; mv < MV; ++mv) {
                        sl[2 * nd][mv] = narrow4<T>(accS[mv][nd] - widen4_packed(sv[2 * nd][mv]));
                        sl[2 * nd + 1][mv] = narrow4<T>(accM[mv][nd] - widen4_packed(sv[2 * nd + 1][mv]));
                    }
            }
        }
    };
    // portion PORTION of the stores of sv (and sl) as the start states of chunk block sblk
    size_t sblk = 0;
    auto emit_states = [&](auto PORTION) {
        if (!a.states_saved) return;
        T *st = static_cast<T *>(a.states_saved) + sblk * (2 * DK * DV);
        T *stl = static_cast<T *>(a.states_lo) + sblk * (2 * DK * DV);
        static_for<NS>([&](auto IDX) {
            constexpr int idx = decltype(IDX)::value, nd = idx >> 1;
            if ((REBUILD ? idx * 8 / NS : 0) == decltype(PORTION)::value) {
                // (dv0 is a multiple of 16: the workgroup's first column block is part of the uniform base)
                const unsigned off = (unsigned)vblk(DK, (w * ND + nd) * 16 + r, kg * (4 * MV));
                const size_t base = ((idx & 1) ? DK * DV : 0) + vblk(DK, 0, dv0);
                store_cols_raw<MV>(at32(st + base, off), sv[idx]);
                if constexpr (LO) {
                    if (a.states_lo) store_cols_raw<MV>(at32(stl + base, off), sl[idx]);
                }
            }
        });
        __builtin_amdgcn_sched_barrier(0);
    };
    // one chunk: its operands are in `cur`; those of the next chunk go on their way into `nxt`, portion by portion.
    // The k tile of chunk n+2 is requested first of all; each wave waits for its part of that transfer before the
    // first barrier of the NEXT step (see the wait there), and that step's barriers publish the tile before chunk
    // n+2 begins.
    if constexpr (!REBUILD) {
        if (a.states_saved) { // the start states of the first chunk: what came in
            narrow_states();
            sblk = (size_t)bh * d.N + d.n0;
            emit_states(std::integral_constant<int, 0>{});
        }
    }
    int slot = 0;
    auto step = [&](int n, const CO &cur, CO &nxt) {
        const size_t blk = (size_t)bh * d.N + n;
        const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h; // (uniform base + 32-bit lane offset, as in fetch_part)
        const unsigned itok = (unsigned)(i * d.H);
        const int nn = (n + 1 < d.n1) ? n + 1 : n;
        const T *kc = sKr + slot * (64 * DK);
        if (n + 2 < d.n1) request_k(n + 2, slot >= 1 ? slot - 1 : 2);
        slot = slot == 2 ? 0 : slot + 1;
        fetch_part<T, DK, DV, DVB, REBUILD, 0, KTILE>(nxt, d, a, bh, b, h, nn, dv0);

        sblk = blk;
        auto emit_in_step = [&](auto PORTION) {
            if constexpr (REBUILD) emit_states(PORTION);
        };
        if constexpr (REBUILD) {
            if (a.states_saved) narrow_states();
        }
        emit_in_step(std::integral_constant<int, 0>{});

        fetch_part<T, DK, DV, DVB, REBUILD, 4, KTILE>(nxt, d, a, bh, b, h, nn, dv0);
        emit_in_step(std::integral_constant<int, 1>{});
        // ---------------- stage 1: R^T = (V - a.(K S) + pb.(K M))^T and the inter-chunk read-outs for token i,
        //                  then V~^T = R^T T^T over all 64 tokens
        f32x4 accO[MV], vt[MV]; // vt = V~ rounded to the storage type
        typename Raw4<T>::type vb[MV]; // (the same in storage form: narrowed once, for HBM, for LDS and for vt)
        if (!REBUILD) {
            f32x4 x1[MV], x2[MV], accOS[MV], accOM[MV];
            zero_acc(x1);
            zero_acc(x2);
            zero_acc(accOS);
            zero_acc(accOM);
#pragma unroll
            for (int s = 0; s < CO::KS; ++s) {
                typename O::Frag fk;
                if constexpr (KTILE) fk = token_tile_row_frag<DK>(kc, i, s, kg);
                else fk = cur.kr[s];
#pragma unroll
                for (int mv = 0; mv < MV; ++mv) {
                    const typename O::Frag fs = TS::frag(sSt, mv, s * O::KSTEP, r, kg);
                    const typename O::Frag fm = TS::frag(sSt, mv, DK + s * O::KSTEP, r, kg);
                    x1[mv] = O::mma(fs, fk, x1[mv]);
                    accOS[mv] = O::mma(fs, cur.q[s], accOS[mv]);
                    x2[mv] = O::mma(fm, fk, x2[mv]);
                    accOM[mv] = O::mma(fm, cur.q[s], accOM[mv]);
                }
            }
            fetch_part<T, DK, DV, DVB, REBUILD, 1, KTILE>(nxt, d, a, bh, b, h, nn, dv0);
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) {
                accO[mv] = d.scale * (cur.c0[COEF_A] * accOS[mv] - cur.c0[COEF_B] * accOM[mv]);
                TV::put4(sRt, mv * 16 + kg * 4, i, widen4(cur.u[mv]) - cur.c0[COEF_A] * x1[mv] + cur.c0[COEF_PB] * x2[mv]);
            }
            if constexpr (KTILE) {
                // This wave's part of the k tile requested at the start of the PREVIOUS step has landed: at least
                // AFTER vector-memory instructions were issued behind it (previous step: coefficients and V 3, q KS,
                // T and Bm 4, o 1; this step: coefficients and V 3, q KS; more with the optional stores and the next
                // tile's request), they complete in order, and no more than AFTER of them are younger than this
                // step's own requests (the tile's D/32, 3, the 2 ND state stores, KS) -- so the wait never holds a
                // wave for a load it has only just issued.
                constexpr int AFTER = 11 + 2 * CO::KS;
                static_assert(AFTER <= 63 && DK / 32 + 3 + 2 * ND + CO::KS <= AFTER, "vmcnt immediate");
                __builtin_amdgcn_s_waitcnt(0x0F70 | (AFTER & 15) | ((AFTER >> 4) << 14));
            }
            __syncthreads();
            f32x4 accV[MV];
            zero_acc(accV);
#pragma unroll
            for (int s = 0; s < CO::KS2; ++s)
#pragma unroll
                for (int mv = 0; mv < MV; ++mv)
                    accV[mv] = O::mma(TV::frag(sRt, mv, s * O::KSTEP, r, kg), cur.tm[s], accV[mv]);
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) {
                vb[mv] = narrow4<T>(accV[mv]);
                vt[mv] = widen4_packed(vb[mv]);
            }
            if (a.vt_saved) {
                store_cols_raw<MV>(at32(static_cast<T *>(a.vt_saved) + tok0 * DV + dv0, itok * DV + kg * (4 * MV)), vb);
            }
        } else {
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) {
                vb[mv] = cur.u[mv];
                vt[mv] = widen4(cur.u[mv]);
            }
        }
        emit_in_step(std::integral_constant<int, 2>{});
        // V~^T to LDS in the three scalings of stage 2
#pragma unroll
        for (int mv = 0; mv < MV; ++mv) {
            if (!REBUILD) TV::put4_raw(sV0, mv * 16 + kg * 4, i, vb[mv]);
            TV::put4(sVg, mv * 16 + kg * 4, i, cur.c1[COEF_GC - 4] * vt[mv]);
            TV::put4(sVr, mv * 16 + kg * 4, i, -cur.c1[COEF_RC - 4] * vt[mv]);
        }
        emit_in_step(std::integral_constant<int, 3>{});
        __syncthreads();

        // ---------------- stage 2: intra-chunk output and the state update
        fetch_part<T, DK, DV, DVB, REBUILD, 2, KTILE>(nxt, d, a, bh, b, h, nn, dv0);
        emit_in_step(std::integral_constant<int, 4>{});
        const float aC = cur.c0[COEF_AC], bC = cur.c1[COEF_BC - 4], mC = cur.c1[COEF_MC - 4];
#pragma unroll
        for (int mv = 0; mv < MV; ++mv)
#pragma unroll
            for (int nd = 0; nd < ND; ++nd) {
                accS[mv][nd] = aC * accS[mv][nd] - bC * accM[mv][nd];
                accM[mv][nd] = mC * accM[mv][nd];
            }
#pragma unroll
        for (int s = 0; s < CO::KS2; ++s) {
            typename O::Frag fkt[ND];
#pragma unroll
            for (int nd = 0; nd < ND; ++nd) {
                if constexpr (KTILE) fkt[nd] = token_tile_col_frag<DK>(kc, w * ND + nd, s, r, kg);
                else fkt[nd] = cur.kt[nd][s];
            }
#pragma unroll
            for (int mv = 0; mv < MV; ++mv) {
                const typename O::Frag fg = TV::frag(sVg, mv, s * O::KSTEP, r, kg);
                const typename O::Frag fr = TV::frag(sVr, mv, s * O::KSTEP, r, kg);
#pragma unroll
                for (int nd = 0; nd < ND; ++nd) {
                    accS[mv][nd] = O::mma(fg, fkt[nd], accS[mv][nd]);
                    accM[mv][nd] = O::mma(fr, fkt[nd], accM[mv][nd]);
                }
                if (!REBUILD) {
                    accO[mv] = O::mma(TV::frag(sV0, mv, s * O::KSTEP, r, kg), cur.bm[s], accO[mv]);
                }
            }
        }
        emit_in_step(std::integral_constant<int, 5>{});
        fetch_part<T, DK, DV, DVB, REBUILD, 3, KTILE>(nxt, d, a, bh, b, h, nn, dv0);
        emit_in_step(std::integral_constant<int, 6>{});
        if constexpr (!REBUILD) {
            // the states after this chunk, narrowed once: the LDS copy for the next chunk's stage 1 and, in HBM, that
            // chunk's start states
            narrow_states();
#pragma unroll
            for (int mv = 0; mv < MV; ++mv)
#pragma unroll
                for (int nd = 0; nd < ND; ++nd) {
                    const int dk = (w * ND + nd) * 16 + r;
                    TS::put4_raw(sSt, mv * 16 + kg * 4, dk, sv[2 * nd][mv]);
                    TS::put4_raw(sSt, mv * 16 + kg * 4, DK + dk, sv[2 * nd + 1][mv]);
                }
            if (n + 1 < d.n1) {
                sblk = blk + 1;
                emit_states(std::integral_constant<int, 0>{});
            }
            store_cols<T, MV>(at32(static_cast<T *>(a.o) + tok0 * DV + dv0, itok * DV + kg * (4 * MV)), accO);
        }
        emit_in_step(std::integral_constant<int, 7>{});
        __syncthreads();
    };
    // two operand sets used alternately: handing one set over to the other by assignment would touch every
    // register of the set that was just requested, i.e. wait for all of its loads
    {
        CO opsA, opsB;
        fetch_chunk<T, DK, DV, DVB, REBUILD, KTILE>(opsA, d, a, bh, b, h, d.n0, dv0);
        int n = d.n0;
        for (; n + 1 < d.n1; n += 2) {
            step(n, opsA, opsB);
            step(n + 1, opsB, opsA);
        }
        if (n < d.n1) step(n, opsA, opsB);
    }

#pragma unroll
    for (int mv = 0; mv < MV; ++mv)
#pragma unroll
        for (int nd = 0; nd < ND; ++nd) {
            const size_t g = ((size_t)bh * DK + (w * ND + nd) * 16 + r) * DV + dv0 + kg * (4 * MV) + mv * 4;
            if (a.S_final) *reinterpret_cast<f32x4 *>(a.S_final + g) = accS[mv][nd];
            if (a.M_final) *reinterpret_cast<f32x4 *>(a.M_final + g) = accM[mv][nd];
        }
}


template <typename T, int DK, int DV, int DVB, bool REBUILD>
hipError_t launch_scan_t(const Dims &d, const ScanFwdArgs &a, hipStream_t s) {
    constexpr int G = DV / DVB;
    dim3 grid(((d.BH + 7) / 8) * 8 * G), block(kThreads);
    static const size_t spread = lds_bytes_for_one_workgroup_per_cu(
        reinterpret_cast<const void *>(&scan_fwd_kernel<T, DK, DV, DVB, REBUILD>));
    const size_t dyn = (int)grid.x <= num_cus() ? spread : 0; // no more workgroups than CUs: one per CU
    hipLaunchKernelGGL((scan_fwd_kernel<T, DK, DV, DVB, REBUILD>), grid, block, dyn, s, d, a);
    return hipGetLastError();
}

template <typename T, int DK, int DV, bool REBUILD>
hipError_t pick_dvb(const Dims &d, const ScanFwdArgs &a, hipStream_t s) {
    if (scan_dvb(d) == 16) return launch_scan_t<T, DK, DV, 16, REBUILD>(d, a, s);
    return launch_scan_t<T, DK, DV, 32, REBUILD>(d, a, s);
}

template <bool REBUILD> hipError_t dispatch_scan(const Dims &d, const ScanFwdArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (!a.coef || !a.k || ((f32 || REBUILD) && !a.KT)) return hipErrorInvalidValue;
    if (d.dk == 64 && d.dv == 64)
        return f32 ? pick_dvb<float, 64, 64, REBUILD>(d, a, s) : pick_dvb<bf16_t, 64, 64, REBUILD>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? pick_dvb<float, 128, 128, REBUILD>(d, a, s) : pick_dvb<bf16_t, 128, 128, REBUILD>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace

int num_cus() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
            v = 256;
        return v;
    }();
    return n;
}

int scan_dvb(const Dims &d) {
    const bool f32 = d.dtype == 1;
    return (4 * d.BH * (d.dv / 32) < 3 * num_cus() || (f32 && d.dk == 128)) ? 16 : 32;
}

int scan_workgroups(const Dims &d) { return (d.BH + 7) / 8 * 8 * (d.dv / scan_dvb(d)); }

size_t lds_bytes_for_one_workgroup_per_cu(const void *kernel) {
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, kernel) != hipSuccess) return 0;
    const size_t half = 80 * 1024, want = half + 1024; // two workgroups of more than 80 KB do not fit the 160 KB of a CU
    return fa.sharedSizeBytes > half ? 0 : want - fa.sharedSizeBytes;
}

hipError_t launch_scan_fwd(const Dims &d, const ScanFwdArgs &a, hipStream_t s) { return dispatch_scan<false>(d, a, s); }

bool scan_fwd_reads_KT(const Dims &d) { return d.dtype == 1; }

hipError_t launch_rebuild(const Dims &d, const RebuildArgs &r, hipStream_t s) {
    ScanFwdArgs a = {};
    a.coef = r.coef;
    a.k = r.k;
    a.KT = r.KT;
    a.vt_saved = const_cast<void *>(r.vt_saved);
    a.S0 = r.S0;
    a.M0 = r.M0;
    a.states_saved = r.states;
    a.states_lo = r.states_lo;
    a.S_final = r.S_final;
    a.M_final = r.M_final;
    return dispatch_scan<true>(d, a, s);
}

} // namespace mdn
