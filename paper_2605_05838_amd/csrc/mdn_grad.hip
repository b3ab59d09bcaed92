// Chunk-parallel gradient kernel: everything of the backward pass that is not on the serial
// chain.  The paper gives no backward equations ("Practical Considerations" of Sec. 3.1 only says
// the states are reconstructed from V~); the formulas below are the reverse-mode adjoint of the
// chunk formulas of Sec. 3.1 / Appendix C, with S, M the chunk-START states, dS', dM' the adjoints
// of the chunk-END states, dV~ from the reverse scan, K~ = eta k, P = alpha k, Q~ = scale q:
//
//   dR  = T^T dV~   (= dV, formed by the reverse scan)   dBm = tril(dO V~^T)   dA = -tril_strict(dR V~^T)
//   W1  = dBm .* Gamma                  W2  = dA .* Gamma^-
//   dQ~ = W1 K~ + a.(dO S^T) - b.(dO M^T)
//   dK~ = W1^T Q~ + W2^T P + Gamma_C.(V~ dS'^T) - Rho_C.(V~ dM'^T)
//   dP  = W2 K~ - a^-.(dR S^T) + b^-.(dR M^T)
//   dq = scale dQ~,  dk = eta dK~ + alpha dP,  deta_i = k_i.dK~_i,  dalpha_i += k_i.dP_i
//   coefficient adjoints: da_i = Q~_i.(S dO_i), db_i = -Q~_i.(M dO_i), da^-_i = -P_i.(S dR_i),
//   db^-_i = P_i.(M dR_i), da_C += <dS',S>, db_C -= <dS',M>, dm_C = <dM',M>,
//   dGamma = dBm .* (Q~K~^T), dGamma^- = dA .* (P K~^T), dGamma_{C,j} += K~_j.(dS' V~_j),
//   dRho_{C,j} -= K~_j.(dM' V~_j); then the reverse of the coefficient scans
//   a_i = alpha_i a_{i-1}, m_i = mu_i m_{i-1}, Rho_ij = mu_i Rho_{i-1,j},
//   b_i = alpha_i b_{i-1} + beta_i m_i, Gamma_ij = alpha_i Gamma_{i-1,j} + beta_i Rho_ij.
//
// One workgroup (8 waves) per (chunk, batch*head).  A wave owns 16 tokens and half of the dk (or j)
// tiles of every product, and every product is formed transposed, tokens as the MFMA column index: the operands all waves share
// (V~, K, K^T, Q^T, S, M, dS', dM') are the A operands and go through one LDS staging buffer,
// tile after tile, each fetched from HBM with coalesced 16-byte loads while the previous tile is
// being consumed; the wave's own rows of dO, dR, V~, q, k are B fragments held in registers.
// An accumulator lane then holds 4 consecutive dk of one token: dq, dk leave as 8-byte stores and
// the row dots against q, k need two shuffles.  (fp32 storage does not fit the staging buffer in
// LDS: it reads the shared operands straight from HBM/L2 with the same code.)
#include "mdn_coef.h"
#include "mdn_device.h"
#include "mdn_kernels.h"

#include <type_traits>

namespace mdn {

namespace {

constexpr int LDG = 65; // row stride of the fp32 64x64 coefficient matrices in LDS
constexpr int GT = 512;  // threads per workgroup: 8 waves = 4 token tiles x 2 halves of the dk (or j) tiles

// sum over the 4 lanes (kg = 0..3) that hold the same token column r
__device__ __forceinline__ float reduce_kg(float v) {
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// sum over dk of t^T[dk][i] * X[i][dk] for this lane's token; t tile mt holds dk = mt*16 + kg*4 + x
template <int NK> __device__ __forceinline__ float coldot(const f32x4 (&t)[NK], const f32x4 (&xv)[NK]) {
    float s = 0.f;
#pragma unroll
    for (int mt = 0; mt < NK; ++mt)
#pragma unroll
        for (int x = 0; x < 4; ++x) s += t[mt][x] * xv[mt][x];
    return reduce_kg(s);
}

template <typename T, int DK, int DV, bool STAGED>
__global__ __launch_bounds__(GT) void grad_kernel(Dims d, GradArgs a) {
    typedef Op<T> O;
    typedef typename O::Frag Frag;
    constexpr int E = O::EPL;
    constexpr int LDW = 64 + O::PAD, LDNV = DV + O::PAD, LDNK = DK + O::PAD;
    constexpr int NK = DK / 16, KSV = DV / O::KSTEP, KSK = DK / O::KSTEP, KS2 = 64 / O::KSTEP;
    constexpr int NAT_ELEMS = 64 * LDNV + 64 * LDNK, BLK_ELEMS = 2 * DK * 64, ST_ELEMS = DK * DV;
    constexpr int SB_ELEMS0 = NAT_ELEMS > BLK_ELEMS ? NAT_ELEMS : BLK_ELEMS;
    constexpr int SB_ELEMS = STAGED ? (SB_ELEMS0 > ST_ELEMS ? SB_ELEMS0 : ST_ELEMS) : 8;
    // 16-byte vectors per thread of each staged tile
    constexpr int NV_V = 64 * DV / E / GT, NV_K = 64 * DK / E / GT, NV_B = DK * 64 / E / GT, NV_S = DK * DV / E / GT;
    constexpr int NH = NK / 2; // dk tiles per wave
    constexpr int NREG0 = (NV_V + NV_K) > 2 * NV_B ? (NV_V + NV_K) : 2 * NV_B;
    constexpr int NREG = NREG0 > NV_S ? NREG0 : NV_S;

    __shared__ float sG[64 * LDG];     // Gamma
    __shared__ float sRho[64 * LDG];   // Rho
    __shared__ float sDG1[64 * LDG];   // direct dGamma from Bm
    __shared__ float sDG2[65 * LDG];   // direct dGamma^- (row i here belongs to Gamma row i-1)
    __shared__ __align__(16) T sW[4 * 64 * LDW];
    T *sW1e = sW;                 // W1 . eta_j         [i][j]
    T *sW2e = sW + 64 * LDW;      // W2 . eta_j         [i][j]
    T *sW1T = sW + 2 * 64 * LDW;  // scale W1^T         [j][i]
    T *sW2T = sW + 3 * 64 * LDW;  // (W2 . alpha_i)^T   [j][i]
    // after the W products: accumulated adjoints of Gamma and Rho
    float *sGa = reinterpret_cast<float *>(sW), *sRa = sGa + 64 * LDG;
    static_assert(sizeof(T) * 4 * 64 * LDW >= sizeof(float) * 2 * 64 * LDG, "adjoint matrices do not fit the W space");
    __shared__ __align__(16) T sB[SB_ELEMS];   // staging buffer of the shared operands
    __shared__ float s_al[64], s_et[64], s_a[64], s_b[64];
    // row dots come in two halves (one per dk half): [hf][token]
    __shared__ float s_da[2][64], s_db[2][64], s_dam[2][64], s_dbm[2][64], s_dgc[2][64], s_drc[2][64], s_dalk[2][64], s_detk[2][64];
    __shared__ float s_gC[64], s_rC[64];
    __shared__ float s_ga[64], s_gb[64], s_gm[64];
    __shared__ float s_red[8][3];

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id(), r = lane & 15, kg = lane >> 4;
    const int wt = w & 3, hf = w >> 2;
    const int i = wt * 16 + r; // this lane's token (MFMA column)
    const int n = blockIdx.x, bh = blockIdx.y, b = bh / d.H, h = bh % d.H;
    const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
    const size_t blk = (size_t)bh * d.N + n;
    const size_t rsk = (size_t)d.H * DK, rsv = (size_t)d.H * DV;
    const T *qg = static_cast<const T *>(a.q) + tok0 * DK;
    const T *kgl = static_cast<const T *>(a.k) + tok0 * DK;
    const T *vtg = static_cast<const T *>(a.vt_saved) + tok0 * DV;
    const T *dog = static_cast<const T *>(a.dO) + tok0 * DV;
    const T *drg = static_cast<const T *>(a.dv) + tok0 * DV; // dR = T^T dV~ (= dV), from the reverse scan
    const T *KTg = static_cast<const T *>(a.KT) + blk * (DK * 64);
    const T *QTg = static_cast<const T *>(a.QT) + blk * (DK * 64);
    const T *Sg = static_cast<const T *>(a.states) + blk * (2 * DK * DV), *Mg = Sg + DK * DV;
    const T *dSg = static_cast<const T *>(a.dstates) + blk * (2 * DK * DV), *dMg = dSg + DK * DV;

    // ---- cooperative tile movement: HBM -> registers (issue), registers -> LDS (commit)
    Vec16<T> P[NREG], Q[NREG];
    auto issue_natural = [&](Vec16<T> *dst, const T *src, size_t rs, auto D_, auto NV_) {
        // [64][D] rows of the chunk; D/E vectors per row
        constexpr int cpr = decltype(D_)::value / E;
#pragma unroll
        for (int u = 0; u < decltype(NV_)::value; ++u) {
            const int c = tid + u * GT, row = c / cpr, cc = c % cpr;
            dst[u] = *reinterpret_cast<const Vec16<T> *>(src + row * rs + cc * E);
        }
    };
    auto commit_natural = [&](const Vec16<T> *src, T *dstl, int ld, auto D_, auto NV_) {
        constexpr int cpr = decltype(D_)::value / E;
#pragma unroll
        for (int u = 0; u < decltype(NV_)::value; ++u) {
            const int c = tid + u * GT, row = c / cpr, cc = c % cpr;
            *reinterpret_cast<Vec16<T> *>(dstl + row * ld + cc * E) = src[u];
        }
    };
    auto issue_linear = [&](Vec16<T> *dst, const T *src, auto NV_) {
#pragma unroll
        for (int u = 0; u < decltype(NV_)::value; ++u)
            dst[u] = *reinterpret_cast<const Vec16<T> *>(src + (size_t)(tid + u * GT) * E);
    };
    auto commit_linear = [&](const Vec16<T> *src, T *dstl, auto NV_) {
#pragma unroll
        for (int u = 0; u < decltype(NV_)::value; ++u)
            *reinterpret_cast<Vec16<T> *>(dstl + (size_t)(tid + u * GT) * E) = src[u];
    };
    typedef std::integral_constant<int, DV> cDV;
    typedef std::integral_constant<int, DK> cDK;
    typedef std::integral_constant<int, NV_V> cNV_V;
    typedef std::integral_constant<int, NV_K> cNV_K;
    typedef std::integral_constant<int, NV_B> cNV_B;
    typedef std::integral_constant<int, NV_S> cNV_S;
    auto dot_regs = [&](const Vec16<T> *x, const Vec16<T> *y) {
        float s = 0.f;
#pragma unroll
        for (int u = 0; u < NV_S; ++u)
#pragma unroll
            for (int e = 0; e < E; ++e) s += to_f32(x[u].e[e]) * to_f32(y[u].e[e]);
        return s;
    };

    // ---------------- prologue: first tiles in flight, gates, this wave's own rows
    if (STAGED) {
        issue_natural(P, vtg, rsv, cDV{}, cNV_V{});
        issue_natural(P + NV_V, kgl, rsk, cDK{}, cNV_K{});
    }
    // gates of token `lane` (used by wave 0 for the coefficient scans)
    const size_t gl = tok0 + (size_t)lane * d.H;
    const float g_al = a.alpha[gl], g_be = a.beta[gl], g_mu = a.mu[gl], g_et = a.eta ? a.eta[gl] : 1.f;
    for (int c = tid; c < LDG; c += GT) sDG2[64 * LDG + c] = 0.f;
    Frag fdO[KSV], fdR[KSV], fq[KSK], fk[KSK]; // B fragments: row = token i
#pragma unroll
    for (int s = 0; s < KSV; ++s) {
        fdO[s] = O::load(dog + (size_t)i * rsv + s * O::KSTEP + kg * E);
        fdR[s] = O::load(drg + (size_t)i * rsv + s * O::KSTEP + kg * E);
    }
#pragma unroll
    for (int s = 0; s < KSK; ++s) {
        fq[s] = O::load(qg + (size_t)i * rsk + s * O::KSTEP + kg * E);
        fk[s] = O::load(kgl + (size_t)i * rsk + s * O::KSTEP + kg * E);
    }
    // k_i and q_i in accumulator layout: element x of tile mt is dk = mt*16 + kg*4 + x
    f32x4 kv[NH];
#pragma unroll
    for (int mt = 0; mt < NH; ++mt) kv[mt] = load4(kgl + (size_t)i * rsk + (hf * NH + mt) * 16 + kg * 4);

    const T *tVt = STAGED ? sB : vtg;
    const T *tK = STAGED ? sB + 64 * LDNV : kgl;
    const int ldVt = STAGED ? LDNV : (int)rsv, ldK = STAGED ? LDNK : (int)rsk;
    if (STAGED) {
        commit_natural(P, sB, LDNV, cDV{}, cNV_V{});
        commit_natural(P + NV_V, sB + 64 * LDNV, LDNK, cDK{}, cNV_K{});
        issue_linear(P, KTg, cNV_B{});
        issue_linear(P + NV_B, QTg, cNV_B{});
    }
    __syncthreads();

    // ---------------- phase 0: forward coefficients: vectors by wave scans, matrices by a column scan
    float pa = 0.f, pm = 0.f, pb = 0.f; // a_lane, m_lane, b_lane (wave 0)
    if (w == 0) {
        pa = scan_prod(g_al);
        pm = scan_prod(g_mu);
        float c = g_al;
        pb = g_be * pm;
        scan_affine_fwd(c, pb);
        s_al[lane] = g_al;
        s_et[lane] = g_et;
        s_a[lane] = pa;
        s_b[lane] = pb;
        float gC, rC;
        coef_column_scan<true>(g_al, g_be, g_mu, sG, sRho, LDG, gC, rC);
        s_gC[lane] = gC; // Gamma_{C,j}
        s_rC[lane] = rC; // Rho_{C,j}
    }
    __syncthreads();

    // ---------------- phase A: the four 64x64 products (transposed: rows j, column i) and the
    //                  masked matrices built from them
    {
        const float al_i = s_al[i];
#pragma unroll
        for (int mh = 0; mh < 2; ++mh) {
            const int mt = hf * 2 + mh;
            f32x4 accB = {0.f, 0.f, 0.f, 0.f}, accA = accB, accQK = accB, accKK = accB;
            const T *vp = tVt + (size_t)(mt * 16 + r) * ldVt + kg * E;
            const T *kp = tK + (size_t)(mt * 16 + r) * ldK + kg * E;
#pragma unroll
            for (int s = 0; s < KSV; ++s) {
                const Frag fv = O::load(vp + s * O::KSTEP);
                accB = O::mma(fv, fdO[s], accB);
                accA = O::mma(fv, fdR[s], accA);
            }
#pragma unroll
            for (int s = 0; s < KSK; ++s) {
                const Frag fkk = O::load(kp + s * O::KSTEP);
                accQK = O::mma(fkk, fq[s], accQK);
                accKK = O::mma(fkk, fk[s], accKK);
            }
            f32x4 w1e, w2e;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int j = mt * 16 + kg * 4 + x;
                const float gam = sG[i * LDG + j], gprev = (i > 0) ? sG[(i - 1) * LDG + j] : 0.f;
                const float et = s_et[j];
                const float dBm = (j <= i) ? accB[x] : 0.f;
                const float dA = (j < i) ? -accA[x] : 0.f;
                sDG1[i * LDG + j] = dBm * (d.scale * et * accQK[x]);
                sDG2[i * LDG + j] = dA * (al_i * et * accKK[x]);
                const float w1 = dBm * gam, w2 = dA * gprev;
                w1e[x] = w1 * et;
                w2e[x] = w2 * et;
                sW1T[j * LDW + i] = from_f32<T>(w1 * d.scale);
                sW2T[j * LDW + i] = from_f32<T>(w2 * al_i);
            }
            store4(sW1e + i * LDW + mt * 16 + kg * 4, w1e);
            store4(sW2e + i * LDW + mt * 16 + kg * 4, w2e);
        }
    }
    __syncthreads();

    // ---------------- phase B: the token-contractions W1 K~, W2 K~, W1^T Q~, W2^T P
    const T *tKT = STAGED ? sB : KTg, *tQT = STAGED ? sB + DK * 64 : QTg;
    if (STAGED) {
        commit_linear(P, sB, cNV_B{});
        commit_linear(P + NV_B, sB + DK * 64, cNV_B{});
        issue_linear(Q, Sg, cNV_S{});
        __syncthreads();
    }
    f32x4 accQ[NH], accP[NH], accK[NH]; // dQ~^T, dP^T, dK~^T: [dk tile of this half][token i]
    zero_acc(accQ);
    zero_acc(accP);
    zero_acc(accK);
#pragma unroll
    for (int s = 0; s < KS2; ++s) {
        const Frag b1e = O::load(sW1e + i * LDW + s * O::KSTEP + kg * E);
        const Frag b2e = O::load(sW2e + i * LDW + s * O::KSTEP + kg * E);
        const Frag b1t = O::load(sW1T + i * LDW + s * O::KSTEP + kg * E);
        const Frag b2t = O::load(sW2T + i * LDW + s * O::KSTEP + kg * E);
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) {
            const Frag aK = O::load(tKT + kblk<T>(DK, (hf * NH + mt) * 16 + r, s * O::KSTEP + kg * E));
            const Frag aQ = O::load(tQT + kblk<T>(DK, (hf * NH + mt) * 16 + r, s * O::KSTEP + kg * E));
            accQ[mt] = O::mma(aK, b1e, accQ[mt]);
            accP[mt] = O::mma(aK, b2e, accP[mt]);
            accK[mt] = O::mma(aQ, b1t, accK[mt]);
            accK[mt] = O::mma(aK, b2t, accK[mt]);
        }
    }

    // ---------------- phases C-F: products with the four state matrices, one staged tile each
    // two products X^T[dk][i] = sum_dv St[dk][dv] f[i][dv] sharing the A fragments of one state tile
    auto state_products = [&](const T *tile, const Frag (&f1)[KSV], const Frag (&f2)[KSV], f32x4 (&t1)[NH],
                              f32x4 (&t2)[NH], bool second) {
        zero_acc(t1);
        zero_acc(t2);
#pragma unroll
        for (int s = 0; s < KSV; ++s)
#pragma unroll
            for (int mt = 0; mt < NH; ++mt) {
                const Frag as = O::load(tile + vblk(DK, (hf * NH + mt) * 16 + r, s * O::KSTEP + kg * E));
                t1[mt] = O::mma(as, f1[s], t1[mt]);
                if (second) t2[mt] = O::mma(as, f2[s], t2[mt]);
            }
    };
    float p1 = 0.f, p2 = 0.f, p3 = 0.f; // partial <dS',S>, <dS',M>, <dM',M>
    f32x4 t1[NH], t2[NH];
    const float a_i = s_a[i], b_i = s_b[i], am_i = (i > 0) ? s_a[i - 1] : 1.f, bm_i = (i > 0) ? s_b[i - 1] : 0.f;
    const float al_i = s_al[i], et_i = s_et[i];

    // C: S
    if (STAGED) {
        __syncthreads(); // phase B done with the staging buffer
        commit_linear(Q, sB, cNV_S{});
        issue_linear(P, dSg, cNV_S{});
        __syncthreads();
    }
    state_products(STAGED ? sB : Sg, fdO, fdR, t1, t2, true);
    {
        f32x4 qv[NH];
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) qv[mt] = load4(qg + (size_t)i * rsk + (hf * NH + mt) * 16 + kg * 4);
        const float da = d.scale * coldot<NH>(t1, qv);
        const float dam = -al_i * coldot<NH>(t2, kv);
        if (kg == 0) { s_da[hf][i] = da; s_dam[hf][i] = dam; }
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) {
            accQ[mt] += a_i * t1[mt];
            accP[mt] -= am_i * t2[mt];
        }
    }
    // E: dS'
    Frag fVt[KSV];
#pragma unroll
    for (int s = 0; s < KSV; ++s) fVt[s] = O::load(vtg + (size_t)i * rsv + s * O::KSTEP + kg * E);
    if (STAGED) {
        __syncthreads();
        p1 = dot_regs(P, Q);
        commit_linear(P, sB, cNV_S{});
        issue_linear(Q, Mg, cNV_S{});
        __syncthreads();
    }
    state_products(STAGED ? sB : dSg, fVt, fVt, t1, t2, false);
    const float gC_i = s_gC[i], rC_i = s_rC[i];
    {
        const float dgc = et_i * coldot<NH>(t1, kv);
        if (kg == 0) s_dgc[hf][i] = dgc;
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) accK[mt] += gC_i * t1[mt];
    }
    // D: M
    if (STAGED) {
        __syncthreads();
        p2 = dot_regs(P, Q);
        commit_linear(Q, sB, cNV_S{});
        issue_linear(P, dMg, cNV_S{});
        __syncthreads();
    }
    state_products(STAGED ? sB : Mg, fdO, fdR, t1, t2, true);
    {
        f32x4 qv[NH];
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) qv[mt] = load4(qg + (size_t)i * rsk + (hf * NH + mt) * 16 + kg * 4);
        const float db = -d.scale * coldot<NH>(t1, qv);
        const float dbm = al_i * coldot<NH>(t2, kv);
        if (kg == 0) { s_db[hf][i] = db; s_dbm[hf][i] = dbm; }
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) {
            accQ[mt] -= b_i * t1[mt];
            accP[mt] += bm_i * t2[mt];
        }
        T *dqg = static_cast<T *>(a.dq) + (tok0 + (size_t)i * d.H) * DK + hf * NH * 16 + kg * 4;
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) store4(dqg + mt * 16, d.scale * accQ[mt]);
        const float dalk = coldot<NH>(accP, kv);
        if (kg == 0) s_dalk[hf][i] = dalk;
    }
    // F: dM'
    if (STAGED) {
        __syncthreads();
        p3 = dot_regs(P, Q);
        commit_linear(P, sB, cNV_S{});
        __syncthreads();
    }
    state_products(STAGED ? sB : dMg, fVt, fVt, t1, t2, false);
    {
        const float drc = -et_i * coldot<NH>(t1, kv);
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) accK[mt] -= rC_i * t1[mt];
        const float detk = coldot<NH>(accK, kv);
        if (kg == 0) { s_drc[hf][i] = drc; s_detk[hf][i] = detk; }
        T *dkg = static_cast<T *>(a.dk) + (tok0 + (size_t)i * d.H) * DK + hf * NH * 16 + kg * 4;
#pragma unroll
        for (int mt = 0; mt < NH; ++mt) store4(dkg + mt * 16, et_i * accK[mt] + al_i * accP[mt]);
    }
    if (!STAGED) {
        // <dS',S>, <dS',M>, <dM',M> straight from memory
        for (int c = tid * E; c < DK * DV; c += GT * E) {
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const float s = to_f32(Sg[c + e]), m = to_f32(Mg[c + e]);
                const float ds = to_f32(dSg[c + e]), dm = to_f32(dMg[c + e]);
                p1 += ds * s;
                p2 += ds * m;
                p3 += dm * m;
            }
        }
    }
    p1 = reduce64(p1);
    p2 = reduce64(p2);
    p3 = reduce64(p3);
    if (lane == 0) { s_red[w][0] = p1; s_red[w][1] = p2; s_red[w][2] = p3; }
    __syncthreads();

    // ---------------- phase 4: reverse of the coefficient scans
    if (w == 0)
        coef_column_scan_reverse(g_al, g_be, g_mu, sDG1, sDG2, s_dgc[0][lane] + s_dgc[1][lane],
                                 s_drc[0][lane] + s_drc[1][lane], sGa, sRa, LDG);
    __syncthreads();
    {
        // dalpha_i += sum_{j<i} G_ij Gamma_{i-1,j};  dbeta_i += sum_{j<=i} G_ij Rho_ij;
        // dmu_i += sum_{j<i} R_ij Rho_{i-1,j}: 8 threads per row
        const int row = tid >> 3, part = tid & 7;
        float ga = 0.f, gb = 0.f, gm = 0.f;
        for (int j = part; j <= row; j += 8) {
            const float G = sGa[row * LDG + j], R = sRa[row * LDG + j];
            gb += G * sRho[row * LDG + j];
            if (j < row) {
                ga += G * sG[(row - 1) * LDG + j];
                gm += R * sRho[(row - 1) * LDG + j];
            }
        }
        ga += __shfl_xor(ga, 1); ga += __shfl_xor(ga, 2); ga += __shfl_xor(ga, 4);
        gb += __shfl_xor(gb, 1); gb += __shfl_xor(gb, 2); gb += __shfl_xor(gb, 4);
        gm += __shfl_xor(gm, 1); gm += __shfl_xor(gm, 2); gm += __shfl_xor(gm, 4);
        if (part == 0) { s_ga[row] = ga; s_gb[row] = gb; s_gm[row] = gm; }
    }
    __syncthreads();
    if (w == 0) {
        // vectors (lane i = token i): reverse of b_i = alpha_i b_{i-1} + beta_i m_i, a_i = alpha_i a_{i-1},
        // m_i = mu_i m_{i-1}, with a^-_i = a_{i-1}, b^-_i = b_{i-1}:
        //   db_i = Db_i + alpha_{i+1} db_{i+1},  da_i = Da_i + alpha_{i+1} da_{i+1},
        //   dm_i = Dm_i + beta_i db_i + mu_{i+1} dm_{i+1}
        float dS_S = 0.f, dS_M = 0.f, dM_M = 0.f;
#pragma unroll
        for (int ww = 0; ww < 8; ++ww) {
            dS_S += s_red[ww][0];
            dS_M += s_red[ww][1];
            dM_M += s_red[ww][2];
        }
        const int li = lane;
        const float al_next = __shfl_down(g_al, 1), mu_next = __shfl_down(g_mu, 1);
        const float dbm_next = (li < 63) ? s_dbm[0][li + 1] + s_dbm[1][li + 1] : -dS_M;
        const float dam_next = (li < 63) ? s_dam[0][li + 1] + s_dam[1][li + 1] : dS_S;
        float cb = (li < 63) ? al_next : 0.f, db = s_db[0][li] + s_db[1][li] + dbm_next;
        scan_affine_rev(cb, db);
        float ca = (li < 63) ? al_next : 0.f, da = s_da[0][li] + s_da[1][li] + dam_next;
        scan_affine_rev(ca, da);
        float cm = (li < 63) ? mu_next : 0.f, dm = (li == 63 ? dM_M : 0.f) + g_be * db;
        scan_affine_rev(cm, dm);
        const float aprev = __shfl_up(pa, 1), bprev = __shfl_up(pb, 1), mprev = __shfl_up(pm, 1);
        const float a_prev = (li > 0) ? aprev : 1.f, b_prev = (li > 0) ? bprev : 0.f, m_prev = (li > 0) ? mprev : 1.f;
        const size_t g = tok0 + (size_t)li * d.H;
        a.dalpha[g] = s_ga[li] + db * b_prev + da * a_prev + s_dalk[0][li] + s_dalk[1][li];
        a.dbeta[g] = s_gb[li] + db * pm;
        a.dmu[g] = s_gm[li] + dm * m_prev;
        if (a.deta) a.deta[g] = s_detk[0][li] + s_detk[1][li];
    }
}

template <typename T, int DK, int DV, bool STAGED>
hipError_t launch_t(const Dims &d, const GradArgs &a, hipStream_t s) {
    dim3 grid(d.N, d.BH), block(GT);
    hipLaunchKernelGGL((grad_kernel<T, DK, DV, STAGED>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_grad(const Dims &d, const GradArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64)
        return f32 ? launch_t<float, 64, 64, false>(d, a, s) : launch_t<bf16_t, 64, 64, true>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_t<float, 128, 128, false>(d, a, s) : launch_t<bf16_t, 128, 128, true>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
