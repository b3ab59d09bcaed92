// Chunk-parallel precompute kernel ("intra"): everything of one 64-token chunk that does not
// depend on the incoming states S, M.
//
//   coefficients (Sec. 3.1 Eq. "coefficients", Appendix D), computed WITHOUT the log domain:
//       a_i = prod alpha,  m_i = prod mu,  b_i = alpha_i b_{i-1} + beta_i m_i,
//       Rho_jj = 1, Rho_ij = mu_i Rho_{i-1,j},  Gamma_ij = alpha_i Gamma_{i-1,j} + beta_i Rho_ij
//     (equal to (a_i/m_j)(c_i - c_{j-1}); only positive terms, no division, valid at mu = 0)
//   masked products (Sec. 3.1 "Chunkwise Algorithm"):
//       A  = (P K~^T) .* Gamma^-   (strictly lower; Gamma^-_ij = Gamma_{i-1,j}),  P = alpha k, K~ = eta k
//       Bm = (Q~ K~^T) .* Gamma    (lower incl. diagonal),                         Q~ = scale q
//   triangular solve  T = (I + A)^{-1}
//
// The WY-style factors U = T V, Y = T diag(a^-) P, Z = T diag(b^-) P of Sec. 3.1 are NOT formed: the scans
// apply T themselves,  V~ = T (V - a.(K S) + pb.(K M))  with  alpha_i a_{i-1} = a_i,  pb_i = alpha_i b_{i-1}
// (the same expression with T pulled out; Appendix C, Eq. "apx.v.before" solved for V~), and the reverse scan
// uses Y^T dV~ = K^T (a . T^T dV~).  That trades three 64 x d products and their 1.3 KB per token of HBM
// round trips for one 64 x 64 x dv product inside the scan.
//
// One workgroup (4 waves) per (chunk, batch*head).  Forward mode writes T, Bm and K^T; backward mode writes
// the transposed operands the reverse scan needs (Bm^T, T^T, K^T, Q^T); a training forward writes both sets
// at once, so that the backward need not recompute them.  Everything is written in the blocked layout of
// mdn_device.h (kblk), in which the serial scans' fragment loads are contiguous.
#include "mdn_coef.h"
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

constexpr int LDA = 68; // row stride (floats) of the fp32 A / T matrix in LDS
constexpr int LDG = 65; // row stride (floats) of Gamma in LDS

// LDS [R][ld] (first 64 columns) -> global, kblk layout of an [R][64] operand.  Consecutive lanes write
// consecutive 16-byte pieces of the destination (the pieces of one row's contraction step, then the next
// row's): every store instruction covers whole cache lines.
template <typename T>
__device__ __forceinline__ void store_tile_64cols(T *dst, const T *src, int ld, int rows, int tid) {
    constexpr int E = Op<T>::EPL, PPS = Op<T>::KSTEP / E, CPR = 64 / E; // pieces per contraction step, per row
    for (int c = tid; c < rows * CPR; c += kThreads) {
        const int p = c % PPS, row = (c / PPS) % rows, ks = c / (PPS * rows), cc = ks * PPS + p;
        *reinterpret_cast<Vec16<T> *>(dst + kblk<T>(rows, row, cc * E)) =
            *reinterpret_cast<const Vec16<T> *>(src + row * ld + cc * E);
    }
}

// MODE 0: forward operands; 1: operands of the reverse pass; 2: both (training forward that keeps the
// reverse pass's operands instead of recomputing them)
template <typename T, int DK, int DV, int MODE>
__global__ __launch_bounds__(kThreads) void intra_kernel(Dims d, IntraArgs a) {
    constexpr bool FWD = MODE != 1, BWD = MODE != 0;
    typedef Op<T> O;
    constexpr int E = O::EPL;
    constexpr int LDN = DK + O::PAD; // natural tiles
    constexpr int LDT = 64 + O::PAD; // transposed tiles (32-bit storage)
    constexpr int DX = BWD ? DK : 0; // second transposed tile: Q^T (reverse-pass operands only)
    // (16-bit storage reads the transposed tiles out of the natural ones and needs no space for them)
    constexpr int REG_NAT = 2 * 64 * LDN, REG_TR = sizeof(T) == 2 ? 0 : (DK + DX) * LDT;
    constexpr int REGION = REG_NAT > REG_TR ? REG_NAT : REG_TR;
    constexpr int NVK = 64 * DK / E / kThreads, NVX = BWD ? NVK : 1; // 16-byte vectors per thread

    __shared__ __align__(16) T sR[REGION];
    // Gamma (row stride LDG); later scratch of the block inverse
    __shared__ __align__(16) float sG[64 * LDA];
    // A, then T: in the space of the K, Q tiles, once every wave is done with those (70 -> 53 KB of LDS for 16-bit
    // storage at d = 128: three workgroups per CU instead of two)
    static_assert(sizeof(T) * REGION >= sizeof(float) * 64 * LDA, "A does not fit the tile region");
    float *sA = reinterpret_cast<float *>(sR);
    float *sTT = sG;
    __shared__ __align__(16) float s_al[64], s_be[64], s_et[64], s_a[64], s_b[64];

    T *sK = sR, *sQ = sR + 64 * LDN;      // phase A
    T *sKT = sR, *sXT = sR + DK * LDT;    // phase B (aliases phase A)

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int n = d.n0 + blockIdx.x, bh = blockIdx.y;
    const int b = bh / d.H, h = bh % d.H;
    const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
    const size_t blk = (size_t)bh * d.N + n; // chunk-block index into the workspace tensors
    const T *qg = static_cast<const T *>(a.q) + tok0 * DK;
    const T *kg_ = static_cast<const T *>(a.k) + tok0 * DK;
    const size_t rsk = (size_t)d.H * DK;
    float *coef = a.coef + blk * (kCoefRows * 64);

    // ---- the gates first, then the K, Q tiles: all loads in flight at once; the coefficient scans below need
    //      only the gates and run while the tiles are on their way
    const size_t gtok = tok0 + (size_t)lane * d.H;
    const float g_al = a.alpha[gtok], g_be = a.beta[gtok], g_mu = a.mu[gtok], g_et = a.eta ? a.eta[gtok] : 1.f;
    typename O::Frag rk[NVK], rq[NVK];
    {
        constexpr int CPR = DK / E;
#pragma unroll
        for (int u = 0; u < NVK; ++u) {
            const int c = tid + u * kThreads, row = c / CPR, cc = c % CPR;
            rk[u] = O::load(kg_ + row * rsk + cc * E);
            rq[u] = O::load(qg + row * rsk + cc * E);
        }
    }
    // 16-bit storage: the transposed tiles K^T, Q^T come straight out of the natural tiles in LDS through
    // transposing reads (a fragment of such a read is one 16-byte piece of the blocked layout).  32-bit storage:
    // the rows are loaded a second time in the order of the transposed tiles (in flight until the K, Q tiles are
    // no longer needed) and transposed through LDS.
    constexpr bool TRT = sizeof(T) == 2;
    Vec16<T> rkt[TRT ? 1 : NVK], rxt[TRT ? 1 : NVX];
    if constexpr (!TRT) {
#pragma unroll
        for (int u = 0; u < NVK; ++u) {
            const int c = tid + u * kThreads, row = c % 64, cc = c / 64;
            rkt[u] = *reinterpret_cast<const Vec16<T> *>(kg_ + row * rsk + cc * E);
        }
        if (BWD) {
#pragma unroll
            for (int u = 0; u < NVX; ++u) {
                const int c = tid + u * kThreads, row = c % 64, cc = c / 64;
                rxt[u] = *reinterpret_cast<const Vec16<T> *>(qg + row * rsk + cc * E);
            }
        }
    }

    // ---- gate coefficients.  Matrix Gamma: every wave 16 rows (column scans started from segment maps);
    //      vectors: wave 0, by wave scans (lane i = token i).
    {
        const float al = g_al, be = g_be, mu = g_mu, et = g_et;
        if (w == 0) {
            const float pa = scan_prod(al), pm = scan_prod(mu);
            float c = al, pb = be * pm;
            scan_affine_fwd(c, pb); // b_i = alpha_i b_{i-1} + beta_i m_i
            s_al[lane] = al;
            s_be[lane] = be;
            s_et[lane] = et;
            s_a[lane] = pa;
            s_b[lane] = pb;
            // alpha_i b_{i-1} (b_{-1} = 0), and the chunk-end values a_C, b_C, m_C into every row
            const f32x4 c0 = {pa, pb, al * wave_up1(pb, 0.f, lane), lane_value(pa, 63)};
            *reinterpret_cast<f32x4 *>(coef + lane * kCoefRows + COEF_A) = c0;
            coef[lane * kCoefRows + COEF_BC] = lane_value(pb, 63);
            coef[lane * kCoefRows + COEF_MC] = lane_value(pm, 63);
        }
        float gC, rC;
        coef_column_scan_blocked<false>(al, be, mu, sG, nullptr, LDG, w, gC, rC);
        if (w == 3) {
            coef[lane * kCoefRows + COEF_GC] = gC * et;
            coef[lane * kCoefRows + COEF_RC] = rC * et;
        }
    }
    {
        constexpr int CPR = DK / E;
#pragma unroll
        for (int u = 0; u < NVK; ++u) {
            const int c = tid + u * kThreads, row = c / CPR, cc = c % CPR;
            *reinterpret_cast<typename O::Frag *>(sK + row * LDN + cc * E) = rk[u];
            *reinterpret_cast<typename O::Frag *>(sQ + row * LDN + cc * E) = rq[u];
        }
    }
    __syncthreads();

    // ---- K^T, Q^T first (they only need the tiles), so that the tile region is free once the products are done
    if constexpr (TRT) {
        // in the blocked layout, where asked for (the reverse scan and the state reconstruction read
        // them; the forward scan makes K^T itself out of the k rows): (dk tile, 32-token step) blocks dealt over
        // the waves; lane (r, kq) reads (dk = 16 dt + r, tokens 32 ks + 8 kq ..) and owns exactly that
        // 16-byte piece of the blocked layout, so a wave stores 1 KB of consecutive bytes
        if (a.KT || (BWD && a.QT)) {
            const int r = lane & 15, kq = lane >> 4;
            T *KTo = a.KT ? static_cast<T *>(a.KT) + blk * (DK * 64) : nullptr;
            T *QTo = BWD && a.QT ? static_cast<T *>(a.QT) + blk * (DK * 64) : nullptr;
#pragma unroll
            for (int t = 0; t < (DK / 16) * 2 / 4; ++t) {
                const int tt = w + 4 * t, dt = tt >> 1, ks = tt & 1;
                const size_t o = kblk<T>(DK, dt * 16 + r, ks * 32 + kq * 8);
                if (KTo) *reinterpret_cast<typename O::Frag *>(KTo + o) = tr_frag(sK, LDN, ks * 32, dt * 16, r, kq);
                if (QTo) *reinterpret_cast<typename O::Frag *>(QTo + o) = tr_frag(sQ, LDN, ks * 32, dt * 16, r, kq);
            }
        }
    }

    // ---- masked intra-chunk products: wave w owns rows i0..i0+15.
    //      The Q K^T product is formed in the orientation whose accumulator lanes hold 4 consecutive
    //      entries along the contraction index of the consumer (j for Bm, i for Bm^T).
    const int r = lane & 15, kq = lane >> 4, i0 = w * 16;
    {
        f32x4 kk[4], qk[4];
        zero_acc(kk);
        zero_acc(qk);
        mma_rows<T, 4, DK>(kk, sK + i0 * LDN, LDN, sK, LDN);
        if (BWD) {
            // qk[nt][x] = q_i . k_j, i = i0 + kq*4 + x, j = nt*16 + r  ->  Bm^T row j, k = i
            mma_rows<T, 4, DK>(qk, sQ + i0 * LDN, LDN, sK, LDN);
            T *out = static_cast<T *>(a.BmT) + blk * 4096;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const int j = nt * 16 + r;
                f32x4 v;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int i = i0 + kq * 4 + x;
                    v[x] = (j <= i) ? d.scale * s_et[j] * sG[i * LDG + j] * qk[nt][x] : 0.f;
                }
                store4(out + kblk<T>(64, j, i0 + kq * 4), v);
            }
        }
        if (FWD) {
            // qk[nt][x] = k_j . q_i, j = i0 + kq*4 + x, i = nt*16 + r  ->  Bm row i, k = j
            zero_acc(qk);
            mma_rows<T, 4, DK>(qk, sK + i0 * LDN, LDN, sQ, LDN);
            T *out = static_cast<T *>(a.Bm) + blk * 4096;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const int i = nt * 16 + r, j0 = i0 + kq * 4;
                const float *gr = &sG[i * LDG + j0];
                const f32x4 et = *reinterpret_cast<const f32x4 *>(&s_et[j0]);
                f32x4 v;
#pragma unroll
                for (int x = 0; x < 4; ++x) v[x] = (j0 + x <= i) ? d.scale * et[x] * gr[x] * qk[nt][x] : 0.f;
                store4(out + kblk<T>(64, i, i0 + kq * 4), v);
            }
        }
        if constexpr (!TRT) {
            // ---- 32-bit storage: the transposed tiles take the space of the K, Q tiles (dst[d][row] = src[row][d]),
            //      go out from there, and only then does A move in
            __syncthreads();
#pragma unroll
            for (int u = 0; u < NVK; ++u) {
                const int c = tid + u * kThreads, row = c % 64, cc = c / 64;
#pragma unroll
                for (int e = 0; e < E; ++e) sKT[(cc * E + e) * LDT + row] = rkt[u].e[e];
            }
            if (BWD) {
#pragma unroll
                for (int u = 0; u < NVX; ++u) {
                    const int c = tid + u * kThreads, row = c % 64, cc = c / 64;
#pragma unroll
                    for (int e = 0; e < E; ++e) sXT[(cc * E + e) * LDT + row] = rxt[u].e[e];
                }
            }
            __syncthreads();
            store_tile_64cols<T>(static_cast<T *>(a.KT) + blk * (DK * 64), sKT, LDT, DK, tid);
            if (BWD) store_tile_64cols<T>(static_cast<T *>(a.QT) + blk * (DK * 64), sXT, LDT, DK, tid);
        }
        __syncthreads(); // every wave is done with the tiles: A takes their place
        // K K^T is symmetric: element x of tile nt is read as k_i . k_j with i = nt*16 + r (row of A) and
        // j = i0 + kq*4 + x, so that a lane holds 4 consecutive j of one row: eta and the row of A are one 16-byte
        // LDS access each
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
            const int i = nt * 16 + r, j0 = i0 + kq * 4;
            // (Gamma's rows have an odd stride, for the column accesses of the reverse-pass product above: its four
            //  values are read one by one)
            const float *gr = &sG[(i > 0 ? i - 1 : 0) * LDG + j0];
            const f32x4 et = *reinterpret_cast<const f32x4 *>(&s_et[j0]);
            const float al_i = s_al[i];
            f32x4 v;
#pragma unroll
            for (int x = 0; x < 4; ++x) v[x] = (j0 + x < i) ? al_i * et[x] * gr[x] * kk[nt][x] : 0.f;
            *reinterpret_cast<f32x4 *>(&sA[i * LDA + j0]) = v;
        }
    }
    __syncthreads();

    // ---- T = (I + A)^{-1} by 16x16 blocks, wave w = block row w
    tri_inverse_blocked(sA, sTT, LDA, w);
    __syncthreads();

    if (BWD) {
        T *tt = static_cast<T *>(a.TmT) + blk * 4096; // T^T: row j, k = i
        constexpr int E = O::EPL;
        constexpr int PPS = O::KSTEP / E; // 16-byte pieces per contraction step: consecutive lanes, consecutive pieces
        for (int c = tid; c < 64 * (64 / E); c += kThreads) {
            const int pp = c % PPS, jj = (c / PPS) & 63, cc = (c / (PPS * 64)) * PPS + pp;
            Vec16<T> v;
#pragma unroll
            for (int e = 0; e < E; ++e) v.e[e] = from_f32<T>(sA[(cc * E + e) * LDA + jj]);
            *reinterpret_cast<Vec16<T> *>(tt + kblk<T>(64, jj, cc * E)) = v;
        }
    }

    if (FWD) {
        T *tm = static_cast<T *>(a.Tm) + blk * 4096; // T: row i, k = j
        constexpr int PPS = O::KSTEP / E;
        for (int c = tid; c < 64 * (64 / E); c += kThreads) {
            const int pp = c % PPS, ii = (c / PPS) & 63, cc = (c / (PPS * 64)) * PPS + pp;
            Vec16<T> v;
#pragma unroll
            for (int e = 0; e < E; ++e) v.e[e] = from_f32<T>(sA[ii * LDA + cc * E + e]);
            *reinterpret_cast<Vec16<T> *>(tm + kblk<T>(64, ii, cc * E)) = v;
        }
    }
}

template <typename T, int DK, int DV>
hipError_t launch_intra_t(const Dims &d, int mode, const IntraArgs &a, hipStream_t s) {
    dim3 grid(d.n1 - d.n0, d.BH), block(kThreads);
    if (mode == 0) hipLaunchKernelGGL((intra_kernel<T, DK, DV, 0>), grid, block, 0, s, d, a);
    else if (mode == 1) hipLaunchKernelGGL((intra_kernel<T, DK, DV, 1>), grid, block, 0, s, d, a);
    else hipLaunchKernelGGL((intra_kernel<T, DK, DV, 2>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_intra(const Dims &d, int mode, const IntraArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64)
        return f32 ? launch_intra_t<float, 64, 64>(d, mode, a, s) : launch_intra_t<bf16_t, 64, 64>(d, mode, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_intra_t<float, 128, 128>(d, mode, a, s) : launch_intra_t<bf16_t, 128, 128>(d, mode, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
