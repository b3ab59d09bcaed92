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
//   WY-style factors  U = T V,  Y = T diag(a^-) P = (T diag(a)) K,  Z = T diag(b^-) P = (T diag(b^- alpha)) K
//
// One workgroup (4 waves) per (chunk, batch*head).  Forward mode writes U, -Y, Z, Bm and K^T;
// backward mode writes the transposed operands the reverse scan needs (-Y^T, Z^T, Bm^T, T^T, K^T, Q^T).
// Everything is written in the blocked layouts of mdn_device.h (kblk / vblk), in which the serial
// scans' fragment loads are contiguous.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

constexpr int LDA = 68; // row stride (floats) of the fp32 A / T matrix in LDS
constexpr int LDG = 65; // row stride (floats) of Gamma in LDS

// natural [64][D] tile: rows of the chunk -> LDS [64][ld]
template <typename T, int D>
__device__ __forceinline__ void load_tile_natural(T *dst, int ld, const T *src, size_t row_stride, int tid,
                                                  int nthreads) {
    constexpr int E = Op<T>::EPL, CPR = D / E;
    for (int c = tid; c < 64 * CPR; c += nthreads) {
        const int row = c / CPR, cc = c % CPR;
        const Vec16<T> v = *reinterpret_cast<const Vec16<T> *>(src + row * row_stride + cc * E);
        *reinterpret_cast<Vec16<T> *>(dst + row * ld + cc * E) = v;
    }
}

// transposed: LDS [D][ld] with dst[d][row] = src[row][d]
template <typename T, int D>
__device__ __forceinline__ void load_tile_transposed(T *dst, int ld, const T *src, size_t row_stride, int tid,
                                                     int nthreads) {
    constexpr int E = Op<T>::EPL, CPR = D / E;
    for (int c = tid; c < 64 * CPR; c += nthreads) {
        const int row = c % 64, cc = c / 64; // consecutive threads -> consecutive rows (LDS-friendly)
        const Vec16<T> v = *reinterpret_cast<const Vec16<T> *>(src + row * row_stride + cc * E);
#pragma unroll
        for (int e = 0; e < E; ++e) dst[(cc * E + e) * ld + row] = v.e[e];
    }
}

// LDS [R][ld] (first 64 columns) -> global, kblk layout of an [R][64] operand
template <typename T>
__device__ __forceinline__ void store_tile_64cols(T *dst, const T *src, int ld, int rows, int tid) {
    constexpr int E = Op<T>::EPL, CPR = 64 / E;
    for (int c = tid; c < rows * CPR; c += kThreads) {
        const int row = c % rows, cc = c / rows;
        *reinterpret_cast<Vec16<T> *>(dst + kblk<T>(rows, row, cc * E)) =
            *reinterpret_cast<const Vec16<T> *>(src + row * ld + cc * E);
    }
}

template <typename T, int DK, int DV, bool BWD>
__global__ __launch_bounds__(kThreads) void intra_kernel(Dims d, IntraArgs a) {
    typedef Op<T> O;
    constexpr int LDN = DK + O::PAD; // natural tiles
    constexpr int LDT = 64 + O::PAD; // transposed tiles and the operand copy of T
    constexpr int DX = BWD ? DK : DV;
    constexpr int REG_NAT = 2 * 64 * LDN, REG_TR = (DK + DX) * LDT;
    constexpr int REGION = REG_NAT > REG_TR ? REG_NAT : REG_TR;

    __shared__ __align__(16) T sR[REGION];
    __shared__ __align__(16) float sG[64 * LDG];
    __shared__ __align__(16) float sA[64 * LDA];
    __shared__ __align__(16) T sTop[64 * LDT];
    __shared__ float s_al[64], s_be[64], s_mu[64], s_et[64], s_a[64], s_b[64], s_cs[64];

    T *sK = sR, *sQ = sR + 64 * LDN;      // phase A
    T *sKT = sR, *sXT = sR + DK * LDT;    // phase B (aliases phase A)

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int n = blockIdx.x, bh = blockIdx.y;
    const int b = bh / d.H, h = bh % d.H;
    const size_t tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
    const size_t blk = (size_t)bh * d.N + n; // chunk-block index into the workspace tensors
    const T *qg = static_cast<const T *>(a.q) + tok0 * DK;
    const T *kg_ = static_cast<const T *>(a.k) + tok0 * DK;
    const T *vg = static_cast<const T *>(a.v) + tok0 * DV;
    const size_t rsk = (size_t)d.H * DK, rsv = (size_t)d.H * DV;
    float *coef = a.coef + blk * (kCoefRows * 64);

    if (tid < 64) {
        const size_t g = tok0 + (size_t)tid * d.H;
        s_al[tid] = a.alpha[g];
        s_be[tid] = a.beta[g];
        s_mu[tid] = a.mu[g];
        s_et[tid] = a.eta ? a.eta[g] : 1.f;
    }
    load_tile_natural<T, DK>(sK, LDN, kg_, rsk, tid, kThreads);
    load_tile_natural<T, DK>(sQ, LDN, qg, rsk, tid, kThreads);
    __syncthreads();

    // ---- gate coefficients: wave 0, lane j owns column j of Gamma / Rho
    if (w == 0) {
        const int j = lane;
        float pa = 1.f, pm = 1.f, pb = 0.f, my_a = 0.f, my_b = 0.f;
        float g = 0.f, rho = 0.f;
        for (int i = 0; i < 64; ++i) {
            const float al = s_al[i], be = s_be[i], mu = s_mu[i];
            pa *= al;
            pm *= mu;
            pb = al * pb + be * pm;
            if (i == j) { my_a = pa; my_b = pb; }
            rho = (i == j) ? 1.f : rho * mu;
            g = al * g + be * rho;
            sG[i * LDG + j] = g;
        }
        s_a[j] = my_a;
        s_b[j] = my_b;
        const float et = s_et[j];
        coef[COEF_A * 64 + j] = my_a;
        coef[COEF_B * 64 + j] = my_b;
        coef[COEF_GC * 64 + j] = g * et;
        coef[COEF_RC * 64 + j] = rho * et;
        coef[COEF_ETA * 64 + j] = et;
        if (j < 3) coef[COEF_SCALAR * 64 + j] = (j == 0) ? pa : (j == 1) ? pb : pm;
    }
    __syncthreads();

    // ---- masked intra-chunk products: wave w owns rows i0..i0+15.
    //      The Q K^T product is formed in the orientation whose accumulator lanes hold 4 consecutive
    //      entries along the contraction index of the consumer (j for Bm, i for Bm^T).
    const int r = lane & 15, kq = lane >> 4, i0 = w * 16;
    {
        f32x4 kk[4], qk[4];
        zero_acc(kk);
        zero_acc(qk);
        mma_rows<T, 4, DK>(kk, sK + i0 * LDN, LDN, sK, LDN);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + kq * 4 + x, j = nt * 16 + r;
                const float gprev = (i > 0) ? sG[(i - 1) * LDG + j] : 0.f;
                sA[i * LDA + j] = (j < i) ? s_al[i] * s_et[j] * gprev * kk[nt][x] : 0.f;
            }
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
        } else {
            // qk[nt][x] = k_j . q_i, j = i0 + kq*4 + x, i = nt*16 + r  ->  Bm row i, k = j
            mma_rows<T, 4, DK>(qk, sK + i0 * LDN, LDN, sQ, LDN);
            T *out = static_cast<T *>(a.Bm) + blk * 4096;
#pragma unroll
            for (int nt = 0; nt < 4; ++nt) {
                const int i = nt * 16 + r;
                f32x4 v;
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int j = i0 + kq * 4 + x;
                    v[x] = (j <= i) ? d.scale * s_et[j] * sG[i * LDG + j] * qk[nt][x] : 0.f;
                }
                store4(out + kblk<T>(64, i, i0 + kq * 4), v);
            }
        }
    }
    __syncthreads();

    // ---- T = (I + A)^{-1}: wave 0, lane j solves column j by forward substitution
    //      t_i = [i == j] - sum_{k < i} A_ik t_k   (entries above the diagonal come out as 0);
    //      meanwhile waves 1..3 stage the transposed tiles.
    if (w == 0) {
        const int j = lane;
        float t[64];
#pragma unroll
        for (int i = 0; i < 64; ++i) t[i] = 0.f;
#pragma unroll
        for (int i = 0; i < 64; ++i) {
            float acc = (i == j) ? 1.f : 0.f;
#pragma unroll
            for (int k4 = 0; k4 < (i + 3) / 4; ++k4) {
                const f32x4 av = *reinterpret_cast<const f32x4 *>(&sA[i * LDA + 4 * k4]);
                acc -= av[0] * t[4 * k4 + 0];
                acc -= av[1] * t[4 * k4 + 1];
                acc -= av[2] * t[4 * k4 + 2];
                acc -= av[3] * t[4 * k4 + 3];
            }
            t[i] = acc;
        }
#pragma unroll
        for (int i = 0; i < 64; ++i) sA[i * LDA + j] = t[i];
    } else {
        load_tile_transposed<T, DK>(sKT, LDT, kg_, rsk, tid - 64, kThreads - 64);
        if (BWD) load_tile_transposed<T, DK>(sXT, LDT, qg, rsk, tid - 64, kThreads - 64);
        else load_tile_transposed<T, DV>(sXT, LDT, vg, rsv, tid - 64, kThreads - 64);
    }
    __syncthreads();

    // raw transposed copies for the scans
    store_tile_64cols<T>(static_cast<T *>(a.KT) + blk * (DK * 64), sKT, LDT, DK, tid);
    if (BWD) {
        store_tile_64cols<T>(static_cast<T *>(a.QT) + blk * (DK * 64), sXT, LDT, DK, tid);
        T *tt = static_cast<T *>(a.TmT) + blk * 4096; // T^T: row j, k = i
        constexpr int E = O::EPL;
        for (int c = tid; c < 64 * (64 / E); c += kThreads) {
            const int jj = c & 63, cc = c >> 6;
            Vec16<T> v;
#pragma unroll
            for (int e = 0; e < E; ++e) v.e[e] = from_f32<T>(sA[(cc * E + e) * LDA + jj]);
            *reinterpret_cast<Vec16<T> *>(tt + kblk<T>(64, jj, cc * E)) = v;
        }
    }

    // ---- WY-style factors.  pass 0: U = T V (forward only); pass 1: Y; pass 2: Z.
    //      Each product is formed in the orientation whose accumulator lanes hold 4 consecutive
    //      entries along the index that is contiguous in the consumer's layout.
    for (int pass = BWD ? 1 : 0; pass < 3; ++pass) {
        if (tid < 64) {
            const float bprev = (tid > 0) ? s_b[tid - 1] : 0.f;
            s_cs[tid] = (pass == 0) ? 1.f : (pass == 1) ? s_a[tid] : bprev * s_al[tid];
        }
        __syncthreads();
        for (int c = tid; c < 4096; c += kThreads) {
            const int ii = c >> 6, jj = c & 63;
            sTop[ii * LDT + jj] = from_f32<T>(sA[ii * LDA + jj] * s_cs[jj]);
        }
        __syncthreads();
        const float sgn = pass == 1 ? -1.f : 1.f;
        if (!BWD) {
            if (pass == 0) {
                // U^T[dv][i] = sum_j V^T[dv][j] T[i][j]  ->  vblk [dv/16][token][16]
#pragma unroll
                for (int mt = 0; mt < DV / 64; ++mt) {
                    const int m0 = (w * (DV / 64) + mt) * 16;
                    f32x4 u[4];
                    zero_acc(u);
                    mma_rows<T, 4, 64>(u, sXT + m0 * LDT, LDT, sTop, LDT);
                    T *out = static_cast<T *>(a.U) + blk * (64 * DV);
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) store4(out + vblk(64, nt * 16 + r, m0 + kq * 4), u[nt]);
                }
            } else {
                // Y^T[dk][i] = sum_j K^T[dk][j] (T diag(cs))[i][j]  ->  kblk: row i, k = dk
#pragma unroll
                for (int mt = 0; mt < DK / 64; ++mt) {
                    const int m0 = (w * (DK / 64) + mt) * 16;
                    f32x4 y[4];
                    zero_acc(y);
                    mma_rows<T, 4, 64>(y, sKT + m0 * LDT, LDT, sTop, LDT);
                    T *out = static_cast<T *>(pass == 1 ? a.nY : a.Z) + blk * (64 * DK);
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) store4(out + kblk<T>(64, nt * 16 + r, m0 + kq * 4), sgn * y[nt]);
                }
            }
        } else {
            // Y[i][dk] = sum_j (T diag(cs))[i][j] K^T[dk][j]  ->  Y^T in kblk: row dk, k = i
            f32x4 y[DK / 16];
            zero_acc(y);
            mma_rows<T, DK / 16, 64>(y, sTop + i0 * LDT, LDT, sKT, LDT);
            T *out = static_cast<T *>(pass == 1 ? a.nYT : a.ZT) + blk * (DK * 64);
#pragma unroll
            for (int nt = 0; nt < DK / 16; ++nt) store4(out + kblk<T>(DK, nt * 16 + r, i0 + kq * 4), sgn * y[nt]);
        }
        __syncthreads();
    }
}

template <typename T, int DK, int DV>
hipError_t launch_intra_t(const Dims &d, bool bwd, const IntraArgs &a, hipStream_t s) {
    dim3 grid(d.N, d.BH), block(kThreads);
    if (bwd) hipLaunchKernelGGL((intra_kernel<T, DK, DV, true>), grid, block, 0, s, d, a);
    else hipLaunchKernelGGL((intra_kernel<T, DK, DV, false>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_intra(const Dims &d, bool bwd, const IntraArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64)
        return f32 ? launch_intra_t<float, 64, 64>(d, bwd, a, s) : launch_intra_t<bf16_t, 64, 64>(d, bwd, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_intra_t<float, 128, 128>(d, bwd, a, s) : launch_intra_t<bf16_t, 128, 128>(d, bwd, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
