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
// 16-bit storage ("staged"): one workgroup (8 waves) per CU walks its share of the (chunk, batch*head) pairs and
// requests the next chunk's gates and token tiles during the coefficient phases of the current one; 32-bit storage:
// one workgroup per chunk.  Every product is formed transposed (dk or j as the MFMA row index, tokens as the column
// index), so an accumulator lane holds 4 consecutive dk of one token: dq, dk leave as 8-byte stores and the row
// dots against q, k need two shuffles.
//   * 64x64 products (phase A): wave = (token tile, half of the j tiles); operands V~, k, q, dO, dR from LDS.
//   * everything with a dk row index (phases B-F): wave = (dk tile, token group).  Its A operands are
//     the wave's own 16 rows of S, M, dS', dM' (nobody else needs them, so they go from HBM straight into
//     fragment registers, in flight long before their use: no LDS copy, no barrier between the state products)
//     and of K^T, Q^T (transposing LDS reads of the k, q tiles, taken while those tiles are still there).  The B
//     operands are token rows that every wave needs: W1, W2 (built in phase A) and the natural-layout tiles of
//     dO, dR, V~ in LDS.
//   * the token tiles V~, k, q, dO, dR go HBM -> LDS without passing through registers (global_load_lds,
//     16 bytes per lane into consecutive LDS slots).  Rows are stored unpadded; to keep the fragment
//     reads (16 rows x one 16-byte piece) off each other's banks, piece c of row i sits at position
//     c ^ (i mod 16): the permutation is applied on the global side, where each lane is free to fetch
//     any address.  The kernel asks HBM for no byte twice.
// (fp32 storage does not fit the token tiles in LDS: it reads them, and K^T, Q^T, from HBM/L2 with the same code,
// and keeps only two state tiles in registers at a time.)
#include "mdn_coef.h"
#include "mdn_device.h"
#include "mdn_kernels.h"

#include <type_traits>

namespace mdn {

namespace {

constexpr int LDG = 68; // row stride of the fp32 64x64 coefficient matrices in LDS (rows 16-byte aligned)
constexpr int GT = 512; // threads per workgroup: 8 waves

// row-dot partial sums, one [dk tiles][64] block each
enum { P_DA = 0, P_DB, P_DAM, P_DBM, P_DGC, P_DRC, P_DALK, P_DETK, P_COUNT };

// this lane's share of the sum over the 16 dk of one accumulator tile of t^T[dk][i] * X[i][dk] for its token
__device__ __forceinline__ float dot4(f32x4 t, f32x4 xv) { return t[0] * xv[0] + t[1] * xv[1] + t[2] * xv[2] + t[3] * xv[3]; }

// Sums over the 4 lane groups kg = 0..3 (lanes r, r + 16, r + 32, r + 48) of TT values at once: on return the lanes of
// group kg (kg < TT) hold the complete sum of v[kg].  The row swaps exchange one value's odd rows for the other value's
// even rows, so one swap and one add halve TWO values: 3 swaps + 3 adds for four sums instead of 8 + 8, in the same
// association ((row 0 + row 1) + (row 2 + row 3)) as the sum of a single value by two exchanges.
__device__ __forceinline__ float reduce_tiles(const float (&v)[4]) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    u32x2 p = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[0]), __float_as_uint(v[1]), false, false);
    const float s01 = __uint_as_float(p[0]) + __uint_as_float(p[1]); // rows 0, 2: halves of v0; rows 1, 3: of v1
    p = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[2]), __float_as_uint(v[3]), false, false);
    const float s23 = __uint_as_float(p[0]) + __uint_as_float(p[1]);
    p = __builtin_amdgcn_permlane32_swap(__float_as_uint(s01), __float_as_uint(s23), false, false);
    return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}
__device__ __forceinline__ float reduce_tiles(const float (&v)[2]) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 p = __builtin_amdgcn_permlane16_swap(__float_as_uint(v[0]), __float_as_uint(v[1]), false, false);
    return add_xor32(__uint_as_float(p[0]) + __uint_as_float(p[1])); // rows 0, 2: v0; rows 1, 3: v1
}

// keeps the compiler from moving instructions across this point (used to stop the fragment loads of
// later contraction steps from piling up in registers)
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// LO: the rounding remainders of the four state tensors are given as well (GradArgs::states_lo, dstates_lo): the three
// state traces and the products of dS', dM' with V~ then take hi + lo of their factors.
template <typename T, int DK, int DV, bool STAGED, bool LO>
__global__ __launch_bounds__(GT) void grad_kernel(Dims d, GradArgs a) {
    typedef Op<T> O;
    typedef typename O::Frag Frag;
    constexpr int E = O::EPL;
    constexpr int LDW = 64 + O::PAD;
    static_assert(DK == DV, "token tiles share one row length");
    constexpr int D = DK, CPR = D / E;                 // 16-byte pieces per token row
    constexpr int XM = (CPR < 16 ? CPR : 16) - 1;      // piece c of row i is stored at c ^ (i & XM)
    constexpr int CPS = O::KSTEP / E;                  // pieces per contraction step
    constexpr int KSV = DV / O::KSTEP, KSK = DK / O::KSTEP, KS2 = 64 / O::KSTEP;
    constexpr int NKW = DK / 16;  // dk tiles = waves along dk
    constexpr int TG = 8 / NKW;   // token groups
    constexpr int TT = 4 / TG;    // token tiles per wave
    constexpr bool DEEP = STAGED; // all four state tiles in registers at once
    constexpr bool WTR = sizeof(T) == 2; // 16-bit storage: transposing LDS reads instead of transposed LDS writes
    static_assert(NKW * TG == 8 && TT * TG == 4, "8 waves = dk tiles x token groups");

    __shared__ __align__(16) float sG[64 * LDG];     // Gamma
    __shared__ __align__(16) float sRho[64 * LDG];   // Rho
    __shared__ __align__(16) float sDG1[64 * LDG];   // direct dGamma from Bm
    __shared__ __align__(16) float sDG2[65 * LDG];   // direct dGamma^- (row i here belongs to Gamma row i-1)
    __shared__ __align__(16) T sW[4 * 64 * LDW];
    T *sW1e = sW;                 // W1 . eta_j         [i][j]
    T *sW2e = sW + 64 * LDW;      // W2 . eta_j         [i][j]
    T *sW1T = sW + 2 * 64 * LDW;  // scale W1: [i][j] in 16-bit storage (read transposed), else its transpose [j][i]
    T *sW2T = sW + 3 * 64 * LDW;  // W2 . alpha_i: likewise
    // after the W products the space holds the row-dot partial sums, then the accumulated adjoints of Gamma, Rho
    float *spart = reinterpret_cast<float *>(sW);
    float *sGa = reinterpret_cast<float *>(sW), *sRa = sGa + 64 * LDG;
    float *sTop = sRa + 64 * LDG; // [4][2][64]: top rows of the four row segments of the reverse scan
    static_assert(sizeof(T) * 4 * 64 * LDW >= sizeof(float) * (2 * 64 * LDG + 512), "adjoint matrices do not fit the W space");
    static_assert(sizeof(T) * 4 * 64 * LDW >= sizeof(float) * P_COUNT * NKW * 64, "partial sums do not fit the W space");
    // token tiles [64][D] (pieces permuted, see above): V~, dO, dR; k sits in the W space until the W matrices are written
    __shared__ __align__(16) T sVt[STAGED ? 64 * D : 8];
    __shared__ __align__(16) T sDO[STAGED ? 64 * D : 8];
    __shared__ __align__(16) T sDR[STAGED ? 64 * D : 8];
    T *sK = sW, *sQ = sW + 64 * D;
    static_assert(4 * LDW >= 2 * D, "k and q tiles do not fit the W space");
    __shared__ __align__(16) float s_al[64], s_et[64], s_a[64], s_b[64];
    __shared__ float sRowC[3 * 64]; // reverse scan: the three per-row coefficients
    __shared__ float s_gC[64], s_rC[64];
    __shared__ float s_ga[64], s_gb[64], s_gm[64];
    __shared__ float s_da[64], s_de[64]; // wave 5's share of dalpha, and deta, for wave 4's final sums
    __shared__ float s_red[8][3];

    // Wave and lane indices, re-derived at the start of every chunk from values the compiler cannot see
    // through: otherwise every address and every wave-uniform offset this kernel ever forms is hoisted out of
    // the chunk loop and kept in a register for its whole duration (hundreds of them, vector and scalar).
    int w;              // wave-uniform by construction (a scalar register): branches on it are scalar
    // phase A: token tile wt (rows i of the 64 x 64 matrices), first column tile jA, whether the wave also forms column
    // tile 1 (two waves do), and the column tiles of its rows that lie above the diagonal and are only zeroed (bit jt of
    // zt).  Only the 10 tile pairs on or below the diagonal are multiplied out; they are dealt so that the two waves of a
    // SIMD (w, w + 4) share at most three of them (by rows alone SIMD 3 would have four and SIMD 0 one):
    //   w:  0  1  2    3    4  5  6  7
    //   wt: 0  1  2    3    3  1  2  3
    //   j:  0  0  0,1  0,1  3  1  2  2        zeroed: w0 -> 1, 2, 3; w1 -> 2; w5 -> 3; w6 -> 3
    int wt, jA, zt;
    bool hasB;
    int kt, tg; // phases B-F: dk tile, token group
    int tid, lane, r, kg, i; // i: this lane's token (MFMA column) in phase A
    unsigned gl;
    auto refresh_ids = [&]() {
        int ws = __builtin_amdgcn_readfirstlane(wave_id());
        asm volatile("" : "+s"(ws));
        w = ws;
        wt = (0xE7E4 >> (2 * w)) & 3;       // 0 1 2 3 3 1 2 3
        jA = (0xA700 >> (2 * w)) & 3;       // 0 0 0 0 3 1 2 2
        hasB = w == 2 || w == 3;
        zt = (0x0880004E >> (4 * w)) & 15;  // E 4 0 0 0 8 8 0
        kt = w % NKW;
        tg = TG == 1 ? 0 : w / NKW;
        int t = threadIdx.x;
        asm volatile("" : "+v"(t));
        tid = t;
        lane = t & 63;
        r = lane & 15;
        kg = lane >> 4;
        i = wt * 16 + r;
        gl = (unsigned)(lane * d.H);
    };
    refresh_ids();
    // per-lane offsets inside the chunk stay 32-bit (a uniform 64-bit base plus a 32-bit lane offset is
    // one address register instead of two)
    const unsigned rsk = (unsigned)d.H * DK, rsv = (unsigned)d.H * DV;

    // The workgroup walks the chunks c, c + gridDim.x, ... of this launch (c counts the chunks [n0, n1) of all
    // (batch, head) pairs, chunk index fastest).
    const int nper = d.n1 - d.n0, nchunks = nper * d.BH;
    int chunk = blockIdx.x;
    if (chunk >= nchunks) return;
    size_t tok0, blk;
    const T *qg, *kgl, *vtg, *dog, *drg, *KTg, *QTg, *Sg, *Mg, *dSg, *dMg, *Slg = nullptr, *dSlg = nullptr;
    auto set_chunk = [&](int c) {
        const int n = d.n0 + c % nper, bh = c / nper, b = bh / d.H, h = bh % d.H;
        tok0 = ((size_t)b * d.T + (size_t)n * 64) * d.H + h;
        blk = (size_t)bh * d.N + n;
        qg = static_cast<const T *>(a.q) + tok0 * DK;
        kgl = static_cast<const T *>(a.k) + tok0 * DK;
        vtg = static_cast<const T *>(a.vt_saved) + tok0 * DV;
        dog = static_cast<const T *>(a.dO) + tok0 * DV;
        drg = static_cast<const T *>(a.dv) + tok0 * DV; // dR = T^T dV~ (= dV), from the reverse scan
        KTg = static_cast<const T *>(a.KT) + blk * (DK * 64);
        QTg = static_cast<const T *>(a.QT) + blk * (DK * 64);
        Sg = static_cast<const T *>(a.states) + blk * (2 * DK * DV);
        Mg = Sg + DK * DV;
        dSg = static_cast<const T *>(a.dstates) + blk * (2 * DK * DV);
        dMg = dSg + DK * DV;
        if constexpr (LO) {
            Slg = static_cast<const T *>(a.states_lo) + blk * (2 * DK * DV);
            dSlg = static_cast<const T *>(a.dstates_lo) + blk * (2 * DK * DV);
        }
    };
    set_chunk(chunk);

    // fragment of row `row`, contraction step st of a token tile (in LDS, or in global memory with row stride ld)
    auto tfrag = [&](const T *tile, int ld, int row, int st) -> Frag {
        if (STAGED) return O::load(tile + row * D + (((st * CPS + kg) ^ (row & XM)) * E));
        return O::load(at32(tile, row * ld + st * O::KSTEP + kg * E));
    };
    // A fragment (row dk = 16 kt + r, tokens 32 s + 8 kg ..) of the transpose of a token tile in LDS: two transposing
    // reads; lane 4e + c of a 16-lane group addresses tokens 32 s + 8 kg (+ 4) + e, dk 16 kt + 4c .. 4c+3
    auto tile_tr_frag = [&](const T *tile, int s) -> Frag {
        if constexpr (STAGED) {
            const int row = s * 32 + kg * 8 + (r >> 2), c = kt * (16 / E) + ((r & 3) * 4) / E, sub = ((r & 3) * 4) % E;
            return tr_pair(tile + row * D + ((c ^ (row & XM)) * E) + sub,
                           tile + (row + 4) * D + ((c ^ ((row + 4) & XM)) * E) + sub);
        } else {
            return Frag{};
        }
    };
    // this wave's 16 rows (dk tile kt) of a [dk][dv] state tile as A fragments
    auto load_state = [&](Frag(&f)[KSV], const T *tile) {
#pragma unroll
        for (int s = 0; s < KSV; ++s) f[s] = O::load(at32(tile, (unsigned)vblk(DK, kt * 16 + r, s * O::KSTEP + kg * E)));
    };
    // this lane's share of <X, Y> = sum over the wave's 16 rows and all dv of X[dk][dv] Y[dk][dv] for two state tiles
    // held as fragments: the matrix unit forms X Y^T (16 x 16, contraction over dv; a fragment serves as A and as B
    // operand alike) and the trace is picked off the accumulators, element (m, m) sitting in lane r = m, kg = m / 4.
    // (Multiplying the 2 x 512 register elements out on the vector unit took ~100 instructions per product, a
    // sixth of the kernel's longest phase.)
    auto dot_frags = [&](const Frag(&x)[KSV], const Frag(&y)[KSV]) {
        f32x4 dd = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < KSV; ++u) dd = O::mma(x[u], y[u], dd);
        const int c = r & 3;
        const float v = c == 0 ? dd[0] : c == 1 ? dd[1] : c == 2 ? dd[2] : dd[3];
        return (r >> 2) == kg ? v : 0.f;
    };

    // ---- what a chunk needs first is requested as early as possible: its gates, its token tiles (straight into
    //      LDS, waves 6 and 7) and its q fragments.  For every chunk but the workgroup's first that is during
    //      the coefficient phase of the chunk before, which has no memory traffic of its own.
    float n_al = 0.f, n_be = 0.f, n_mu = 0.f, n_et = 1.f; // gates of token `lane` of the chunk being requested
    auto request_gates = [&]() {
        if (w < 6) { // waves 6, 7 never use them, and must not wait for anything behind their tile transfers
            n_al = *at32(a.alpha + tok0, gl);
            n_be = *at32(a.beta + tok0, gl);
            n_mu = *at32(a.mu + tok0, gl);
            n_et = a.eta ? *at32(a.eta + tok0, gl) : 1.f;
        }
    };
    // ---- phase 0: forward coefficients of the chunk whose gates are in n_*: waves 0-3 the matrices Gamma, Rho
    //      (16 rows each), wave 4 the vectors by wave scans
    float g_al = 0.f, g_be = 0.f, g_mu = 0.f, g_et = 1.f; // gates of token `lane` of the current chunk
    float pa = 0.f, pm = 0.f, pb = 0.f;                   // a_lane, m_lane, b_lane of the current chunk (wave 4)
    auto phase0 = [&]() {
        g_al = n_al;
        g_be = n_be;
        g_mu = n_mu;
        g_et = n_et;
        if (w < 4) {
            float gC, rC;
            coef_column_scan_blocked<true>(g_al, g_be, g_mu, sG, sRho, LDG, w, gC, rC, lane);
            if (w == 3) {
                s_gC[lane] = gC; // Gamma_{C,j}
                s_rC[lane] = rC; // Rho_{C,j}
            }
        }
        if (w == 4) {
            pa = scan_prod(g_al, lane);
            pm = scan_prod(g_mu, lane);
            float c = g_al;
            pb = g_be * pm;
            scan_affine_fwd(c, pb, lane);
            s_al[lane] = g_al;
            s_et[lane] = g_et;
            s_a[lane] = pa;
            s_b[lane] = pb;
        }
    };

    for (int c = tid; c < LDG; c += GT) sDG2[64 * LDG + c] = 0.f;
    request_gates();
    if (STAGED && w >= 6) {
        dma_token_tile<T, D>(sVt, vtg, rsv, w - 6, lane);
        dma_token_tile<T, D>(sK, kgl, rsk, w - 6, lane);
        dma_token_tile<T, D>(sQ, qg, rsk, w - 6, lane);
        dma_token_tile<T, D>(sDO, dog, rsv, w - 6, lane);
        dma_token_tile<T, D>(sDR, drg, rsv, w - 6, lane);
    }
    phase0();

    const int ldV = (int)rsv, ldK = (int)rsk; // row strides of the global tiles (fp32 path)
    for (;;) {
    refresh_ids();
    const T *tVt = STAGED ? sVt : vtg, *tK = STAGED ? sK : kgl, *tQ = STAGED ? sQ : qg, *tDR = STAGED ? sDR : drg, *tDO = STAGED ? sDO : dog;
    if (STAGED && w >= 6) __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): this chunk's tiles have landed
    __syncthreads(); // token tiles in LDS, coefficients ready
    // what the later phases read goes on its way now, in order of use
    Frag aK[KS2], aQ[KS2]; // this wave's rows of K^T, Q^T (A fragments: row dk = 16 kt + r, contraction over tokens)
#pragma unroll
    for (int s = 0; s < KS2; ++s) {
        if constexpr (STAGED) {
            // out of the k, q tiles in LDS by transposing reads (the tiles give way to the W matrices after
            // phase A, so now): no second trip to HBM for bytes the CU already holds
            aK[s] = tile_tr_frag(sK, s);
            aQ[s] = tile_tr_frag(sQ, s);
        } else {
            aK[s] = O::load(at32(KTg, (unsigned)kblk<T>(DK, kt * 16 + r, s * O::KSTEP + kg * E)));
            aQ[s] = O::load(at32(QTg, (unsigned)kblk<T>(DK, kt * 16 + r, s * O::KSTEP + kg * E)));
        }
    }
    Frag fS[KSV], fM[KSV], fdS[KSV], fdM[KSV];
    load_state(fS, Sg);
    if (DEEP) load_state(fM, Mg);
    sched_fence();

    // ---------------- phase A: the four 64x64 products (transposed: rows j, column i) and the
    //                  masked matrices built from them
    f32x4 accB[2], accA[2], accQK[2], accKK[2];
    {
        Frag fdO[KSV], fdR[KSV], fk[KSK], fq[KSK];
#pragma unroll
        for (int s = 0; s < KSV; ++s) {
            fdO[s] = tfrag(tDO, ldV, i, s);
            fdR[s] = tfrag(tDR, ldV, i, s);
        }
#pragma unroll
        for (int s = 0; s < KSK; ++s) {
            fk[s] = tfrag(tK, ldK, i, s);
            fq[s] = tfrag(tQ, ldK, i, s);
        }
#pragma unroll
        for (int mh = 0; mh < 2; ++mh) {
            accB[mh] = accA[mh] = accQK[mh] = accKK[mh] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (mh == 1 && !hasB) continue;
            const int j0 = (mh == 0 ? jA : 1) * 16 + r;
#pragma unroll
            for (int s = 0; s < KSV; ++s) {
                const Frag fv = tfrag(tVt, ldV, j0, s);
                accB[mh] = O::mma(fv, fdO[s], accB[mh]);
                accA[mh] = O::mma(fv, fdR[s], accA[mh]);
            }
#pragma unroll
            for (int s = 0; s < KSK; ++s) {
                const Frag fkk = tfrag(tK, ldK, j0, s);
                accQK[mh] = O::mma(fkk, fq[s], accQK[mh]);
                accKK[mh] = O::mma(fkk, fk[s], accKK[mh]);
            }
        }
    }
    // k and q of this wave's tokens in accumulator layout: element x is dk = kt*16 + kg*4 + x
    //  (kept in storage form: widening them here would make the wave wait for every load issued so far)
    typename Raw4<T>::type kv[TT], qv[TT];
    if (STAGED) {
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const int it = (tg * TT + t) * 16 + r, c = kt * (16 / E) + (kg * 4) / E; // 16-byte piece of the row
            const int o = it * D + ((c ^ (it & XM)) * E) + (kg * 4) % E;
            kv[t] = load4_raw(sK + o);
            qv[t] = load4_raw(sQ + o);
        }
    }
    if (STAGED) __syncthreads(); // everybody is done with the k and q tiles: the W matrices take their place
    {
        // this lane: token i (row of the masked matrices), columns j0 .. j0+3 of tile mt; everything a row needs
        // is 16 contiguous bytes, read and written as such
        const float al_i = s_al[i];
#pragma unroll
        for (int mh = 0; mh < 2; ++mh) {
            if (mh == 1 && !hasB) continue;
            const int mt = mh == 0 ? jA : 1, j0 = mt * 16 + kg * 4;
            const f32x4 gam = *reinterpret_cast<const f32x4 *>(&sG[i * LDG + j0]);
            const f32x4 gprev = (i > 0) ? *reinterpret_cast<const f32x4 *>(&sG[(i - 1) * LDG + j0]) : f32x4{0.f, 0.f, 0.f, 0.f};
            const f32x4 et = *reinterpret_cast<const f32x4 *>(&s_et[j0]);
            f32x4 w1e, w2e, w1s, w2a, dg1, dg2;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int j = j0 + x;
                const float dBm = (j <= i) ? accB[mh][x] : 0.f;
                const float dA = (j < i) ? -accA[mh][x] : 0.f;
                dg1[x] = dBm * (d.scale * et[x] * accQK[mh][x]);
                dg2[x] = dA * (al_i * et[x] * accKK[mh][x]);
                const float w1 = dBm * gam[x], w2 = dA * gprev[x];
                w1e[x] = w1 * et[x];
                w2e[x] = w2 * et[x];
                w1s[x] = w1 * d.scale;
                w2a[x] = w2 * al_i;
            }
            *reinterpret_cast<f32x4 *>(&sDG1[i * LDG + j0]) = dg1;
            *reinterpret_cast<f32x4 *>(&sDG2[i * LDG + j0]) = dg2;
            store4(sW1e + i * LDW + j0, w1e);
            store4(sW2e + i * LDW + j0, w2e);
            if (WTR) { // kept [i][j] like the others; the products that contract over i read them transposed
                store4(sW1T + i * LDW + j0, w1s);
                store4(sW2T + i * LDW + j0, w2a);
            } else {
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    sW1T[(j0 + x) * LDW + i] = from_f32<T>(w1s[x]);
                    sW2T[(j0 + x) * LDW + i] = from_f32<T>(w2a[x]);
                }
            }
        }
        // the tiles of this wave's rows above the diagonal: zeros in all six matrices
#pragma unroll
        for (int mt = 1; mt < 4; ++mt) {
            if (!((zt >> mt) & 1)) continue;
            const int j0 = mt * 16 + kg * 4;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<f32x4 *>(&sDG1[i * LDG + j0]) = z;
            *reinterpret_cast<f32x4 *>(&sDG2[i * LDG + j0]) = z;
            store4(sW1e + i * LDW + j0, z);
            store4(sW2e + i * LDW + j0, z);
            if (WTR) {
                store4(sW1T + i * LDW + j0, z);
                store4(sW2T + i * LDW + j0, z);
            } else {
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    sW1T[(j0 + x) * LDW + i] = from_f32<T>(0.f);
                    sW2T[(j0 + x) * LDW + i] = from_f32<T>(0.f);
                }
            }
        }
    }
    __syncthreads();
    if (!STAGED) { // (staged: taken from the tiles in LDS before the W matrices replaced them)
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const int it = (tg * TT + t) * 16 + r;
            kv[t] = load4_raw(at32(kgl, it * rsk + kt * 16 + kg * 4));
            qv[t] = load4_raw(at32(qg, it * rsk + kt * 16 + kg * 4));
        }
        sched_fence(); // q, k rows are needed first: keep them ahead of the state tiles in the return order
    }
    if (DEEP) {
        load_state(fdS, dSg); // dM' follows once S is no longer needed
    }
    sched_fence(); // these loads leave now, not after the products below
    // ---------------- phase B: the token-contractions W1 K~, W2 K~, W1^T Q~, W2^T P
    // B fragment (column j = j0 + r, contraction over i, step s) of W1^T / W2^T
    auto wt_frag = [&](const T *m, int j0, int s) -> Frag {
        if constexpr (WTR)
            return tr_frag(m, LDW, s * O::KSTEP, j0, r, kg);
        else
            return O::load(m + (j0 + r) * LDW + s * O::KSTEP + kg * E);
    };
    f32x4 accQ[TT], accP[TT], accK[TT]; // dQ~^T, dP^T, dK~^T: [dk tile kt][token tile t of this group]
    zero_acc(accQ);
    zero_acc(accP);
    zero_acc(accK);
    // W1, W2 are lower triangular ([i][j], zero for j > i): a contraction step whose 32 source tokens all lie on the zero
    // side of the token tile adds exact zeros and is left out (a quarter of the phase's products)
#pragma unroll
    for (int s = 0; s < KS2; ++s)
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const int tile = tg * TT + t, j_lo = s * O::KSTEP, j_hi = j_lo + O::KSTEP - 1; // the step's source tokens
            const int wo = (tile * 16 + r) * LDW + s * O::KSTEP + kg * E;
            if (j_lo <= tile * 16 + 15) { // rows i of this tile against columns j of the step: some j <= i
                accQ[t] = O::mma(aK[s], O::load(sW1e + wo), accQ[t]);
                accP[t] = O::mma(aK[s], O::load(sW2e + wo), accP[t]);
            }
            if (j_hi >= tile * 16) { // columns j of this tile against rows i of the step: some i >= j
                accK[t] = O::mma(aQ[s], wt_frag(sW1T, tile * 16, s), accK[t]);
                accK[t] = O::mma(aK[s], wt_frag(sW2T, tile * 16, s), accK[t]);
            }
        }
    __syncthreads(); // the W space is free for the partial sums

    // ---------------- phases C-F: products with the four state matrices.  X^T[dk][i] = sum_dv St[dk][dv] f[i][dv]
    // two products sharing their B fragments (LDS reads are what bounds these phases):
    //   t1^T[dk][i] = sum_dv Fa[dk][dv] X[i][dv],  t2^T likewise with Fb
    auto state_product2 = [&](const Frag(&fa)[KSV], const Frag(&fb)[KSV], const T *tile, f32x4(&t1)[TT], f32x4(&t2)[TT],
                              bool add = false) {
        if (!add) {
            zero_acc(t1);
            zero_acc(t2);
        }
#pragma unroll
        for (int s = 0; s < KSV; ++s) {
#pragma unroll
            for (int t = 0; t < TT; ++t) {
                const Frag x = tfrag(tile, ldV, (tg * TT + t) * 16 + r, s);
                t1[t] = O::mma(fa[s], x, t1[t]);
                t2[t] = O::mma(fb[s], x, t2[t]);
            }
            sched_fence();
        }
    };
    auto part = [&](int q, int it) -> float & { return spart[(q * NKW + kt) * 64 + it]; };
    float p1 = 0.f, p2 = 0.f, p3 = 0.f; // partial <dS',S>, <dS',M>, <dM',M>
    f32x4 t1[TT], t2[TT];

    // C: S and M against dO
    if (!DEEP) load_state(fM, Mg);
    state_product2(fS, fM, tDO, t1, t2);
    // the row dots of a phase: every lane's share per token tile first, then all token tiles' sums over the lane groups
    // at once; group kg ends up with the sums of token tile kg and writes them
    const int itg = (tg * TT + (kg & (TT - 1))) * 16 + r;
    float ra[TT], rb[TT], rc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const int it = (tg * TT + t) * 16 + r;
        const f32x4 qw = widen4(qv[t]);
        ra[t] = dot4(t1[t], qw);
        rb[t] = dot4(t2[t], qw);
        accQ[t] += s_a[it] * t1[t] - s_b[it] * t2[t];
        store4(at32(static_cast<T *>(a.dq) + tok0 * DK, it * rsk + kt * 16 + kg * 4), d.scale * accQ[t]);
    }
    {
        const float da = d.scale * reduce_tiles(ra), db = -d.scale * reduce_tiles(rb);
        if (kg < TT) {
            part(P_DA, itg) = da;
            part(P_DB, itg) = db;
        }
    }
    // D: S and M against dR
    load_state(fdM, dMg);
    if (!DEEP) load_state(fdS, dSg);
    state_product2(fS, fM, tDR, t1, t2);
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const int it = (tg * TT + t) * 16 + r;
        const f32x4 kw = widen4(kv[t]);
        ra[t] = dot4(t1[t], kw);
        rb[t] = dot4(t2[t], kw);
        accP[t] += ((it > 0) ? s_b[it - 1] : 0.f) * t2[t] - ((it > 0) ? s_a[it - 1] : 1.f) * t1[t];
        rc[t] = dot4(accP[t], kw);
    }
    {
        const float al_i = s_al[itg];
        const float dam = -al_i * reduce_tiles(ra), dbm = al_i * reduce_tiles(rb), dalk = reduce_tiles(rc);
        if (kg < TT) {
            part(P_DAM, itg) = dam;
            part(P_DBM, itg) = dbm;
            part(P_DALK, itg) = dalk;
        }
    }
    if (tg == 0) {
        p1 = dot_frags(fdS, fS);
        p2 = dot_frags(fdS, fM);
        p3 = dot_frags(fdM, fM);
    }
    // E: dS' and dM' against V~
    state_product2(fdS, fdM, tVt, t1, t2);
    if constexpr (LO) {
        // the remainders: (hi + lo)(hi + lo) without the lo lo term, one tile of remainders in registers at a time
        Frag fx[KSV];
        load_state(fx, Slg);
        if (tg == 0) p1 += dot_frags(fdS, fx);
        load_state(fx, Slg + DK * DV);
        if (tg == 0) {
            p2 += dot_frags(fdS, fx);
            p3 += dot_frags(fdM, fx);
        }
        load_state(fdS, dSlg);
        if (tg == 0) {
            p1 += dot_frags(fdS, fS);
            p2 += dot_frags(fdS, fM);
        }
        load_state(fdM, dSlg + DK * DV);
        if (tg == 0) p3 += dot_frags(fdM, fM);
        state_product2(fdS, fdM, tVt, t1, t2, true);
    }
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const int it = (tg * TT + t) * 16 + r;
        const f32x4 kw = widen4(kv[t]);
        ra[t] = dot4(t1[t], kw);
        rb[t] = dot4(t2[t], kw);
        accK[t] += s_gC[it] * t1[t] - s_rC[it] * t2[t];
        rc[t] = dot4(accK[t], kw);
        store4(at32(static_cast<T *>(a.dk) + tok0 * DK, it * rsk + kt * 16 + kg * 4), s_et[it] * accK[t] + s_al[it] * accP[t]);
    }
    {
        const float et_i = s_et[itg];
        const float dgc = et_i * reduce_tiles(ra), drc = -et_i * reduce_tiles(rb), detk = reduce_tiles(rc);
        if (kg < TT) {
            part(P_DGC, itg) = dgc;
            part(P_DRC, itg) = drc;
            part(P_DETK, itg) = detk;
        }
    }
    p1 = reduce64(p1);
    p2 = reduce64(p2);
    p3 = reduce64(p3);
    if (lane == 0) { s_red[w][0] = p1; s_red[w][1] = p2; s_red[w][2] = p3; }
    __syncthreads();

    // ---------------- phase 4: reverse of the coefficient scans.  Waves 0-3: the matrices (16 rows each, two
    //                  parts around a barrier); wave 4 (which holds a, b, m): the vectors.
    auto total = [&](int q) { // sum over the dk tiles of one row dot of token `lane`
        float s = 0.f;
#pragma unroll
        for (int k2 = 0; k2 < NKW; ++k2) s += spart[(q * NKW + k2) * 64 + lane];
        return s;
    };
    // the workgroup's next chunk: gates and three of the four token tiles go on their way now
    // (the LDS space of V~, dO, dR is free; that of k holds this phase's matrices until the row sums are done)
    const size_t tok0_cur = tok0;
    const int next = chunk + (int)gridDim.x;
    const bool has_next = STAGED && next < nchunks; // (the unstaged kernel is launched with one workgroup per chunk)
    if (has_next) {
        set_chunk(next);
        request_gates();
        if (STAGED && w >= 6) {
            dma_token_tile<T, D>(sVt, vtg, rsv, w - 6, lane);
            dma_token_tile<T, D>(sDO, dog, rsv, w - 6, lane);
            dma_token_tile<T, D>(sDR, drg, rsv, w - 6, lane);
        }
    }
    RevScanRows rr;
    float db = 0.f, dm = 0.f;
    if (w < 4) {
        float dgc = 0.f, drc = 0.f;
        if (w == 3) {
            dgc = total(P_DGC);
            drc = total(P_DRC);
        }
        coef_scan_reverse_part1(g_al, g_be, g_mu, sDG1, sDG2, dgc, drc, LDG, w, rr, sTop, lane);
    }
    if (w == 5) {
        coef_scan_reverse_rowcoefs(g_al, g_be, g_mu, sRowC, lane);
        // the vector chain of a (it does not meet those of b and m before the final sums): reverse of
        // a_i = alpha_i a_{i-1} with a^-_i = a_{i-1}:  da_i = Da_i + Da^-_{i+1} + alpha_{i+1} da_{i+1}; its share of
        // dalpha_i, da_i a_{i-1} + k_i.dP_i, and deta_i go to wave 4 through LDS
        float dS_S = 0.f;
#pragma unroll
        for (int ww = 0; ww < 8; ++ww) dS_S += s_red[ww][0];
        const float t_da = total(P_DA), t_dam = total(P_DAM), t_dalk = total(P_DALK);
        const int li = lane;
        const float al_next = wave_down1(g_al, 0.f, lane), dam_dn = wave_down1(t_dam, 0.f, lane);
        float ca = (li < 63) ? al_next : 0.f;
        float da5 = t_da + ((li < 63) ? dam_dn : dS_S);
        scan_affine_rev(ca, da5, lane);
        s_da[li] = da5 * ((li > 0) ? s_a[li - 1] : 1.f) + t_dalk;
        s_de[li] = total(P_DETK);
    }
    if (w == 4) {
        // vectors (lane i = token i): reverse of b_i = alpha_i b_{i-1} + beta_i m_i, m_i = mu_i m_{i-1}, with
        // b^-_i = b_{i-1}:
        //   db_i = Db_i + Db^-_{i+1} + alpha_{i+1} db_{i+1},  dm_i = Dm_i + beta_i db_i + mu_{i+1} dm_{i+1}
        float dS_M = 0.f, dM_M = 0.f;
#pragma unroll
        for (int ww = 0; ww < 8; ++ww) {
            dS_M += s_red[ww][1];
            dM_M += s_red[ww][2];
        }
        const float t_db = total(P_DB), t_dbm = total(P_DBM);
        const int li = lane;
        const float al_next = wave_down1(g_al, 0.f, lane), mu_next = wave_down1(g_mu, 0.f, lane);
        const float dbm_dn = wave_down1(t_dbm, 0.f, lane);
        float cb = (li < 63) ? al_next : 0.f;
        db = t_db + ((li < 63) ? dbm_dn : -dS_M);
        scan_affine_rev(cb, db, lane);
        float cm = (li < 63) ? mu_next : 0.f;
        dm = (li == 63 ? dM_M : 0.f) + g_be * db;
        scan_affine_rev(cm, dm, lane);
    }
    __syncthreads(); // segment top rows exchanged; every partial sum has been read (their space is reused now)
    if (w < 4) coef_scan_reverse_part2(LDG, w, rr, sTop, sRowC, sGa, sRa, lane);
    __syncthreads();
    {
        // dalpha_i += sum_{j<i} G_ij Gamma_{i-1,j};  dbeta_i += sum_{j<=i} G_ij Rho_ij;
        // dmu_i += sum_{j<i} R_ij Rho_{i-1,j}: 8 threads per row, 8 consecutive columns each;
        // G, R, Gamma, Rho are zero above the diagonal
        const int row = tid >> 3, pt = tid & 7, rowm = row > 0 ? row - 1 : 0;
        float ga = 0.f, gb = 0.f, gm = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int j = pt * 8 + u * 4;
            const f32x4 G = *reinterpret_cast<const f32x4 *>(&sGa[row * LDG + j]);
            const f32x4 R = *reinterpret_cast<const f32x4 *>(&sRa[row * LDG + j]);
            const f32x4 rho = *reinterpret_cast<const f32x4 *>(&sRho[row * LDG + j]);
            const f32x4 gp = *reinterpret_cast<const f32x4 *>(&sG[rowm * LDG + j]);
            const f32x4 rp = *reinterpret_cast<const f32x4 *>(&sRho[rowm * LDG + j]);
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                gb += G[x] * rho[x];
                ga += (j + x < row) ? G[x] * gp[x] : 0.f;
                gm += (j + x < row) ? R[x] * rp[x] : 0.f;
            }
        }
        // sum over the 8 lanes of a token (quad exchanges, then the neighbouring quad by a row rotation each way:
        // lanes 0-3 of an aligned group of 8 take the quad to their right, lanes 4-7 the one to their left)
        auto sum8 = [&](float v) {
            v += dpp_move<0xB1>(v);
            v += dpp_move<0x4E>(v);
            const float up = dpp_move<0x12C>(v), dn = dpp_move<0x124>(v); // row_ror 12 = lane + 4, row_ror 4 = lane - 4
            return v + ((lane & 4) ? dn : up);
        };
        ga = sum8(ga);
        gb = sum8(gb);
        gm = sum8(gm);
        if (pt == 0) { s_ga[row] = ga; s_gb[row] = gb; s_gm[row] = gm; }
    }
    __syncthreads();
    if (w == 4) {
        const int li = lane;
        const float bprev = wave_up1(pb, 0.f, lane), mprev = wave_up1(pm, 1.f, lane);
        const float b_prev = (li > 0) ? bprev : 0.f, m_prev = (li > 0) ? mprev : 1.f;
        const unsigned g = (unsigned)(li * d.H);
        *at32(a.dalpha + tok0_cur, g) = s_ga[li] + db * b_prev + s_da[li];
        *at32(a.dbeta + tok0_cur, g) = s_gb[li] + db * pm;
        *at32(a.dmu + tok0_cur, g) = s_gm[li] + dm * m_prev;
        if (a.deta) *at32(a.deta + tok0_cur, g) = s_de[li];
    }
    if (!has_next) break;
    chunk = next;
    if (STAGED && w >= 6) { // the row sums are done with the space of the k and q tiles
        dma_token_tile<T, D>(sK, kgl, rsk, w - 6, lane);
        dma_token_tile<T, D>(sQ, qg, rsk, w - 6, lane);
    }
    phase0(); // Gamma, Rho are free again after the row sums; the next chunk's gates arrived long ago
    } // chunks of this workgroup
}

template <typename T, int DK, int DV, bool STAGED, bool LO = false>
hipError_t launch_t(const Dims &d, const GradArgs &a, hipStream_t s) {
    // staged (bf16): one workgroup per CU, each walking its share of the chunks; otherwise one per chunk
    const int nchunks = (d.n1 - d.n0) * d.BH;
    dim3 grid(STAGED && nchunks > num_cus() ? num_cus() : nchunks), block(GT);
    hipLaunchKernelGGL((grad_kernel<T, DK, DV, STAGED, LO>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_grad(const Dims &d, const GradArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (!a.states_lo != !a.dstates_lo || (f32 && a.states_lo)) return hipErrorInvalidValue;
    if (a.states_lo) { // 16-bit storage with the rounding remainders of the state tensors
        if (d.dk == 64 && d.dv == 64) return launch_t<bf16_t, 64, 64, true, true>(d, a, s);
        if (d.dk == 128 && d.dv == 128) return launch_t<bf16_t, 128, 128, true, true>(d, a, s);
        return hipErrorInvalidValue;
    }
    if (d.dk == 64 && d.dv == 64)
        return f32 ? launch_t<float, 64, 64, false>(d, a, s) : launch_t<bf16_t, 64, 64, true>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_t<float, 128, 128, false>(d, a, s) : launch_t<bf16_t, 128, 128, true>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
