// Wave-level building blocks for the per-chunk gate coefficients of Sec. 3.1 (Eq. "coefficients")
// in their division-free form, and for the 64x64 unit-lower-triangular solve T = (I + A)^{-1}.
//
//   a_i = prod_{l<=i} alpha_l,  m_i = prod_{l<=i} mu_l,  b_i = alpha_i b_{i-1} + beta_i m_i
//   Rho_ij = prod_{l=j+1..i} mu_l,  Am_ij = prod_{l=j+1..i} alpha_l   (i >= j, 1 on the diagonal)
//   Gamma_ij = alpha_i Gamma_{i-1,j} + beta_i Rho_ij  ( = sum_l Am_il beta_l Rho_lj )
#pragma once
#include "mdn_device.h"

namespace mdn {

// ---- lane shifts inside the 16-lane rows of a wave, as data-parallel-primitive moves (a few clocks; a general
//      cross-lane shuffle goes through the LDS pipeline and costs ~100 clocks on a dependent chain)
// value of lane - N of the same row; `fill` in the N lowest lanes of each row
template <int N> __device__ __forceinline__ float row_up(float v, float fill) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), 0x110 | N, 0xF, 0xF, false));
}
// value of lane + N of the same row; `fill` in the N highest lanes of each row
template <int N> __device__ __forceinline__ float row_down(float v, float fill) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), 0x100 | N, 0xF, 0xF, false));
}

// value held by lane `src` (wave-uniform: a constant or a scalar) as a wave-uniform scalar
__device__ __forceinline__ float lane_bcast(float v, int src) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}

// value of lane + 1 / lane - 1 across the whole wave (`fill` in lane 63 / lane 0): the row shift, with the three
// lanes at the row boundaries patched by scalar broadcasts
__device__ __forceinline__ float wave_down1(float v, float fill, int lane) {
    float r = row_down<1>(v, fill);
    const float b16 = lane_bcast(v, 16), b32 = lane_bcast(v, 32), b48 = lane_bcast(v, 48);
    r = (lane == 15) ? b16 : r;
    r = (lane == 31) ? b32 : r;
    r = (lane == 47) ? b48 : r;
    return r;
}
__device__ __forceinline__ float wave_up1(float v, float fill, int lane) {
    float r = row_up<1>(v, fill);
    const float b15 = lane_bcast(v, 15), b31 = lane_bcast(v, 31), b47 = lane_bcast(v, 47);
    r = (lane == 16) ? b15 : r;
    r = (lane == 32) ? b31 : r;
    r = (lane == 48) ? b47 : r;
    return r;
}

// ---- scans across the 64 lanes of a wave; lane i holds element i.  Inside each 16-lane row by four shift-and-
//      combine steps (the fill value is the identity of the combination, so no lane needs a select), then the
//      rows are chained through three scalar broadcasts.  (The lane index is a parameter so that a caller with
//      a long-running loop can pass its own, loop-variant copy.)

// inclusive prefix product
__device__ __forceinline__ float scan_prod(float v, int lane = lane_id()) {
    v *= row_up<1>(v, 1.f);
    v *= row_up<2>(v, 1.f);
    v *= row_up<4>(v, 1.f);
    v *= row_up<8>(v, 1.f);
#pragma unroll
    for (int row = 1; row < 4; ++row) {
        const float p = lane_bcast(v, 16 * row - 1); // product up to the end of the row before
        if ((lane >> 4) == row) v *= p;
    }
    return v;
}

// x_i = c_i x_{i-1} + d_i with x_{-1} = 0: on return d holds x_i (c is used up)
__device__ __forceinline__ void scan_affine_fwd(float &c, float &d, int lane = lane_id()) {
#define MDN_STEP(N)                                                   \
    {                                                                 \
        const float oc = row_up<N>(c, 1.f), od = row_up<N>(d, 0.f);   \
        d = c * od + d;                                               \
        c = c * oc;                                                   \
    }
    MDN_STEP(1) MDN_STEP(2) MDN_STEP(4) MDN_STEP(8)
#undef MDN_STEP
#pragma unroll
    for (int row = 1; row < 4; ++row) {
        const float x = lane_bcast(d, 16 * row - 1); // x at the end of the row before
        if ((lane >> 4) == row) d = c * x + d;
    }
}

// x_i = c_i x_{i+1} + d_i with x_64 = 0: on return d holds x_i (c is used up)
__device__ __forceinline__ void scan_affine_rev(float &c, float &d, int lane = lane_id()) {
#define MDN_STEP(N)                                                       \
    {                                                                     \
        const float oc = row_down<N>(c, 1.f), od = row_down<N>(d, 0.f);   \
        d = c * od + d;                                                   \
        c = c * oc;                                                       \
    }
    MDN_STEP(1) MDN_STEP(2) MDN_STEP(4) MDN_STEP(8)
#undef MDN_STEP
#pragma unroll
    for (int row = 2; row >= 0; --row) {
        const float x = lane_bcast(d, 16 * (row + 1)); // x at the start of the row after
        if ((lane >> 4) == row) d = c * x + d;
    }
}

// ---- column scans of the 64x64 coefficient matrices; one wave, lane j owns column j and also HOLDS
//      the gates of token j (al, be, mu); the gates of row i reach all lanes through v_readlane.
//      sG[i*ldg + j] = Gamma_ij (0 above the diagonal).  The final values (row 63) are returned.
//      If WANT_RHO: sRho[i*ldg + j] = Rho_ij as well.
template <bool WANT_RHO>
__device__ __forceinline__ void coef_column_scan(float al, float be, float mu, float *sG, float *sRho, int ldg,
                                                 float &gC, float &rC) {
    const int j = lane_id();
    float g = 0.f, rho = 0.f;
#pragma unroll
    for (int i = 0; i < 64; ++i) {
        const float a_i = lane_bcast(al, i), b_i = lane_bcast(be, i), m_i = lane_bcast(mu, i);
        rho = (i == j) ? 1.f : rho * m_i;
        g = a_i * g + b_i * rho;
        sG[i * ldg + j] = g;
        if (WANT_RHO) sRho[i * ldg + j] = rho;
    }
    gC = g;
    rC = rho;
}

// ---- the same column scans split over 4 waves: wave w (0..3) produces rows 16w .. 16w+15 of Gamma
//      (and Rho) for all 64 columns, lane j = column j, every wave holding the gates of token `lane`.
//      The state (g, rho) of column j moves from row i-1 to row i by the triangular map
//        T_i = [alpha_i, beta_i mu_i; 0, mu_i],   starting from (beta_j, 1) in row j.
//      A wave gets the state its columns have in row 16w-1 without walking there: products of the T_i
//      inside each 16-row segment by a segmented suffix scan over the lanes, then at most two whole
//      segment maps on top.  After that, 16 dependent steps instead of 64.
//      gC, rC (row 63) are returned by wave 3 only.
template <bool WANT_RHO>
__device__ __forceinline__ void coef_column_scan_blocked(float al, float be, float mu, float *sG, float *sRho, int ldg,
                                                         int w, float &gC, float &rC, int j = lane_id()) {
    const int jl = j & 15;
    // inclusive suffix products inside the 16-lane segment: (A, B, M)_j = T_end o ... o T_j
    // ((A2, B2, M2) o (A, B, M): this lane's map first, the later rows' after it; the fill is the identity map)
    float A = al, B = be * mu, M = mu;
#define MDN_STEP(N)                                                                                  \
    {                                                                                                \
        const float A2 = row_down<N>(A, 1.f), B2 = row_down<N>(B, 0.f), M2 = row_down<N>(M, 1.f);    \
        B = A2 * B + B2 * M;                                                                         \
        A = A2 * A;                                                                                  \
        M = M2 * M;                                                                                  \
    }
    MDN_STEP(1) MDN_STEP(2) MDN_STEP(4) MDN_STEP(8)
#undef MDN_STEP
    // exclusive: product of T_{j+1} .. T_end (identity for the last lane of a segment)
    const float Ax = row_down<1>(A, 1.f), Bx = row_down<1>(B, 0.f), Mx = row_down<1>(M, 1.f);
    // state of column j in the last row of its own segment
    float g = (jl < 15) ? Ax * be + Bx : be, rho = (jl < 15) ? Mx : 1.f;
    // on through whole segments up to row 16w - 1 (columns of segment J < I pass through segment I)
#pragma unroll
    for (int I = 1; I < 3; ++I) {
        const float As = lane_bcast(A, 16 * I), Bs = lane_bcast(B, 16 * I), Ms = lane_bcast(M, 16 * I);
        if (I < w && j < 16 * I) {
            g = As * g + Bs * rho;
            rho = Ms * rho;
        }
    }
    if (j >= 16 * w) { // columns that start inside (or below) this wave's rows
        g = 0.f;
        rho = 0.f;
    }
    // (w is wave-uniform: the lane selects below are scalar operands)
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int i = w * 16 + u;
        const float a_i = lane_bcast(al, i), b_i = lane_bcast(be, i), m_i = lane_bcast(mu, i);
        rho = (i == j) ? 1.f : rho * m_i;
        g = a_i * g + b_i * rho;
        sG[i * ldg + j] = g;
        if (WANT_RHO) sRho[i * ldg + j] = rho;
    }
    gC = g;
    rC = rho;
}

// ---- reverse of the column scans (adjoint): lane j owns column j.  With D_ij the direct adjoint of
//      Gamma_ij (sD1[i][j] + sD2[i+1][j], plus dgc_j in row 63) and drc_j the direct adjoint of Rho_63,j:
//        G_ij = D_ij + alpha_{i+1} G_{i+1,j}            R_ij = [i = 63] drc_j + beta_i G_ij + mu_{i+1} R_{i+1,j}
//      for i = 63 .. j.  Writes sGa[i][j] = G_ij, sRa[i][j] = R_ij (zero for i < j).
__device__ __forceinline__ void coef_column_scan_reverse(float al, float be, float mu, const float *sD1,
                                                         const float *sD2, float dgc, float drc, float *sGa,
                                                         float *sRa, int ldg) {
    const int j = lane_id();
    float cg = 0.f, cr = 0.f; // alpha_{i+1} G_{i+1,j}, mu_{i+1} R_{i+1,j}
    // 16 rows at a time: all direct adjoints of the block are read before its dependent chain starts
    // (every entry of sD1 / sD2 is defined, zero above the diagonal), so no LDS wait sits on the chain
#pragma unroll
    for (int i0 = 48; i0 >= 0; i0 -= 16) {
        float dir[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) dir[u] = sD1[(i0 + u) * ldg + j] + sD2[(i0 + u + 1) * ldg + j];
#pragma unroll
        for (int u = 15; u >= 0; --u) {
            const int i = i0 + u;
            const float a_i = lane_bcast(al, i), b_i = lane_bcast(be, i), m_i = lane_bcast(mu, i);
            float G = dir[u] + cg, R = cr;
            if (i == 63) {
                G += dgc;
                R += drc;
            }
            R += b_i * G;
            G = (i >= j) ? G : 0.f;
            R = (i >= j) ? R : 0.f;
            sGa[i * ldg + j] = G;
            sRa[i * ldg + j] = R;
            cg = a_i * G;
            cr = m_i * R;
        }
    }
}

// ---- the reverse column scans split over 4 waves: wave w (0..3) owns rows 16w .. 16w+15, lane j = column j.
//      Part 1 walks the wave's rows upwards with nothing coming in from the rows below (16 dependent
//      steps).  With the three coefficients with which an incoming pair (Gin, Rin) = (G, R) of the row below
//      the segment enters each row,
//        G_ij = Gloc_ij + gc_i Gin_j          R_ij = Rloc_ij + ec_i Gin_j + mc_i Rin_j
//        gc_i = alpha_{i+1} gc_{i+1},  mc_i = mu_{i+1} mc_{i+1},  ec_i = beta_i gc_i + mu_{i+1} ec_{i+1}
//      (gc = mc = 1, ec = 0 below the segment's last row; alpha_64 = mu_64 = 0: nothing comes in below row 63),
//      part 2, after a workgroup barrier, chains the top rows of the segments below to get what comes in, and
//      completes and stores the wave's rows.  The coefficients are the same for all columns: ONE wave forms
//      them for all 64 rows at once (lane = row, suffix scans inside the 16-lane segments) beside part 1.
struct RevScanRows {
    float G[16], R[16];
};
// sRowC: [3][64] floats (gc, ec, mc of every row); called by one whole wave, lane = row
__device__ __forceinline__ void coef_scan_reverse_rowcoefs(float al, float be, float mu, float *sRowC, int lane = lane_id()) {
    float gc = wave_down1(al, 0.f, lane), mc = wave_down1(mu, 0.f, lane); // alpha_{i+1}, mu_{i+1}; nothing below row 63
    const float y = mc;
    // inclusive suffix products inside the segment
#define MDN_STEP(N)                   \
    {                                 \
        gc *= row_down<N>(gc, 1.f);   \
        mc *= row_down<N>(mc, 1.f);   \
    }
    MDN_STEP(1) MDN_STEP(2) MDN_STEP(4) MDN_STEP(8)
#undef MDN_STEP
    float c = y, ec = be * gc; // ec_i = y_i ec_{i+1} + beta_i gc_i
#define MDN_STEP(N)                                                        \
    {                                                                      \
        const float oc = row_down<N>(c, 1.f), od = row_down<N>(ec, 0.f);   \
        ec = c * od + ec;                                                  \
        c = c * oc;                                                        \
    }
    MDN_STEP(1) MDN_STEP(2) MDN_STEP(4) MDN_STEP(8)
#undef MDN_STEP
    sRowC[lane] = gc;
    sRowC[64 + lane] = ec;
    sRowC[128 + lane] = mc;
}
// sTop: [4][2][64] floats (top rows: G, R)
__device__ __forceinline__ void coef_scan_reverse_part1(float al, float be, float mu, const float *sD1, const float *sD2,
                                                        float dgc, float drc, int ldg, int w, RevScanRows &rr, float *sTop,
                                                        int j = lane_id()) {
    const int i0 = w * 16; // (w is wave-uniform: the lane selects below are scalar operands)
    float dir[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) dir[u] = sD1[(i0 + u) * ldg + j] + sD2[(i0 + u + 1) * ldg + j];
    float cg = 0.f, cr = 0.f; // alpha_{i+1} Gloc_{i+1,j}, mu_{i+1} Rloc_{i+1,j}
#pragma unroll
    for (int u = 15; u >= 0; --u) {
        const int i = i0 + u;
        const float b_i = lane_bcast(be, i);
        float G = dir[u] + cg, R = cr;
        if (i == 63) {
            G += dgc;
            R += drc;
        }
        R += b_i * G;
        rr.G[u] = G;
        rr.R[u] = R;
        if (u > 0) {
            cg = lane_bcast(al, i) * G;
            cr = lane_bcast(mu, i) * R;
        }
    }
    sTop[(w * 2 + 0) * 64 + j] = (j <= i0) ? rr.G[0] : 0.f;
    sTop[(w * 2 + 1) * 64 + j] = (j <= i0) ? rr.R[0] : 0.f;
}

// Writes sGa[i][j] = G_ij, sRa[i][j] = R_ij for the wave's 16 rows (zero for i < j).
__device__ __forceinline__ void coef_scan_reverse_part2(int ldg, int w, const RevScanRows &rr, const float *sTop,
                                                        const float *sRowC, float *sGa, float *sRa, int j = lane_id()) {
    float Gin = 0.f, Rin = 0.f; // G, R of the row just below this wave's segment
#pragma unroll
    for (int seg = 3; seg >= 1; --seg) {
        if (seg > w) {
            const float gct = sRowC[seg * 16], ect = sRowC[64 + seg * 16], mct = sRowC[128 + seg * 16];
            const bool act = j <= seg * 16;
            const float Gt = sTop[(seg * 2 + 0) * 64 + j] + (act ? gct * Gin : 0.f);
            const float Rt = sTop[(seg * 2 + 1) * 64 + j] + (act ? ect * Gin + mct * Rin : 0.f);
            Gin = Gt;
            Rin = Rt;
        }
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int i = w * 16 + u;
        const float G = rr.G[u] + sRowC[i] * Gin;
        const float R = rr.R[u] + sRowC[64 + i] * Gin + sRowC[128 + i] * Rin;
        sGa[i * ldg + j] = (i >= j) ? G : 0.f;
        sRa[i * ldg + j] = (i >= j) ? R : 0.f;
    }
}

// ---- T = (I + A)^{-1}, A strictly lower triangular 64x64 fp32 in LDS (row-major, stride lda, zeros on
//      and above the diagonal), by 16x16 blocks.  Called by 4 waves (w = 0..3); wave w owns block row w.
//      On return sA holds T (row-major).  sTT is scratch of 64*lda floats.
//        T_ii = (I + A_ii)^{-1}                              (forward substitution, lane = column)
//        T_ij = -T_ii * sum_{k=j..i-1} A_ik T_kj   (i > j)    (fp32 MFMA; levels i - j = 1, 2, 3)
//      The accumulator of the inner sum is, lane for lane, the B fragment of the product with T_ii.
__device__ __forceinline__ void tri_inverse_blocked(float *sA, float *sTT, int lda, int w) {
    typedef Op<float> O;
    const int lane = lane_id(), r = lane & 15, kg = lane >> 4;
    const int b0 = w * 16;
    // diagonal block: lanes 0..15, lane r solves column r of block w; t[k] = T_ww[k][r]
    if (lane < 16) {
        float t[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) t[i] = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float acc = (i == r) ? 1.f : 0.f;
#pragma unroll
            for (int k4 = 0; k4 < (i + 3) / 4; ++k4) {
                const f32x4 av = *reinterpret_cast<const f32x4 *>(&sA[(b0 + i) * lda + b0 + 4 * k4]);
                acc -= av[0] * t[4 * k4 + 0];
                acc -= av[1] * t[4 * k4 + 1];
                acc -= av[2] * t[4 * k4 + 2];
                acc -= av[3] * t[4 * k4 + 3];
            }
            t[i] = acc;
        }
        // T^T storage: sTT[col * lda + row]
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
            *reinterpret_cast<f32x4 *>(&sTT[(b0 + r) * lda + b0 + 4 * i4]) =
                f32x4{t[4 * i4], t[4 * i4 + 1], t[4 * i4 + 2], t[4 * i4 + 3]};
    }
    __syncthreads();
    // own diagonal block as A fragments: row r, k = 4*kg + s  ->  sTT[(b0 + k) * lda + b0 + r]
    f32x4 tii;
#pragma unroll
    for (int s = 0; s < 4; ++s) tii[s] = sTT[(b0 + 4 * kg + s) * lda + b0 + r];
    // write the diagonal block of T row-major (replacing A_ww, which is no longer needed)
#pragma unroll
    for (int s = 0; s < 4; ++s) sA[(b0 + r) * lda + b0 + 4 * kg + s] = tii[s];

    for (int dlt = 1; dlt < 4; ++dlt) {
        const int jb = w - dlt; // block column handled at this level
        if (jb >= 0) {
            f32x4 x = {0.f, 0.f, 0.f, 0.f};
            for (int kb = jb; kb < w; ++kb) {
                // A_{w,kb} (row-major, k contiguous) times T_{kb,jb} (from sTT: column-major, k contiguous)
                const f32x4 fa = *reinterpret_cast<const f32x4 *>(&sA[(b0 + r) * lda + kb * 16 + 4 * kg]);
                const f32x4 fb = *reinterpret_cast<const f32x4 *>(&sTT[(jb * 16 + r) * lda + kb * 16 + 4 * kg]);
                x = O::mma(fa, fb, x);
            }
            f32x4 t = {0.f, 0.f, 0.f, 0.f};
            t = O::mma(tii, x, t); // x is, lane for lane, the B fragment (k = 4*kg + s, n = r)
            // t[xx] = -T_{w,jb}[row 4*kg + xx][col r]
#pragma unroll
            for (int xx = 0; xx < 4; ++xx) {
                sTT[(jb * 16 + r) * lda + b0 + 4 * kg + xx] = -t[xx];
            }
        }
        __syncthreads();
    }
    // T_{w,jb} row-major into sA for the off-diagonal blocks of this block row
    for (int jb = 0; jb < w; ++jb) {
#pragma unroll
        for (int s = 0; s < 4; ++s) sA[(b0 + 4 * kg + s) * lda + jb * 16 + r] = sTT[(jb * 16 + r) * lda + b0 + 4 * kg + s];
    }
}

} // namespace mdn
