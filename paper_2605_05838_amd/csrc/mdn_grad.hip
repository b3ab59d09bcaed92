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
// One workgroup (4 waves) per (chunk, batch*head); wave w owns token rows 16w..16w+15 of every
// row-parallel product.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

constexpr int LDG = 65; // row stride of the fp32 64x64 coefficient matrices in LDS

// out[x] = sum over the columns of row (kg*4+x) of t .* X, X(m, c) = X[m*ldx + c]; every lane of a
// 16-lane group ends up with the row sums of its 4 rows.
template <typename T, int NT>
__device__ __forceinline__ f32x4 rowdot(const f32x4 (&t)[NT], const T *X, size_t ldx) {
    const int r = lane_id() & 15, kg = lane_id() >> 4;
    f32x4 out;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        float s = 0.f;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) s += t[nt][x] * to_f32(X[(size_t)(kg * 4 + x) * ldx + nt * 16 + r]);
        out[x] = reduce16(s);
    }
    return out;
}

template <typename T, int DK, int DV>
__global__ __launch_bounds__(kThreads) void grad_kernel(Dims d, GradArgs a) {
    typedef Op<T> O;
    constexpr int LDW = 64 + O::PAD;
    constexpr int NK = DK / 16;
    constexpr size_t ALIAS_BYTES = sizeof(float) * 64 * LDG;

    __shared__ float sG[64 * LDG];     // Gamma; recycled as the per-entry products of dmu
    __shared__ float sDG1[64 * LDG];   // direct dGamma from Bm; recycled as the products of dalpha
    __shared__ float sDG2[65 * LDG];   // direct dGamma^- (row i here belongs to Gamma row i-1); recycled for dbeta
    __shared__ __align__(16) T sW1e[64 * LDW]; // W1 . eta_j         [i][j]
    __shared__ __align__(16) T sW2e[64 * LDW]; // W2 . eta_j         [i][j]
    __shared__ __align__(16) T sW1T[64 * LDW]; // scale W1^T         [j][i]
    __shared__ __align__(16) T sW2T[64 * LDW]; // (W2 . alpha_i)^T   [j][i]
    __shared__ __align__(16) unsigned char sAlias[ALIAS_BYTES];
    __shared__ float s_al[64], s_be[64], s_mu[64], s_et[64], s_a[64], s_b[64], s_m[64];
    __shared__ float s_da[64], s_db[64], s_dam[64], s_dbm[64], s_dgc[64], s_drc[64], s_dalk[64], s_detk[64];
    __shared__ float s_ga[64], s_gb[64], s_gm[64];
    __shared__ float s_red[4][3];

    float *sRho = reinterpret_cast<float *>(sAlias); // Rho [64][LDG]                (phase 4)

    const int tid = threadIdx.x, lane = lane_id(), w = wave_id(), r = lane & 15, kg = lane >> 4, i0 = w * 16;
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

    // ---------------- phase 0: gates and the forward coefficient scan (Gamma, a, b, m)
    if (tid < 64) {
        const size_t g = tok0 + (size_t)tid * d.H;
        s_al[tid] = a.alpha[g];
        s_be[tid] = a.beta[g];
        s_mu[tid] = a.mu[g];
        s_et[tid] = a.eta ? a.eta[g] : 1.f;
    }
    for (int c = tid; c < LDG; c += kThreads) sDG2[64 * LDG + c] = 0.f;
    __syncthreads();
    if (w == 0) {
        const int j = lane;
        float pa = 1.f, pm = 1.f, pb = 0.f, g = 0.f, rho = 0.f;
        for (int i = 0; i < 64; ++i) {
            const float al = s_al[i], be = s_be[i], mu = s_mu[i];
            pa *= al;
            pm *= mu;
            pb = al * pb + be * pm;
            if (i == j) { s_a[j] = pa; s_b[j] = pb; s_m[j] = pm; }
            rho = (i == j) ? 1.f : rho * mu;
            g = al * g + be * rho;
            sG[i * LDG + j] = g;
        }
        s_dgc[j] = g;   // Gamma_{C,j} for now (the adjoint replaces it later)
        s_drc[j] = rho; // Rho_{C,j}
    }

    __syncthreads();

    // ---------------- phase 2: the four 64x64 products and the masked matrices built from them
    {
        f32x4 accB[4], accA[4], accQK[4], accKK[4];
        zero_acc(accB);
        zero_acc(accA);
        zero_acc(accQK);
        zero_acc(accKK);
        mma_rows<T, 4, DV>(accB, dog + (size_t)i0 * rsv, (int)rsv, vtg, (int)rsv);
        mma_rows<T, 4, DV>(accA, drg + (size_t)i0 * rsv, (int)rsv, vtg, (int)rsv);
        mma_rows<T, 4, DK>(accQK, qg + (size_t)i0 * rsk, (int)rsk, kgl, (int)rsk);
        mma_rows<T, 4, DK>(accKK, kgl + (size_t)i0 * rsk, (int)rsk, kgl, (int)rsk);
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + kg * 4 + x, j = nt * 16 + r;
                const float gam = sG[i * LDG + j], gprev = (i > 0) ? sG[(i - 1) * LDG + j] : 0.f;
                const float et = s_et[j], al = s_al[i];
                const float dBm = (j <= i) ? accB[nt][x] : 0.f;
                const float dA = (j < i) ? -accA[nt][x] : 0.f;
                sDG1[i * LDG + j] = dBm * (d.scale * et * accQK[nt][x]);
                sDG2[i * LDG + j] = dA * (al * et * accKK[nt][x]);
                const float w1 = dBm * gam, w2 = dA * gprev;
                sW1e[i * LDW + j] = from_f32<T>(w1 * et);
                sW2e[i * LDW + j] = from_f32<T>(w2 * et);
                sW1T[j * LDW + i] = from_f32<T>(w1 * d.scale);
                sW2T[j * LDW + i] = from_f32<T>(w2 * al);
            }
    }
    __syncthreads();

    // ---------------- phase 3: products with the states; dq, dk and the direct coefficient adjoints
    f32x4 accP[NK]; // dP rows i0..i0+15
    {
        f32x4 accQ[NK], t[NK];
        zero_acc(accQ);
        mma_rows_kblk<T, NK, 64>(accQ, sW1e + i0 * LDW, LDW, KTg, DK);
        // a . (dO S^T), b . (dO M^T)
        zero_acc(t);
        mma_rows_vblk<T, NK, DV>(t, dog + (size_t)i0 * rsv, (int)rsv, Sg, DK);
        f32x4 da = rowdot<T, NK>(t, qg + (size_t)i0 * rsk, rsk);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float ai = s_a[i0 + kg * 4 + x];
#pragma unroll
            for (int nt = 0; nt < NK; ++nt) accQ[nt][x] += ai * t[nt][x];
        }
        zero_acc(t);
        mma_rows_vblk<T, NK, DV>(t, dog + (size_t)i0 * rsv, (int)rsv, Mg, DK);
        f32x4 db = rowdot<T, NK>(t, qg + (size_t)i0 * rsk, rsk);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float bi = s_b[i0 + kg * 4 + x];
#pragma unroll
            for (int nt = 0; nt < NK; ++nt) accQ[nt][x] -= bi * t[nt][x];
        }
        if (r == 0)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                s_da[i0 + kg * 4 + x] = d.scale * da[x];
                s_db[i0 + kg * 4 + x] = -d.scale * db[x];
            }
        T *dqg = static_cast<T *>(a.dq) + (tok0 + (size_t)i0 * d.H) * DK;
#pragma unroll
        for (int nt = 0; nt < NK; ++nt)
#pragma unroll
            for (int x = 0; x < 4; ++x)
                dqg[(size_t)(kg * 4 + x) * rsk + nt * 16 + r] = from_f32<T>(d.scale * accQ[nt][x]);

        // dP = W2 K~ - a^- . (dR S^T) + b^- . (dR M^T)
        zero_acc(accP);
        mma_rows_kblk<T, NK, 64>(accP, sW2e + i0 * LDW, LDW, KTg, DK);
        zero_acc(t);
        mma_rows_vblk<T, NK, DV>(t, drg + (size_t)i0 * rsv, (int)rsv, Sg, DK);
        f32x4 dam = rowdot<T, NK>(t, kgl + (size_t)i0 * rsk, rsk); // k_i . (S dR_i); P_i = alpha_i k_i
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int i = i0 + kg * 4 + x;
            const float am = (i > 0) ? s_a[i - 1] : 1.f;
#pragma unroll
            for (int nt = 0; nt < NK; ++nt) accP[nt][x] -= am * t[nt][x];
        }
        zero_acc(t);
        mma_rows_vblk<T, NK, DV>(t, drg + (size_t)i0 * rsv, (int)rsv, Mg, DK);
        f32x4 dbm = rowdot<T, NK>(t, kgl + (size_t)i0 * rsk, rsk);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int i = i0 + kg * 4 + x;
            const float bm = (i > 0) ? s_b[i - 1] : 0.f;
#pragma unroll
            for (int nt = 0; nt < NK; ++nt) accP[nt][x] += bm * t[nt][x];
        }
        f32x4 dalk = rowdot<T, NK>(accP, kgl + (size_t)i0 * rsk, rsk);
        if (r == 0)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + kg * 4 + x;
                s_dam[i] = -s_al[i] * dam[x];
                s_dbm[i] = s_al[i] * dbm[x];
                s_dalk[i] = dalk[x];
            }
    }
    {
        // dK~ = W1^T Q~ + W2^T P + Gamma_C . (V~ dS'^T) - Rho_C . (V~ dM'^T), rows j = i0..i0+15
        f32x4 accK[NK], t[NK];
        zero_acc(accK);
        mma_rows_kblk<T, NK, 64>(accK, sW1T + i0 * LDW, LDW, QTg, DK);
        mma_rows_kblk<T, NK, 64>(accK, sW2T + i0 * LDW, LDW, KTg, DK);
        zero_acc(t);
        mma_rows_vblk<T, NK, DV>(t, vtg + (size_t)i0 * rsv, (int)rsv, dSg, DK);
        f32x4 dgc = rowdot<T, NK>(t, kgl + (size_t)i0 * rsk, rsk);
        float gC[4], rC[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            gC[x] = s_dgc[i0 + kg * 4 + x];
            rC[x] = s_drc[i0 + kg * 4 + x];
#pragma unroll
            for (int nt = 0; nt < NK; ++nt) accK[nt][x] += gC[x] * t[nt][x];
        }
        zero_acc(t);
        mma_rows_vblk<T, NK, DV>(t, vtg + (size_t)i0 * rsv, (int)rsv, dMg, DK);
        f32x4 drc = rowdot<T, NK>(t, kgl + (size_t)i0 * rsk, rsk);
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
            for (int nt = 0; nt < NK; ++nt) accK[nt][x] -= rC[x] * t[nt][x];
        f32x4 detk = rowdot<T, NK>(accK, kgl + (size_t)i0 * rsk, rsk);
        __syncthreads(); // every wave has read Gamma_C / Rho_C out of s_dgc / s_drc
        if (r == 0)
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int j = i0 + kg * 4 + x;
                s_dgc[j] = s_et[j] * dgc[x];   // adjoint of Gamma_{C,j}
                s_drc[j] = -s_et[j] * drc[x];  // adjoint of Rho_{C,j}
                s_detk[j] = detk[x];
            }
        T *dkg = static_cast<T *>(a.dk) + (tok0 + (size_t)i0 * d.H) * DK;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int j = i0 + kg * 4 + x;
            const float et = s_et[j], al = s_al[j];
#pragma unroll
            for (int nt = 0; nt < NK; ++nt)
                dkg[(size_t)(kg * 4 + x) * rsk + nt * 16 + r] = from_f32<T>(et * accK[nt][x] + al * accP[nt][x]);
        }
    }
    // <dS',S>, <dS',M>, <dM',M>
    {
        float p1 = 0.f, p2 = 0.f, p3 = 0.f;
        for (int c = tid * O::EPL; c < DK * DV; c += kThreads * O::EPL) {
#pragma unroll
            for (int e = 0; e < O::EPL; ++e) {
                const float s = to_f32(Sg[c + e]), m = to_f32(Mg[c + e]);
                const float ds = to_f32(dSg[c + e]), dm = to_f32(dMg[c + e]);
                p1 += ds * s;
                p2 += ds * m;
                p3 += dm * m;
            }
        }
        p1 = reduce64(p1);
        p2 = reduce64(p2);
        p3 = reduce64(p3);
        if (lane == 0) { s_red[w][0] = p1; s_red[w][1] = p2; s_red[w][2] = p3; }
    }
    __syncthreads();

    // ---------------- phase 4: reverse of the coefficient scans (wave 0)
    if (w == 0) {
        const int j = lane;
        {
            float rho = 0.f;
            for (int i = 0; i < 64; ++i) {
                rho = (i == j) ? 1.f : rho * s_mu[i];
                sRho[i * LDG + j] = rho;
            }
        }
        // column j of the accumulated adjoints G^ (of Gamma) and R^ (of Rho), rows 63 .. j
        float carryG = 0.f, carryR = 0.f;
        for (int i = 63; i >= 0; --i) {
            if (i >= j) {
                const float G = sDG1[i * LDG + j] + sDG2[(i + 1) * LDG + j] + (i == 63 ? s_dgc[j] : 0.f) + carryG;
                const float R = (i == 63 ? s_drc[j] : 0.f) + s_be[i] * G + carryR;
                const float gprev = (i > j) ? sG[(i - 1) * LDG + j] : 0.f;
                const float rprev = (i > j) ? sRho[(i - 1) * LDG + j] : 0.f;
                sDG1[i * LDG + j] = G * gprev;                    // -> dalpha_i
                sDG2[(i + 1) * LDG + j] = G * sRho[i * LDG + j];  // -> dbeta_i
                sG[i * LDG + j] = R * rprev;                      // -> dmu_i
                carryG = s_al[i] * G;
                carryR = s_mu[i] * R;
            }
        }
    }
    __syncthreads();
    if (tid < 64) {
        const int i = tid;
        float ga = 0.f, gb = 0.f, gm = 0.f;
        for (int j = 0; j <= i; ++j) {
            gb += sDG2[(i + 1) * LDG + j];
            if (j < i) {
                ga += sDG1[i * LDG + j];
                gm += sG[i * LDG + j];
            }
        }
        s_ga[i] = ga;
        s_gb[i] = gb;
        s_gm[i] = gm;
    }
    __syncthreads();
    if (w == 0) {
        // vectors: b_i = alpha_i b_{i-1} + beta_i m_i, a_i = alpha_i a_{i-1}, m_i = mu_i m_{i-1};
        // a^-_i = a_{i-1}, b^-_i = b_{i-1}.  Every lane runs the same 64 steps, lane i keeps step i.
        const float dS_S = s_red[0][0] + s_red[1][0] + s_red[2][0] + s_red[3][0];
        const float dS_M = s_red[0][1] + s_red[1][1] + s_red[2][1] + s_red[3][1];
        const float dM_M = s_red[0][2] + s_red[1][2] + s_red[2][2] + s_red[3][2];
        float cb = 0.f, ca = 0.f, cm = 0.f; // carried adjoints arriving from step i+1
        float my_al = 0.f, my_be = 0.f, my_mu = 0.f;
        for (int i = 63; i >= 0; --i) {
            const float al = s_al[i], be = s_be[i], mu = s_mu[i];
            const float aprev = (i > 0) ? s_a[i - 1] : 1.f, bprev = (i > 0) ? s_b[i - 1] : 0.f;
            const float mprev = (i > 0) ? s_m[i - 1] : 1.f;
            float db = s_db[i] + (i < 63 ? s_dbm[i + 1] : -dS_M) + cb;
            float da = s_da[i] + (i < 63 ? s_dam[i + 1] : dS_S) + ca;
            float dm = (i == 63 ? dM_M : 0.f) + be * db + cm;
            const float g_al = s_ga[i] + db * bprev + da * aprev;
            const float g_be = s_gb[i] + db * s_m[i];
            const float g_mu = s_gm[i] + dm * mprev;
            if (i == lane) { my_al = g_al; my_be = g_be; my_mu = g_mu; }
            cb = al * db;
            ca = al * da;
            cm = mu * dm;
        }
        const size_t g = tok0 + (size_t)lane * d.H;
        a.dalpha[g] = my_al + s_dalk[lane];
        a.dbeta[g] = my_be;
        a.dmu[g] = my_mu;
        if (a.deta) a.deta[g] = s_detk[lane];
    }
}

template <typename T, int DK, int DV>
hipError_t launch_t(const Dims &d, const GradArgs &a, hipStream_t s) {
    dim3 grid(d.N, d.BH), block(kThreads);
    hipLaunchKernelGGL((grad_kernel<T, DK, DV>), grid, block, 0, s, d, a);
    return hipGetLastError();
}

} // namespace

hipError_t launch_grad(const Dims &d, const GradArgs &a, hipStream_t s) {
    const bool f32 = d.dtype == 1;
    if (d.dk == 64 && d.dv == 64) return f32 ? launch_t<float, 64, 64>(d, a, s) : launch_t<bf16_t, 64, 64>(d, a, s);
    if (d.dk == 128 && d.dv == 128)
        return f32 ? launch_t<float, 128, 128>(d, a, s) : launch_t<bf16_t, 128, 128>(d, a, s);
    return hipErrorInvalidValue;
}

} // namespace mdn
