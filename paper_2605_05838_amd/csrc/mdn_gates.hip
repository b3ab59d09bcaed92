// Stability-aware gate parameterisation (Sec. 3.3, "Stability Aware Gating Parameterization") and its adjoint:
// from the four per-head projections of a token to the linear-domain gates the momentum delta rule takes,
//     eta   = tanh(x_eta / tau) + 1
//     alpha_max = cos^2 theta = 1 / (1 + (eta s)^2),  beta_max = sin^2 theta = (eta s)^2 / (1 + (eta s)^2),  theta = arctan(eta s)
//     alpha = alpha_max exp(-a_alpha softplus(x_alpha + b_alpha)),  mu = exp(max(-a_mu softplus(x_mu + b_mu), mu_log_min))
//     beta  = sigmoid(x_beta) beta_max
// Elementwise over [B,T,H] in fp32 (16 bytes in, 16 bytes out per token-head: nothing beside the 11 KB per token-head
// of the chunkwise path).  The adjoint also sums the gradients of the four per-head parameter vectors: per
// workgroup in LDS, then one atomic add per head and workgroup.
#include "../../include/mdn.h"
#include "mdn_device.h"

#include <hip/hip_runtime.h>

namespace mdn {

namespace {

constexpr int GT = 256;

__device__ __forceinline__ float softplus_f(float x) { return x > 20.f ? x : log1pf(__expf(x)); }
__device__ __forceinline__ float sigmoid_f(float x) { return 1.f / (1.f + __expf(-x)); }

struct GateArgs {
    const float *xa, *xm, *xb, *xe;
    const float *a_alpha, *b_alpha, *a_mu, *b_mu;
    float s, tau, mu_log_min;
    long long n; // B*T*H
    int H;
};

__global__ __launch_bounds__(GT) void gates_fwd_kernel(GateArgs g, float *alpha, float *beta, float *mu, float *eta) {
    for (long long i = (long long)blockIdx.x * GT + threadIdx.x; i < g.n; i += (long long)gridDim.x * GT) {
        const int h = (int)(i % g.H);
        const float e = tanhf(g.xe[i] / g.tau) + 1.f, u = e * g.s, den = 1.f + u * u;
        eta[i] = e;
        alpha[i] = __expf(-g.a_alpha[h] * softplus_f(g.xa[i] + g.b_alpha[h])) / den;
        mu[i] = __expf(fmaxf(-g.a_mu[h] * softplus_f(g.xm[i] + g.b_mu[h]), g.mu_log_min));
        beta[i] = sigmoid_f(g.xb[i]) * (u * u / den);
    }
}

// dpar: [4][H] = da_alpha, db_alpha, da_mu, db_mu (accumulated: the caller's launch sequence zeroes it first)
__global__ __launch_bounds__(GT) void gates_bwd_kernel(GateArgs g, const float *dalpha, const float *dbeta, const float *dmu,
                                                        const float *deta, float *dxa, float *dxm, float *dxb, float *dxe,
                                                        float *dpar) {
    extern __shared__ float s_par[]; // [4][H]
    const int lane = threadIdx.x & 63;
    for (int c = threadIdx.x; c < 4 * g.H; c += GT) s_par[c] = 0.f;
    __syncthreads();
    for (long long i = (long long)blockIdx.x * GT + threadIdx.x; i < g.n; i += (long long)gridDim.x * GT) {
        const int h = (int)(i % g.H);
        const float th = tanhf(g.xe[i] / g.tau), e = th + 1.f, u = e * g.s, den = 1.f + u * u;
        const float dmax = 2.f * u * g.s / (den * den); // d beta_max / d eta = - d alpha_max / d eta
        const float za = g.xa[i] + g.b_alpha[h], zm = g.xm[i] + g.b_mu[h];
        const float spa = softplus_f(za), spm = softplus_f(zm);
        const float decay = __expf(-g.a_alpha[h] * spa), sb = sigmoid_f(g.xb[i]);
        const float fm = -g.a_mu[h] * spm;
        const float da = dalpha[i], db = dbeta[i];
        const float dfa = da * decay / den;                                      // d L / d f_alpha = dalpha * alpha
        const float dfm = fm > g.mu_log_min ? dmu[i] * __expf(fm) : 0.f;         // the clamp passes no gradient
        const float gxa = dfa * (-g.a_alpha[h] * sigmoid_f(za)), gxm = dfm * (-g.a_mu[h] * sigmoid_f(zm));
        dxa[i] = gxa;
        dxm[i] = gxm;
        dxb[i] = db * (u * u / den) * sb * (1.f - sb);
        dxe[i] = (deta[i] - da * decay * dmax + db * sb * dmax) * (1.f - th * th) / g.tau;
        if (dpar) {
            // lanes 32 (16) apart hold the same head when H divides 32 (16): their contributions are summed across
            // the wave's halves (rows) first, so that one lane per head and wave goes to the LDS atomics instead of four
            // (a loop trip is taken by whole waves except in the last one, whose stragglers take the plain path)
            float p0 = dfa * -spa, p1 = gxa, p2 = dfm * -spm, p3 = gxm;
            const bool whole = i - lane + 63 < g.n;
            int active = 64;
            if (whole && 32 % g.H == 0) {
                p0 = add_xor32(p0); p1 = add_xor32(p1); p2 = add_xor32(p2); p3 = add_xor32(p3);
                active = 32;
                if (16 % g.H == 0) {
                    p0 = add_xor16(p0); p1 = add_xor16(p1); p2 = add_xor16(p2); p3 = add_xor16(p3);
                    active = 16;
                }
            }
            if (lane < active) {
                atomicAdd(&s_par[0 * g.H + h], p0);
                atomicAdd(&s_par[1 * g.H + h], p1);
                atomicAdd(&s_par[2 * g.H + h], p2);
                atomicAdd(&s_par[3 * g.H + h], p3);
            }
        }
    }
    __syncthreads();
    if (dpar)
        for (int c = threadIdx.x; c < 4 * g.H; c += GT) atomicAdd(&dpar[c], s_par[c]);
}

__global__ void gates_zero_kernel(float *p, int n) {
    for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < n; c += gridDim.x * blockDim.x) p[c] = 0.f;
}

int check(const mdn_gate_params *p, GateArgs *g) {
    if (!p) return MDN_ERR_NULL;
    if (p->B < 1 || p->T < 1 || p->H < 1 || p->H > 1024 || !(p->tau > 0.f)) return MDN_ERR_SHAPE;
    if (!p->a_alpha || !p->b_alpha || !p->a_mu || !p->b_mu) return MDN_ERR_NULL;
    g->a_alpha = p->a_alpha; g->b_alpha = p->b_alpha; g->a_mu = p->a_mu; g->b_mu = p->b_mu;
    g->s = p->s; g->tau = p->tau; g->mu_log_min = p->mu_log_min;
    g->n = (long long)p->B * p->T * p->H;
    g->H = p->H;
    return MDN_OK;
}

int grid_for(long long n) {
    const long long b = (n + GT - 1) / GT;
    return (int)(b < 4096 ? b : 4096);
}

} // namespace

} // namespace mdn

using namespace mdn;

extern "C" {

int mdn_gates_fwd(const mdn_gate_params *params, const float *x_alpha, const float *x_mu, const float *x_beta,
                  const float *x_eta, float *alpha, float *beta, float *mu, float *eta, void *stream) {
    GateArgs g = {};
    const int rc = check(params, &g);
    if (rc) return rc;
    if (!x_alpha || !x_mu || !x_beta || !x_eta || !alpha || !beta || !mu || !eta) return MDN_ERR_NULL;
    g.xa = x_alpha; g.xm = x_mu; g.xb = x_beta; g.xe = x_eta;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(gates_fwd_kernel, dim3(grid_for(g.n)), dim3(GT), 0, s, g, alpha, beta, mu, eta);
    return hipGetLastError() == hipSuccess ? MDN_OK : MDN_ERR_LAUNCH;
}

int mdn_gates_bwd(const mdn_gate_params *params, const float *x_alpha, const float *x_mu, const float *x_beta,
                  const float *x_eta, const float *dalpha, const float *dbeta, const float *dmu, const float *deta,
                  float *dx_alpha, float *dx_mu, float *dx_beta, float *dx_eta, float *dparams, void *stream) {
    GateArgs g = {};
    const int rc = check(params, &g);
    if (rc) return rc;
    if (!x_alpha || !x_mu || !x_beta || !x_eta || !dalpha || !dbeta || !dmu || !deta || !dx_alpha || !dx_mu || !dx_beta ||
        !dx_eta)
        return MDN_ERR_NULL;
    g.xa = x_alpha; g.xm = x_mu; g.xb = x_beta; g.xe = x_eta;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dparams) hipLaunchKernelGGL(gates_zero_kernel, dim3(1), dim3(256), 0, s, dparams, 4 * g.H);
    // (with parameter gradients every workgroup ends in 4 H atomic adds on the same 4 H addresses, which the L2 takes one
    //  after the other: few workgroups with many tokens each)
    const int wgs = dparams ? (grid_for(g.n) < 256 ? grid_for(g.n) : 256) : grid_for(g.n);
    hipLaunchKernelGGL(gates_bwd_kernel, dim3(wgs), dim3(GT), 4 * g.H * sizeof(float), s, g, dalpha, dbeta, dmu,
                       deta, dx_alpha, dx_mu, dx_beta, dx_eta, dparams);
    return hipGetLastError() == hipSuccess ? MDN_OK : MDN_ERR_LAUNCH;
}

} // extern "C"
