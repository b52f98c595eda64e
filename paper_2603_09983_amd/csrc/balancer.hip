// Heterogeneous Workload Balancer (Sec. 3.3; appendix "Solution Derivation"):
// per layer, the integer threshold tau* in [1,K] that minimises
// |T_cpu(tau) - T_gpu(tau)| under the I/O-window and the memory constraint,
// K when no tau is feasible.  K <= 64, so instead of the appendix's
// four-candidate shortcut (which leans on convexity) one wavefront per layer
// evaluates EVERY tau, one lane each, and takes the minimum: same result where
// the shortcut's premise holds, and still the definition's answer where it
// does not.  Inputs are what the two upstream kernels leave in device memory:
// the activation frequencies (for b) and the prefetch counts n(tau).
//
// The decision is a comparison of floating-point values, so the arithmetic is
// fp64 in a fixed operation order with contraction off: the threshold is the
// same integer as a plain CPU evaluation of the printed formulas.
#include "../../include/moe_spac.h"
#include "moe_internal.h"

namespace moe {

namespace {

struct BalanceArgs {
    const int32_t *f;       // [L,N]
    const int32_t *n_tau;   // [L,K+1]
    const double *r_c;      // [L,K+1]
    const double *r_g;      // [L,K+1]
    int32_t *tau_out;       // [L]
    int32_t *b_out;         // [L] or null
    int N, K, gamma, k, l_target;
    double t_cpu, t_gpu, t_io, t_draft;
    long long w_expert, vram_left;
};

__global__ __launch_bounds__(kWave) void balance_kernel(BalanceArgs a)
{
#pragma clang fp contract(off)
    __shared__ double obj_s[kWave + 1];
    __shared__ int ok_s[kWave + 1];
    const int l = blockIdx.x, lane = threadIdx.x;
    // b: de-duplicated activated experts of this layer
    int b = 0;
    for (int i0 = 0; i0 < a.N; i0 += kWave) {
        const int i = i0 + lane;
        const bool on = i < a.N && a.f[(size_t)l * a.N + i] > 0;
        b += __popcll(__ballot(on));
    }
    // lane tau - 1 evaluates threshold tau
    const int tau = lane + 1;
    if (tau <= a.K) {
        const size_t j = (size_t)l * (a.K + 1) + tau;
        const double tc = ((a.r_c[j] * (double)a.gamma) * (double)a.k) * a.t_cpu;
        const double tg = (a.r_g[j] * (double)b) * a.t_gpu;
        const double total = tc > tg ? tc : tg;
        const double window = total + ((double)a.gamma * a.t_draft) / (double)a.l_target;
        const int n = a.n_tau[j];
        const bool io_ok = a.t_io * (double)n <= window;
        const bool mem_ok = a.w_expert * (long long)n <= a.vram_left;
        obj_s[tau] = fabs(tc - tg);
        ok_s[tau] = io_ok && mem_ok;
    }
    __syncthreads();
    if (lane == 0) {
        int best = -1;
        double best_f = 0.0;
        for (int t = 1; t <= a.K; ++t) {
            if (!ok_s[t]) continue;
            if (best < 0 || obj_s[t] < best_f) {   // strict: ties stay with the smaller tau
                best = t;
                best_f = obj_s[t];
            }
        }
        a.tau_out[l] = best < 0 ? a.K : best;
        if (a.b_out) a.b_out[l] = b;
    }
}

}  // namespace

}  // namespace moe

using namespace moe;

extern "C" int moe_balance_threshold(const int32_t *f, const int32_t *n_tau, const double *r_c, const double *r_g,
                                     int L, int N, int K, int gamma, int k, const moe_balance_params_t *p,
                                     int32_t *tau_out, int32_t *b_out, void *stream)
{
    if (!f || !n_tau || !r_c || !r_g || !p || !tau_out) return MOE_ERR_NULL;
    if (L < 1 || L > 65535 || N < 1 || K < 1 || K > 64 || gamma < 0 || k < 1 || p->l_target < 1 ||
        p->w_expert_bytes < 0 || (size_t)L * N > (size_t)1 << 30)
        return MOE_ERR_SHAPE;
    BalanceArgs a = {f, n_tau, r_c, r_g, tau_out, b_out, N, K, gamma, k, p->l_target, p->t_cpu, p->t_gpu,
                     p->t_io, p->t_draft, (long long)p->w_expert_bytes, (long long)p->vram_left_bytes};
    void *params[] = {&a};
    hipError_t e = launch_timed((const void *)balance_kernel, dim3(L), dim3(kWave), params, 0, (hipStream_t)stream,
                                MOE_KERNEL_BALANCER);
    if (e == hipSuccess) e = hipGetLastError();
    return e == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}
