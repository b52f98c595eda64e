// Speculative Utility Estimator (Sec. 3.2, Alg. 1 and the utility-transition
// equation): the consumer of the activation frequencies that the routing step
// produces.  One call advances the estimator of L layers by one inference
// step; per expert it is a handful of integer operations on five words of
// state, so one workgroup per layer walks that layer's N experts and the
// launch is bound by its one trip to memory.  The same pass counts, per
// layer, the experts a prefetcher would have to fetch for each threshold:
// n(tau) = #{i : s_i >= tau, expert i holds no cache slot} (Sec. 3.3,
// notation table), so the balancer's input needs no second pass over s.
//
// Readings: f_{i,0} = 0 (moe_utility_init); the forgetting factor is the
// rational lam_num / lam_den and the floor is taken in integer arithmetic;
// the upward test comes first, so with a boundary of 0 a fluctuation of 0
// raises the utility (the listing's ">=").
#include "moe_internal.h"
#include "../../include/moe_spac.h"

namespace moe {

namespace {

constexpr int kEstThreads = 256;
constexpr int kMaxUtility = 64;   // K <= gamma, and gamma is a draft length

__global__ __launch_bounds__(kEstThreads) void utility_init_kernel(int32_t *f_prev, int32_t *s, int32_t *th_up,
                                                                   int32_t *th_dn, int n, int theta0)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        f_prev[i] = 0;
        s[i] = 0;
        th_up[i] = theta0;
        th_dn[i] = theta0;
    }
}

__global__ __launch_bounds__(kEstThreads) void utility_update_kernel(const int32_t *f, int32_t *f_prev, int32_t *s,
                                                                     int32_t *th_up, int32_t *th_dn,
                                                                     const int32_t *slot_table, int32_t *n_tau,
                                                                     int N, int K, int lam_num, int lam_den)
{
    __shared__ int level_s[kMaxUtility + 1];   // non-resident experts per utility level
    const int l = blockIdx.x, tid = threadIdx.x;
    const size_t base = (size_t)l * N;
    if (n_tau && tid <= K) level_s[tid] = 0;
    __syncthreads();
    for (int i = tid; i < N; i += kEstThreads) {
        const size_t j = base + i;
        const int fi = f[j], fp = f_prev[j];
        int si = s[j], up = th_up[j], dn = th_dn[j];
        const long long d = (long long)fi - (long long)fp;   // fluctuation
        // inertial utility transition (boundaries of this step)
        if (d >= (long long)up) si = si + 1 < K ? si + 1 : K;
        else if (-d >= (long long)dn) si = si - 1 > 0 ? si - 1 : 0;
        // adaptive boundary calibration (boundaries of the next step)
        if (d > 0) up = (int)(((long long)(lam_den - lam_num) * up + (long long)lam_num * d) / lam_den);
        else if (d < 0) dn = (int)(((long long)(lam_den - lam_num) * dn + (long long)lam_num * (-d)) / lam_den);
        s[j] = si;
        th_up[j] = up;
        th_dn[j] = dn;
        f_prev[j] = fi;
        if (n_tau && slot_table[j] < 0) {
            const int lv = si < 0 ? 0 : si > K ? K : si;   // (a caller-supplied state outside [0,K] stays in bounds)
            atomicAdd(&level_s[lv], 1);
        }
    }
    if (!n_tau) return;
    __syncthreads();
    if (tid <= K) {
        int n = 0;
        for (int lv = tid; lv <= K; ++lv) n += level_s[lv];
        n_tau[(size_t)l * (K + 1) + tid] = n;
    }
}

}  // namespace

}  // namespace moe

using namespace moe;

extern "C" int moe_utility_init(int32_t *f_prev, int32_t *s, int32_t *theta_up, int32_t *theta_dn, int L, int N,
                                int gamma, void *stream)
{
    if (!f_prev || !s || !theta_up || !theta_dn) return MOE_ERR_NULL;
    if (L < 1 || N < 1 || gamma < 0 || (size_t)L * N > (size_t)1 << 30) return MOE_ERR_SHAPE;
    const int n = L * N;
    int blocks = (n + kEstThreads - 1) / kEstThreads;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(utility_init_kernel, dim3(blocks), dim3(kEstThreads), 0, (hipStream_t)stream, f_prev, s,
                       theta_up, theta_dn, n, gamma / 2);
    return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}

extern "C" int moe_utility_update(const int32_t *f, int32_t *f_prev, int32_t *s, int32_t *theta_up,
                                  int32_t *theta_dn, const int32_t *slot_table, int32_t *n_tau, int L, int N, int K,
                                  int lam_num, int lam_den, void *stream)
{
    if (!f || !f_prev || !s || !theta_up || !theta_dn) return MOE_ERR_NULL;
    if (n_tau && !slot_table) return MOE_ERR_NULL;
    if (L < 1 || N < 1 || K < 0 || K > kMaxUtility || lam_den < 1 || lam_num < 0 || lam_num > lam_den ||
        L > 65535 || (size_t)L * N > (size_t)1 << 30)
        return MOE_ERR_SHAPE;
    const void *fn = (const void *)utility_update_kernel;
    void *params[] = {&f, &f_prev, &s, &theta_up, &theta_dn, &slot_table, &n_tau, &N, &K, &lam_num, &lam_den};
    hipError_t e = launch_timed(fn, dim3(L), dim3(kEstThreads), params, 0, (hipStream_t)stream, MOE_KERNEL_ESTIMATOR);
    if (e == hipSuccess) e = hipGetLastError();
    return e == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}
