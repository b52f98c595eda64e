// Routing side of the verify-step MoE layer (gfx950):
//   router GEMM  s = W_g h            (Sec. 2.2, first line of the MoE equation)
//   Top-k and the gate over the k picks  (second and third line)
//   activation-frequency histogram     (Sec. 2.3)
//   expert id -> cache slot, miss list, per-slot token lists   (App. D)
//
// These steps move a few hundred kilobytes; what they cost is the chain of
// dependent trips to memory and of workgroup barriers, so the kernel is built
// to keep that chain short.  The T*E dot products are dealt one per wavefront,
// round-robin over as many workgroups as the device has CUs (a CU that had to
// fetch the operands of sixteen of them takes microseconds longer than one
// that fetches two or three).  Each logit goes to memory together with the
// number of the call as ONE 64-bit atomic store; workgroup 0, one wavefront
// per token, reads the entries with atomic loads until they carry that number
// (a bounded number of times), so the hand-over needs no counter, no fence and
// no cache write-back.  It then picks each token's Top-k out of registers (k
// maxima over the wavefront) and produces histogram, slot counts, miss list and
// per-slot lists out of LDS with independent threads between a few barriers.
// On this one serial path every instruction counts: a wavefront issues one
// about every four cycles.
#include "moe_internal.h"
#include "route_device.h"

namespace moe {

namespace {

__global__ __launch_bounds__(kRouteThreads) void route_kernel(RouteArgs a)
{
    extern __shared__ int dyn[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int b = blockIdx.x, G = gridDim.x;
    const int T = a.T, H = a.H, E = a.E, TE = T * E;
    const int A = T * a.k;
    const unsigned tag = *a.epoch + 1u;   // number of this call
    // (two words of the control block that only a test sets: the bound of the polls, and a number added to
    // what producers stamp their entries with, so that the host can make every wait run out)
    const unsigned *ctrl = a.epoch - kCtrlEpoch;
    const int spin = ctrl[kCtrlSpin] ? (int)ctrl[kCtrlSpin] : kSpinLimit;
    const unsigned wtag = tag + ctrl[kCtrlSkew];   // stamps this call's logits
    if (b == 0 && tid == 0) check_layout(a.epoch - kCtrlEpoch, a.layout);

    // (workgroup 0) the slot table rides along with the first trip to memory
    int tab_v = -1;
    if (b == 0 && a.slot_table && tid < E) tab_v = a.slot_table[tid];   // (E <= kMaxE <= kRouteThreads)

    // s[t,e] = W_g[e,:] . h[t,:]: one wavefront per dot product, lanes stride H four at a time
    const uint16_t *x = (const uint16_t *)a.hidden;
    for (int q = b + w * G; q < TE; q += G * kRouteWaves) {
        const int t = q / E, e = q - t * E;
        const float *wrow = a.router_w + (size_t)e * H;
        const uint16_t *xr = x + (size_t)t * H;
        const float bias = a.router_bias ? a.router_bias[e] : 0.f;
        float acc = 0.f;
#pragma unroll 8
        for (int h = lane * 4; h < H; h += kWave * 4) {
            float4 wv = *(const float4 *)(wrow + h);
            uint2 xv = *(const uint2 *)(xr + h);
            acc += wv.x * bf16_lo(xv.x) + wv.y * bf16_hi(xv.x) + wv.z * bf16_lo(xv.y) + wv.w * bf16_hi(xv.y);
        }
#pragma unroll
        for (int m = kWave / 2; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, kWave);
        acc += bias;
        if (lane == 0) {
            __hip_atomic_store(a.tagged_logits + q, ((unsigned long long)wtag << 32) | __float_as_uint(acc),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (a.logits_opt) a.logits_opt[q] = acc;
        }
    }
    // ---- ranking: workgroup b ranks tokens 16b .. 16b+15, one wavefront each ----
    const int n_rank = (T + kRouteWaves - 1) / kRouteWaves;
    const bool share_ids = n_rank > 1 && A <= kTagIdxEntries;   // ids handed to workgroup 0 as stamped entries
    if (b >= (share_ids ? n_rank : 1)) return;
    PostLds L = carve_lds(dyn, E, a.C, A);
    const bool small = a.slot_table && a.hist && T <= 128 && A <= kRouteThreads && a.C <= kRouteThreads;
    if (b == 0) {
        if (a.slot_table && tid < E) L.tab_s[tid] = tab_v;
        if (small) {
            if (tid < E) L.hist_s[tid] = 0;
            for (int i = tid; i < a.C * ((T + 31) >> 5); i += kRouteThreads) L.cnt_s[i] = 0;   // (the token masks)
        }
    }
    const bool idx_in_lds = A <= kLdsCopy;
    lds_f32 *lg = L.lg_s + w * lg_stride(E);
    for (int t = share_ids ? b * kRouteWaves + w : w; t < T; t += share_ids ? T : kRouteWaves) {
        // wait (a bounded number of polls) until every logit of token t carries the tag
        const unsigned long long *src = a.tagged_logits + (size_t)t * E;
        for (int e0 = 0; e0 < E; e0 += kWave) {
            const int e = e0 + lane;
            unsigned long long v = (unsigned long long)tag << 32;
            int polls = 0;
            for (;;) {
                if (e < E) v = __hip_atomic_load(src + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (__ballot((unsigned)(v >> 32) != tag) == 0ull) break;
                if (++polls > spin) {   // cannot happen on a healthy device; never wait for ever
                    if (lane == 0) atomicOr(a.error_flag, 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (e < E) {
                const float f = __uint_as_float((unsigned)v);
                lg[e] = (f == f) ? f : -INFINITY;   // NaN cannot win a comparison; rank it last
            }
        }
        __builtin_amdgcn_wave_barrier();
        wave_topk_gate(E, a.k, a.topk_idx + (size_t)t * a.k, idx_in_lds ? L.idx_s + t * a.k : nullptr,
                       a.topk_w + (size_t)t * a.k, lg);
        if (share_ids) {
            // (LDS operations of one wavefront execute in order: the ids written above are visible)
            __builtin_amdgcn_wave_barrier();
            for (int j = lane; j < a.k; j += kWave)
                __hip_atomic_store(a.tagged_idx + (size_t)t * a.k + j,
                                   ((unsigned long long)wtag << 32) | (unsigned)L.idx_s[t * a.k + j], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (b != 0) return;

    // ---- workgroup 0: everything after the Top-k ----
    __syncthreads();
    if (share_ids) {
        // collect the ids the other workgroups ranked (its own come back the same way)
        for (int i = tid; i < A; i += kRouteThreads) {
            unsigned long long v = 0;
            int polls = 0;
            for (;;) {
                v = __hip_atomic_load(a.tagged_idx + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((unsigned)(v >> 32) == tag) break;
                if (++polls > spin) {
                    atomicOr(a.error_flag, 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            const unsigned e = (unsigned)v;
            L.idx_s[i] = e < (unsigned)E ? (int)e : 0;   // (a bound that ran out leaves garbage: stay in range)
        }
        __syncthreads();
    }

    const int32_t *idx = idx_in_lds ? (const int32_t *)L.idx_s : a.topk_idx;
    if (small) {
        block_post_small<false>(L.idx_s, L.tab_s, T, a.k, E, a.C, a, L.hist_s, L.cnt_s, L.scan_s, L.off_s, tag);
    } else if (a.slot_table) {
        // ids and slot table are read through LDS-typed pointers when they are in LDS (the usual case)
        if (idx_in_lds)
            block_post(L.idx_s, L.tab_s, A, E, a.C, a.hist, a.slot_idx, a.miss_list, a.miss_count, a.slot_count,
                       a.slot_offset, a.perm, a.pos, a.active_slots, a.n_active, L.hist_s, L.cnt_s, L.off_s,
                       L.scan_s, L.sidx_s);
        else
            block_post(idx, L.tab_s, A, E, a.C, a.hist, a.slot_idx, a.miss_list, a.miss_count, a.slot_count,
                       a.slot_offset, a.perm, a.pos, a.active_slots, a.n_active, L.hist_s, L.cnt_s, L.off_s,
                       L.scan_s, L.sidx_s);
    } else if (a.hist) {
        block_histogram(idx, A, E, a.hist, L.hist_s);
    }
    if (tid == 0) {
        *a.epoch = tag;
        // a wait ran out somewhere in this call: what it wrote is not a result, and says so
        if (a.miss_count && __hip_atomic_load(a.error_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) *a.miss_count = -1;
    }
}

__global__ __launch_bounds__(kRouteThreads) void histogram_kernel(const int32_t *idx, int A, int E,
                                                                   int32_t *hist)
{
    extern __shared__ int dyn[];
    block_histogram(idx, A, E, hist, (lds_i32 *)dyn);
}

// large inputs: zero, then per-workgroup LDS histograms merged with integer atomics
__global__ void zero_kernel(int32_t *p, int n)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

__global__ __launch_bounds__(kRouteThreads) void histogram_multi_kernel(const int32_t *idx, int A, int E,
                                                                         int32_t *hist)
{
    extern __shared__ int dyn[];
    for (int e = threadIdx.x; e < E; e += blockDim.x) dyn[e] = 0;
    __syncthreads();
    for (size_t a = (size_t)blockIdx.x * blockDim.x + threadIdx.x; a < (size_t)A;
         a += (size_t)gridDim.x * blockDim.x) {
        int e = idx[a];
        if ((unsigned)e < (unsigned)E) atomicAdd(&dyn[e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x)
        if (dyn[e]) atomicAdd(&hist[e], dyn[e]);
}

__global__ __launch_bounds__(kRouteThreads) void resolve_kernel(const int32_t *idx, const int32_t *slot_table,
                                                                 int A, int E, int C, int32_t *slot_idx,
                                                                 int32_t *miss_list, int32_t *miss_count,
                                                                 int32_t *slot_count, int32_t *slot_offset,
                                                                 int32_t *perm, int32_t *pos,
                                                                 int32_t *active_slots, unsigned *n_active,
                                                                 unsigned *epoch, unsigned layout)
{
    extern __shared__ int dyn[];
    if (epoch && threadIdx.x == 0) check_layout(epoch - kCtrlEpoch, layout);
    PostLds L = carve_lds(dyn, 0, C, A);
    block_post(idx, slot_table, A, E, C, nullptr, slot_idx, miss_list, miss_count, slot_count, slot_offset,
               perm, pos, active_slots, n_active, L.hist_s, L.cnt_s, L.off_s, L.scan_s, L.sidx_s);
    if (epoch && threadIdx.x == 0) *epoch += 1u;   // the kernels that follow stamp their entries with this number
}

__global__ void clear_ctrl_kernel(unsigned *ws, int words)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < words; i += gridDim.x * blockDim.x) ws[i] = 0u;
}

}  // namespace


size_t route_lds_bytes(int E, int C, int A) { return post_lds_bytes(E, C, A, true); }

hipError_t launch_route(const RouteArgs &a, hipStream_t s)
{
    size_t lds = post_lds_bytes(a.E, a.slot_table ? a.C : 0, a.T * a.k, true);
    hipError_t e = allow_full_lds((const void *)route_kernel, kLdsBytes - 1024);
    if (e != hipSuccess) return e;
    int grid = device_cus(&e);
    if (e != hipSuccess) return e;
    if (grid > a.T * a.E) grid = a.T * a.E;
    RouteArgs args = a;
    void *params[] = {&args};
    e = launch_timed((const void *)route_kernel, dim3(grid), dim3(kRouteThreads), params, lds, s, 0);
    return e != hipSuccess ? e : hipGetLastError();
}

hipError_t launch_histogram(const int32_t *topk_idx, int A, int E, int32_t *hist, hipStream_t s)
{
    size_t lds = (size_t)E * sizeof(int);
    if (A <= (1 << 16)) {
        hipLaunchKernelGGL(histogram_kernel, dim3(1), dim3(kRouteThreads), lds, s, topk_idx, A, E, hist);
    } else {
        hipLaunchKernelGGL(zero_kernel, dim3((E + 255) / 256), dim3(256), 0, s, hist, E);
        int blocks = (A + kRouteThreads * 16 - 1) / (kRouteThreads * 16);
        if (blocks > 1024) blocks = 1024;
        hipLaunchKernelGGL(histogram_multi_kernel, dim3(blocks), dim3(kRouteThreads), lds, s, topk_idx, A,
                           E, hist);
    }
    return hipGetLastError();
}

hipError_t launch_resolve(const int32_t *topk_idx, const int32_t *slot_table, int A, int E, int C,
                          int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, int32_t *slot_count,
                          int32_t *slot_offset, int32_t *perm, int32_t *pos, int32_t *active_slots,
                          unsigned *n_active, hipStream_t s)
{
    size_t lds = post_lds_bytes(0, C, A, false);
    if (lds > (size_t)kLdsBytes - 1024) return hipErrorInvalidValue;
    hipError_t e = allow_full_lds((const void *)resolve_kernel, kLdsBytes - 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(kRouteThreads), lds, s, topk_idx, slot_table, A, E, C,
                       slot_idx, miss_list, miss_count, slot_count, slot_offset, perm, pos, active_slots,
                       n_active, (unsigned *)nullptr, 0u);
    return hipGetLastError();
}

hipError_t launch_lists_from_slots(unsigned layout, const int32_t *slot_idx, int A, int C, int32_t *slot_count,
                                   int32_t *slot_offset, int32_t *perm, int32_t *pos, int32_t *active_slots,
                                   unsigned *n_active, unsigned *epoch, hipStream_t s)
{
    size_t lds = post_lds_bytes(0, C, A, false);
    if (lds > (size_t)kLdsBytes - 1024) return hipErrorInvalidValue;
    hipError_t e = allow_full_lds((const void *)resolve_kernel, kLdsBytes - 1024);
    if (e != hipSuccess) return e;
    prof_begin(1, s);
    hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(kRouteThreads), lds, s, (const int32_t *)nullptr,
                       (const int32_t *)nullptr, A, 0, C, const_cast<int32_t *>(slot_idx),
                       (int32_t *)nullptr, (int32_t *)nullptr, slot_count, slot_offset, perm, pos,
                       active_slots, n_active, epoch, layout);
    prof_end(1, s);
    return hipGetLastError();
}

hipError_t launch_clear_ctrl(void *workspace, size_t bytes, hipStream_t s)
{
    // everything: a stale 64-bit entry anywhere in the workspace must not carry a future call number
    const size_t words = bytes / 4;
    if (words > (size_t)1 << 31) return hipErrorInvalidValue;
    int blocks = (int)((words + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(clear_ctrl_kernel, dim3(blocks), dim3(256), 0, s, (unsigned *)workspace, (int)words);
    return hipGetLastError();
}

}  // namespace moe
