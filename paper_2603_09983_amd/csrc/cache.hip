// Utility-guided cache manager (Sec. 3.4 "Unified Asynchronous Execution
// Engine"; appendix on its implementation), the part that runs on the device:
//
//  plan_kernel  one planning step per layer, one workgroup each: evict the
//               residents whose utility fell below the layer's threshold tau
//               (never one that is in use: the frozen tag), then hand the free
//               slots to the non-resident experts of utility >= tau, level K
//               first, request order (expert id) inside a level, at most
//               `budget` of them; writes the eviction list, the fetch list
//               with its slots, and the new slot table that the next verify
//               step's slot lookup reads.
//  load_kernel  moves the fetched experts' three matrices from a backing
//               store into their slots of the pools.  The store can be device
//               memory or pinned host memory mapped into the device: the
//               kernel only sees pointers, so the same launch on a second
//               stream overlaps the copy with the verify steps of other
//               layers, which is the paper's asynchronous prefetch.
//
// The paper keeps a multi-level FIFO queue and a red-black tree on the host;
// with N <= 512 experts per layer the same order falls out of counting: the
// position of an expert in a list is the number of list members with a
// smaller (level, id) key, which every thread counts for its own expert from
// a copy of the keys in LDS.  No queue, no tree, no host round trip.
#include "../../include/moe_spac.h"
#include "moe_internal.h"

namespace moe {

namespace {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;

struct PlanArgs {
    const int32_t *s;        // [L,N]
    const int32_t *in_use;   // [L,N] or null
    int32_t *slot_table;     // [L,N] in/out
    const int32_t *tau;      // [L]
    const int32_t *budget;   // [L] or null (no limit)
    int32_t *evict_list;     // [L,N]
    int32_t *n_evict;        // [L]
    int32_t *fetch_list;     // [L,C]
    int32_t *fetch_slot;     // [L,C]
    int32_t *n_fetch;        // [L]
    int N, C, K;
};

// number of set keys below `key` among key_s[0..N) (entries < 0 are not members)
__device__ inline int rank_below(const int *key_s, int N, int key)
{
    int r = 0;
    for (int i = 0; i < N; ++i) {
        const int k2 = key_s[i];
        r += (k2 >= 0 && k2 < key) ? 1 : 0;
    }
    return r;
}

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(PlanArgs a)
{
    __shared__ int ekey_s[kMaxE];        // eviction key  s*N + id, or -1
    __shared__ int fkey_s[kMaxE];        // fetch key  (K-s)*N + id, or -1
    __shared__ int used_s[kMaxC];        // slot still held after the evictions
    __shared__ int free_s[kMaxC];        // free slots, ascending
    __shared__ int scan_s[kPlanWaves];
    __shared__ int tot_s[3];             // evicted, candidates, free
    const int l = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const int N = a.N, C = a.C, K = a.K;
    const int tau = a.tau[l];
    // (asked for with the other inputs, not where it is needed: one trip to memory instead of two)
    int bud = 0x7fffffff;
    if (a.budget) {
        bud = a.budget[l];
        bud = bud < 0 ? 0 : bud;
    }
    const size_t base = (size_t)l * N;

    int s = 0, slot = -1;
    bool frozen = false;
    if (tid < N) {
        s = a.s[base + tid];
        slot = a.slot_table[base + tid];
        if ((unsigned)slot >= (unsigned)C) slot = -1;
        frozen = a.in_use && a.in_use[base + tid] != 0;
    }
    const bool evict = tid < N && slot >= 0 && !frozen && s < tau;
    const bool cand = tid < N && slot < 0 && s >= tau && s <= K;
    if (tid < kMaxE) {
        ekey_s[tid] = evict ? s * N + tid : -1;
        fkey_s[tid] = cand ? (K - s) * N + tid : -1;
    }
    for (int c = tid; c < C; c += kPlanThreads) used_s[c] = 0;
    if (tid < 3) tot_s[tid] = 0;
    __syncthreads();
    if (tid < N && slot >= 0 && !evict) used_s[slot] = 1;   // (a table that is not one-to-one just marks the slot once)
    if (evict) atomicAdd(&tot_s[0], 1);
    if (cand) atomicAdd(&tot_s[1], 1);
    __syncthreads();
    // free slots in ascending order: prefix sum of the free flags (C <= 1024 = one slot per thread)
    const int is_free = (tid < C && !used_s[tid]) ? 1 : 0;
    int inc = is_free;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int t = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += t;
    }
    if (lane == kWave - 1) scan_s[w] = inc;
    __syncthreads();
    int wave_base = 0, n_free = 0;
    for (int i = 0; i < kPlanWaves; ++i) {
        const int v = scan_s[i];
        if (i < w) wave_base += v;
        n_free += v;
    }
    if (is_free) free_s[wave_base + inc - 1] = tid;
    __syncthreads();

    if (evict) {
        a.evict_list[base + rank_below(ekey_s, N, s * N + tid)] = tid;
        a.slot_table[base + tid] = -1;
    }
    int n_fetch = tot_s[1] < n_free ? tot_s[1] : n_free;
    n_fetch = n_fetch < bud ? n_fetch : bud;
    if (cand) {
        const int r = rank_below(fkey_s, N, (K - s) * N + tid);
        if (r < n_fetch) {
            const int c = free_s[r];
            a.fetch_list[(size_t)l * C + r] = tid;
            a.fetch_slot[(size_t)l * C + r] = c;
            a.slot_table[base + tid] = c;
        }
    }
    if (tid == 0) {
        a.n_evict[l] = tot_s[0];
        a.n_fetch[l] = n_fetch;
    }
}

struct LoadArgs {
    const uint16_t *store_gate, *store_up, *store_down;   // [E,F,H], [E,F,H], [E,H,F]
    uint16_t *pool_gate, *pool_up, *pool_down;             // [C,F,H], [C,F,H], [C,H,F]
    const int32_t *fetch_list, *fetch_slot, *n_fetch;      // one layer's lists
    size_t words16;                                         // 16-byte words per matrix (F*H*2/16)
};

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// grid (chunks, max_fetch): block (x, j) copies its share of the three matrices of fetch entry j
__global__ __launch_bounds__(256) void load_kernel(LoadArgs a)
{
    const int j = blockIdx.y;
    if (j >= *a.n_fetch) return;
    const size_t e = (size_t)a.fetch_list[j], c = (size_t)a.fetch_slot[j];
    const u32x4 *src[3] = {(const u32x4 *)a.store_gate + e * a.words16, (const u32x4 *)a.store_up + e * a.words16,
                           (const u32x4 *)a.store_down + e * a.words16};
    u32x4 *dst[3] = {(u32x4 *)a.pool_gate + c * a.words16, (u32x4 *)a.pool_up + c * a.words16,
                     (u32x4 *)a.pool_down + c * a.words16};
    // four 16-byte words per thread in flight (words i, i + 256, ..: a wavefront's accesses stay contiguous)
    const size_t bd = blockDim.x, stride = (size_t)gridDim.x * bd * 4;
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        size_t i = (size_t)blockIdx.x * bd * 4 + threadIdx.x;
        for (; i + 3 * bd < a.words16; i += stride) {
            const u32x4 v0 = __builtin_nontemporal_load(src[m] + i), v1 = __builtin_nontemporal_load(src[m] + i + bd);
            const u32x4 v2 = __builtin_nontemporal_load(src[m] + i + 2 * bd), v3 = __builtin_nontemporal_load(src[m] + i + 3 * bd);
            __builtin_nontemporal_store(v0, dst[m] + i);
            __builtin_nontemporal_store(v1, dst[m] + i + bd);
            __builtin_nontemporal_store(v2, dst[m] + i + 2 * bd);
            __builtin_nontemporal_store(v3, dst[m] + i + 3 * bd);
        }
        for (; i < a.words16; i += bd)   // the last, partial group of four (only the workgroup that reaches it)
            __builtin_nontemporal_store(__builtin_nontemporal_load(src[m] + i), dst[m] + i);
    }
}

// The same copy for a store in host memory: gridDim.x workgroups walk all fetch entries, one 16-byte word
// per thread in flight.
__global__ __launch_bounds__(256) void load_narrow_kernel(LoadArgs a)
{
    const int n_fetch = *a.n_fetch;
    for (int j = 0; j < n_fetch; ++j) {
        const size_t e = (size_t)a.fetch_list[j], c = (size_t)a.fetch_slot[j];
        const u32x4 *src[3] = {(const u32x4 *)a.store_gate + e * a.words16, (const u32x4 *)a.store_up + e * a.words16,
                               (const u32x4 *)a.store_down + e * a.words16};
        u32x4 *dst[3] = {(u32x4 *)a.pool_gate + c * a.words16, (u32x4 *)a.pool_up + c * a.words16,
                         (u32x4 *)a.pool_down + c * a.words16};
#pragma unroll
        for (int m = 0; m < 3; ++m)
            for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.words16; i += (size_t)gridDim.x * blockDim.x)
                __builtin_nontemporal_store(__builtin_nontemporal_load(src[m] + i), dst[m] + i);
    }
}

}  // namespace

}  // namespace moe

using namespace moe;

extern "C" int moe_cache_plan(const int32_t *s, const int32_t *in_use, int32_t *slot_table, const int32_t *tau,
                              const int32_t *budget, int L, int N, int C, int K, int32_t *evict_list,
                              int32_t *n_evict, int32_t *fetch_list, int32_t *fetch_slot, int32_t *n_fetch,
                              void *stream)
{
    if (!s || !slot_table || !tau || !evict_list || !n_evict || !fetch_list || !fetch_slot || !n_fetch)
        return MOE_ERR_NULL;
    if (L < 1 || L > 65535 || N < 1 || N > kMaxE || C < 0 || C > kMaxC || K < 0 || K > 64) return MOE_ERR_SHAPE;
    PlanArgs a = {s, in_use, slot_table, tau, budget, evict_list, n_evict, fetch_list, fetch_slot, n_fetch, N, C, K};
    void *params[] = {&a};
    hipError_t e = launch_timed((const void *)plan_kernel, dim3(L), dim3(kPlanThreads), params, 0,
                                (hipStream_t)stream, MOE_KERNEL_CACHE_PLAN);
    if (e == hipSuccess) e = hipGetLastError();
    return e == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}

extern "C" int moe_pool_load(const void *store_gate, const void *store_up, const void *store_down, void *pool_gate,
                             void *pool_up, void *pool_down, const int32_t *fetch_list, const int32_t *fetch_slot,
                             const int32_t *n_fetch, int max_fetch, int H, int F, void *stream)
{
    if (!store_gate || !store_up || !store_down || !pool_gate || !pool_up || !pool_down || !fetch_list ||
        !fetch_slot || !n_fetch)
        return MOE_ERR_NULL;
    if (max_fetch < 1 || max_fetch > kMaxC || H < 1 || F < 1) return MOE_ERR_SHAPE;
    if (((size_t)H * F * 2) % 16 != 0) return MOE_ERR_ALIGN;
    auto al = [](const void *p) { return ((uintptr_t)p & 15) == 0; };
    if (!al(store_gate) || !al(store_up) || !al(store_down) || !al(pool_gate) || !al(pool_up) || !al(pool_down))
        return MOE_ERR_ALIGN;
    LoadArgs a = {(const uint16_t *)store_gate, (const uint16_t *)store_up, (const uint16_t *)store_down,
                  (uint16_t *)pool_gate, (uint16_t *)pool_up, (uint16_t *)pool_down, fetch_list, fetch_slot, n_fetch,
                  (size_t)H * F * 2 / 16};
    void *params[] = {&a};
    int chunks = (int)((a.words16 + 256 * 8 - 1) / (256 * 8));   // eight 16-byte words per thread and matrix
    if (chunks > 512) chunks = 512;
    if (chunks < 1) chunks = 1;
    // A store in host memory is read at the rate of the link to the host, a hundred times below HBM's: a
    // chip-wide launch would hold every wavefront slot for a millisecond and keep the verify steps'
    // workgroups waiting.  Sixteen workgroups with one 16-byte word per thread in flight (64 KB) reach 9/10
    // of the link's rate (51 of 56 GB/s) and disturb the verify steps least.  Measured per cfg2 layer with a
    // copy always in flight: +5.7 us; 32 workgroups +7.5, 64 +11.5, a chip-wide launch +15; four words per
    // thread in flight +8 (4 workgroups) to +12 (16).
    bool narrow = false;
    {
        hipPointerAttribute_t attr;
        if (hipPointerGetAttributes(&attr, store_gate) == hipSuccess)
            narrow = attr.type == hipMemoryTypeHost;
        else
            (void)hipGetLastError();   // not a pointer the runtime knows: launch as for device memory
    }
    if (narrow) {
        hipError_t e = launch_timed((const void *)load_narrow_kernel, dim3(16), dim3(256), params, 0,
                                    (hipStream_t)stream, MOE_KERNEL_POOL_LOAD);
        if (e == hipSuccess) e = hipGetLastError();
        return e == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
    }
    hipError_t e = launch_timed((const void *)load_kernel, dim3(chunks, max_fetch), dim3(256), params, 0,
                                (hipStream_t)stream, MOE_KERNEL_POOL_LOAD);
    if (e == hipSuccess) e = hipGetLastError();
    return e == hipSuccess ? MOE_OK : MOE_ERR_LAUNCH;
}
