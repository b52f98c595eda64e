// Routing side of the verify-step MoE layer (gfx950):
//   router GEMM  s = W_g h            (Sec. 2.2, first line of the MoE equation)
//   Top-k and the gate over the k picks  (second and third line)
//   activation-frequency histogram     (Sec. 2.3)
//   expert id -> cache slot, miss list, per-slot token lists   (App. D)
//
// The fused kernel spreads the [T,H]x[H,E] contraction over one workgroup per
// expert row; the workgroup that finishes last (ticket in the workspace
// control block) owns every logit and runs the small integer steps out of LDS,
// so a layer needs one launch for all of them, no grid-wide wait, and only
// three dependent trips to memory (weights, logits, results).
#include "moe_internal.h"

namespace moe {

namespace {

constexpr int kRouteThreads = 512;
constexpr int kRouteWaves = kRouteThreads / kWave;
constexpr int kTokBlock = 8;
constexpr int kLdsCopy = 4096;  // assignments whose ids are mirrored in LDS

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ inline float load_coherent(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One wavefront ranks the E logits of one token: rank(e) = number of experts
// that beat e (larger logit, or equal logit and lower id).  The experts of
// rank 0..k-1 are the Top-k in descending-logit order; their gate is
// exp(s - s_max) normalised over those k.  Lane l owns experts l, l+64, ...;
// every value is broadcast once through a scalar register (no LDS traffic).
template <int NLOC>
__device__ void wave_topk_gate_n(const float *row, bool coherent, int E, int k, int32_t *idx_out,
                                 int32_t *idx_lds, float *w_out)
{
    const int lane = threadIdx.x & (kWave - 1);
    constexpr int nloc = NLOC;
    float v[NLOC];
    int rank[NLOC];
#pragma unroll
    for (int i = 0; i < NLOC; ++i) {
        int e = lane + kWave * i;
        v[i] = -INFINITY;
        rank[i] = 0;
        if (i < nloc && e < E) {
            float x = coherent ? load_coherent(row + e) : row[e];
            v[i] = (x == x) ? x : -INFINITY;   // NaN cannot win a comparison; rank it last
        }
    }
#pragma unroll
    for (int i2 = 0; i2 < NLOC; ++i2) {
        if (i2 < nloc) {
            for (int l = 0; l < kWave; ++l) {
                int e2 = l + kWave * i2;
                if (e2 >= E) break;
                float o = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v[i2]), l));
#pragma unroll
                for (int i = 0; i < NLOC; ++i) {
                    int e = lane + kWave * i;
                    rank[i] += (o > v[i] || (o == v[i] && e2 < e)) ? 1 : 0;
                }
            }
        }
    }
    // s_max = the logit of rank 0
    float smax_c = -INFINITY;
#pragma unroll
    for (int i = 0; i < NLOC; ++i) {
        int e = lane + kWave * i;
        if (i < nloc && e < E && rank[i] == 0) smax_c = v[i];
    }
    float smax = smax_c;
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) smax = fmaxf(smax, __shfl_xor(smax, m, kWave));
    float p[NLOC];
    float den = 0.f;
#pragma unroll
    for (int i = 0; i < NLOC; ++i) {
        int e = lane + kWave * i;
        p[i] = 0.f;
        if (i < nloc && e < E && rank[i] < k) p[i] = expf(v[i] - smax);
        den += p[i];
    }
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) den += __shfl_xor(den, m, kWave);
#pragma unroll
    for (int i = 0; i < NLOC; ++i) {
        int e = lane + kWave * i;
        if (i < nloc && e < E && rank[i] < k) {
            idx_out[rank[i]] = e;
            if (idx_lds) idx_lds[rank[i]] = e;
            w_out[rank[i]] = p[i] / den;
        }
    }
}

__device__ void wave_topk_gate(const float *row, bool coherent, int E, int k, int32_t *idx_out,
                               int32_t *idx_lds, float *w_out)
{
    if (E <= kWave) wave_topk_gate_n<1>(row, coherent, E, k, idx_out, idx_lds, w_out);
    else if (E <= 2 * kWave) wave_topk_gate_n<2>(row, coherent, E, k, idx_out, idx_lds, w_out);
    else if (E <= 4 * kWave) wave_topk_gate_n<4>(row, coherent, E, k, idx_out, idx_lds, w_out);
    else wave_topk_gate_n<kMaxEPL>(row, coherent, E, k, idx_out, idx_lds, w_out);
}

// hist[e] = number of assignments naming expert e (LDS integer atomics).
__device__ void block_histogram(const int32_t *idx, int A, int E, int32_t *hist, int *hist_s)
{
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist_s[e] = 0;
    __syncthreads();
    for (int a = threadIdx.x; a < A; a += blockDim.x) {
        int e = idx[a];
        if ((unsigned)e < (unsigned)E) atomicAdd(&hist_s[e], 1);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist[e] = hist_s[e];
}

// Slot lookup, ascending miss list, per-slot assignment lists and the list of
// active slots.  idx / slot_table may point to LDS copies.
// slot_table == nullptr: slot_idx is an input (lists only).
// LDS: cnt_s[C], off_s[C+1], scan_s[16], sidx_s[min(A, kLdsCopy)].
__device__ void block_resolve(const int32_t *idx, const int32_t *slot_table, int A, int E, int C,
                              int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count,
                              int32_t *slot_count, int32_t *slot_offset, int32_t *perm, int32_t *pos,
                              int32_t *active_slots, unsigned *n_active, int *cnt_s, int *off_s, int *scan_s,
                              int *sidx_s)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const int nw = blockDim.x / kWave;
    for (int c = tid; c < C; c += blockDim.x) cnt_s[c] = 0;
    __syncthreads();
    int running = 0;
    for (int base = 0; base < A; base += blockDim.x) {
        int a = base + tid;
        bool valid = a < A;
        int c = -1;
        if (valid) {
            if (slot_table) {
                int e = idx[a];
                c = ((unsigned)e < (unsigned)E) ? slot_table[e] : -1;
            } else {
                c = slot_idx[a];
            }
            if ((unsigned)c >= (unsigned)C) c = -1;
            if (slot_table) slot_idx[a] = c;
            if (a < kLdsCopy) sidx_s[a] = c;
            if (c >= 0) atomicAdd(&cnt_s[c], 1);
        }
        bool miss = valid && c < 0;
        unsigned long long bal = __ballot(miss);
        int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) scan_s[w] = __popcll(bal);
        __syncthreads();
        int wave_base = 0, total = 0;
        for (int i = 0; i < nw; ++i) {
            int s = scan_s[i];
            if (i < w) wave_base += s;
            total += s;
        }
        if (miss && miss_list) miss_list[running + wave_base + before] = a;
        running += total;
        __syncthreads();
    }
    if (tid == 0) {
        if (miss_count) *miss_count = running;
        int o = 0, na = 0;
        for (int c = 0; c < C; ++c) {
            off_s[c] = o;
            o += cnt_s[c];
            if (cnt_s[c] > 0) active_slots[na++] = c;
        }
        off_s[C] = o;
        *n_active = (unsigned)na;
    }
    __syncthreads();
    for (int c = tid; c <= C; c += blockDim.x) {
        slot_offset[c] = off_s[c];
        if (c < C) slot_count[c] = cnt_s[c];
    }
    // stable: the list of a slot holds its assignments in ascending flat id
    for (int c = tid; c < C; c += blockDim.x) {
        if (cnt_s[c] == 0) continue;
        int cur = off_s[c];
        for (int a = 0; a < A; ++a) {
            int s = (a < kLdsCopy) ? sidx_s[a] : slot_idx[a];
            if (s == c) { perm[cur] = a; pos[a] = cur; ++cur; }
        }
    }
    for (int a = tid; a < A; a += blockDim.x) {
        int s = (a < kLdsCopy) ? sidx_s[a] : slot_idx[a];
        if ((unsigned)s >= (unsigned)C) pos[a] = -1;
    }
}

// dynamic LDS: hist_s[E] tab_s[E] cnt_s[C] off_s[C+1] scan_s[16] sidx_s[cap] idx_s[cap], cap = min(A, kLdsCopy)
struct PostLds {
    int *hist_s, *tab_s, *cnt_s, *off_s, *scan_s, *sidx_s, *idx_s;
};

__device__ inline PostLds carve_lds(int *dyn, int E, int C, int A)
{
    const int cap = A < kLdsCopy ? A : kLdsCopy;
    PostLds p;
    p.hist_s = dyn;
    p.tab_s = p.hist_s + E;
    p.cnt_s = p.tab_s + E;
    p.off_s = p.cnt_s + C;
    p.scan_s = p.off_s + C + 1;
    p.sidx_s = p.scan_s + 16;
    p.idx_s = p.sidx_s + cap;
    return p;
}

size_t post_lds_bytes(int E, int C, int A)
{
    const int cap = A < kLdsCopy ? A : kLdsCopy;
    return (size_t)(2 * E + C + (C + 1) + 16 + 2 * cap) * sizeof(int);
}

__global__ __launch_bounds__(kRouteThreads) void route_kernel(RouteArgs a)
{
    extern __shared__ int dyn[];
    __shared__ float red[kRouteWaves][kTokBlock];
    __shared__ int is_last;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const int e = blockIdx.x;
    const int T = a.T, H = a.H, E = a.E;
    const int A = T * a.k;
    const float *wrow = a.router_w + (size_t)e * H;
    const uint16_t *x = (const uint16_t *)a.hidden;
    PostLds L = carve_lds(dyn, E, a.C, A);

    // the slot table rides along with the first trip to memory (only the last workgroup uses it)
    if (a.slot_table)
        for (int i = tid; i < E; i += kRouteThreads) L.tab_s[i] = a.slot_table[i];

    // s[t,e] for every token t: the wavefronts split H, lanes stride it 4 at a time
    for (int t0 = 0; t0 < T; t0 += kTokBlock) {
        float acc[kTokBlock];
#pragma unroll
        for (int u = 0; u < kTokBlock; ++u) acc[u] = 0.f;
        for (int h = (w * kWave + lane) * 4; h < H; h += kRouteThreads * 4) {
            float4 wv = *(const float4 *)(wrow + h);
#pragma unroll
            for (int u = 0; u < kTokBlock; ++u) {
                int t = t0 + u;
                if (t < T) {
                    uint2 xv = *(const uint2 *)(x + (size_t)t * H + h);
                    acc[u] += wv.x * bf16_lo(xv.x) + wv.y * bf16_hi(xv.x) + wv.z * bf16_lo(xv.y) +
                              wv.w * bf16_hi(xv.y);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kTokBlock; ++u) {
#pragma unroll
            for (int m = kWave / 2; m >= 1; m >>= 1) acc[u] += __shfl_xor(acc[u], m, kWave);
            if (lane == 0) red[w][u] = acc[u];
        }
        __syncthreads();
        if (tid < kTokBlock && t0 + tid < T) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < kRouteWaves; ++i) s += red[i][tid];
            if (a.router_bias) s += a.router_bias[e];
            a.logits_ws[(size_t)(t0 + tid) * E + e] = s;
            if (a.logits_opt) a.logits_opt[(size_t)(t0 + tid) * E + e] = s;
        }
        __syncthreads();
    }

    // the last workgroup to arrive sees every logit.  The logits were written by wavefront 0, so
    // only it publishes them (a release fence per wavefront costs a cache write-back each)
    if (w == 0) __threadfence();
    __syncthreads();
    if (tid == 0) {
        unsigned old = atomicAdd(a.ticket, 1u);
        is_last = (old == gridDim.x - 1);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    const bool idx_in_lds = A <= kLdsCopy;
    for (int t = w; t < T; t += kRouteWaves)
        wave_topk_gate(a.logits_ws + (size_t)t * E, true, E, a.k, a.topk_idx + (size_t)t * a.k,
                       idx_in_lds ? L.idx_s + t * a.k : nullptr, a.topk_w + (size_t)t * a.k);
    __syncthreads();

    const int32_t *idx = idx_in_lds ? L.idx_s : a.topk_idx;
    if (a.hist) block_histogram(idx, A, E, a.hist, L.hist_s);
    if (a.slot_table)
        block_resolve(idx, L.tab_s, A, E, a.C, a.slot_idx, a.miss_list, a.miss_count, a.slot_count,
                      a.slot_offset, a.perm, a.pos, a.active_slots, a.n_active, L.cnt_s, L.off_s, L.scan_s,
                      L.sidx_s);
    if (tid == 0) atomicExch(a.ticket, 0u);
}

__global__ __launch_bounds__(kRouteThreads) void histogram_kernel(const int32_t *idx, int A, int E,
                                                                   int32_t *hist)
{
    extern __shared__ int dyn[];
    block_histogram(idx, A, E, hist, dyn);
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
                                                                 int32_t *active_slots, unsigned *n_active)
{
    extern __shared__ int dyn[];
    PostLds L = carve_lds(dyn, 0, C, A);
    block_resolve(idx, slot_table, A, E, C, slot_idx, miss_list, miss_count, slot_count, slot_offset, perm,
                  pos, active_slots, n_active, L.cnt_s, L.off_s, L.scan_s, L.sidx_s);
}

__global__ void clear_ctrl_kernel(unsigned *ctrl)
{
    if (threadIdx.x < kCtrlBytes / 4) ctrl[threadIdx.x] = 0u;
}

}  // namespace

hipError_t launch_route(const RouteArgs &a, hipStream_t s)
{
    size_t lds = post_lds_bytes(a.E, a.slot_table ? a.C : 0, a.T * a.k);
    prof_begin(0, s);
    hipLaunchKernelGGL(route_kernel, dim3(a.E), dim3(kRouteThreads), lds, s, a);
    prof_end(0, s);
    return hipGetLastError();
}

hipError_t launch_histogram(const int32_t *topk_idx, int A, int E, int32_t *hist, hipStream_t s)
{
    size_t lds = (size_t)E * sizeof(int);
    if (A <= (1 << 16)) {
        hipLaunchKernelGGL(histogram_kernel, dim3(1), dim3(kRouteThreads), lds, s, topk_idx, A, E, hist);
    } else {
        hipLaunchKernelGGL(zero_kernel, dim3((E + 255) / 256), dim3(256), 0, s, hist, E);
        int blocks = (A + kRouteThreads * 64 - 1) / (kRouteThreads * 64);
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
    size_t lds = post_lds_bytes(0, C, A);
    hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(kRouteThreads), lds, s, topk_idx, slot_table, A, E, C,
                       slot_idx, miss_list, miss_count, slot_count, slot_offset, perm, pos, active_slots,
                       n_active);
    return hipGetLastError();
}

hipError_t launch_lists_from_slots(const int32_t *slot_idx, int A, int C, int32_t *slot_count,
                                   int32_t *slot_offset, int32_t *perm, int32_t *pos, int32_t *active_slots,
                                   unsigned *n_active, hipStream_t s)
{
    size_t lds = post_lds_bytes(0, C, A);
    prof_begin(1, s);
    hipLaunchKernelGGL(resolve_kernel, dim3(1), dim3(kRouteThreads), lds, s, (const int32_t *)nullptr,
                       (const int32_t *)nullptr, A, 0, C, const_cast<int32_t *>(slot_idx),
                       (int32_t *)nullptr, (int32_t *)nullptr, slot_count, slot_offset, perm, pos,
                       active_slots, n_active);
    prof_end(1, s);
    return hipGetLastError();
}

hipError_t launch_clear_ctrl(void *ctrl, hipStream_t s)
{
    hipLaunchKernelGGL(clear_ctrl_kernel, dim3(1), dim3(64), 0, s, (unsigned *)ctrl);
    return hipGetLastError();
}

}  // namespace moe
