// Device-side pieces of the routing steps (Top-k and gate of one token per wavefront, histogram, slot
// lookup, miss list and per-slot lists of a whole batch per workgroup), shared by the routing kernel and
// by the gate/up kernel that does the routing itself.  Included inside an unnamed namespace of each
// translation unit.
#pragma once
#include "moe_internal.h"

namespace moe {

namespace {

constexpr int kRouteThreads = 1024;
constexpr int kRouteWaves = kRouteThreads / kWave;
constexpr int kLdsCopy = 4096;  // assignments whose ids are mirrored in LDS

__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// LDS and global pointers carry their address space: a generic pointer would turn every access into
// a flat instruction, and the dependent LDS reads below would each cost a trip through the memory
// pipeline instead of an LDS access.
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) int lds_i32;
typedef float f32x4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const f32x4v lds_f32x4;
typedef __attribute__((address_space(1))) int32_t g_i32;
typedef __attribute__((address_space(1))) float g_f32;

// Value of v in the lane n places further on inside the row of 16 lanes, wrapping round (register to
// register, no trip through LDS): data-parallel-primitive control row_ror:n = 0x120 + n.
template <int N>
__device__ __forceinline__ unsigned row_rotate(unsigned v)
{
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x120 + N, 0xf, 0xf, false);
}

// Maximum of x over the 64 lanes of a wavefront (all of them active), as a uniform value.  Four
// rotations leave each row's maximum in every lane of the row; the four row results are then read
// into scalar registers.
__device__ __forceinline__ unsigned wave_max_u32(unsigned x)
{
    unsigned y;
    y = row_rotate<1>(x); x = x > y ? x : y;
    y = row_rotate<2>(x); x = x > y ? x : y;
    y = row_rotate<4>(x); x = x > y ? x : y;
    y = row_rotate<8>(x); x = x > y ? x : y;
    const unsigned a = (unsigned)__builtin_amdgcn_readlane((int)x, 0), b = (unsigned)__builtin_amdgcn_readlane((int)x, 16);
    const unsigned c = (unsigned)__builtin_amdgcn_readlane((int)x, 32), d = (unsigned)__builtin_amdgcn_readlane((int)x, 48);
    const unsigned ab = a > b ? a : b, cd = c > d ? c : d;
    return ab > cd ? ab : cd;
}

// One wavefront picks the Top-k of the E logits of one token, best first: k times the maximum over the
// wavefront, ties to the lower expert id, the winner taken out.  Logits are compared as unsigned keys
// that order like the floats (-0 counted as +0; key 0 = taken or no expert, below every float).  The
// gate is exp(s - s_max) normalised over the k, summed in rank order.  Lane l owns experts l, l+64, ...;
// the caller has put the logits into `lg` (LDS private to the wavefront: E floats, NaN replaced by -inf).
// Lane j < k ends up with the j-th expert and writes it out.  Needs k <= E and all 64 lanes active.
// Returns the gate weight of the lane's pick (lanes >= k: unspecified).
template <int NLOC>
__device__ __forceinline__ float wave_topk_gate_n(int E, int k, int32_t *idx_out_, lds_i32 *idx_lds,
                                                  float *w_out_, lds_f32 *lg)
{
    g_i32 *idx_out = (g_i32 *)(uintptr_t)idx_out_;
    g_f32 *w_out = (g_f32 *)(uintptr_t)w_out_;
    const int lane = threadIdx.x & (kWave - 1);
    unsigned key[NLOC];
#pragma unroll
    for (int i = 0; i < NLOC; ++i) {
        const int e = lane + kWave * i;
        float f = e < E ? lg[e] : 0.f;
        f = f == 0.f ? 0.f : f;
        const unsigned u = __float_as_uint(f);
        key[i] = e < E ? ((u & 0x80000000u) ? ~u : (u | 0x80000000u)) : 0u;
    }
    unsigned my_key = 0x80000000u;   // (the key of 0.0f)
    int my_e = 0;
    for (int j = 0; j < k; ++j) {
        unsigned m = key[0];
#pragma unroll
        for (int i = 1; i < NLOC; ++i) m = m > key[i] ? m : key[i];
        const unsigned best = wave_max_u32(m);
        // lowest id among the experts that hold it: the lowest i that has one, then the lowest lane
        int win_i = 0;
        unsigned long long win_bal = 0ull;
#pragma unroll
        for (int i = NLOC - 1; i >= 0; --i) {
            const unsigned long long bal = __ballot(key[i] == best);
            if (bal) {
                win_bal = bal;
                win_i = i;
            }
        }
        const int win_lane = win_bal ? __ffsll((long long)win_bal) - 1 : 0;
        int e = win_lane + kWave * win_i;
        e = e < E ? e : E - 1;   // (only if k > E: stay inside every table)
        if (lane == j) {
            my_key = best;
            my_e = e;
        }
#pragma unroll
        for (int i = 0; i < NLOC; ++i)
            if (i == win_i && lane == win_lane) key[i] = 0u;
    }
    const float my_s = __uint_as_float((my_key & 0x80000000u) ? (my_key ^ 0x80000000u) : ~my_key);
    const float smax = __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)__float_as_uint(my_s), 0));
    const float ex = lane < k ? __expf(my_s - smax) : 0.f;
    float den = 0.f;
    for (int j = 0; j < k; ++j) den += __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)__float_as_uint(ex), j));
    const float gate = ex / den;
    if (lane < k) {
        if (idx_lds) idx_lds[lane] = my_e;
        if (idx_out_) {   // (null: the ids are wanted in LDS only)
            idx_out[lane] = my_e;
            w_out[lane] = gate;
        }
    }
    return gate;
}

__device__ __forceinline__ void wave_topk_gate(int E, int k, int32_t *idx_out, lds_i32 *idx_lds, float *w_out,
                                               lds_f32 *lg)
{
    if (E <= kWave) wave_topk_gate_n<1>(E, k, idx_out, idx_lds, w_out, lg);
    else if (E <= 2 * kWave) wave_topk_gate_n<2>(E, k, idx_out, idx_lds, w_out, lg);
    else if (E <= 4 * kWave) wave_topk_gate_n<4>(E, k, idx_out, idx_lds, w_out, lg);
    else wave_topk_gate_n<kMaxEPL>(E, k, idx_out, idx_lds, w_out, lg);
}

// logits of one token in LDS: E floats, each wavefront's row starting on a multiple of four
__host__ __device__ inline int lg_stride(int E) { return (E + 3) & ~3; }


// hist[e] = number of assignments naming expert e (LDS integer atomics).
__device__ void block_histogram(const int32_t *idx, int A, int E, int32_t *hist, lds_i32 *hist_s)
{
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist_s[e] = 0;
    __syncthreads();
    for (int a = threadIdx.x; a < A; a += blockDim.x) {
        int e = idx[a];
        if ((unsigned)e < (unsigned)E) __hip_atomic_fetch_add(&hist_s[e], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < E; e += blockDim.x) hist[e] = hist_s[e];
}

// Histogram (optional), slot lookup, ascending miss list, per-slot assignment lists and the
// list of active slots, by one workgroup.  idx / slot_table may point to LDS copies.
//   hist == nullptr: no histogram.   slot_table == nullptr: slot_idx is an input (lists only).
// LDS: hist_s[E], cnt_s[C], off_s[C+1], scan_s[32], sidx_s[min(A, kLdsCopy)].
template <typename IdxPtr, typename TabPtr>
__device__ void block_post(IdxPtr idx, TabPtr slot_table, int A, int E, int C, int32_t *hist,
                           int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, int32_t *slot_count,
                           int32_t *slot_offset, int32_t *perm, int32_t *pos, int32_t *active_slots,
                           unsigned *n_active, lds_i32 *hist_s, lds_i32 *cnt_s, lds_i32 *off_s, lds_i32 *scan_s,
                           lds_i32 *sidx_s)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const int nw = blockDim.x / kWave;
    if (hist)
        for (int e = tid; e < E; e += blockDim.x) hist_s[e] = 0;
    for (int c = tid; c < C; c += blockDim.x) cnt_s[c] = 0;
    __syncthreads();
    // pass over the assignments: histogram, slot of each, slot counts, miss list
    int running = 0;
    for (int base = 0; base < A; base += blockDim.x) {
        int a = base + tid;
        bool valid = a < A;
        int c = -1;
        if (valid) {
            if (slot_table) {
                int e = idx[a];
                bool e_ok = (unsigned)e < (unsigned)E;
                if (hist && e_ok) __hip_atomic_fetch_add(&hist_s[e], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                c = e_ok ? slot_table[e] : -1;
            } else {
                c = slot_idx[a];
            }
            if ((unsigned)c >= (unsigned)C) c = -1;
            if (slot_table) slot_idx[a] = c;
            if (a < kLdsCopy) sidx_s[a] = c;
            if (c >= 0) __hip_atomic_fetch_add(&cnt_s[c], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        bool miss = valid && c < 0;
        unsigned long long bal = __ballot(miss);
        int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (A > kWave) {
            // more than one wavefront holds assignments: offsets across wavefronts through LDS
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
        } else {
            if (miss && miss_list) miss_list[before] = a;
            if (w == 0 && lane == 0) scan_s[0] = __popcll(bal);
        }
    }
    __syncthreads();
    if (A <= kWave) running = scan_s[0];
    if (tid == 0 && miss_count) *miss_count = running;
    if (hist)
        for (int e = tid; e < E; e += blockDim.x) hist[e] = hist_s[e];
    // offsets and active list: thread c looks at the slots before it
    for (int c = tid; c <= C; c += blockDim.x) {
        int o = 0, na = 0;
#pragma unroll 8
        for (int c2 = 0; c2 < c; ++c2) {
            int v = cnt_s[c2];
            o += v;
            na += v > 0 ? 1 : 0;
        }
        off_s[c] = o;
        slot_offset[c] = o;
        if (c < C) {
            int v = cnt_s[c];
            slot_count[c] = v;
            if (v > 0) active_slots[na] = c;
        } else {
            *n_active = (unsigned)na;
        }
    }
    __syncthreads();
    // lists: assignment a goes to position off[slot] + (number of earlier assignments of that slot),
    // so the list of a slot holds its assignments in ascending flat id
    for (int a = tid; a < A; a += blockDim.x) {
        int s = (a < kLdsCopy) ? sidx_s[a] : slot_idx[a];
        if ((unsigned)s >= (unsigned)C) {
            pos[a] = -1;
            continue;
        }
        int r = 0;
#pragma unroll 8
        for (int a2 = 0; a2 < a; ++a2) {
            int s2 = (a2 < kLdsCopy) ? sidx_s[a2] : slot_idx[a2];
            if ((unsigned)s2 >= (unsigned)C) s2 = -1;
            r += s2 == s ? 1 : 0;
        }
        int p = off_s[s] + r;
        perm[p] = a;
        pos[a] = p;
    }
}

// dynamic LDS: hist_s[E] tab_s[E] cnt_s[4C] off_s[C+1] scan_s[48] sidx_s[cap] idx_s[cap] lg_s[waves*E]
struct PostLds {
    lds_i32 *hist_s, *tab_s, *cnt_s, *off_s, *scan_s, *sidx_s, *idx_s;
    lds_f32 *lg_s;
};

__device__ inline PostLds carve_lds(int *dyn_, int E, int C, int A)
{
    const int cap = A < kLdsCopy ? A : kLdsCopy;
    lds_i32 *dyn = (lds_i32 *)dyn_;
    PostLds p;
    p.hist_s = dyn;
    p.tab_s = p.hist_s + E;
    p.cnt_s = p.tab_s + E;
    p.off_s = p.cnt_s + 4 * C;   // (counters of the general builder, or up to four mask words per slot)
    p.scan_s = p.off_s + C + 1;
    p.sidx_s = p.scan_s + 48;
    p.idx_s = p.sidx_s + cap;
    p.lg_s = (lds_f32 *)(dyn + ((2 * E + 5 * C + 49 + 2 * cap + 3) & ~3));
    return p;
}

inline size_t post_lds_bytes(int E, int C, int A, bool with_topk)
{
    const int cap = A < kLdsCopy ? A : kLdsCopy;
    size_t n = (size_t)2 * E + 4 * C + (C + 1) + 48 + 2 * cap;
    if (with_topk) n += (size_t)kRouteWaves * lg_stride(E) + 4;
    return n * sizeof(int);
}

constexpr int kSpinLimit = 1 << 20;   // polls of an entry in memory before a waiting workgroup gives up

// Small batches (T <= 128, one thread per assignment and per slot): the tokens of each slot as a
// bit mask of NW = ceil(T/32) words (a token names a slot at most once, the slot table being
// one-to-one), so counts, offsets and list positions are population counts.  Same outputs as
// block_post.
// PUBLISH: every word of the per-slot lists also goes, stamped with the call's number, into each of the
// kListReplicas copies behind r.lists_pub (entries no expert fills are stamped too, with -1, so that a
// reader can wait for all of them).
// What block_post_small found, in registers: thread tid < C holds slot tid's count, offset and place among the
// active slots (-1: no token); thread tid < T*k holds its assignment's slot and list position (-1: not
// resident); every thread holds the totals.
struct SmallLists {
    int count, offset, active_rank, n_active, n_listed, slot, pos;
};

// to_memory false: nothing is written to global memory (a workgroup that only wants the lists for itself).
template <bool PUBLISH>
__device__ __forceinline__ SmallLists block_post_small(lds_i32 *idx_s, lds_i32 *tab_s, int T, int kk, int E, int C, const RouteArgs &r,
                                 lds_i32 *hist_s, lds_i32 *mask_s, lds_i32 *scan_s, lds_i32 *off_s, unsigned tag,
                                 bool to_memory = true)
{
    auto publish = [&](int word, int value) {
        if (!PUBLISH) return;
        const unsigned long long e = ((unsigned long long)tag << 32) | (unsigned)value;
        const size_t stride = list_pub_entries(T, kk, C);
        for (int rep = 0; rep < kListReplicas; ++rep)
            __hip_atomic_store(r.lists_pub + rep * stride + word, e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const int A = T * kk, NW = (T + 31) >> 5;
    const bool valid = tid < A;
    const int tok = valid ? tid / kk : 0;
    int c = -1;
    if (valid) {
        const int e = idx_s[tid];
        __hip_atomic_fetch_add(&hist_s[e], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        c = tab_s[e];
        if ((unsigned)c >= (unsigned)C) c = -1;
        if (c >= 0)
            __hip_atomic_fetch_or(&mask_s[c * NW + (tok >> 5)], 1 << (tok & 31), __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_WORKGROUP);
        if (to_memory) r.slot_idx[tid] = c;
    }
    const bool miss = valid && c < 0;
    const unsigned long long bal = __ballot(miss);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) scan_s[w] = __popcll(bal);
    __syncthreads();
    // slot `tid`: its token count; prefix sums of (count, count > 0) inside the wavefront, from ballots:
    // of the flag, and of each bit of the count (a count is at most T <= 128)
    int cntv = 0;
    if (tid < C)
        for (int wd = 0; wd < NW; ++wd) cntv += __popc((unsigned)mask_s[tid * NW + wd]);
    const unsigned long long upto = (2ull << lane) - 1ull;   // lanes 0..lane
    const int inc_a = __popcll(__ballot(cntv > 0) & upto);
    int inc_o = 0;
    for (int bit = 0; (1 << bit) <= T; ++bit) inc_o += __popcll(__ballot((cntv >> bit) & 1) & upto) << bit;
    if (lane == kWave - 1) {
        scan_s[16 + w] = inc_o;
        scan_s[32 + w] = inc_a;
    }
    // (only the wavefronts that hold an assignment or a slot have anything to add)
    const int nwv = ((A > C ? A : C) + kWave - 1) / kWave;
    {
        int wave_base = 0, total = 0;
        for (int i = 0; i < nwv; ++i) {
            const int v = scan_s[i];
            if (i < w) wave_base += v;
            total += v;
        }
        if (to_memory) {
            if (miss) r.miss_list[wave_base + before] = tid;
            if (tid == 0) *r.miss_count = total;
            if (tid < E) r.hist[tid] = hist_s[tid];
        }
    }
    __syncthreads();
    int base_o = 0, base_a = 0, tot_o = 0, tot_a = 0;
    for (int i = 0; i < nwv; ++i) {
        const int vo = scan_s[16 + i], va = scan_s[32 + i];
        if (i < w) {
            base_o += vo;
            base_a += va;
        }
        tot_o += vo;
        tot_a += va;
    }
    SmallLists out = {0, 0, -1, tot_a, tot_o, c, -1};
    if (tid < C) {
        const int off = base_o + inc_o - cntv, na = base_a + inc_a - (cntv > 0 ? 1 : 0);
        off_s[tid] = off;
        out.count = cntv;
        out.offset = off;
        out.active_rank = cntv > 0 ? na : -1;
        if (to_memory) {
            r.slot_count[tid] = cntv;
            r.slot_offset[tid] = off;
            if (cntv > 0) r.active_slots[na] = tid;
        }
        publish(1 + tid, cntv);
        publish(1 + C + tid, off);
        if (cntv > 0) publish(1 + 2 * C + na, tid);
        if (tid >= tot_a) publish(1 + 2 * C + tid, -1);
    }
    if (tid == 0) {
        if (to_memory) {
            r.slot_offset[C] = tot_o;
            *r.n_active = (unsigned)tot_a;
        }
        publish(0, tot_a);
    }
    __syncthreads();
    // position of an assignment = offset of its slot + number of earlier tokens of that slot
    if (valid) {
        int p = -1;
        if (c >= 0) {
            p = off_s[c] + __popc((unsigned)mask_s[c * NW + (tok >> 5)] & ((1u << (tok & 31)) - 1u));
            for (int wd = 0; wd < (tok >> 5); ++wd) p += __popc((unsigned)mask_s[c * NW + wd]);
            if (to_memory) r.perm[p] = tid;
            publish(1 + 3 * C + p, tid);
        }
        if (to_memory) r.pos[tid] = p;
        out.pos = p;
        if (tid >= tot_o) publish(1 + 3 * C + tid, -1);
    }
    return out;
}

}  // namespace

}  // namespace moe
