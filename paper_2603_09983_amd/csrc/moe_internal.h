// Internal declarations shared by the translation units of libmoe_spac.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <mutex>

namespace moe {

constexpr int kWave = 64;
constexpr int kMaxE = 512;        // logits of one token live in one wavefront: E <= 64 * kMaxEPL
constexpr int kMaxEPL = kMaxE / kWave;
constexpr int kMaxK = 64;
constexpr int kMaxC = 1024;
constexpr int kSliceF = 128;      // FFN rows (gate/up outputs) owned by one workgroup
constexpr int kFfnThreads = 512;  // 8 wavefronts, 16 FFN rows each
constexpr int kLdsBytes = 160 * 1024;
constexpr int kCtrlBytes = 256;
// contraction lengths up to this many columns are parked in LDS whole (one panel per item)
constexpr int kPanelMax = 2048;

int stream_panel_width(int K);     // columns of a contraction parked in LDS at a time; 0 when K has no panel split

// LDS of one workgroup of a streaming kernel: the tile (16 rows of a panel of KP columns, padded), the
// partial results, the per-slot lists and the token list, the output buffer with its records.
constexpr int kStreamRowPad = 16;   // bytes of padding per LDS tile row
constexpr int kStreamOutCap = 16;   // items whose results wait in LDS between two batches of stores
static inline size_t stream_lds_need(int KP, int T, int k, int C, bool gateup)
{
    const size_t groups = T > 16 ? 2 : 1;
    return (size_t)16 * (2 * (size_t)KP + kStreamRowPad) + groups * 16 * kWave * 16 +
           ((size_t)3 * C + (size_t)T * k) * 4 + (size_t)kStreamOutCap * (groups * (gateup ? 128 : 256) + 8) * 4;
}

// The streaming kernels (stream.hip) take every batch of up to 32 tokens, and larger batches when
// every item is a single panel, as long as the lists fit their LDS; the rest (wide matrices with large
// batches, ragged row lengths, very long lists) falls back to ffn.hip.
static inline bool use_stream_kernels(int T, int k, int C, int H, int F, int n_shared, int F_shared)
{
    // (their 1 KB pieces must not straddle the middle of a 16-row tile: row bytes a multiple of 128)
    if (H % 64 != 0 || F % 64 != 0 || (n_shared > 0 && F_shared % 64 != 0)) return false;
    if (T > 32 && !(H <= kPanelMax && F <= kPanelMax && (n_shared == 0 || F_shared <= kPanelMax))) return false;
    const int kp_h = stream_panel_width(H), kp_f = stream_panel_width(F);
    const int kp_s = n_shared > 0 ? stream_panel_width(F_shared) : 0;
    if (kp_h == 0 || kp_f == 0 || (n_shared > 0 && kp_s == 0)) return false;
    return stream_lds_need(kp_h, T, k, C, true) <= (size_t)kLdsBytes &&
           stream_lds_need(kp_f > kp_s ? kp_f : kp_s, T, k, C, false) <= (size_t)kLdsBytes;
}

static inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// Small batches: the routing steps run inside a larger launch (dot products by all workgroups).  In the
// one-launch kernel workgroup 0 ranks and hands the lists to the others as stamped 64-bit words, kListReplicas
// copies so that not all workgroups poll the same lines; one copy: n_active | slot_count[C] | slot_offset[C] |
// active_slots[C] | perm[T*k].  In the gate/up kernel of the two-launch form every workgroup ranks the stamped
// logits for itself (kLogitReplicas copies of those) and only the per-workgroup words behind the copies are used.
constexpr int kListReplicas = 16;
constexpr int kLogitReplicas = 16;  // copies of the stamped logits when every workgroup ranks them itself (<= lanes that store)
constexpr int kMaxGroups = 1024;   // workgroups of that launch (one stamped word each, behind the copies)
__host__ __device__ static inline size_t list_pub_entries(int T, int k, int C) { return (size_t)1 + 3 * (size_t)C + (size_t)T * k; }
size_t route_lds_bytes(int E, int C, int A);   // LDS of the routing steps of one batch (route.hip)
static inline bool use_fused_route(int T, int k, int E, int C, int H, int F, int n_shared, int F_shared)
{
    if (T > 32 || E < 1 || E > 2 * kWave || (size_t)T * k > 1024 || C < 1 || C > kMaxC) return false;
    if (!use_stream_kernels(T, k, C, H, F, n_shared, F_shared)) return false;
    return route_lds_bytes(E, C, T * k) <= (size_t)kLdsBytes - 1024;
}

// Inside the routing kernel the logits travel from the workgroups that compute them to the one
// that ranks them as 64-bit (tag, value) entries, tag = number of the call on this workspace: an
// entry that carries the call's tag holds the call's value, so no counter and no fence is needed.
// The region has a fixed size and sits right behind the control block; moe_workspace_init clears
// it (no stale entry may carry a future tag).
constexpr int kTagEntries = 65536;   // 512 KB: T*E of the largest routing call that uses them
static_assert(32 * (2 * kWave) * kLogitReplicas <= kTagEntries, "the copies of the logits of the largest batch that ranks them in every workgroup");
// Behind them, the same kind of entries for the Top-k ids when more than one workgroup ranks
// (batches above 16 tokens): T*k of them.
constexpr int kTagIdxEntries = 4096;   // (at most as many as the routing kernel mirrors in LDS)

// Byte offsets of the scratch arrays inside the caller's workspace.
struct WsLayout {
    size_t ctrl, tagged, tagged_idx, perm, pos, slot_count, slot_offset, active, part, part_sh, act, act_sh, o, o_sh, total;
    size_t lists_pub;   // stamped copies of the per-slot lists (gate/up kernel that does the routing itself), or 0
};

// control block words
constexpr int kCtrlNActive = 1;   // number of resident slots that received at least one token
constexpr int kCtrlError = 2;     // non-zero once a bounded wait inside a kernel has run out
constexpr int kCtrlEpoch = 3;     // routing calls completed on this workspace (the tag of the last one)
// Two words that only a test sets (moe_workspace_init clears them): with them the host forces every bounded
// wait inside a kernel to run out, so that the failure path can be exercised while every kernel still exits.
constexpr int kCtrlSpin = 4;      // polls before a wait gives up (0 = the built-in bound)
constexpr int kCtrlSkew = 5;      // added to the call number that producers stamp their entries with (0)
constexpr int kCtrlLayout = 6;    // hash of the layout the workspace has been used with since it was initialised (0: none yet)
constexpr unsigned kErrWait = 1u, kErrLayout = 2u;   // bits of the error word

// The first kernel of a call: the workspace serves one layout between two initialisations (a region that held
// other data may hold words that look like entries of the current call).
__device__ static inline void check_layout(unsigned *ctrl, unsigned layout)
{
    if (layout == 0u) return;
    const unsigned old = ctrl[kCtrlLayout];
    if (old == 0u) ctrl[kCtrlLayout] = layout;
    else if (old != layout) atomicOr(ctrl + kCtrlError, kErrLayout);
}
constexpr int kMaxDevices = 64;   // devices the per-device launch state is kept for
constexpr int kKindLayer = 9;     // measurement aid: the one-launch layer kernel (MOE_KERNEL_LAYER)

static inline int n_slices(int F) { return (F + kSliceF - 1) / kSliceF; }

static inline WsLayout ws_layout(int T, int E, int k, int C, int H, int F, int n_shared, int F_shared)
{
    WsLayout w;
    size_t A = (size_t)T * k;
    size_t o = 0;
    w.lists_pub = 0;
    w.ctrl = o;        o += kCtrlBytes;
    w.tagged = o;      o += (size_t)kTagEntries * 8;   // (same place whatever the entry point and shape)
    w.tagged_idx = o;  o += (size_t)kTagIdxEntries * 8;
    w.perm = o;        o += align256(A * 4);
    w.pos = o;         o += align256(A * 4);
    w.slot_count = o;  o += align256((size_t)(C > 0 ? C : 1) * 4);
    w.slot_offset = o; o += align256((size_t)(C + 1) * 4);
    w.active = o;      o += align256((size_t)(C > 0 ? C : 1) * 4);
    if (!use_stream_kernels(T, k, C, H, F, n_shared, F_shared)) {
        // large batches: per-slice partial sums of the fused FFN kernel
        w.part = o;    o += align256((size_t)n_slices(F) * A * H * 4);
        w.part_sh = o; o += align256((size_t)n_shared * n_slices(F_shared) * T * H * 4);
        w.act = w.act_sh = w.o = w.o_sh = o;
    } else {
        // activations and per-assignment outputs of the streaming kernels
        w.part = w.part_sh = o;
        // (4 bytes per element: the one-launch kernel stores (call number, two bf16 values) entries)
        w.act = o;     o += align256(A * F * 4);
        w.act_sh = o;  o += align256((size_t)n_shared * T * F_shared * 4);
        // (8 bytes per element: small batches store (call number, value) entries, see JoinArgs)
        w.o = o;       o += align256(A * H * 8);
        w.o_sh = o;    o += align256((size_t)n_shared * T * H * 8);
        if (use_fused_route(T, k, E, C, H, F, n_shared, F_shared)) {
            w.lists_pub = o;
            // (..., one stamped word per workgroup of the launch, and the gate weights, stamped, kListReplicas copies)
            o += align256((list_pub_entries(T, k, C) * kListReplicas + kMaxGroups + A * kListReplicas) * 8);
        }
    }
    w.total = o;
    return w;
}

// Non-zero hash of where the regions of a layout lie: two shapes with the same offsets keep the same kind of
// entry in every place, and may share a workspace without a new initialisation.
static inline unsigned layout_hash(const WsLayout &w)
{
    const size_t f[] = {w.perm, w.pos, w.slot_count, w.slot_offset, w.active, w.part, w.part_sh, w.act, w.act_sh,
                        w.o, w.o_sh, w.lists_pub, w.total};
    unsigned long long h = 1469598103934665603ull;   // FNV-1a over the offsets
    for (size_t v : f)
        for (int i = 0; i < 8; ++i) {
            h ^= (v >> (8 * i)) & 0xffu;
            h *= 1099511628211ull;
        }
    const unsigned r = (unsigned)(h ^ (h >> 32));
    return r ? r : 1u;
}

// What the routing kernel should do after the logits are complete.
struct RouteArgs {
    const void *hidden;        // [T,H] bf16
    const float *router_w;     // [E,H]
    const float *router_bias;  // [E] or null
    int T, H, E, k;
    unsigned layout;           // hash of the workspace layout of this call (0: not checked)
    int32_t *topk_idx;         // [T,k]
    float *topk_w;             // [T,k]
    float *logits_opt;         // [T,E] or null
    int32_t *hist;             // [E] or null (skip)
    // slot resolve (skipped when slot_table is null)
    const int32_t *slot_table; // [E]
    int C;
    int32_t *slot_idx;         // [T,k]
    int32_t *miss_list;        // [T*k]
    int32_t *miss_count;       // [1]
    int32_t *slot_count;       // [C]
    int32_t *slot_offset;      // [C+1]
    int32_t *perm;             // [T*k]
    int32_t *pos;              // [T*k]
    int32_t *active_slots;     // [C] slots with at least one token, ascending
    unsigned *n_active;        // [1]
    unsigned *error_flag;      // control word set when a bounded wait inside a kernel ran out
    unsigned long long *tagged_logits;   // [T*E] (tag << 32 | value bits)
    unsigned long long *tagged_idx;      // [T*k] (tag << 32 | expert id), batches above 16 tokens
    unsigned *epoch;           // control word: tag of the last completed call
    unsigned long long *lists_pub;   // kListReplicas x list_pub_entries stamped words, or null (nothing published)
};

// Arguments of the streaming kernels (gate/up: R = F rows, K = H; down: R = H rows, K = F).
struct StreamArgs {
    const uint16_t *w0, *w1;   // routed pools: gate, up | down, unused
    const uint16_t *s0, *s1;   // shared experts: same roles
    const uint16_t *bsrc;      // gate/up: hidden [T,H]; down: act [A,F]
    const uint16_t *bsrc_sh;   // down: act_sh [n_shared,T,F_shared]
    void *out, *out_sh;        // gate/up: act, act_sh (bf16); down: o [A,H], o_sh [n_shared,T,H] (fp32)
    const int32_t *slot_count, *slot_offset, *perm, *active_slots;
    const unsigned *n_active;
    int T, k;
    int R, K, R_sh, K_sh, n_shared, C;
    int KP, KP_sh;             // panel widths (columns parked in LDS at a time)
    // Filled in by the launch functions: panels per routed / shared item, and floor(2^32 / d) for the divisors of
    // the kernel's index arithmetic (grid size, items per routed / shared expert, k, k + n_shared).  A division by a
    // value only known at run time is ~30 instructions, and in the prologue of a launch sixteen wavefronts execute
    // them one after the other on the compute unit's one scalar unit.
    int np, np_sh;
    unsigned rcp_G, rcp_tiles, rcp_tiles_sh, rcp_k, rcp_S;
};

// n / d with rcp = floor(2^32 / d) (d = 1: 2^32 - 1): the estimate is never too large and at most one short.
__host__ __device__ static inline unsigned rcp32(unsigned d) { return d <= 1u ? 0xffffffffu : (unsigned)((1ull << 32) / d); }
__device__ static inline int udiv_rcp(int n, int d, unsigned rcp)
{
    unsigned q = __umulhi((unsigned)n, rcp);
    if ((unsigned)n - q * (unsigned)d >= (unsigned)d) ++q;
    return (int)q;
}

// The weighted sum back into token order at the end of the down kernel (small batches).
struct JoinArgs {
    const float *topk_w;       // [T,k]
    const int32_t *pos;        // [T*k] row of the per-assignment outputs, or -1
    void *out;                 // [T,H] fp32 or bf16
    const unsigned *epoch;     // control word: number of this call (stamps the 64-bit entries)
    unsigned *error_flag;      // control word set when a bounded wait ran out
    int32_t *miss_count;       // [1] or null: set to -1 when a bounded wait ran out
    int out_bf16, accumulate;
};

// Arguments of the one-launch kernel of small batches (layer.hip): gate/up and down as one weight stream,
// the final sum at its end, optionally the routing steps at its head.
struct LayerArgs {
    const uint16_t *w_gate, *w_up, *w_down;      // slot-major pools
    const uint16_t *sh_gate, *sh_up, *sh_down;   // shared experts or null
    const uint16_t *hidden;                      // [T,H] bf16
    unsigned long long *act, *act_sh;            // [A][F/2], [n_shared][T][F_sh/2]: call number << 32 | two bf16
    unsigned long long *o, *o_sh;                // [A][H], [n_shared][T][H]: call number << 32 | fp32
    const int32_t *slot_count, *slot_offset, *perm, *pos, *active_slots;   // lists left by a routing / list kernel
    const unsigned *n_active;                    // (unused when the kernel does the routing itself)
    const float *topk_w;                         // [T,k]
    void *out;                                   // [T,H] fp32 or bf16
    int32_t *miss_count;                         // [1] or null: set to -1 when a bounded wait ran out
    unsigned *ctrl;                              // control block of the workspace
    int T, k, H, F, F_sh, n_shared, C;
    int KP_h, KP_f, KP_fs, RD, RDS, tile_lds_bytes, tab_cap;   // (filled in by launch_layer)
    int out_bf16, accumulate;
};

struct FfnArgs {
    const void *hidden;        // [T,H] bf16
    const void *w_gate, *w_up, *w_down;        // slot-major pools
    const void *sh_gate, *sh_up, *sh_down;     // shared experts or null
    const int32_t *slot_count, *slot_offset, *perm;
    float *part;               // [n_slices(F)][A][H]
    float *part_sh;            // [n_shared][n_slices(F_shared)][T][H]
    int T, H, F, k, C, n_shared, F_shared;
};

struct CombineArgs {
    const float *topk_w;       // [T,k]
    const int32_t *pos;        // [T*k] row of `part` or -1
    const float *part, *part_sh;
    void *out;
    const unsigned *error_flag;   // control word set when a bounded wait ran out (then `out` is filled with NaN), or null
    int32_t *miss_count;          // [1] or null: set to -1 in that case
    int T, H, F, k, n_shared, F_shared, out_bf16, accumulate;
};

hipError_t launch_route(const RouteArgs &a, hipStream_t s);
hipError_t launch_histogram(const int32_t *topk_idx, int A, int E, int32_t *hist, hipStream_t s);
hipError_t launch_resolve(const int32_t *topk_idx, const int32_t *slot_table, int A, int E, int C,
                          int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, int32_t *slot_count,
                          int32_t *slot_offset, int32_t *perm, int32_t *pos, int32_t *active_slots,
                          unsigned *n_active, hipStream_t s);
// (epoch: control word stepped by one, so that the FFN kernels of this call have a number of their own)
// (layout: hash of the workspace layout of this call, checked against the one the workspace has served so far)
hipError_t launch_lists_from_slots(unsigned layout, const int32_t *slot_idx, int A, int C, int32_t *slot_count,
                                   int32_t *slot_offset, int32_t *perm, int32_t *pos, int32_t *active_slots,
                                   unsigned *n_active, unsigned *epoch, hipStream_t s);
// join != null (down kernel only, stream_can_join() true): outputs leave as stamped 64-bit entries
// and the kernel ends with the weighted sum into `out`; no combine launch is needed then
hipError_t launch_stream(const StreamArgs &a, bool gateup, const JoinArgs *join, hipStream_t s);
// gate/up kernel that first does the routing steps described by `r` (use_fused_route() true, r.lists_pub set)
hipError_t launch_stream_routed(const StreamArgs &a, const RouteArgs &r, hipStream_t s);
bool stream_can_join(const StreamArgs &d);
hipError_t launch_combine_rows(const CombineArgs &a, const float *o, const float *o_sh, hipStream_t s);
// one-launch form (batches of up to 16 tokens): use_layer_kernel() must hold; route != null: the kernel does
// the routing steps itself (use_fused_route() true, route->lists_pub set)
bool use_layer_kernel(int T, int k, int E, int C, int H, int F, int n_shared, int F_shared);
hipError_t launch_layer(const LayerArgs &a, const RouteArgs *route, hipStream_t s);
hipError_t read_layer_timeline(void *dst, size_t bytes);   // [kTimelineGroups][kLayerTimelineWords], tracing builds only
// Timeline stamps of the last gate/up and down launches: [2][kTimelineGroups][kTimelineWords] 64-bit words
// (start, lists in LDS, first tile done, loop done, results stored, end: 100 MHz ticks; items, tiles).
// hipErrorNotSupported unless the library was built with -DMOE_STREAM_TRACE.
constexpr int kTimelineGroups = 1024, kTimelineWords = 8;
constexpr int kLayerTimelineWords = 24;   // the one-launch kernel's record per workgroup
hipError_t read_stream_timeline(void *dst, size_t bytes);
hipError_t launch_ffn(const FfnArgs &a, hipStream_t s);
hipError_t launch_combine(const CombineArgs &a, hipStream_t s);
// zero-fills the workspace (control block, stamped-entry regions and everything else)
hipError_t launch_clear_ctrl(void *workspace, size_t bytes, hipStream_t s);
// a launch that the measurement aid times by the dispatch's own start and end stamps when enabled
hipError_t launch_timed(const void *fn, dim3 grid, dim3 block, void **params, size_t lds, hipStream_t s, int kind);
// event bracketing for the measurement aid (no-ops unless enabled)
// Per-device state of the library (each guarded by one mutex; any host thread may call):
// compute units of the current device = workgroups of the chip-wide launches (capped at kMaxGroups; 0 and
// *err when the runtime would not say), ...
int device_cus(hipError_t *err);
// ... and the kernels that have been allowed `bytes` of dynamic LDS on the current device (set once each).
hipError_t allow_full_lds(const void *fn, int bytes = kLdsBytes);
void prof_begin(int kind, hipStream_t s);
void prof_end(int kind, hipStream_t s);
size_t ffn_lds_bytes(int H, int nt);
int ffn_token_tiles(int T, int H);   // 0 when H does not fit the LDS

}  // namespace moe
