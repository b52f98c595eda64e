// C-ABI of libmoe_spac.so: argument checks and launch sequencing only.
#include "../../include/moe_spac.h"
#include "moe_internal.h"
#include <mutex>
#include <unordered_map>
#include <vector>

using namespace moe;

namespace {

thread_local char g_launch_msg[160] = "HIP launch error";

int launch_failed(hipError_t e)
{
    snprintf(g_launch_msg, sizeof g_launch_msg, "HIP launch error: %s", hipGetErrorString(e));
    return MOE_ERR_LAUNCH;
}

// ---- measurement aid: event pairs around each launch ----
constexpr int kProfMax = 8192;
struct ProfState {
    bool on = false;
    hipEvent_t ev[MOE_KERNEL_KINDS][kProfMax][2];
    int created[MOE_KERNEL_KINDS] = {};   // pairs made so far, per kind
    int used[MOE_KERNEL_KINDS] = {};
} g_prof;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_route_shape(int T, int H, int E, int k)
{
    if (T < 1 || H < 1 || E < 1 || k < 1 || k > E || E > kMaxE || k > kMaxK) return MOE_ERR_SHAPE;
    if ((size_t)T * k > (size_t)1 << 30 || (size_t)T * E > (size_t)kTagEntries) return MOE_ERR_SHAPE;
    if (H % 8 != 0) return MOE_ERR_ALIGN;
    return MOE_OK;
}

int check_ffn_shape(int T, int H, int F, int k, int C, int n_shared, int F_shared)
{
    if (T < 1 || H < 1 || F < 1 || k < 1 || C < 0 || C > kMaxC || T > 65535) return MOE_ERR_SHAPE;
    if (H % 8 != 0 || F % 8 != 0 || (n_shared > 0 && F_shared % 8 != 0)) return MOE_ERR_ALIGN;   // 16-byte rows
    // the kernel that takes what the streaming kernels do not keeps a token tile's hidden rows in LDS
    if (!use_stream_kernels(T, k, C, H, F, n_shared, F_shared) && ffn_token_tiles(T, H) == 0) return MOE_ERR_SHAPE;
    return MOE_OK;
}

}  // namespace

namespace {
struct DeviceState {
    int n_cus = 0;
    std::unordered_map<const void *, int> lds_allowed;   // kernel -> dynamic LDS bytes it has been allowed
};
DeviceState g_device[kMaxDevices];
std::mutex g_device_mutex;

hipError_t current_device(int *dev)
{
    hipError_t e = hipGetDevice(dev);
    if (e == hipSuccess && (*dev < 0 || *dev >= kMaxDevices)) e = hipErrorInvalidDevice;
    return e;
}
}  // namespace

int moe::device_cus(hipError_t *err)
{
    int dev = 0, n = 0;
    hipError_t e = current_device(&dev);
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(g_device_mutex);
        DeviceState &d = g_device[dev];
        if (d.n_cus == 0) {
            int nc = 0;
            e = hipDeviceGetAttribute(&nc, hipDeviceAttributeMultiprocessorCount, dev);
            if (e == hipSuccess) d.n_cus = nc > 0 ? (nc < kMaxGroups ? nc : kMaxGroups) : 256;
        }
        n = d.n_cus;
    }
    if (err) *err = e;
    return n;
}

hipError_t moe::allow_full_lds(const void *fn, int bytes)
{
    int dev = 0;
    hipError_t e = current_device(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(g_device_mutex);
    DeviceState &d = g_device[dev];
    auto it = d.lds_allowed.find(fn);
    if (it != d.lds_allowed.end() && it->second >= bytes) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) d.lds_allowed[fn] = bytes;
    return e;
}

// One kernel launch, bracketed by a pair of events on its stream while the measurement aid is on.
hipError_t moe::launch_timed(const void *fn, dim3 grid, dim3 block, void **params, size_t lds, hipStream_t s,
                             int kind)
{
    prof_begin(kind, s);
    hipError_t e = hipLaunchKernel(fn, grid, block, params, lds, s);
    prof_end(kind, s);
    return e;
}

void moe::prof_begin(int kind, hipStream_t s)
{
    if (!g_prof.on || g_prof.used[kind] >= kProfMax) return;
    // (event pairs are made when first needed: a process that never measures makes none)
    int &made = g_prof.created[kind];
    if (g_prof.used[kind] >= made) {
        hipEvent_t *pair = g_prof.ev[kind][made];
        if (hipEventCreate(&pair[0]) != hipSuccess) return;
        if (hipEventCreate(&pair[1]) != hipSuccess) {
            (void)hipEventDestroy(pair[0]);
            return;
        }
        ++made;
    }
    (void)hipEventRecord(g_prof.ev[kind][g_prof.used[kind]][0], s);
}

void moe::prof_end(int kind, hipStream_t s)
{
    if (g_prof.on && g_prof.used[kind] < g_prof.created[kind]) {
        (void)hipEventRecord(g_prof.ev[kind][g_prof.used[kind]][1], s);
        ++g_prof.used[kind];
    }
}

extern "C" int moe_profile_enable(int on)
{
    if (on)
        for (int k = 0; k < MOE_KERNEL_KINDS; ++k) g_prof.used[k] = 0;
    g_prof.on = on != 0;
    return MOE_OK;
}

extern "C" int moe_profile_read(int kind, double *total_ms, int *launches)
{
    if (!total_ms || !launches) return MOE_ERR_NULL;
    if (kind < 0 || kind >= MOE_KERNEL_KINDS) return MOE_ERR_SHAPE;
    double sum = 0.0;
    for (int i = 0; i < g_prof.used[kind]; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.ev[kind][i][0], g_prof.ev[kind][i][1]) != hipSuccess)
            return MOE_ERR_LAUNCH;
        sum += ms;
    }
    *total_ms = sum;
    *launches = g_prof.used[kind];
    return MOE_OK;
}

extern "C" int moe_profile_event_overhead(void *stream, int pairs, double *avg_ms)
{
    if (!avg_ms) return MOE_ERR_NULL;
    if (pairs < 1 || pairs > kProfMax) return MOE_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    // event pairs of its own, nothing between the two records of a pair
    std::vector<hipEvent_t> ev((size_t)2 * pairs, nullptr);
    int rc = MOE_OK;
    for (auto &e : ev)
        if (rc == MOE_OK && hipEventCreate(&e) != hipSuccess) rc = MOE_ERR_LAUNCH;
    for (int i = 0; i < 2 * pairs && rc == MOE_OK; ++i)
        if (hipEventRecord(ev[i], s) != hipSuccess) rc = MOE_ERR_LAUNCH;
    if (rc == MOE_OK && hipStreamSynchronize(s) != hipSuccess) rc = MOE_ERR_LAUNCH;
    double sum = 0.0;
    for (int i = 0; i < pairs && rc == MOE_OK; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1]) != hipSuccess) rc = MOE_ERR_LAUNCH;
        sum += ms;
    }
    for (auto &e : ev)
        if (e) (void)hipEventDestroy(e);
    if (rc == MOE_OK) *avg_ms = sum / pairs;
    return rc;
}

extern "C" int moe_profile_stream_timeline(unsigned long long *words, size_t n_words)
{
    if (!words) return MOE_ERR_NULL;
    const size_t plane = (size_t)kTimelineGroups * kTimelineWords, lplane = (size_t)kTimelineGroups * kLayerTimelineWords;
    if (n_words != 2 * plane + lplane) return MOE_ERR_SHAPE;
    hipError_t e = read_stream_timeline(words, 2 * plane * sizeof(unsigned long long));
    if (e == hipErrorNotSupported) return MOE_ERR_SHAPE;   // not a tracing build
    if (e == hipSuccess) e = read_layer_timeline(words + 2 * plane, lplane * sizeof(unsigned long long));
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

extern "C" const char *moe_profile_kernel_name(int kind)
{
    switch (kind) {
    case MOE_KERNEL_ROUTE: return "route_kernel";
    case MOE_KERNEL_LISTS: return "resolve_kernel";
    case MOE_KERNEL_FFN: return "ffn_gate_up";
    case MOE_KERNEL_COMBINE: return "combine_kernel";
    case MOE_KERNEL_DOWN: return "ffn_down";
    case MOE_KERNEL_ESTIMATOR: return "utility_update_kernel";
    case MOE_KERNEL_BALANCER: return "balance_kernel";
    case MOE_KERNEL_CACHE_PLAN: return "plan_kernel";
    case MOE_KERNEL_POOL_LOAD: return "load_kernel";
    case MOE_KERNEL_LAYER: return "layer_kernel";
    default: return "?";
    }
}

extern "C" const char *moe_status_string(int status)
{
    switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_SHAPE: return "a size is outside the supported range";
    case MOE_ERR_ALIGN: return "H or F is not a multiple of 8, or a pointer is not 16-byte aligned";
    case MOE_ERR_WORKSPACE: return "workspace is smaller than moe_workspace_bytes() asks for, or has served another shape since moe_workspace_init";
    case MOE_ERR_LAUNCH: return g_launch_msg;
    case MOE_ERR_SCRATCH: return "the shape needs more scratch memory than the library's static array holds";
    default: return "unknown status";
    }
}

extern "C" int moe_workspace_bytes(const moe_shape_t *sh, size_t *bytes_out)
{
    if (!sh || !bytes_out) return MOE_ERR_NULL;
    if (sh->T < 1 || sh->H < 1 || sh->E < 1 || sh->k < 1 || sh->k > sh->E || sh->F < 1 || sh->C < 0 ||
        sh->n_shared < 0 || (sh->n_shared > 0 && sh->F_shared < 1))
        return MOE_ERR_SHAPE;
    *bytes_out = ws_layout(sh->T, sh->E, sh->k, sh->C, sh->H, sh->F, sh->n_shared, sh->F_shared).total;
    return MOE_OK;
}

extern "C" int moe_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return MOE_ERR_NULL;
    if (workspace_bytes < (size_t)kCtrlBytes) return MOE_ERR_WORKSPACE;
    if (!aligned16(workspace)) return MOE_ERR_ALIGN;
    hipError_t e = launch_clear_ctrl(workspace, workspace_bytes, (hipStream_t)stream);
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

extern "C" int moe_workspace_status(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return MOE_ERR_NULL;
    if (workspace_bytes < (size_t)kCtrlBytes) return MOE_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    unsigned ctrl[kCtrlBytes / 4];
    hipError_t e = hipMemcpyAsync(ctrl, workspace, sizeof ctrl, hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return launch_failed(e);
    if (ctrl[kCtrlError] == 0u) return MOE_OK;
    // a wait ran out part-way through a call: clear the flag, and step the call counter by two, so that no
    // entry which a workgroup of the failed call stamped late (with that call's number, or the next one when the
    // counter had not been stepped yet) can pass for an entry of a later call
    const unsigned cleared = 0u, epoch = ctrl[kCtrlEpoch] + 2u;
    e = hipMemcpyAsync((unsigned *)workspace + kCtrlError, &cleared, sizeof cleared, hipMemcpyHostToDevice, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync((unsigned *)workspace + kCtrlEpoch, &epoch, sizeof epoch, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    if (e != hipSuccess) return launch_failed(e);
    if (ctrl[kCtrlError] & kErrLayout)   // (the layout word stays: the next call with that other shape says so again)
        return MOE_ERR_WORKSPACE;
    snprintf(g_launch_msg, sizeof g_launch_msg, "a bounded wait inside a kernel ran out (results of that call are invalid)");
    return MOE_ERR_LAUNCH;
}

extern "C" int moe_workspace_wait_test(void *workspace, size_t workspace_bytes, unsigned poll_limit,
                                       unsigned stamp_skew, void *stream)
{
    if (!workspace) return MOE_ERR_NULL;
    if (workspace_bytes < (size_t)kCtrlBytes) return MOE_ERR_WORKSPACE;
    static_assert(kCtrlSkew == kCtrlSpin + 1, "the two words are written with one copy");
    hipStream_t s = (hipStream_t)stream;
    const unsigned words[2] = {poll_limit, stamp_skew};
    hipError_t e = hipMemcpyAsync((unsigned *)workspace + kCtrlSpin, words, sizeof words, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

extern "C" int moe_route_topk(const void *hidden, const float *router_w, const float *router_bias, int T,
                              int H, int E, int k, int32_t *topk_idx, float *topk_w, float *logits_opt,
                              void *workspace, size_t workspace_bytes, void *stream)
{
    if (!hidden || !router_w || !topk_idx || !topk_w || !workspace) return MOE_ERR_NULL;
    int rc = check_route_shape(T, H, E, k);
    if (rc) return rc;
    if (!aligned16(hidden) || !aligned16(router_w) || !aligned16(workspace)) return MOE_ERR_ALIGN;
    WsLayout w = ws_layout(T, E, k, 0, 0, 0, 0, 0);
    if (workspace_bytes < w.perm) return MOE_ERR_WORKSPACE;   // control block + tagged logits
    char *ws = (char *)workspace;
    RouteArgs a = {};
    a.hidden = hidden; a.router_w = router_w; a.router_bias = router_bias;
    a.T = T; a.H = H; a.E = E; a.k = k;
    a.tagged_logits = (unsigned long long *)(ws + w.tagged);
    a.tagged_idx = (unsigned long long *)(ws + w.tagged_idx);
    a.epoch = (unsigned *)(ws + w.ctrl) + kCtrlEpoch;
    a.error_flag = (unsigned *)(ws + w.ctrl) + kCtrlError;
    a.topk_idx = topk_idx; a.topk_w = topk_w; a.logits_opt = logits_opt;
    hipError_t e = launch_route(a, (hipStream_t)stream);
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

extern "C" int moe_expert_histogram(const int32_t *topk_idx, int T, int k, int E, int32_t *hist, void *stream)
{
    if (!topk_idx || !hist) return MOE_ERR_NULL;
    if (T < 1 || k < 1 || E < 1 || E > 8192 || (size_t)T * k > (size_t)1 << 30) return MOE_ERR_SHAPE;
    hipError_t e = launch_histogram(topk_idx, T * k, E, hist, (hipStream_t)stream);
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

extern "C" int moe_slot_resolve(const int32_t *topk_idx, const int32_t *slot_table, int T, int k, int E, int C,
                                int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    if (!topk_idx || !slot_table || !slot_idx || !miss_list || !miss_count || !workspace) return MOE_ERR_NULL;
    if (T < 1 || k < 1 || E < 1 || C < 0 || C > kMaxC || (size_t)T * k > (size_t)1 << 30) return MOE_ERR_SHAPE;
    if (!aligned16(workspace)) return MOE_ERR_ALIGN;
    WsLayout w = ws_layout(T, E, k, C, 0, 0, 0, 0);
    if (workspace_bytes < w.part) return MOE_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    hipError_t e = launch_resolve(topk_idx, slot_table, T * k, E, C, slot_idx, miss_list, miss_count,
                                  (int32_t *)(ws + w.slot_count), (int32_t *)(ws + w.slot_offset),
                                  (int32_t *)(ws + w.perm), (int32_t *)(ws + w.pos),
                                  (int32_t *)(ws + w.active), (unsigned *)(ws + w.ctrl) + kCtrlNActive,
                                  (hipStream_t)stream);
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

namespace {

// The expert FFN and the combine, given the per-slot lists in the workspace.
// Shapes the LDS-staged streaming kernels take (use_stream_kernels) run gate/up,
// then down with the combine inside it (small batches) or followed by it; the
// rest takes the fused per-slice kernel and its combine.
int run_ffn(const void *hidden, const float *topk_w, const void *w_gate, const void *w_up, const void *w_down,
            const void *sh_gate, const void *sh_up, const void *sh_down, int T, int H, int F, int k, int C,
            int n_shared, int F_shared, const WsLayout &w, char *ws, void *out, int out_bf16, int accumulate,
            hipStream_t s, const RouteArgs *routing = nullptr, bool one_launch = false, int32_t *miss_count = nullptr)
{
    // (the caller's routing / list kernel has given this call its number in the control block)
    int32_t *slot_count = (int32_t *)(ws + w.slot_count), *slot_offset = (int32_t *)(ws + w.slot_offset);
    int32_t *perm = (int32_t *)(ws + w.perm), *pos = (int32_t *)(ws + w.pos);
    CombineArgs c = {};
    c.topk_w = topk_w; c.pos = pos; c.out = out;
    c.T = T; c.H = H; c.F = F; c.k = k; c.n_shared = n_shared; c.F_shared = F_shared;
    c.out_bf16 = out_bf16; c.accumulate = accumulate;
    c.error_flag = (const unsigned *)(ws + w.ctrl) + kCtrlError;
    c.miss_count = miss_count;
    hipError_t e;
    if (one_launch) {
        // small batch: gate/up, down and the final sum as one weight stream (routing != null: the routing steps too)
        LayerArgs l = {};
        l.w_gate = (const uint16_t *)w_gate; l.w_up = (const uint16_t *)w_up; l.w_down = (const uint16_t *)w_down;
        l.sh_gate = (const uint16_t *)sh_gate; l.sh_up = (const uint16_t *)sh_up; l.sh_down = (const uint16_t *)sh_down;
        l.hidden = (const uint16_t *)hidden;
        l.act = (unsigned long long *)(ws + w.act); l.act_sh = (unsigned long long *)(ws + w.act_sh);
        l.o = (unsigned long long *)(ws + w.o); l.o_sh = (unsigned long long *)(ws + w.o_sh);
        l.slot_count = slot_count; l.slot_offset = slot_offset; l.perm = perm; l.pos = pos;
        l.active_slots = (const int32_t *)(ws + w.active);
        l.n_active = (const unsigned *)(ws + w.ctrl) + kCtrlNActive;
        l.topk_w = topk_w; l.out = out; l.miss_count = miss_count;
        l.ctrl = (unsigned *)(ws + w.ctrl);
        l.T = T; l.k = k; l.H = H; l.F = F; l.F_sh = F_shared; l.n_shared = n_shared; l.C = C;
        l.out_bf16 = out_bf16; l.accumulate = accumulate;
        e = launch_layer(l, routing, s);
        return e == hipSuccess ? MOE_OK : launch_failed(e);
    }
    if (use_stream_kernels(T, k, C, H, F, n_shared, F_shared)) {
        StreamArgs g = {};
        g.w0 = (const uint16_t *)w_gate; g.w1 = (const uint16_t *)w_up;
        g.s0 = (const uint16_t *)sh_gate; g.s1 = (const uint16_t *)sh_up;
        g.bsrc = (const uint16_t *)hidden; g.bsrc_sh = nullptr;
        g.out = ws + w.act; g.out_sh = ws + w.act_sh;
        g.slot_count = slot_count; g.slot_offset = slot_offset; g.perm = perm;
        g.active_slots = (const int32_t *)(ws + w.active);
        g.n_active = (const unsigned *)(ws + w.ctrl) + kCtrlNActive;
        g.T = T; g.k = k; g.C = C;
        g.R = F; g.K = H; g.R_sh = F_shared; g.K_sh = H; g.n_shared = n_shared;
        g.KP = g.KP_sh = stream_panel_width(H);
        // (routing != null: the gate/up launch does the routing steps itself)
        e = routing ? launch_stream_routed(g, *routing, s) : launch_stream(g, true, nullptr, s);
        if (e != hipSuccess) return launch_failed(e);
        StreamArgs d = g;
        d.w0 = (const uint16_t *)w_down; d.w1 = nullptr;
        d.s0 = (const uint16_t *)sh_down; d.s1 = nullptr;
        d.bsrc = (const uint16_t *)(ws + w.act); d.bsrc_sh = (const uint16_t *)(ws + w.act_sh);
        d.out = ws + w.o; d.out_sh = ws + w.o_sh;
        d.R = H; d.K = F; d.R_sh = H; d.K_sh = F_shared;
        d.KP = stream_panel_width(F); d.KP_sh = n_shared ? stream_panel_width(F_shared) : 0;
        if (stream_can_join(d)) {
            // small batch: the down kernel also sums the per-assignment outputs into `out`
            JoinArgs j = {};
            j.topk_w = topk_w; j.pos = pos; j.out = out;
            j.epoch = (const unsigned *)(ws + w.ctrl) + kCtrlEpoch;
            j.error_flag = (unsigned *)(ws + w.ctrl) + kCtrlError;
            j.miss_count = miss_count;
            j.out_bf16 = out_bf16; j.accumulate = accumulate;
            e = launch_stream(d, false, &j, s);
            return e == hipSuccess ? MOE_OK : launch_failed(e);
        }
        e = launch_stream(d, false, nullptr, s);
        if (e != hipSuccess) return launch_failed(e);
        e = launch_combine_rows(c, (const float *)(ws + w.o), (const float *)(ws + w.o_sh), s);
        return e == hipSuccess ? MOE_OK : launch_failed(e);
    }
    FfnArgs f = {};
    f.hidden = hidden; f.w_gate = w_gate; f.w_up = w_up; f.w_down = w_down;
    f.sh_gate = sh_gate; f.sh_up = sh_up; f.sh_down = sh_down;
    f.slot_count = slot_count; f.slot_offset = slot_offset; f.perm = perm;
    f.part = (float *)(ws + w.part); f.part_sh = (float *)(ws + w.part_sh);
    f.T = T; f.H = H; f.F = F; f.k = k; f.C = C; f.n_shared = n_shared; f.F_shared = F_shared;
    e = launch_ffn(f, s);
    if (e != hipSuccess) return launch_failed(e);
    c.part = f.part; c.part_sh = f.part_sh;
    e = launch_combine(c, s);
    return e == hipSuccess ? MOE_OK : launch_failed(e);
}

}  // namespace

extern "C" int moe_grouped_ffn(const void *hidden, const float *topk_w, const int32_t *slot_idx,
                               const void *w_gate, const void *w_up, const void *w_down, int T, int H, int F,
                               int k, int C, void *out, int out_bf16, int accumulate, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    if (!hidden || !topk_w || !slot_idx || !out || !workspace) return MOE_ERR_NULL;
    if (C > 0 && (!w_gate || !w_up || !w_down)) return MOE_ERR_NULL;
    int rc = check_ffn_shape(T, H, F, k, C, 0, 0);
    if (rc) return rc;
    if (!aligned16(hidden) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) ||
        !aligned16(out) || !aligned16(workspace))
        return MOE_ERR_ALIGN;
    // the single-step call has no routing scratch: lay the workspace out with E = 0
    WsLayout w = ws_layout(T, 0, k, C, H, F, 0, 0);
    if (workspace_bytes < w.total) return MOE_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = launch_lists_from_slots(layout_hash(w), slot_idx, T * k, C, (int32_t *)(ws + w.slot_count),
                                           (int32_t *)(ws + w.slot_offset), (int32_t *)(ws + w.perm),
                                           (int32_t *)(ws + w.pos), (int32_t *)(ws + w.active),
                                           (unsigned *)(ws + w.ctrl) + kCtrlNActive,
                                           (unsigned *)(ws + w.ctrl) + kCtrlEpoch, s);
    if (e != hipSuccess) return launch_failed(e);
    return run_ffn(hidden, topk_w, w_gate, w_up, w_down, nullptr, nullptr, nullptr, T, H, F, k, C, 0, 0, w, ws,
                   out, out_bf16, accumulate, s);
}

namespace {

// Argument checks of a whole-layer call that do not concern the workspace.
int check_layer_args(const moe_shape_t *sh, const void *hidden, const float *router_w, const int32_t *slot_table,
                     const void *w_gate, const void *w_up, const void *w_down, const void *shared_gate,
                     const void *shared_up, const void *shared_down, const int32_t *topk_idx, const float *topk_w,
                     const int32_t *hist, const int32_t *slot_idx, const int32_t *miss_list,
                     const int32_t *miss_count, const void *out)
{
    if (!sh || !hidden || !router_w || !slot_table || !topk_idx || !topk_w || !hist || !slot_idx ||
        !miss_list || !miss_count || !out)
        return MOE_ERR_NULL;
    if (sh->C > 0 && (!w_gate || !w_up || !w_down)) return MOE_ERR_NULL;
    if (sh->n_shared < 0 || (sh->n_shared > 0 && sh->F_shared < 1)) return MOE_ERR_SHAPE;
    if (sh->launch_form < MOE_LAUNCH_AUTO || sh->launch_form > MOE_LAUNCH_ROUTE_PLUS_ONE) return MOE_ERR_SHAPE;
    if (sh->n_shared > 0 && (!shared_gate || !shared_up || !shared_down)) return MOE_ERR_NULL;
    int rc = check_route_shape(sh->T, sh->H, sh->E, sh->k);
    if (rc) return rc;
    rc = check_ffn_shape(sh->T, sh->H, sh->F, sh->k, sh->C, sh->n_shared, sh->n_shared ? sh->F_shared : 0);
    if (rc) return rc;
    if (!aligned16(hidden) || !aligned16(router_w) || !aligned16(w_gate) || !aligned16(w_up) ||
        !aligned16(w_down) || !aligned16(shared_gate) || !aligned16(shared_up) || !aligned16(shared_down) ||
        !aligned16(out))
        return MOE_ERR_ALIGN;
    return MOE_OK;
}

// Steps 1-4 on a workspace that has been checked (size, alignment) and initialised for this shape.
int run_layer(const moe_shape_t *sh, const void *hidden, const float *router_w, const float *router_bias,
              const int32_t *slot_table, const void *w_gate, const void *w_up, const void *w_down,
              const void *shared_gate, const void *shared_up, const void *shared_down, int32_t *topk_idx,
              float *topk_w, int32_t *hist, int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, void *out,
              int out_bf16, int accumulate, const WsLayout &w, char *ws, hipStream_t s)
{
    RouteArgs r = {};
    r.hidden = hidden; r.router_w = router_w; r.router_bias = router_bias;
    r.T = sh->T; r.H = sh->H; r.E = sh->E; r.k = sh->k;
    r.tagged_logits = (unsigned long long *)(ws + w.tagged);
    r.tagged_idx = (unsigned long long *)(ws + w.tagged_idx);
    r.epoch = (unsigned *)(ws + w.ctrl) + kCtrlEpoch;
    r.error_flag = (unsigned *)(ws + w.ctrl) + kCtrlError;
    r.topk_idx = topk_idx; r.topk_w = topk_w; r.logits_opt = nullptr; r.hist = hist;
    r.layout = layout_hash(w);
    r.slot_table = slot_table; r.C = sh->C;
    r.slot_idx = slot_idx; r.miss_list = miss_list; r.miss_count = miss_count;
    r.slot_count = (int32_t *)(ws + w.slot_count); r.slot_offset = (int32_t *)(ws + w.slot_offset);
    r.perm = (int32_t *)(ws + w.perm); r.pos = (int32_t *)(ws + w.pos);
    r.active_slots = (int32_t *)(ws + w.active); r.n_active = (unsigned *)(ws + w.ctrl) + kCtrlNActive;
    // The launch forms (moe_shape_t::launch_form): three launches (routing kernel, gate/up stream, down stream with
    // the final sum), two (routing steps at the head of the gate/up kernel), one (routing, gate/up, down and the
    // final sum in one kernel: batches of up to 16 tokens), or the routing kernel followed by the one-launch FFN.
    const int n_sh = sh->n_shared, F_sh = sh->n_shared ? sh->F_shared : 0;
    const bool can_layer = use_layer_kernel(sh->T, sh->k, sh->E, sh->C, sh->H, sh->F, n_sh, F_sh);
    const bool can_route_inside = w.lists_pub != 0;
    int form = sh->launch_form;
    // (the library's choice: routing inside the gate/up launch where the shape allows, one launch less per layer)
    if (form == MOE_LAUNCH_AUTO) form = can_route_inside ? MOE_LAUNCH_TWO : MOE_LAUNCH_THREE;
    if (form == MOE_LAUNCH_ONE && !(can_layer && can_route_inside)) return MOE_ERR_SHAPE;
    if (form == MOE_LAUNCH_ROUTE_PLUS_ONE && !can_layer) return MOE_ERR_SHAPE;
    if (form == MOE_LAUNCH_TWO && !can_route_inside) return MOE_ERR_SHAPE;
    if (form == MOE_LAUNCH_ONE || form == MOE_LAUNCH_TWO) {
        r.lists_pub = (unsigned long long *)(ws + w.lists_pub);
        return run_ffn(hidden, topk_w, w_gate, w_up, w_down, shared_gate, shared_up, shared_down, sh->T, sh->H,
                       sh->F, sh->k, sh->C, n_sh, F_sh, w, ws, out, out_bf16, accumulate, s, &r,
                       form == MOE_LAUNCH_ONE, miss_count);
    }
    hipError_t e = launch_route(r, s);
    if (e != hipSuccess) return launch_failed(e);
    return run_ffn(hidden, topk_w, w_gate, w_up, w_down, shared_gate, shared_up, shared_down, sh->T, sh->H,
                   sh->F, sh->k, sh->C, n_sh, F_sh, w, ws, out, out_bf16, accumulate, s, nullptr,
                   form == MOE_LAUNCH_ROUTE_PLUS_ONE, miss_count);
}

}  // namespace

extern "C" int moe_verify_layer(const moe_shape_t *sh, const void *hidden, const float *router_w,
                                const float *router_bias, const int32_t *slot_table, const void *w_gate,
                                const void *w_up, const void *w_down, const void *shared_gate,
                                const void *shared_up, const void *shared_down, int32_t *topk_idx,
                                float *topk_w, int32_t *hist, int32_t *slot_idx, int32_t *miss_list,
                                int32_t *miss_count, void *out, int out_bf16, int accumulate, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    if (!workspace) return MOE_ERR_NULL;
    int rc = check_layer_args(sh, hidden, router_w, slot_table, w_gate, w_up, w_down, shared_gate, shared_up,
                              shared_down, topk_idx, topk_w, hist, slot_idx, miss_list, miss_count, out);
    if (rc) return rc;
    if (!aligned16(workspace)) return MOE_ERR_ALIGN;
    WsLayout w = ws_layout(sh->T, sh->E, sh->k, sh->C, sh->H, sh->F, sh->n_shared, sh->F_shared);
    if (workspace_bytes < w.total) return MOE_ERR_WORKSPACE;
    return run_layer(sh, hidden, router_w, router_bias, slot_table, w_gate, w_up, w_down, shared_gate, shared_up,
                     shared_down, topk_idx, topk_w, hist, slot_idx, miss_list, miss_count, out, out_bf16,
                     accumulate, w, (char *)workspace, (hipStream_t)stream);
}

// ---- the whole layer for callers that cannot allocate ----
// Same steps and kernels as moe_verify_layer, with the workspace in a device array that is part of the
// library's image (every device that loads the library holds its own copy, at an address of its own).
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t kScratchBytes = (size_t)MOE_STATIC_SCRATCH_BYTES;

struct ScratchState {
    void *ptr = nullptr;          // device address of `scratch` on this device
    bool laid_out = false;        // the array has been cleared for `shape`
    moe_shape_t shape = {};
};
ScratchState g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

bool same_shape(const moe_shape_t &a, const moe_shape_t &b)
{
    return a.T == b.T && a.H == b.H && a.E == b.E && a.k == b.k && a.F == b.F && a.C == b.C &&
           a.n_shared == b.n_shared && a.F_shared == b.F_shared && a.launch_form == b.launch_form;
}

}  // namespace

extern "C" int moe_verify_layer_static(const moe_shape_t *sh, const void *hidden, const float *router_w,
                                       const float *router_bias, const int32_t *slot_table, const void *w_gate,
                                       const void *w_up, const void *w_down, const void *shared_gate,
                                       const void *shared_up, const void *shared_down, int32_t *topk_idx,
                                       float *topk_w, int32_t *hist, int32_t *slot_idx, int32_t *miss_list,
                                       int32_t *miss_count, void *out, int out_bf16, int accumulate, void *stream)
{
    int rc = check_layer_args(sh, hidden, router_w, slot_table, w_gate, w_up, w_down, shared_gate, shared_up,
                              shared_down, topk_idx, topk_w, hist, slot_idx, miss_list, miss_count, out);
    if (rc) return rc;
    const WsLayout w = ws_layout(sh->T, sh->E, sh->k, sh->C, sh->H, sh->F, sh->n_shared, sh->F_shared);
    if (w.total > kScratchBytes) return MOE_ERR_SCRATCH;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return launch_failed(e);
    if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ScratchState &st = g_scratch[dev];
    if (!st.ptr) {
        // (in host code the array's name is only a handle: the device address comes from the runtime)
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return launch_failed(e != hipSuccess ? e : hipErrorInvalidSymbol);
        st.ptr = p;
    }
    if (!st.laid_out || !same_shape(st.shape, *sh)) {
        // another layout than the last call's (or the first call): no stale entry may carry a future
        // call number, so everything this layout uses starts at zero (a fill kernel on the caller's stream)
        st.laid_out = false;
        e = launch_clear_ctrl(st.ptr, w.total, s);
        if (e != hipSuccess) return launch_failed(e);
        st.shape = *sh;
        st.laid_out = true;
    }
    return run_layer(sh, hidden, router_w, router_bias, slot_table, w_gate, w_up, w_down, shared_gate, shared_up,
                     shared_down, topk_idx, topk_w, hist, slot_idx, miss_list, miss_count, out, out_bf16,
                     accumulate, w, (char *)st.ptr, s);
}
