/*
 * moe_spac.h -- C-ABI of the MI355X (gfx950) verify-step MoE layer.
 *
 * One call of moe_verify_layer is the MoE layer forward for one speculative-
 * decoding verification batch of T = gamma + 1 tokens (Sec. 2.1): routing and
 * gating (Sec. 2.2), the activation-frequency histogram that the Speculative
 * Utility Estimator consumes (Sec. 2.3, Alg. 1 "observe activation
 * frequencies"), the rewrite of expert ids into cache slots with non-resident
 * experts marked by a sentinel and listed for the host (App. D), and the
 * gate/up/down expert FFN over the resident experts with the weighted
 * combine back into token order (Sec. 2.2 last line; App. D).
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller, unless the
 *     comment says "host".  The library never allocates, frees or keeps a
 *     pointer.  Scratch comes from the caller's `workspace`.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; no call synchronises.  Outputs (miss_count
 *     included) are valid once the caller has synchronised the stream.
 *   - Layouts are row-major, innermost index last.  bf16 tensors are raw
 *     16-bit patterns (void*).  Notation: T tokens, H hidden size, E routed
 *     experts, k experts per token, F expert FFN width, C cache capacity in
 *     slots, A = T*k assignments (flat id a = t*k + j).
 *   - Return value: MOE_OK, or a negative code; on a negative code nothing
 *     was launched.  No exceptions, no abort, nothing printed.
 *   - Supported sizes: 1 <= k <= min(E, 64); E <= 512; T*E <= 65536;
 *     C <= 1024; H, F and F_shared multiples of 8 (rows of 16 bytes); bf16
 *     tensors and `out` 16-byte aligned.  Batches of up to 32 tokens with
 *     H, F and F_shared multiples of 64 run in the weight-streaming kernels
 *     at any H; every other shape runs in a kernel that keeps a token tile's
 *     hidden rows in LDS, which limits it to H <= 4992 (MOE_ERR_SHAPE beyond).
 *   - Two calls that share a workspace must not overlap in time.  A
 *     workspace holds state between calls (a call counter and regions whose
 *     entries are stamped with it): initialise it with moe_workspace_init
 *     over its full size, and again after anything else wrote into it or
 *     before using it with a different shape.  moe_grouped_ffn lays the
 *     workspace out differently from moe_verify_layer with the same sizes
 *     (it has no shared experts): initialise between the two as well.  A
 *     call that finds the workspace laid out for something else marks its
 *     results and moe_workspace_status returns MOE_ERR_WORKSPACE.
 *   - The routing kernel and the down kernel hand results from one workgroup
 *     to another inside a launch (stamped entries in the workspace, bounded
 *     polling).  They are sized to occupy the whole device.  Layer calls on
 *     different streams of one device are legal, but if they really run at
 *     the same time the bounded waits can run out (moe_workspace_status then
 *     reports it, nothing hangs): issue the layer calls of one device in
 *     stream order.
 *   - The slot table maps distinct resident experts to distinct slots (it is
 *     a cache directory); with two experts on one slot the per-slot lists are
 *     unspecified (every access still stays in bounds).
 */
#ifndef MOE_SPAC_H
#define MOE_SPAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOE_OK = 0,
    MOE_ERR_NULL = -1,      /* a required pointer is NULL                              */
    MOE_ERR_SHAPE = -2,     /* a size is out of the supported range                    */
    MOE_ERR_ALIGN = -3,     /* H or F not a multiple of 8, or a misaligned pointer      */
    MOE_ERR_WORKSPACE = -4, /* workspace_bytes is smaller than the call needs          */
    MOE_ERR_LAUNCH = -5,    /* the HIP runtime refused a launch or an attribute        */
    MOE_ERR_SCRATCH = -6    /* moe_verify_layer_static: the shape needs more scratch memory
                               than MOE_STATIC_SCRATCH_BYTES                            */
};

/* Problem sizes of one layer call.  n_shared always-on experts of width
 * F_shared each (0 = none); they are not routed, not cached and not counted. */
typedef struct moe_shape {
    int T, H, E, k, F, C;
    int n_shared, F_shared;
    int launch_form;   /* moe_verify_layer only: MOE_LAUNCH_* (0 = the library chooses) */
} moe_shape_t;

/* How moe_verify_layer cuts the layer into kernel launches (same results in
 * every form).  A form that the shape does not allow is refused with
 * MOE_ERR_SHAPE; MOE_LAUNCH_AUTO never is.  A workspace that has been used in
 * one form must be initialised again before it is used in another. */
enum {
    MOE_LAUNCH_AUTO = 0,
    MOE_LAUNCH_THREE = 1,         /* routing | gate/up stream | down stream + final sum (+ a combine launch above 32 tokens) */
    MOE_LAUNCH_TWO = 2,           /* routing steps at the head of the gate/up kernel: T <= 32, E <= 128 */
    MOE_LAUNCH_ONE = 3,           /* routing, gate/up, down and final sum as one kernel: T <= 16, E <= 128, H, F multiples of 64 */
    MOE_LAUNCH_ROUTE_PLUS_ONE = 4 /* routing kernel, then gate/up, down and final sum as one kernel: T <= 16 */
};

/* Host-only, pure.  Static text for a status code (never NULL). */
const char *moe_status_string(int status);

/* Host-only, pure.  Bytes of workspace that any entry point needs for `shape`
 * (an upper bound for the single-step entry points).  shape: host pointer. */
int moe_workspace_bytes(const moe_shape_t *shape, size_t *bytes_out);

/* Zero-fills a freshly allocated workspace (control block, call counter and
 * every region whose entries the kernels stamp with the call number).  Call
 * once per workspace, over its full size, before its first use. */
int moe_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Synchronous health check: waits for `stream`, then reads the control block.
 * Inside a launch workgroups hand results to one another through stamped
 * entries of the workspace (the logits and the lists of the routing steps,
 * the per-assignment outputs before the final sum); each wait polls a bounded
 * number of times and, should that bound ever run out, sets a flag in the
 * control block and finishes instead of waiting for ever.  The call that it
 * happened in marks its results: every element of `out` that is written after
 * the flag was set is NaN, and *miss_count is -1.  Returns MOE_OK when no
 * flag is set; MOE_ERR_LAUNCH when one is, or when the copy fails;
 * MOE_ERR_WORKSPACE when a call found that the workspace had served a shape
 * with another layout since its last moe_workspace_init (that call's results
 * are marked in the same way; initialise the workspace again).  The flag
 * is then cleared and the call counter stepped past every number the failed
 * call may have used, so the workspace stays usable; no call on this
 * workspace may be in flight meanwhile.  workspace: device pointer. */
int moe_workspace_status(void *workspace, size_t workspace_bytes, void *stream);

/* Test hook for the failure path above: makes the bounded waits of later
 * calls on this workspace poll at most `poll_limit` times (0 = the built-in
 * bound) and adds `stamp_skew` to the call number that producers stamp their
 * entries with (0 = none), so that with a small limit and a skew of 1 no wait
 * ever finds its entry, every one runs out quickly, and every kernel still
 * ends by itself.  moe_workspace_init clears both.  Synchronous.
 * workspace: device pointer. */
int moe_workspace_wait_test(void *workspace, size_t workspace_bytes, unsigned poll_limit,
                            unsigned stamp_skew, void *stream);

/* Step 1 -- Sec. 2.2, lines one to three of the MoE equation.
 *   s = W_g h (+ bias), the k largest logits per token (listed by descending
 *   logit, ties to the lower expert id; -0 equals +0; a NaN logit ranks as
 *   minus infinity), g = softmax restricted to those k.
 * hidden [T,H] bf16; router_w [E,H] fp32; router_bias [E] fp32 or NULL (NULL
 * is the paper's equation); topk_idx [T,k] int32 out; topk_w [T,k] fp32 out;
 * logits_opt [T,E] fp32 out or NULL. */
int moe_route_topk(const void *hidden, const float *router_w, const float *router_bias, int T, int H,
                   int E, int k, int32_t *topk_idx, float *topk_w, float *logits_opt, void *workspace,
                   size_t workspace_bytes, void *stream);

/* Step 2 -- Sec. 2.3 "Activation Frequency": hist[e] = number of assignments
 * that selected expert e over the T tokens of this step (the f_{e,t} that
 * Alg. 1 observes).  topk_idx [T,k] int32 with values in [0,E); hist [E] int32
 * out (overwritten).  Ids outside [0,E) are ignored. */
int moe_expert_histogram(const int32_t *topk_idx, int T, int k, int E, int32_t *hist, void *stream);

/* Step 3 -- App. D: the ids rewrite.  slot_idx[a] = slot_table[topk_idx[a]],
 * -1 when the expert is not resident; miss_list = the flat ids a of the
 * missed assignments in ascending order (the host's share of the layer);
 * miss_count [1].  slot_table [E] int32: -1 or a slot in [0,C), distinct
 * experts in distinct slots; a value outside [0,C) is treated as -1.
 * miss_list must hold T*k entries.  The per-slot token lists (the
 * expert-sorted permutation that step 4 consumes) are left in `workspace`. */
int moe_slot_resolve(const int32_t *topk_idx, const int32_t *slot_table, int T, int k, int E, int C,
                     int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, void *workspace,
                     size_t workspace_bytes, void *stream);

/* Step 4 -- Sec. 2.2 last line, restricted to resident experts (App. D):
 *   out[t,:] (+)= sum over j with slot_idx[t,j] >= 0 of
 *        topk_w[t,j] * W_down[c] ( silu(W_gate[c] x_t) * (W_up[c] x_t) ),  c = slot_idx[t,j].
 * Pools are slot-major: w_gate, w_up [C,F,H] bf16, w_down [C,H,F] bf16 (each
 * matrix [out,in]).  bf16 products, fp32 accumulation; the activation is
 * rounded to bf16 before the down projection.  Missed assignments add
 * nothing.  out [T,H] fp32, or bf16 when out_bf16 != 0; accumulate != 0 adds
 * to what `out` holds (the join with the host's partial result), else `out`
 * is overwritten.  Slots outside [0,C) in slot_idx are treated as -1. */
int moe_grouped_ffn(const void *hidden, const float *topk_w, const int32_t *slot_idx, const void *w_gate,
                    const void *w_up, const void *w_down, int T, int H, int F, int k, int C, void *out,
                    int out_bf16, int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* Steps 1-4 for one verification batch on `stream`, in the launch form that
 * shape->launch_form names (MOE_LAUNCH_AUTO: two launches, the routing steps
 * at the head of the gate/up kernel, for batches of up to 32 tokens and 128
 * experts with a non-empty pool; else three launches; four above 32 tokens).
 * Every form computes the same outputs to the same bar.
 * The workspace carries state from call to call (see moe_workspace_init): it
 * must have been initialised once, be used by one call at a time, and be
 * initialised again before it serves another shape.
 * shape: host pointer.  shared_gate/up [n_shared,F_shared,H] and shared_down
 * [n_shared,H,F_shared] bf16 (NULL when n_shared = 0) are added with weight 1
 * for every token.  All step outputs are produced: topk_idx, topk_w [T,k];
 * hist [E]; slot_idx [T,k]; miss_list [T*k]; miss_count [1]; out [T,H]. */
int moe_verify_layer(const moe_shape_t *shape, const void *hidden, const float *router_w,
                     const float *router_bias, const int32_t *slot_table, const void *w_gate,
                     const void *w_up, const void *w_down, const void *shared_gate, const void *shared_up,
                     const void *shared_down, int32_t *topk_idx, float *topk_w, int32_t *hist,
                     int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, void *out, int out_bf16,
                     int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* moe_verify_layer for callers that cannot allocate device memory or hand a
 * workspace over: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments (without the workspace), same steps,
 * same kernels and the same results as moe_verify_layer; the scratch memory is
 * an array of MOE_STATIC_SCRATCH_BYTES bytes inside the library's own device
 * image, which every GPU the library runs on holds from the first call until
 * the process ends.  The call allocates and frees nothing.
 *   - A shape whose moe_workspace_bytes() exceeds MOE_STATIC_SCRATCH_BYTES is
 *     rejected with MOE_ERR_SCRATCH before anything is launched (16 MiB holds
 *     every shape up to 128 tokens x top-6 at H = 2048, F = 1408).
 *   - The array keeps the last call's contents.  The first call on a device,
 *     and every call whose shape differs from the previous call's on that
 *     device, first zero-fills the part of the array the new layout uses (one
 *     small fill kernel on `stream`); moe_workspace_init is not needed.
 *   - All calls on one GPU share that GPU's array: two calls that overlap in
 *     time on one GPU (different streams, or different host threads without
 *     stream order between them) race on it and give unspecified results;
 *     issue them in stream order.  The health flag of the bounded waits is not
 *     readable for this array; use moe_verify_layer where it is needed. */
#define MOE_STATIC_SCRATCH_BYTES (16u << 20)
int moe_verify_layer_static(const moe_shape_t *shape, const void *hidden, const float *router_w,
                            const float *router_bias, const int32_t *slot_table, const void *w_gate,
                            const void *w_up, const void *w_down, const void *shared_gate,
                            const void *shared_up, const void *shared_down, int32_t *topk_idx, float *topk_w,
                            int32_t *hist, int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, void *out,
                            int out_bf16, int accumulate, void *stream);

/* NEXT STEP AFTER THE HISTOGRAM -- Sec. 3.2, Alg. 1 (Speculative Utility
 * Estimator) and the utility-transition equation; n(tau) as in the notation
 * table of Sec. 3.3.
 *
 * State per (layer, expert), int32, row-major [L,N], owned by the caller:
 * utility s in [0,K], boundaries theta_up and theta_dn, previous frequencies
 * f_prev.  moe_utility_init sets s = 0, f_prev = 0 (the reading taken for
 * f_{i,0}) and both boundaries to floor(gamma/2).
 *
 * moe_utility_update advances all L layers by one inference step from the
 * observed frequencies f [L,N] (for one layer: the `hist` output of step 2):
 *   d = f - f_prev;
 *   d >= theta_up: s <- min(K, s+1);  else -d >= theta_dn: s <- max(0, s-1);
 *   d > 0: theta_up <- floor((1-lam) theta_up + lam d);
 *   d < 0: theta_dn <- floor((1-lam) theta_dn + lam |d|);   f_prev <- f.
 * The transition uses the boundaries as they were before this call.  lam =
 * lam_num / lam_den (0 <= lam_num <= lam_den, e.g. 1/10); the floor is exact
 * integer arithmetic.  0 <= K <= 64.
 * Optional: slot_table [L,N] (expert -> slot or -1) and n_tau [L,K+1] out:
 * n_tau[l,tau] = number of experts of layer l with s >= tau (after the
 * update) that hold no slot, tau = 0..K.  Pass both or n_tau = NULL.
 * One launch on `stream`; nothing is allocated. */
int moe_utility_init(int32_t *f_prev, int32_t *s, int32_t *theta_up, int32_t *theta_dn, int L, int N, int gamma,
                     void *stream);
int moe_utility_update(const int32_t *f, int32_t *f_prev, int32_t *s, int32_t *theta_up, int32_t *theta_dn,
                       const int32_t *slot_table, int32_t *n_tau, int L, int N, int K, int lam_num, int lam_den,
                       void *stream);

/* Sec. 3.3 (the two time equations, the objective, its constraints) and the
 * appendix on its solution: the per-layer threshold tau* that balances host
 * and device time.  For each layer l (one launch for all L):
 *   b          = number of experts with f[l,i] > 0
 *   T_cpu(tau) = r_c[l,tau] * gamma * k * t_cpu
 *   T_gpu(tau) = r_g[l,tau] * b * t_gpu
 *   feasible   : t_io * n_tau[l,tau] <= max(T_cpu, T_gpu) + gamma * t_draft / l_target
 *                and w_expert_bytes * n_tau[l,tau] <= vram_left_bytes
 *   tau_out[l] = the feasible tau in 1..K with the smallest |T_cpu - T_gpu|
 *                (the smaller tau on ties), K if none is feasible.
 * Every tau is evaluated (K <= 64), in fp64 in the order written above, so
 * the result is the definition's, with or without the convexity the paper's
 * shortcut assumes.  f [L,N] int32 (the histograms); n_tau [L,K+1] int32 (as
 * moe_utility_update writes it); r_c, r_g [L,K+1] fp64 tables indexed by tau
 * (entry 0 unused; the paper learns them in a warm-up run, here they are
 * inputs); params: HOST pointer; b_out [L] int32 or NULL.  All other
 * pointers are device pointers. */
typedef struct moe_balance_params {
    double t_cpu, t_gpu;          /* unit time of one activated expert on host / device */
    double t_io;                  /* unit time to load one expert */
    double t_draft;               /* unit time of one draft-model token */
    int l_target;                 /* layers of the target model */
    int64_t w_expert_bytes;       /* memory of one expert */
    int64_t vram_left_bytes;      /* memory available for prefetched experts */
} moe_balance_params_t;
int moe_balance_threshold(const int32_t *f, const int32_t *n_tau, const double *r_c, const double *r_g, int L,
                          int N, int K, int gamma, int k, const moe_balance_params_t *params, int32_t *tau_out,
                          int32_t *b_out, void *stream);

/* Sec. 3.4 (utility-guided prefetching and eviction) and the appendix on the
 * execution engine: one planning step of the cache manager for L layers, one
 * launch.  For each layer l, with tau = tau[l]:
 *   evicted    = resident experts (slot_table >= 0) with s < tau that are not
 *                in use (in_use != 0 marks the frozen experts; NULL = none),
 *                listed by ascending utility, ascending id inside a utility;
 *   fetched    = non-resident experts with tau <= s <= K, level K first,
 *                ascending id inside a level, as many as there are free slots
 *                (after the evictions) and at most budget[l] (NULL = no limit);
 *   fetch_slot = the free slots in ascending order, one per fetched expert;
 *   slot_table is updated in place (evicted -> -1, fetched -> their slot).
 * s, in_use, slot_table [L,N] int32; tau, budget, n_evict, n_fetch [L];
 * evict_list [L,N]; fetch_list, fetch_slot [L,C].  N <= 512, C <= 1024,
 * K <= 64.  The weights do not move here: see moe_pool_load. */
int moe_cache_plan(const int32_t *s, const int32_t *in_use, int32_t *slot_table, const int32_t *tau,
                   const int32_t *budget, int L, int N, int C, int K, int32_t *evict_list, int32_t *n_evict,
                   int32_t *fetch_list, int32_t *fetch_slot, int32_t *n_fetch, void *stream);

/* Moves the fetched experts of ONE layer into their slots: for j < *n_fetch,
 * pool_x[fetch_slot[j]] = store_x[fetch_list[j]] for x in gate, up [.,F,H] and
 * down [.,H,F] (bf16).  store_*: every expert of the layer, in device memory
 * or in pinned host memory mapped into the device; pool_*: the slot-major
 * pools that moe_verify_layer reads.  fetch_list, fetch_slot, n_fetch: that
 * layer's rows of moe_cache_plan's outputs (device).  max_fetch (host): upper
 * bound of *n_fetch used to size the launch (entries beyond *n_fetch do
 * nothing).  One launch on `stream`; launched on a stream of its own it
 * runs beside other layers' verify steps (a store in host memory gets a
 * launch of few workgroups, so that the slow copy does not occupy the
 * chip).  F*H*2 a multiple of 16. */
int moe_pool_load(const void *store_gate, const void *store_up, const void *store_down, void *pool_gate,
                  void *pool_up, void *pool_down, const int32_t *fetch_list, const int32_t *fetch_slot,
                  const int32_t *n_fetch, int max_fetch, int H, int F, void *stream);

/* Measurement aid (host-side state only; not part of the layer's arithmetic).
 * While enabled, every kernel the library launches is bracketed by a pair of
 * HIP events recorded on the caller's stream.  kind: MOE_KERNEL_*.
 * moe_profile_enable(1) clears the records (event pairs are made with
 * hipEventCreate when a launch first needs one, up to 8192 per kind, and kept;
 * no device memory); moe_profile_enable(0) stops recording.  The records are
 * one set per process, not guarded: measure from one host thread.
 * moe_profile_read sums hipEventElapsedTime over the records of one kind; the
 * caller must have synchronised the stream.  total_ms, launches: host. */
enum { MOE_KERNEL_ROUTE = 0, MOE_KERNEL_LISTS = 1, MOE_KERNEL_FFN = 2 /* gate/up (and down when fused) */,
       MOE_KERNEL_COMBINE = 3, MOE_KERNEL_DOWN = 4, MOE_KERNEL_ESTIMATOR = 5, MOE_KERNEL_BALANCER = 6,
       MOE_KERNEL_CACHE_PLAN = 7, MOE_KERNEL_POOL_LOAD = 8, MOE_KERNEL_LAYER = 9 /* the one-launch layer kernel */,
       MOE_KERNEL_KINDS = 10 };
int moe_profile_enable(int on);
int moe_profile_read(int kind, double *total_ms, int *launches);
const char *moe_profile_kernel_name(int kind);
/* What a pair of events costs by itself: records `pairs` (1..8192) pairs on
 * `stream` with nothing in between, waits for the stream and returns the mean
 * interval in *avg_ms (host).  A bracketed kernel's record contains about this
 * much time that is not the kernel's.  Uses event pairs of its own, which it
 * creates and destroys; independent of moe_profile_enable. */
int moe_profile_event_overhead(void *stream, int pairs, double *avg_ms);
/* Timeline of the last launches of the streaming kernels, for a library built
 * with -DMOE_STREAM_TRACE (the product build returns MOE_ERR_SHAPE and writes
 * nothing).  words: host buffer of 2 x 1024 x 8 + 1024 x 24 64-bit words.
 * First [kernel: 0 gate/up, 1 down][workgroup][8]: ticks of the 100 MHz device
 * wall clock at the workgroup's start, with the per-slot lists in LDS, after
 * its first tile, at the end of its loop, after its results are stored and at
 * its end; then its items and tiles.  Then the one-launch layer kernel,
 * [workgroup][24]: start, lists in LDS, after the first tile, when the walk
 * that multiplies enters the down part, end of the loop, end; (gate/up items
 * << 32 | down items); tiles; then for wavefront 0 and for wavefront 15 eight
 * sums over the loop's steps, in shader clock cycles: waiting for the tile,
 * parking it, storing the previous item's results, requesting a tile and
 * stepping the request walk, first barrier, multiplying, second barrier,
 * stepping the other walk.  Synchronous (a blocking copy from the device);
 * call after synchronising the stream. */
int moe_profile_stream_timeline(unsigned long long *words, size_t n_words);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SPAC_H */
