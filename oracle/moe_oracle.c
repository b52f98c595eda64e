/*
 * CPU oracle for the verify-step MoE layer of MoE-SpAc.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  It shares no code with them and nothing
 * in the product path may link or call it; only the tests, the smoke check
 * and the bench's cpu_baseline leg do.
 *
 * Everything is the defining formula written out, in fp64, on bf16-rounded
 * inputs, with no blocking, fusion or reordering:
 *   - routing, gating, expert mixture: Sec. 2.2, the four-line MoE equation
 *     (s = W_g h; Top-k; g_i = exp(s_i)/sum_{j in Top-k} exp(s_j);
 *      y = sum_{i in Top-k} g_i E_i(h));
 *   - activation frequency f_{i,t}: Sec. 2.3 "Activation Frequency";
 *   - resident / missed split with a sentinel id: App. D (the ids rewrite,
 *     skipped experts, and the join of the two partial results);
 *   - the expert is the gate/up/down FFN named in App. D; the activation is
 *     SiLU on the gate branch (SwiGLU), biases absent.
 *
 * Readings where the paper is silent: ties in Top-k go to the lower expert
 * id; the k ids of a token are listed by descending logit; the sentinel is
 * -1; gates are normalised over the full Top-k set even when some of those
 * experts are not resident (the device result is a partial sum that the
 * host's share completes); shared experts are added with weight 1 for every
 * token and are outside routing, histogram and miss list.
 *
 * Also here, for the consumer of the activation frequencies: one step of the
 * Speculative Utility Estimator (Sec. 3.2, Alg. 1 and the utility-transition
 * equation) and the prefetch count n(tau) of the balancer's notation table
 * (Sec. 3.3).  Readings: f_{i,0} = 0; the forgetting factor is a rational
 * lam_num/lam_den and the floor is taken in exact integer arithmetic; the
 * upward test comes first, so a boundary of 0 lets a fluctuation of 0 raise
 * the utility, as the listing's ">=" says.
 *
 * And the Heterogeneous Workload Balancer's threshold (Sec. 3.3 and the
 * appendix on its formulation): tau* = the feasible integer tau in [1,K] that
 * minimises |T_cpu(tau) - T_gpu(tau)|, by evaluating every tau (the
 * definition; the paper's four-candidate shortcut is a method that relies on
 * convexity and is checked against this in the tests).  Readings: ties go to
 * the smaller tau; b counts the experts with a non-zero frequency; both
 * constraints are "<=" as printed; no feasible tau gives K.
 *
 * And one planning step of the utility-guided cache manager for one layer
 * (Sec. 3.4 "Utility-Guided Prefetching / Eviction"; appendix on the engine:
 * frozen experts): evict the residents whose utility fell below tau, then
 * fetch the non-resident experts of utility >= tau, level K first, into the
 * free slots.  Readings: inside a level requests are served in ascending
 * expert id (the order the estimator emits them); every resident below tau is
 * evicted, not only as many as needed; an expert in use (frozen, the K+1 tag)
 * is never evicted; fetched expert j takes the j-th free slot in ascending
 * slot order; at most `budget` experts are fetched (the balancer's I/O and
 * memory limits expressed as a count).
 *
 * Pinned by tests/test_oracle_pins.py (brute-force dense evaluation in
 * numpy, textbook SwiGLU through torch's own linear/silu, closed forms,
 * the worked example of App. C.1, invariants).  No function here is
 * "parity unpinned".
 *
 * Optional threading: a bare "omp parallel for" over output rows; the
 * per-element summation order does not depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* s[t,e] = sum_h W_g[e,h] * h_t[h] (+ bias[e])      -- Sec. 2.2, first line */
void oracle_router_logits(const uint16_t *hidden, const float *router_w, const float *bias,
                          int T, int H, int E, double *logits)
{
    for (int t = 0; t < T; ++t)
        for (int e = 0; e < E; ++e) {
            double s = 0.0;
            for (int h = 0; h < H; ++h)
                s += (double)router_w[(size_t)e * H + h] * bf16_to_f64(hidden[(size_t)t * H + h]);
            if (bias) s += (double)bias[e];
            logits[(size_t)t * E + e] = s;
        }
}

/* Top-k by k passes of arg-max (larger logit first, lower id on equality) and
 * the gate restricted to the selected set      -- Sec. 2.2, lines two and three */
void oracle_topk_gate(const double *logits, int T, int E, int k, int32_t *topk_idx, double *gate)
{
    char *taken = (char *)malloc((size_t)E);
    for (int t = 0; t < T; ++t) {
        const double *s = logits + (size_t)t * E;
        memset(taken, 0, (size_t)E);
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || s[e] > s[best]) best = e;
            }
            taken[best] = 1;
            topk_idx[(size_t)t * k + j] = best;
        }
        double smax = s[topk_idx[(size_t)t * k]];
        double den = 0.0;
        for (int j = 0; j < k; ++j) den += exp(s[topk_idx[(size_t)t * k + j]] - smax);
        for (int j = 0; j < k; ++j)
            gate[(size_t)t * k + j] = exp(s[topk_idx[(size_t)t * k + j]] - smax) / den;
    }
    free(taken);
}

/* f_i = number of (token, rank) pairs that selected expert i  -- Sec. 2.3 */
void oracle_expert_histogram(const int32_t *topk_idx, int T, int k, int E, int32_t *hist)
{
    for (int e = 0; e < E; ++e) hist[e] = 0;
    for (int a = 0; a < T * k; ++a) hist[topk_idx[a]] += 1;
}

/* ids rewrite: expert id -> cache slot, -1 when not resident; the missed
 * assignments (flat id a = t*k + j) in ascending order      -- App. D */
void oracle_slot_resolve(const int32_t *topk_idx, const int32_t *slot_table, int T, int k,
                         int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count)
{
    int n = 0;
    for (int a = 0; a < T * k; ++a) {
        int32_t c = slot_table[topk_idx[a]];
        slot_idx[a] = c;
        if (c < 0) miss_list[n++] = a;
    }
    *miss_count = n;
}

/* One expert on one token: o = W_down ( silu(W_gate x) * (W_up x) ), added
 * into y with weight g.  w_gate/w_up are [F,H], w_down is [H,F] (row = output). */
static void expert_ffn_add(const uint16_t *x_bits, const uint16_t *w_gate, const uint16_t *w_up,
                           const uint16_t *w_down, int H, int F, double g, double *y)
{
    double *x = (double *)malloc(sizeof(double) * (size_t)H);
    double *m = (double *)malloc(sizeof(double) * (size_t)F);
    for (int h = 0; h < H; ++h) x[h] = bf16_to_f64(x_bits[h]);
#pragma omp parallel for schedule(static)
    for (int f = 0; f < F; ++f) {
        double a = 0.0, u = 0.0;
        for (int h = 0; h < H; ++h) a += bf16_to_f64(w_gate[(size_t)f * H + h]) * x[h];
        for (int h = 0; h < H; ++h) u += bf16_to_f64(w_up[(size_t)f * H + h]) * x[h];
        m[f] = (a / (1.0 + exp(-a))) * u;
    }
#pragma omp parallel for schedule(static)
    for (int h = 0; h < H; ++h) {
        double o = 0.0;
        for (int f = 0; f < F; ++f) o += bf16_to_f64(w_down[(size_t)h * F + f]) * m[f];
        y[h] += g * o;
    }
    free(x);
    free(m);
}

/* y_t = sum over the token's RESIDENT selected experts of g * E_i(h_t)
 *                                     -- Sec. 2.2 last line, restricted per App. D.
 * Weights are indexed by EXPERT id in the full [E,...] set.  slot_table only
 * decides residency.  y is [T,H] fp64 and is overwritten. */
void oracle_routed_ffn(const uint16_t *hidden, const int32_t *topk_idx, const double *gate,
                       const int32_t *slot_table, const uint16_t *w_gate, const uint16_t *w_up,
                       const uint16_t *w_down, int T, int H, int F, int k, double *y)
{
    for (size_t i = 0; i < (size_t)T * H; ++i) y[i] = 0.0;
    for (int t = 0; t < T; ++t)
        for (int j = 0; j < k; ++j) {
            int e = topk_idx[(size_t)t * k + j];
            if (slot_table[e] < 0) continue;
            size_t off = (size_t)e * F * H;
            expert_ffn_add(hidden + (size_t)t * H, w_gate + off, w_up + off, w_down + off, H, F,
                           gate[(size_t)t * k + j], y + (size_t)t * H);
        }
}

/* always-on experts: y_t += E_s(h_t) for every token and every shared expert */
void oracle_shared_ffn_add(const uint16_t *hidden, const uint16_t *sh_gate, const uint16_t *sh_up,
                           const uint16_t *sh_down, int T, int H, int Fs, int n_shared, double *y)
{
    for (int t = 0; t < T; ++t)
        for (int s = 0; s < n_shared; ++s) {
            size_t off = (size_t)s * Fs * H;
            expert_ffn_add(hidden + (size_t)t * H, sh_gate + off, sh_up + off, sh_down + off, H, Fs,
                           1.0, y + (size_t)t * H);
        }
}

/* The whole layer for one verification batch, in the order of the steps. */
void oracle_verify_layer(const uint16_t *hidden, const float *router_w, const float *router_bias,
                         const int32_t *slot_table, const uint16_t *w_gate, const uint16_t *w_up,
                         const uint16_t *w_down, const uint16_t *sh_gate, const uint16_t *sh_up,
                         const uint16_t *sh_down, int T, int H, int E, int k, int F, int n_shared,
                         int Fs, double *logits, int32_t *topk_idx, double *gate, int32_t *hist,
                         int32_t *slot_idx, int32_t *miss_list, int32_t *miss_count, double *y)
{
    oracle_router_logits(hidden, router_w, router_bias, T, H, E, logits);
    oracle_topk_gate(logits, T, E, k, topk_idx, gate);
    oracle_expert_histogram(topk_idx, T, k, E, hist);
    oracle_slot_resolve(topk_idx, slot_table, T, k, slot_idx, miss_list, miss_count);
    oracle_routed_ffn(hidden, topk_idx, gate, slot_table, w_gate, w_up, w_down, T, H, F, k, y);
    if (n_shared > 0)
        oracle_shared_ffn_add(hidden, sh_gate, sh_up, sh_down, T, H, Fs, n_shared, y);
}

/* ---------------------------------------------------------------------------
 * Speculative Utility Estimator, one inference step t for the N experts of one
 * layer (Sec. 3.2, Alg. 1).  State, updated in place: utility s_i in [0,K],
 * boundaries th_up_i, th_dn_i, and the previous frequencies f_prev_i.
 *   fluctuation          d = f_i - f_prev_i
 *   inertial transition  d >= th_up: s <- min(K, s+1);  else -d >= th_dn: s <- max(0, s-1)
 *   boundary calibration d > 0: th_up <- floor((1-lam) th_up + lam d)
 *                        d < 0: th_dn <- floor((1-lam) th_dn + lam |d|)
 * The transition uses the boundaries of step t; calibration produces those of
 * step t+1.  lam = lam_num / lam_den, floor by integer division of
 * non-negative integers.
 * ------------------------------------------------------------------------- */
void oracle_utility_step(const int32_t *f, int32_t *f_prev, int32_t *s, int32_t *th_up, int32_t *th_dn,
                         int N, int K, int lam_num, int lam_den)
{
    for (int i = 0; i < N; ++i) {
        int64_t d = (int64_t)f[i] - (int64_t)f_prev[i];
        if (d >= (int64_t)th_up[i]) {
            s[i] = s[i] + 1 < K ? s[i] + 1 : K;
        } else if (-d >= (int64_t)th_dn[i]) {
            s[i] = s[i] - 1 > 0 ? s[i] - 1 : 0;
        }
        if (d > 0) {
            th_up[i] = (int32_t)(((int64_t)(lam_den - lam_num) * th_up[i] + (int64_t)lam_num * d) / lam_den);
        } else if (d < 0) {
            th_dn[i] = (int32_t)(((int64_t)(lam_den - lam_num) * th_dn[i] + (int64_t)lam_num * (-d)) / lam_den);
        }
        f_prev[i] = f[i];
    }
}

/* n(tau) of the balancer's notation (Sec. 3.3): the number of hot experts (s_i >= tau) that are not
 * on the GPU (slot_table[i] < 0), for tau = 0..K. */
void oracle_prefetch_counts(const int32_t *s, const int32_t *slot_table, int N, int K, int32_t *n_tau)
{
    for (int tau = 0; tau <= K; ++tau) {
        int32_t n = 0;
        for (int i = 0; i < N; ++i)
            if (s[i] >= tau && slot_table[i] < 0) n += 1;
        n_tau[tau] = n;
    }
}

/* ---------------------------------------------------------------------------
 * Heterogeneous Workload Balancer for one layer (Sec. 3.3: the two time
 * equations, the objective and its three constraints; appendix "Solution
 * Derivation": fallback tau = K when nothing is feasible).
 *   b            = number of experts with f_i > 0 (de-duplicated activated experts)
 *   T_cpu(tau)   = r_c(tau) * gamma * k * t_cpu
 *   T_gpu(tau)   = r_g(tau) * b * t_gpu
 *   feasible     : t_io * n(tau) <= max(T_cpu, T_gpu) + gamma * t_draft / l_target
 *                  w_expert * n(tau) <= vram_left           (bytes, integers)
 *   tau*         = argmin over feasible tau in 1..K of |T_cpu - T_gpu|, smaller tau on ties
 * r_c, r_g, n_tau are tables indexed by tau = 0..K (entry 0 unused here).
 * t_cpu_out / t_gpu_out (K+1 doubles each, may be NULL) receive the two times.
 * Returns tau*.
 * ------------------------------------------------------------------------- */
int oracle_balance_threshold(const int32_t *f, const int32_t *n_tau, const double *r_c, const double *r_g,
                             int N, int K, int gamma, int k, double t_cpu, double t_gpu, double t_io,
                             double t_draft, int l_target, int64_t w_expert, int64_t vram_left,
                             int32_t *b_out, double *t_cpu_out, double *t_gpu_out)
{
    int b = 0;
    for (int i = 0; i < N; ++i)
        if (f[i] > 0) b += 1;
    if (b_out) *b_out = b;
    int best = -1;
    double best_f = 0.0;
    for (int tau = 1; tau <= K; ++tau) {
        double tc = ((r_c[tau] * (double)gamma) * (double)k) * t_cpu;
        double tg = (r_g[tau] * (double)b) * t_gpu;
        if (t_cpu_out) t_cpu_out[tau] = tc;
        if (t_gpu_out) t_gpu_out[tau] = tg;
        double total = tc > tg ? tc : tg;
        double window = total + ((double)gamma * t_draft) / (double)l_target;
        int io_ok = t_io * (double)n_tau[tau] <= window;
        int mem_ok = w_expert * (int64_t)n_tau[tau] <= vram_left;
        if (!io_ok || !mem_ok) continue;
        double obj = fabs(tc - tg);
        if (best < 0 || obj < best_f) {
            best = tau;
            best_f = obj;
        }
    }
    return best < 0 ? K : best;
}

/* ---------------------------------------------------------------------------
 * Cache manager, one planning step for one layer (Sec. 3.4; appendix on the
 * execution engine).  s[N]: utilities; in_use[N]: non-zero = frozen;
 * slot_table[N]: expert -> slot or -1, updated in place; C slots.
 *   evict_list  : evicted experts, ascending utility, ascending id inside a utility
 *   fetch_list  : fetched experts, descending utility (K .. tau), ascending id inside a level
 *   fetch_slot  : the slot each fetched expert receives
 * ------------------------------------------------------------------------- */
void oracle_cache_plan(const int32_t *s, const int32_t *in_use, int32_t *slot_table, int N, int C, int K,
                       int tau, int budget, int32_t *evict_list, int32_t *n_evict, int32_t *fetch_list,
                       int32_t *fetch_slot, int32_t *n_fetch)
{
    int ne = 0, nf = 0;
    /* utility-guided eviction */
    for (int level = 0; level < tau; ++level)
        for (int i = 0; i < N; ++i)
            if (slot_table[i] >= 0 && !in_use[i] && s[i] == level) evict_list[ne++] = i;
    for (int j = 0; j < ne; ++j) slot_table[evict_list[j]] = -1;
    /* free slots, ascending */
    int *slot_free = (int *)malloc((size_t)(C > 0 ? C : 1) * sizeof(int));
    for (int c = 0; c < C; ++c) slot_free[c] = 1;
    for (int i = 0; i < N; ++i)
        if (slot_table[i] >= 0 && slot_table[i] < C) slot_free[slot_table[i]] = 0;
    /* utility-guided prefetching: levels K down to tau, request order inside a level */
    int next_slot = 0;
    for (int level = K; level >= tau && level >= 0; --level) {
        for (int i = 0; i < N; ++i) {
            if (slot_table[i] >= 0 || s[i] != level) continue;
            if (nf >= budget) continue;
            while (next_slot < C && !slot_free[next_slot]) ++next_slot;
            if (next_slot >= C) continue;
            slot_free[next_slot] = 0;
            slot_table[i] = next_slot;
            fetch_list[nf] = i;
            fetch_slot[nf] = next_slot;
            ++nf;
        }
    }
    free(slot_free);
    *n_evict = ne;
    *n_fetch = nf;
}
