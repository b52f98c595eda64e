// Weight-streaming kernels of the expert FFN of a verification batch (tuned
// for the regime of a single request, gamma <= 15 draft tokens; larger batches
// take variants of the same kernels):
//      act = silu(W_gate x) * (W_up x)        (gate/up kernel)
//      o   = W_down act                       (down kernel)
// per (token, resident expert) pair -- Sec. 2.2 last line, experts as in App. D.
//
// Both kernels are bound by the bf16 weight bytes, which must come from HBM
// once per layer call.  Measured on MI355X, only loads in which a wavefront
// reads 1 KB of consecutive bytes and the wavefronts of a workgroup read
// neighbouring kilobytes reach the HBM ceiling; the MFMA operand layout read
// straight from row-major weights (16 rows x 64 B per instruction) gets about
// two thirds of it.  So a workgroup streams a tile of 16 weight rows x up to
// 2048 columns (contiguous 64 KB for H = 2048) as 1 KB pieces into registers,
// parks it in LDS, and then every wavefront multiplies ITS share of the
// contraction range (32-wide column blocks dealt round-robin) for all 16 rows
// with MFMA 16x16x32 bf16; the sixteen partial 16x16 results are added through
// LDS in a fixed order.  Tokens sit on the MFMA N axis (16 columns per group,
// zero beyond the routed ones), so the arithmetic is free and nothing is read
// twice.
//
// Work is a flat list of items (expert, tile of 16 MFMA rows) over the shared experts
// and the ACTIVE resident slots only; a fixed grid of one 16-wavefront workgroup per CU
// takes equal contiguous runs of it, so all workgroups are resident at once,
// share the HBM bandwidth evenly and finish together.  (Runs are cut at whole tiles
// on purpose: measured, a tile with fewer rows costs a workgroup as much time as a
// whole one, since its requests wait in the same queues behind everybody's whole tiles.)
#include "moe_internal.h"
#include "route_device.h"

namespace moe {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(1))) uint16_t g_u16;
typedef __attribute__((address_space(1))) float g_f32;

constexpr int kThreads = 1024;
constexpr int kWaves = 16;
constexpr int kPieces = 4;     // 1 KB pieces per wavefront per tile (64 KB tile / 16 wavefronts)
constexpr int kRowPad = kStreamRowPad;
constexpr int kOutCap = kStreamOutCap;

__device__ inline u32x4 ld_stream(const unsigned char *p)
{
    return __builtin_nontemporal_load((const u32x4 *)p);
}

__device__ inline f32x4 mfma(u32x4 a, u32x4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                   c, 0, 0, 0);
}

__device__ inline uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// One item = one expert and one tile of 16 MFMA rows:
//   gate/up kernel: gate rows f..f+7 stacked on up rows f..f+7 (so one MFMA pass yields both
//                   factors of 8 activations, and an item is 64 KB for H = 2048);
//   down kernel:    down rows h..h+15.
// Small items keep the last round of the static schedule short.
//
// NPI = 1 KB pieces each wavefront loads per tile = ceil(pieces of the widest tile / 16).  All NPI
// loads of a tile are issued unconditionally (a wavefront whose piece lies beyond the tile re-reads
// the tile's last piece and parks it on that piece's own bytes), and past the end of its run a
// workgroup keeps "loading" a few cached kilobytes, so the steady state is straight-line code:
// park tile t, put tile t+2 in flight, multiply.  That is what lets the wait before a park leave
// the younger tile in flight.  The state of the two walks over the run (the tile to load next,
// the tile being consumed) lives in plain scalars and is stepped, not recomputed.
// MODE 0: batches up to 16 tokens (one group of 16 token columns per pass); MODE 1: up to 32 tokens
// (two groups); MODE 2: larger batches: two groups per pass, and experts with more than 32 tokens
// take further passes over the parked tile.
//
// JOIN (down kernel, batches of up to 32 tokens): the weighted sum back into token order (Sec. 2.2 last
// line; the join of App. D when `accumulate` is set) rides at the end of the down kernel instead
// of a launch of its own.  Every per-assignment output goes to memory as ONE 64-bit relaxed atomic
// store (call number << 32 | fp32 bits); a workgroup that has finished its items takes a strip of 8
// output columns, reads the entries that strip needs with atomic loads until they carry this
// call's number (a bounded number of times: every other workgroup is resident and none of them
// waits before it has stored), and adds them up in a fixed order.  No counter, no fence: an entry
// with the right number IS the value.
//
//
// Built with -DMOE_STREAM_TRACE the kernel also stamps the 100 MHz wall clock at six points of every
// workgroup's life (moe_profile_stream_timeline reads them back); the product build has none of that.
#ifdef MOE_STREAM_TRACE
__device__ unsigned long long g_timeline[2][kTimelineGroups][kTimelineWords];
#define MOE_STAMP(var) var = wall_clock64()
#else
#define MOE_STAMP(var)
#endif
//
// WSPLIT (down kernel, shared experts whose items have another number of panels than the routed ones):
// the item list is cut into runs of equal numbers of TILES instead of items.
template <bool GATEUP, int NPI, int MODE, bool JOIN, bool WSPLIT, bool FUSED>
__device__ __forceinline__ void stream_body(const StreamArgs &a, const int tile_lds_bytes, const JoinArgs &jn,
                                            const RouteArgs &ra)
{
    static_assert(!WSPLIT || !GATEUP, "gate/up items all have the panels of the hidden size");
    static_assert(!FUSED || (GATEUP && MODE <= 1 && !JOIN && !WSPLIT), "the routing steps ride on the gate/up kernels of up to 32 tokens");
    static_assert(!JOIN || (!GATEUP && MODE < 2), "the join rides on the down kernel of batches up to 32 tokens");
    constexpr int NG = MODE == 0 ? 1 : 2;   // token groups of 16 multiplied per pass
    constexpr bool MULTIPASS = MODE == 2;
    constexpr int RPI = GATEUP ? 8 : 16;    // output rows per item
    constexpr int OB = GATEUP ? 2 : 4;      // bytes per output element
    constexpr int kOutPerItem = RPI * 16;   // results of one item (rows x token columns)
    // Gate/up kernel, batch within one pass: column n of the MFMA result is TOKEN n for every expert
    // (the arithmetic is free), so the B operand never changes and no expert change stalls the
    // stream; the expert's own tokens are picked out when the results are stored.
    constexpr bool ALLTOK = GATEUP && MODE == 1;

    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *tile_s = lds;
    float *red_s = (float *)(lds + tile_lds_bytes);                   // [group][wavefront][lane][4]
    int *ctl_s = (int *)(lds + tile_lds_bytes + NG * kWaves * kWave * 16);
    int *count_s = ctl_s, *offset_s = ctl_s + a.C, *active_s = ctl_s + 2 * a.C, *perm_s = ctl_s + 3 * a.C;
    float *out_s = (float *)(perm_s + a.T * a.k);                     // [kOutCap][NG][kOutPerItem] results waiting to be stored
    int *odesc_s = (int *)(out_s + kOutCap * NG * kOutPerItem);       // [kOutCap][8]: shared?, row of token 0, column bytes, m, first token

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
#ifdef MOE_STREAM_TRACE
    unsigned long long tl_start, tl_lists = 0, tl_first = 0, tl_loop = 0, tl_flush = 0;
#endif
    MOE_STAMP(tl_start);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);   // wavefront id, known to be uniform
    const int n = lane & 15, g = lane >> 4;

    // The shared experts' items need nothing from the routing step, so each workgroup takes its
    // run of them first: their weights are in flight while the slot lists are still being read.
    const int G = gridDim.x, b = blockIdx.x;
    const int tiles = a.R / RPI, tiles_sh = a.n_shared ? a.R_sh / RPI : 0;
    const int n_sh_items = a.n_shared * tiles_sh;
    const int sh_per = udiv_rcp(n_sh_items, G, a.rcp_G), sh_rem = n_sh_items - sh_per * G;
    // (FUSED: workgroup 0 also writes the step outputs and waits for every workgroup's word before it gives the
    // call its number; it takes the last place in the split, whose run is never the longer one)
    const int rk = FUSED ? (b == 0 ? G - 1 : b - 1) : b;
    const int s_cnt = sh_per + (rk < sh_rem ? 1 : 0);
    const int s_start = rk * sh_per + (rk < sh_rem ? rk : sh_rem);
    int r_start = 0, cnt = s_cnt;   // completed once the routing results are in LDS

    // ---- the walk that loads: tile (item pp, panel ppan) is the next one to put in flight ----
    const unsigned char *pw0 = nullptr, *pw1 = nullptr;   // tile rows 0..7 and 8..15, panel 0
    int pK2 = 0, prs = 0, pnpan = 1, ppan = 0;            // row stride, panel row bytes, panels, panel
    int pp = 0, pe = 0, prt = 0;                          // item of the run, expert within class, row tile
    bool psh = false, pvalid = false;
    auto prod_set = [&](bool sh, int e, int rt) {
        psh = sh; pe = e; prt = rt; ppan = 0;
        if (sh) {
            const int K = a.K_sh;
            const size_t eoff = ((size_t)e * a.R_sh + (size_t)rt * RPI) * K;
            pw0 = (const unsigned char *)(a.s0 + eoff);
            pw1 = GATEUP ? (const unsigned char *)(a.s1 + eoff) : pw0 + (size_t)16 * K;
            pK2 = 2 * K; prs = 2 * a.KP_sh; pnpan = a.np_sh;
        } else {
            const int K = a.K;
            const size_t eoff = ((size_t)active_s[e] * a.R + (size_t)rt * RPI) * K;
            pw0 = (const unsigned char *)(a.w0 + eoff);
            pw1 = GATEUP ? (const unsigned char *)(a.w1 + eoff) : pw0 + (size_t)16 * K;
            pK2 = 2 * K; prs = 2 * a.KP; pnpan = a.np;
        }
    };
    auto prod_advance = [&]() {
        if (!pvalid) return;
        if (ppan + 1 < pnpan) { ++ppan; return; }
        ppan = 0;
        ++pp;
        if (pp >= cnt) {            // end of the run: stay on a few cached kilobytes from now on
            pvalid = false;
            pK2 = 0;
            pw1 = pw0;
        } else if (pp == s_cnt) {   // from the shared experts to the routed ones
            const int e = udiv_rcp(r_start, tiles, a.rcp_tiles);
            prod_set(false, e, r_start - e * tiles);
        } else if (prt + 1 == (psh ? tiles_sh : tiles)) {
            prod_set(psh, pe + 1, 0);
        } else {
            ++prt;
            pw0 += (size_t)RPI * pK2;
            pw1 += (size_t)RPI * pK2;
        }
    };

    // ---- the walk that consumes: tile (item cp, panel cpan) is the one parked and multiplied ----
    int c_rs = 0, cK = 0, cnpan = 1, cpan = 0;
    int cp = 0, ce = 0, crt = 0;
    int cm = 0, ckey = -1, corow0 = 0, cbrow0 = 0, cocol = 0;
    bool csh = false;
    auto cons_set = [&](bool sh, int e, int rt) {
        csh = sh; ce = e; crt = rt; cpan = 0;
        cocol = rt * RPI * OB;
        if (sh) {
            cK = a.K_sh; c_rs = 2 * a.KP_sh; cnpan = a.np_sh;
            cm = a.T; ckey = ALLTOK ? 0 : e; corow0 = e * a.T;
            cbrow0 = GATEUP ? 0 : e * a.T;            // hidden[n] | act_sh[e][n]
        } else {
            const int c = active_s[e];
            cK = a.K; c_rs = 2 * a.KP; cnpan = a.np;
            cm = count_s[c]; ckey = ALLTOK ? 0 : a.n_shared + c; corow0 = offset_s[c];
            cbrow0 = ALLTOK ? 0 : GATEUP ? -1 : corow0;   // hidden[n] | hidden[token of list entry n] | act[row]
        }
    };
    auto cons_advance = [&]() {
        if (cpan + 1 < cnpan) { ++cpan; return; }
        cpan = 0;
        ++cp;
        if (cp >= cnt) return;
        if (cp == s_cnt) {
            const int e = udiv_rcp(r_start, tiles, a.rcp_tiles);
            cons_set(false, e, r_start - e * tiles);
        } else if (crt + 1 == (csh ? tiles_sh : tiles)) {
            cons_set(csh, ce + 1, 0);
        } else {
            ++crt;
            cocol += RPI * OB;
        }
    };

    // Piece i of this wavefront covers bytes [(16i+w) KB, +1 KB) of a tile seen as 16 rows of rs
    // bytes (rs a multiple of 128, so a piece lies wholly in tile rows 0..7 or 8..15 and the choice
    // between the two row pointers is uniform).  A tile of rs-byte rows has rs/64 pieces (as many as
    // it has 32-wide column blocks).  For each piece this lane keeps its global byte offset from the
    // half-tile's first row and its LDS byte offset.  Two tiles are in flight per wavefront (st[0],
    // st[1]); each remembers its own geometry.
    // (The two-group variants are short of registers: they keep row and column packed in one word
    // per piece and derive both offsets where they are used.)
    // (The variant for the largest batches and the widest tiles has none to spare at all: it works row
    // and column out again at each use rather than let the compiler spill a register that a load is writing.)
    constexpr bool PACKED = NG == 2;
    constexpr bool LEAN = MODE == 2 && NPI == 4;
    u32x4 st[2][NPI];
    unsigned goff[2][PACKED ? 1 : NPI];   // PACKED: unused
    int loff[2][LEAN ? 1 : NPI];          // PACKED: row << 16 | column; LEAN: unused
    int st_rs[2] = {-1, -1}, st_K2[2] = {-1, -1};
    auto geom = [&](int i, int rs) {      // row << 16 | column of piece i in a tile of rs-byte rows
        const int np = rs / 64;
        int pc = i * kWaves + w;
        pc = pc < np ? pc : np - 1;
        const int off = (pc << 10) + (lane << 4);
        const int row = (int)(((float)(off >> 4) + 0.5f) * (16.0f / (float)rs));
        return row << 16 | (off - row * rs);
    };
    auto issue = [&](int s) {
        if (LEAN) {
            st_rs[s] = prs;
        } else if (prs != st_rs[s] || pK2 != st_K2[s]) {
            st_rs[s] = prs;
            st_K2[s] = pK2;
            const float inv_d = 16.0f / (float)prs;
            const int np = prs / 64;
#pragma unroll
            for (int i = 0; i < NPI; ++i) {
                int pc = i * kWaves + w;
                pc = pc < np ? pc : np - 1;
                int off = (pc << 10) + (lane << 4);
                int row = (int)(((float)(off >> 4) + 0.5f) * inv_d);
                int col = off - row * prs;
                if (PACKED) {
                    loff[s][LEAN ? 0 : i] = row << 16 | col;
                } else {
                    goff[s][i] = (unsigned)((row & 7) * pK2 + col);
                    loff[s][i] = row * (prs + kRowPad) + col;
                }
            }
        }
        const unsigned poff = (unsigned)ppan * (unsigned)prs;
        const int np = prs / 64;
#pragma unroll
        for (int i = 0; i < NPI; ++i) {
            int pc = i * kWaves + w;
            pc = pc < np ? pc : np - 1;
            const unsigned char *base = (pc << 10) < 8 * prs ? pw0 : pw1;   // uniform
            const int rc = LEAN ? geom(i, prs) : loff[s][LEAN ? 0 : i];
            const unsigned go = PACKED ? (unsigned)(((rc >> 16) & 7) * pK2 + (rc & 0xffff)) : goff[s][PACKED ? 0 : i];
            st[s][i] = ld_stream(base + (poff + go));
        }
    };
    auto park = [&](int s) {
        // (a wavefront's re-read of the last piece lands on that piece's own bytes: same data, no test)
#pragma unroll
        for (int i = 0; i < NPI; ++i) {
            const int rc = LEAN ? geom(i, st_rs[s]) : loff[s][LEAN ? 0 : i];
            const int lo = PACKED ? (rc >> 16) * (st_rs[s] + kRowPad) + (rc & 0xffff) : rc;
            *(u32x4 *)(tile_s + lo) = st[s][i];
        }
    };

    u32x4 bx[NG][kPieces];
    int bx_key = -1, bx_panel = -1;   // expert (and panel) whose FIRST token pass the registers hold

    // B operand of this wavefront's column blocks for the token pass starting at token tok0:
    // token tok0 + 16*gr + n sits on column n of group gr.  Drains every load in flight (rare path), unless
    // told to leave the wait to the caller.
    auto load_bx = [&](int tok0, bool wait = true) {
        const int nkb = c_rs / 64;
        const uint16_t *bbase = a.bsrc;
        if (!GATEUP && csh) bbase = a.bsrc_sh;
#pragma unroll
        for (int gr = 0; gr < NG; ++gr) {
            const int tk = tok0 + 16 * gr + n;
            int boff = -1;
            if (tk < (ALLTOK ? a.T : cm))
                boff = (cbrow0 >= 0 ? cbrow0 + tk : perm_s[corow0 + tk]) * cK + cpan * (c_rs / 2);
#pragma unroll
            for (int j = 0; j < kPieces; ++j) {
                int kb = w + kWaves * j;
                bx[gr][j] = (u32x4){0u, 0u, 0u, 0u};
                if (kb < nkb && boff >= 0) bx[gr][j] = *(const u32x4 *)(bbase + (unsigned)(boff + kb * 32 + g * 8));
            }
        }
        if (wait) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    };
    // A shared expert's item needs nothing from the routing step, not even for its B operand (every token,
    // in token order): tile and operand are requested here, and are there by the time the lists are.
    // (FUSED: after the dot products of the routing step have their own loads on the way, not before: behind a
    // tile per workgroup those loads, which everything else waits for, take twice as long)
    bool bx_early = false;
    auto first_shared_item = [&]() {
        if (s_cnt == 0) return;
        const int e = udiv_rcp(s_start, tiles_sh, a.rcp_tiles_sh);
        prod_set(true, e, s_start - e * tiles_sh);
        cons_set(true, e, s_start - e * tiles_sh);
        pvalid = true;
        issue(0);
        load_bx(0, false);
        bx_key = ckey;
        bx_panel = cpan;
        bx_early = true;
    };
    if (!FUSED) first_shared_item();
    // FUSED: steps 1-3 of the layer inside this launch (Sec. 2.2, 2.3, App. D).  Every workgroup computes its
    // share of the T*E dot products and stores each logit, stamped with the call's number, into kLogitReplicas
    // copies; then EVERY workgroup waits for all logits in one of the copies, ranks them and builds the per-slot
    // lists for itself in LDS (the same arithmetic on the same numbers everywhere; workgroup 0 also writes the
    // step outputs to memory).  One hand-over through memory instead of two: the lists are not passed on.
    unsigned rtag = 0, rwtag = 0;
    int rspin = kSpinLimit;
    int n_act = 0;
    if (FUSED) {
        const int T = ra.T, H = ra.H, E = ra.E, TE = T * E, A = T * ra.k, C = ra.C;
        rtag = *ra.epoch + 1u;
        // (two words of the control block that only a test sets: the bound of the polls, and a number added to
        // what producers stamp their entries with, so that the host can make every wait run out)
        rwtag = rtag + (ra.epoch - kCtrlEpoch)[kCtrlSkew];
        if (b == 0 && tid == 0) check_layout(ra.epoch - kCtrlEpoch, ra.layout);
        if ((ra.epoch - kCtrlEpoch)[kCtrlSpin]) rspin = (int)(ra.epoch - kCtrlEpoch)[kCtrlSpin];
        const size_t n_pub = list_pub_entries(T, ra.k, C);
        // (workgroup 0 gives the call its number in the control block only when every workgroup has read the
        // old one: each says so with a stamped word of its own)
        unsigned long long *const seen = ra.lists_pub + (size_t)kListReplicas * n_pub;
        if (tid == 0)
            __hip_atomic_store(seen + b, ((unsigned long long)rtag << 32) | 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int tab_v = -1;
        if (tid < E) tab_v = ra.slot_table[tid];
        const uint16_t *x = (const uint16_t *)ra.hidden;
        for (int q = b + w * G; q < TE; q += G * kWaves) {
            const int t = q / E, e = q - t * E;
            const float *wrow = ra.router_w + (size_t)e * H;
            const uint16_t *xr = x + (size_t)t * H;
            const float bias = ra.router_bias ? ra.router_bias[e] : 0.f;
            float dot = 0.f;
#pragma unroll 8
            for (int h = lane * 4; h < H; h += kWave * 4) {
                const float4 wv = *(const float4 *)(wrow + h);
                const uint2 xv = *(const uint2 *)(xr + h);
                dot += wv.x * bf16_lo(xv.x) + wv.y * bf16_hi(xv.x) + wv.z * bf16_lo(xv.y) + wv.w * bf16_hi(xv.y);
            }
#pragma unroll
            for (int m = kWave / 2; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, kWave);
            dot += bias;
            // lane r: the copy that the workgroups with b % kLogitReplicas == r read
            if (lane < kLogitReplicas)
                __hip_atomic_store(ra.tagged_logits + (size_t)lane * TE + q,
                                   ((unsigned long long)rwtag << 32) | __float_as_uint(dot), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0 && ra.logits_opt) ra.logits_opt[q] = dot;
        }
        first_shared_item();
        {
            // one wavefront per token ranks its logits; then histogram, slot lookup, miss list and per-slot lists
            // out of LDS (which nothing else uses yet: the first tile is still on its way)
            PostLds L = carve_lds((int *)lds, E, C, A);
            if (tid < E) {
                L.tab_s[tid] = tab_v;
                L.hist_s[tid] = 0;
            }
            for (int i = tid; i < C * ((T + 31) >> 5); i += kThreads) L.cnt_s[i] = 0;
            lds_f32 *lg = L.lg_s + w * lg_stride(E);
            for (int t = w; t < T; t += kWaves) {   // (one token per wavefront up to 16 tokens, two up to 32)
                const unsigned long long *src = ra.tagged_logits + (size_t)(b % kLogitReplicas) * TE + (size_t)t * E;
                for (int e0 = 0; e0 < E; e0 += kWave) {
                    const int e = e0 + lane;
                    unsigned long long v = (unsigned long long)rtag << 32;
                    int polls = 0;
                    for (;;) {
                        if (e < E) v = __hip_atomic_load(src + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if (__ballot((unsigned)(v >> 32) != rtag) == 0ull) break;
                        if (++polls > rspin) {   // cannot happen on a healthy device; never wait for ever
                            if (lane == 0) atomicOr(ra.error_flag, 1u);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                    if (e < E) {
                        const float f = __uint_as_float((unsigned)v);
                        lg[e] = (f == f) ? f : -INFINITY;
                    }
                }
                __builtin_amdgcn_wave_barrier();
                // (up to 128 experts here: the ranking of more needs so many registers that the whole
                // kernel would be launched with scratch memory; those batches keep the routing kernel)
                int32_t *const idx_out = b == 0 ? ra.topk_idx + (size_t)t * ra.k : nullptr;
                float *const w_out = b == 0 ? ra.topk_w + (size_t)t * ra.k : nullptr;
                if (E <= kWave)
                    wave_topk_gate_n<1>(E, ra.k, idx_out, L.idx_s + t * ra.k, w_out, lg);
                else
                    wave_topk_gate_n<2>(E, ra.k, idx_out, L.idx_s + t * ra.k, w_out, lg);
            }
            __syncthreads();
            const SmallLists sl = block_post_small<false>(L.idx_s, L.tab_s, T, ra.k, E, C, ra, L.hist_s, L.cnt_s, L.scan_s,
                                                          L.off_s, rwtag, b == 0);
            __syncthreads();   // (the lists' places below may lie where the ranking kept its own data)
            if (tid < C) {
                count_s[tid] = sl.count;
                offset_s[tid] = sl.offset;
                if (sl.active_rank >= 0) active_s[sl.active_rank] = tid;
                if (tid >= sl.n_active) active_s[tid] = 0;       // (never used; stay inside the pool)
            }
            if (tid < A) {
                if (sl.pos >= 0) perm_s[sl.pos] = tid / ra.k;    // token of each list entry
                if (tid >= sl.n_listed) perm_s[tid] = 0;
            }
            n_act = sl.n_active;
            if (b == 0) {
                for (int i = tid; i < G; i += kThreads) {
                    int polls = 0;
                    while ((unsigned)(__hip_atomic_load(seen + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32) != rtag) {
                        if (++polls > rspin) {
                            atomicOr(ra.error_flag, 1u);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
            }
            __syncthreads();
            if (b == 0 && tid == 0) *ra.epoch = rtag;
        }
    }
    if (FUSED) {
        // (the lists are in LDS already)
    } else {
        // one trip to memory for everything the routing step left behind
        for (int i = tid; i < a.C; i += kThreads) {
            count_s[i] = a.slot_count[i];
            offset_s[i] = a.slot_offset[i];
            active_s[i] = a.active_slots[i];
        }
        // token of each list entry (gate/up) | row of each assignment's output, -1 = not resident (join)
        if (GATEUP)
            for (int i = tid; i < a.T * a.k; i += kThreads) perm_s[i] = udiv_rcp(a.perm[i], a.k, a.rcp_k);
        else if (JOIN)
            for (int i = tid; i < a.T * a.k; i += kThreads) perm_s[i] = jn.pos[i];
        n_act = (int)(*a.n_active);
        __syncthreads();
    }

    // equal runs of the whole item list; this workgroup's run = its shared items, then routed ones
    if (!WSPLIT) {
        const int total = n_sh_items + n_act * tiles;
        const int per = udiv_rcp(total, G, a.rcp_G), rem = total - per * G;
        cnt = per + (rk < rem ? 1 : 0);
        r_start = rk * per + (rk < rem ? rk : rem) - s_start;
    } else {
        // Workgroup x starts at routed item max(0, x * total tiles / G - tiles of the shared items
        // before x) / panels per routed item: that never decreases with x, is 0 for x = 0 and the
        // number of routed items for x = G.
        const int np_r = a.np, np_sh = a.np_sh;
        const int n_routed = n_act * tiles;
        const long long total = (long long)n_sh_items * np_sh + (long long)n_routed * np_r;
        auto routed_before = [&](int x) {
            const long long sh = (long long)(x * sh_per + (x < sh_rem ? x : sh_rem)) * np_sh;
            const long long rt = (long long)x * total / G - sh;
            const long long r = rt > 0 ? rt / np_r : 0;
            return (int)(r < n_routed ? r : n_routed);
        };
        r_start = routed_before(b);
        cnt = s_cnt + routed_before(b + 1) - r_start;
    }
    MOE_STAMP(tl_lists);
    const unsigned tag = JOIN ? *jn.epoch : 0u;   // number of this call (set by the routing / list kernel)
    // (two words of the control block that only a test sets: the bound of the polls, and a number added to what
    // producers stamp their entries with, so that the host can make every wait run out)
    const unsigned wtag = JOIN ? tag + (jn.epoch - kCtrlEpoch)[kCtrlSkew] : 0u;
    const int jspin = JOIN && (jn.epoch - kCtrlEpoch)[kCtrlSpin] ? (int)(jn.epoch - kCtrlEpoch)[kCtrlSpin] : kSpinLimit;
    auto join = [&]() {
        if (!JOIN) return;
        typedef unsigned long long u64;
        const int S = a.k + a.n_shared, nent = a.T * 8 * S;
        float *val_s = (float *)tile_s;   // [token][column of the strip][source]; the tile buffer is free by now
        float *gw_s = red_s;              // gate weights, on their way while the entries are waited for
        for (int i = tid; i < a.T * a.k; i += kThreads) gw_s[i] = jn.topk_w[i];
        // set by a thread whose wait ran out: the last word of the partial-sum buffer, which nobody reads any more
        // (not a word of the result descriptors: other wavefronts may still be storing the last batch from them)
        int *gave_up_s = (int *)red_s + NG * kWaves * kWave * 4 - 1;
        if (tid == 0) *gave_up_s = 0;
        for (int u = b; u < a.R / 8; u += G) {
            __syncthreads();
            for (int i = tid; i < nent; i += kThreads) {
                const int tc = udiv_rcp(i, S, a.rcp_S), src = i - tc * S, t = tc >> 3, col = u * 8 + (tc & 7);
                const u64 *p = nullptr;
                if (src < a.k) {
                    const int row = perm_s[t * a.k + src];
                    if (row >= 0) p = (const u64 *)a.out + (size_t)row * a.R + col;
                } else {
                    p = (const u64 *)a.out_sh + ((size_t)(src - a.k) * a.T + t) * a.R_sh + col;
                }
                float v = 0.f;   // an assignment whose expert is not resident adds nothing here
                if (p) {
                    u64 x = 0;
                    int polls = 0;
                    for (;;) {
                        x = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if ((unsigned)(x >> 32) == tag) break;
                        if (++polls > jspin) {   // cannot happen with the whole grid resident; never wait for ever
                            atomicOr(jn.error_flag, 1u);
                            *gave_up_s = 1;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    v = __uint_as_float((unsigned)x);
                }
                val_s[i] = v;
            }
            // a wait ran out, here or (the control block says so) anywhere in this call: what is written is not a result
            __syncthreads();
            const bool poisoned = *gave_up_s != 0 ||
                                  __hip_atomic_load(jn.error_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
            if (poisoned && tid == 0 && jn.miss_count)
                __hip_atomic_store(jn.miss_count, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (tid < a.T * 8) {
                const int t = tid >> 3, col = u * 8 + (tid & 7);
                const size_t o = (size_t)t * a.R + col;
                float acc = 0.f;
                if (jn.accumulate)
                    acc = jn.out_bf16 ? __uint_as_float((uint32_t)((const uint16_t *)jn.out)[o] << 16)
                                      : ((const float *)jn.out)[o];
                for (int jj = 0; jj < a.k; ++jj) acc += gw_s[t * a.k + jj] * val_s[tid * S + jj];
                for (int i = 0; i < a.n_shared; ++i) acc += val_s[tid * S + a.k + i];
                if (poisoned) acc = __uint_as_float(0x7fc00000u);
                if (jn.out_bf16) ((uint16_t *)jn.out)[o] = (uint16_t)f32_to_bf16_rne(acc);
                else ((float *)jn.out)[o] = acc;
            }
        }
    };
    if (cnt == 0) {
        join();
        return;
    }
    const int ntiles = s_cnt * (a.n_shared ? a.np_sh : 0) + (cnt - s_cnt) * a.np;
    if (s_cnt == 0) {
        const int e = udiv_rcp(r_start, tiles, a.rcp_tiles);
        prod_set(false, e, r_start - e * tiles);
        cons_set(false, e, r_start - e * tiles);
        pvalid = true;
        issue(0);
    }

    f32x4 acc[NG];
    int orec = 0, flushed = 0;   // output records written to / flushed from the LDS output buffer

    auto multiply = [&]() {
        const int nkb = c_rs / 64;
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            int kb = w + kWaves * j;
            if (kb < nkb) {
                u32x4 av = *(const u32x4 *)(tile_s + n * (c_rs + kRowPad) + kb * 64 + g * 16);
#pragma unroll
                for (int gr = 0; gr < NG; ++gr) acc[gr] = mfma(av, bx[gr][j], acc[gr]);
            }
        }
    };

    // Results wait in LDS and leave in batches: a store in the steady state would make every
    // later wait on the weight loads a wait for everything (loads and stores share one counter).
    auto flush = [&](bool resume = true) {
        // one wavefront per waiting record, so the whole batch leaves in one round of stores
        for (int r = flushed + w; r < orec; r += kWaves) {
            const int slot = r % kOutCap;
            const int *d = odesc_s + slot * 8;
#pragma unroll
            for (int i = lane; i < NG * kOutPerItem; i += kWave) {
                const int gr = i / kOutPerItem, q = i - gr * kOutPerItem;
                const int tok = d[4] + 16 * gr + ((q >> 2) & 15), row = 4 * (q >> 6) + (q & 3);
                if (tok < d[3]) {
                    int src = i;
                    if (ALLTOK && !d[0]) {   // entry `tok` of the expert's list: its token's column
                        const int t = perm_s[d[1] + tok];
                        src = (t >> 4) * kOutPerItem + ((q >> 6) << 6 | (t & 15) << 2 | (q & 3));
                    }
                    const float v = out_s[slot * (NG * kOutPerItem) + src];
                    // explicit global stores (a generic-pointer store would count as an LDS access too)
                    if (JOIN) {
                        // (call number, value) as one 64-bit entry; d[2] / OB = first column of the item
                        const unsigned long long e = ((unsigned long long)wtag << 32) | __float_as_uint(v);
                        if (d[0])
                            __hip_atomic_store((unsigned long long *)a.out_sh + (size_t)(d[1] + tok) * a.R_sh +
                                                   (d[2] / OB + row), e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        else
                            __hip_atomic_store((unsigned long long *)a.out + (size_t)(d[1] + tok) * a.R +
                                                   (d[2] / OB + row), e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    } else if (d[0]) {
                        unsigned char *orow = (unsigned char *)a.out_sh + (size_t)(d[1] + tok) * (a.R_sh * OB) + d[2];
                        if (GATEUP) ((g_u16 *)(uintptr_t)orow)[row] = (uint16_t)f32_to_bf16_rne(v);
                        else ((g_f32 *)(uintptr_t)orow)[row] = v;
                    } else {
                        unsigned char *orow = (unsigned char *)a.out + (size_t)(d[1] + tok) * (a.R * OB) + d[2];
                        if (GATEUP) ((g_u16 *)(uintptr_t)orow)[row] = (uint16_t)f32_to_bf16_rne(v);
                        else ((g_f32 *)(uintptr_t)orow)[row] = v;
                    }
                }
            }
        }
        flushed = orec;
        if (resume) __builtin_amdgcn_s_waitcnt(0);   // every counter to zero: the stores are done before streaming resumes
    };

    // The sixteen partial 16x16 results of each token group (already posted in red_s, barrier passed),
    // added in wavefront order.  Element q = lane*4 + j of the MFMA result layout is token (q/4)%16,
    // tile row 4*(q/64) + q%4; gate rows are tile rows 0..7 and the up row of the same activation
    // sits 128 elements further on.
    auto reduce_to_record = [&](int tok0) {
        const int slot = orec % kOutCap;
        if (tid < NG * kOutPerItem) {
            const int gr = tid / kOutPerItem, q = tid - gr * kOutPerItem;
            const float *r = red_s + gr * (kWaves * kWave * 4);
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int v = 0; v < kWaves; ++v) {
                s0 += r[v * kWave * 4 + q];
                if (GATEUP) s1 += r[v * kWave * 4 + q + 128];
            }
            out_s[slot * (NG * kOutPerItem) + tid] = GATEUP ? s0 / (1.f + expf(-s0)) * s1 : s0;
        }
        if (tid == 0) {
            int *d = odesc_s + slot * 8;
            d[0] = csh ? 1 : 0; d[1] = corow0; d[2] = cocol; d[3] = cm; d[4] = tok0;
        }
        ++orec;
    };
    auto post_partials = [&]() {
#pragma unroll
        for (int gr = 0; gr < NG; ++gr) *(f32x4 *)(red_s + ((gr * kWaves + w) * kWave + lane) * 4) = acc[gr];
    };

    // one tile: refresh the B operand if the expert changed, park the tile, put the tile two steps
    // ahead in flight, multiply, and on the item's last panel reduce into the output buffer
    auto step = [&](int s) {
        if (bx_key != ckey || bx_panel != cpan) {
            load_bx(0);
            bx_key = ckey;
            bx_panel = cpan;
        }
        park(s);
        issue(s);
        prod_advance();
        __syncthreads();
        if (cpan == 0) {
#pragma unroll
            for (int gr = 0; gr < NG; ++gr) acc[gr] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        multiply();
        const bool last_panel = cpan + 1 == cnpan;
        if (last_panel) post_partials();
        __syncthreads();   // every wavefront is done with the tile in LDS (and its partial result is posted)
        if (last_panel) {
            reduce_to_record(0);
            // more tokens than one pass holds (only reached with a single panel per item): the tile
            // stays parked while further passes reload the B operand
            for (int tok0 = 16 * NG; MULTIPASS && tok0 < cm; tok0 += 16 * NG) {
                if (orec - flushed == kOutCap) { __syncthreads(); flush(); }
                load_bx(tok0);
                bx_key = -1;
#pragma unroll
                for (int gr = 0; gr < NG; ++gr) acc[gr] = (f32x4){0.f, 0.f, 0.f, 0.f};
                multiply();
                __syncthreads();   // the previous pass has been reduced: red_s is free again
                post_partials();
                __syncthreads();
                reduce_to_record(tok0);
            }
        }
        cons_advance();
        if (last_panel && orec - flushed == kOutCap) {
            __syncthreads();
            flush();
        }
    };

    // The first B operand and the second tile are requested together, as soon as the lists say where they
    // are; the wait that follows leaves exactly the second tile's NPI loads in flight (loads complete in
    // order: the first tile and the B operand are there when it ends).  Waiting for the B operand before
    // the second tile is requested would leave the memory system with one tile per workgroup for the
    // two to three microseconds of that round trip.
    if (!bx_early) {
        load_bx(0, false);
        bx_key = ckey;
        bx_panel = cpan;
    }
    prod_advance();
    issue(1);
    prod_advance();
    static_assert(NPI >= 1 && NPI <= 4, "the wait below names the number of loads of one tile");
    __builtin_amdgcn_s_waitcnt(0x0F70 | NPI);   // vmcnt(NPI)

    // (first tile peeled off so that the loop is always entered in the same state: the compiler then
    // counts the loads in flight exactly and each park waits for its own tile only)
    step(0);
    MOE_STAMP(tl_first);
    int t = 1;
    for (; t + 1 < ntiles; t += 2) {
        step(1);
        step(0);
    }
    if (t < ntiles) step(1);
    MOE_STAMP(tl_loop);
    __syncthreads();
    flush(false);
    MOE_STAMP(tl_flush);
    join();
#ifdef MOE_STREAM_TRACE
    if (tid == 0 && blockIdx.x < kTimelineGroups) {
        unsigned long long *tl = g_timeline[GATEUP ? 0 : 1][blockIdx.x];
        tl[0] = tl_start; tl[1] = tl_lists; tl[2] = tl_first; tl[3] = tl_loop; tl[4] = tl_flush; tl[5] = wall_clock64();
        tl[6] = (unsigned long long)cnt; tl[7] = (unsigned long long)ntiles;
    }
#endif
}

template <bool GATEUP, int NPI, int MODE, bool JOIN, bool WSPLIT = false>
__global__ __launch_bounds__(kThreads) void stream_kernel(StreamArgs a, int tile_lds_bytes, JoinArgs jn)
{
    const RouteArgs none = {};
    stream_body<GATEUP, NPI, MODE, JOIN, WSPLIT, false>(a, tile_lds_bytes, jn, none);
}

// The small-batch gate/up kernel with steps 1-3 of the layer in front of it (one launch less per layer, and the
// shared experts' weights stream while the routing runs).
template <int NPI, int MODE>
__global__ __launch_bounds__(kThreads) void routed_stream_kernel(StreamArgs a, int tile_lds_bytes, RouteArgs ra)
{
    const JoinArgs none = {};
    stream_body<true, NPI, MODE, false, false, true>(a, tile_lds_bytes, none, ra);
}

// out[t,:] (+)= sum_j w[t,j] * o[pos[t,j],:] + sum_i o_sh[i,t,:], in a fixed order
__global__ __launch_bounds__(128) void combine_rows_kernel(CombineArgs a, const float *o, const float *o_sh)
{
    const int t = blockIdx.y;
    const int h = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (h >= a.H) return;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (a.accumulate) {
        if (a.out_bf16) {
            u32x2 v = *(const u32x2 *)((const uint16_t *)a.out + (size_t)t * a.H + h);
            acc = (f32x4){__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                          __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u)};
        } else {
            acc = *(const f32x4 *)((const float *)a.out + (size_t)t * a.H + h);
        }
    }
#pragma unroll 8
    for (int j = 0; j < a.k; ++j) {
        int p = a.pos[(size_t)t * a.k + j];
        if (p >= 0) acc += a.topk_w[(size_t)t * a.k + j] * *(const f32x4 *)(o + (size_t)p * a.H + h);
    }
    for (int i = 0; i < a.n_shared; ++i) acc += *(const f32x4 *)(o_sh + ((size_t)i * a.T + t) * a.H + h);
    // a bounded wait of an earlier kernel of this call ran out: what would be written is not a result
    if (a.error_flag && *a.error_flag != 0u) {
        const float qnan = __uint_as_float(0x7fc00000u);
        acc = (f32x4){qnan, qnan, qnan, qnan};
        if (a.miss_count && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *a.miss_count = -1;
    }
    if (a.out_bf16) {
        u32x2 v = {f32_to_bf16_rne(acc[0]) | (f32_to_bf16_rne(acc[1]) << 16),
                   f32_to_bf16_rne(acc[2]) | (f32_to_bf16_rne(acc[3]) << 16)};
        *(u32x2 *)((uint16_t *)a.out + (size_t)t * a.H + h) = v;
    } else {
        *(f32x4 *)((float *)a.out + (size_t)t * a.H + h) = acc;
    }
}



}  // namespace

int stream_panel_width(int K)
{
    // equal panels, each a multiple of 64 columns (128 bytes: a tile's 1 KB pieces must not straddle the middle of
    // the tile, as for whole rows) and at most kPanelMax columns wide
    if (K < 64) return 0;
    for (int np = (K + kPanelMax - 1) / kPanelMax; np <= K / 64; ++np)
        if (K % np == 0 && (K / np) % 64 == 0) return K / np;
    return 0;
}

bool stream_can_join(const StreamArgs &d)
{
    // up to 32 tokens: the 64-bit entries double the bytes of the per-assignment outputs (12.6 MB written
    // and read back at 128 tokens, H = 2048).  Measured per layer against the separate launch, with the
    // entries of a strip requested eight per thread at a time: no difference at 33 and 64 tokens, 4.6 us
    // more at 128 (and that batched form cost the small batches 0.4-1 us).  The strip's entries fit the tile buffer.
    const size_t tile = (size_t)16 * (2 * (d.KP > d.KP_sh ? d.KP : d.KP_sh) + kRowPad);
    return d.T <= 32 && d.R % 8 == 0 && (size_t)d.T * 8 * (d.k + d.n_shared) * 4 <= tile;
}

namespace {
// the fields of StreamArgs that follow from the others and from the grid
void fill_derived(StreamArgs &x, bool gateup, int grid)
{
    const int rpi = gateup ? 8 : 16;
    x.np = x.KP > 0 ? x.K / x.KP : 1;
    x.np_sh = x.n_shared > 0 && x.KP_sh > 0 ? x.K_sh / x.KP_sh : 1;
    x.rcp_G = rcp32((unsigned)grid);
    x.rcp_tiles = rcp32((unsigned)(x.R / rpi));
    x.rcp_tiles_sh = rcp32((unsigned)(x.n_shared > 0 ? x.R_sh / rpi : 1));
    x.rcp_k = rcp32((unsigned)x.k);
    x.rcp_S = rcp32((unsigned)(x.k + x.n_shared));
}
}  // namespace

hipError_t launch_stream(const StreamArgs &a, bool gateup, const JoinArgs *join, hipStream_t s)
{
    if (join && (gateup || !stream_can_join(a))) return hipErrorInvalidValue;
    const int kp_max = a.KP > a.KP_sh ? a.KP : a.KP_sh;
    const size_t tile = (size_t)16 * (2 * kp_max + kRowPad);
    const size_t lds = stream_lds_need(kp_max, a.T, a.k, a.C, gateup);
    if (lds > (size_t)kLdsBytes) return hipErrorInvalidValue;
    const int npi = (kp_max / 32 + kWaves - 1) / kWaves;   // 1..4 pieces per wavefront and tile
    const int mode = a.T > 32 ? 2 : a.T > 16 ? 1 : 0;
#define MOE_STREAM_FN(GU, N)                                                                     \
    {(const void *)stream_kernel<GU, N, 0, false>, (const void *)stream_kernel<GU, N, 1, false>, \
     (const void *)stream_kernel<GU, N, 2, false>}
#define MOE_JOIN_FN(N) {(const void *)stream_kernel<false, N, 0, true>, (const void *)stream_kernel<false, N, 1, true>}
    static const void *const join_fns[4][2] = {MOE_JOIN_FN(1), MOE_JOIN_FN(2), MOE_JOIN_FN(3), MOE_JOIN_FN(4)};
#undef MOE_JOIN_FN
    // down kernel, runs of equal numbers of tiles
#define MOE_WSPLIT_FN(N)                                                                                       \
    {(const void *)stream_kernel<false, N, 0, false, true>, (const void *)stream_kernel<false, N, 1, false, true>, \
     (const void *)stream_kernel<false, N, 2, false, true>}
#define MOE_WSPLIT_JOIN_FN(N) \
    {(const void *)stream_kernel<false, N, 0, true, true>, (const void *)stream_kernel<false, N, 1, true, true>}
    static const void *const wsplit_fns[4][3] = {MOE_WSPLIT_FN(1), MOE_WSPLIT_FN(2), MOE_WSPLIT_FN(3), MOE_WSPLIT_FN(4)};
    static const void *const wsplit_join_fns[4][2] = {MOE_WSPLIT_JOIN_FN(1), MOE_WSPLIT_JOIN_FN(2), MOE_WSPLIT_JOIN_FN(3),
                                                      MOE_WSPLIT_JOIN_FN(4)};
#undef MOE_WSPLIT_FN
#undef MOE_WSPLIT_JOIN_FN
    static const void *const fns[2][4][3] = {
        {MOE_STREAM_FN(false, 1), MOE_STREAM_FN(false, 2), MOE_STREAM_FN(false, 3), MOE_STREAM_FN(false, 4)},
        {MOE_STREAM_FN(true, 1), MOE_STREAM_FN(true, 2), MOE_STREAM_FN(true, 3), MOE_STREAM_FN(true, 4)}};
#undef MOE_STREAM_FN
    const bool wsplit = !gateup && a.n_shared > 0 && a.KP_sh > 0 && a.K_sh / a.KP_sh != a.K / a.KP;
    const void *fn = join ? join_fns[npi - 1][mode] : fns[gateup ? 1 : 0][npi - 1][mode];
    if (wsplit) fn = join ? wsplit_join_fns[npi - 1][mode] : wsplit_fns[npi - 1][mode];
    hipError_t e = allow_full_lds(fn);
    if (e != hipSuccess) return e;
    const int grid = device_cus(&e);
    if (e != hipSuccess) return e;
    int tile_i = (int)tile;
    StreamArgs args = a;
    fill_derived(args, gateup, grid);
    JoinArgs jargs = {};
    if (join) jargs = *join;
    void *params[] = {&args, &tile_i, &jargs};
    hipError_t le = launch_timed(fn, dim3(grid), dim3(kThreads), params, lds, s, gateup ? 2 : 4);
    if (le != hipSuccess) return le;
    return hipGetLastError();
}

hipError_t launch_stream_routed(const StreamArgs &a, const RouteArgs &r, hipStream_t s)
{
    if (!r.lists_pub || a.T > 32) return hipErrorInvalidValue;
    const int kp_max = a.KP > a.KP_sh ? a.KP : a.KP_sh;
    const size_t tile = (size_t)16 * (2 * kp_max + kRowPad);
    size_t lds = stream_lds_need(kp_max, a.T, a.k, a.C, true);
    const size_t lds_route = post_lds_bytes(r.E, r.C, r.T * r.k, true);
    lds = lds > lds_route ? lds : lds_route;
    if (lds > (size_t)kLdsBytes) return hipErrorInvalidValue;
    const int npi = (kp_max / 32 + kWaves - 1) / kWaves;
    static const void *const fns[2][4] = {
        {(const void *)routed_stream_kernel<1, 0>, (const void *)routed_stream_kernel<2, 0>,
         (const void *)routed_stream_kernel<3, 0>, (const void *)routed_stream_kernel<4, 0>},
        {(const void *)routed_stream_kernel<1, 1>, (const void *)routed_stream_kernel<2, 1>,
         (const void *)routed_stream_kernel<3, 1>, (const void *)routed_stream_kernel<4, 1>}};
    const void *fn = fns[a.T > 16 ? 1 : 0][npi - 1];
    hipError_t e = allow_full_lds(fn);
    if (e != hipSuccess) return e;
    const int grid = device_cus(&e);
    if (e != hipSuccess) return e;
    int tile_i = (int)tile;
    StreamArgs args = a;
    fill_derived(args, true, grid);
    RouteArgs rargs = r;
    void *params[] = {&args, &tile_i, &rargs};
    hipError_t le = launch_timed(fn, dim3(grid), dim3(kThreads), params, lds, s, 2);
    if (le != hipSuccess) return le;
    return hipGetLastError();
}

hipError_t read_stream_timeline(void *dst, size_t bytes)
{
#ifdef MOE_STREAM_TRACE
    if (bytes != sizeof(g_timeline)) return hipErrorInvalidValue;
    return hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_timeline), sizeof(g_timeline));
#else
    (void)dst; (void)bytes;
    return hipErrorNotSupported;
#endif
}

hipError_t launch_combine_rows(const CombineArgs &a, const float *o, const float *o_sh, hipStream_t s)
{
    dim3 grid((a.H / 4 + 127) / 128, a.T);
    CombineArgs args = a;
    void *params[] = {&args, &o, &o_sh};
    hipError_t e = launch_timed((const void *)combine_rows_kernel, grid, dim3(128), params, 0, s, 3);
    return e != hipSuccess ? e : hipGetLastError();
}

}  // namespace moe
