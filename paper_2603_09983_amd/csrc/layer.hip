// The expert FFN of a small verification batch (up to 16 tokens: a single request with gamma <= 15 draft
// tokens) as ONE weight stream per layer call:
//      act = silu(W_gate x) * (W_up x)      per (token, resident expert) pair and per shared expert
//      o   = W_down act
//      y_t = sum_j g_{t,j} o_{t,j} + sum_shared o        -- Sec. 2.2 last line, experts as in App. D,
// optionally with steps 1-3 of the layer (logits, Top-k, gate, histogram, slot lookup, miss list, per-slot
// lists: Sec. 2.2 lines 1-3, Sec. 2.3, App. D) at its head.
//
// Why one launch: a launch that streams a few hundred megabytes pays about 5 us before the memory system
// delivers at its steady rate, 2-4 us between its first and its last workgroup leaving the loop, and 1.4 us
// until the next launch starts.  Here the gate/up tiles and the down tiles of a workgroup form ONE list; the
// walk that requests tiles runs two tiles ahead of the walk that multiplies them and crosses from the gate/up
// part into the down part without a pause, so the W_down tiles are in flight while the last gate/up tiles are
// still being multiplied, and a workgroup that is early at the end of its gate/up part simply goes on.
//
// What the down part needs from OTHER workgroups is the activation of an expert.  Every activation leaves the
// workgroup that computed it as ONE 64-bit relaxed atomic store at agent scope: (call number << 32 | two bf16
// values).  An entry that carries the call's number IS the value, so the hand-over needs no counter, no
// release fence (an L2 write-back) and no acquire fence (an L2 invalidate); the reader polls a bounded number
// of times.  The per-assignment outputs go to the final sum the same way ((call number, fp32) entries), and
// every workgroup ends by summing a strip of output columns in a fixed order (no float atomics: the result does
// not depend on scheduling).
//
// Results are stored by the threads that reduce them, item by item.  The memory counter of a wavefront
// counts loads and stores in order, so a store between two tile requests never holds back an older tile, and
// the younger tile is only waited for two steps later, when the store has long been acknowledged.
//
// The tile mechanics are those of the two-launch streaming kernels (stream.hip): a workgroup of 16 wavefronts
// reads a tile of 16 weight rows as 1 KB contiguous pieces into registers, two tiles in flight, parks it in
// LDS, and every wavefront multiplies its 32-wide column blocks for all 16 rows with MFMA 16x16x32 bf16,
// tokens on the N axis.  In the gate/up part column n is TOKEN n for every expert (the arithmetic is free), so
// the B operand never changes there; the expert's own tokens are picked out when the results are stored.
#include "moe_internal.h"
#include "route_device.h"

namespace moe {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef unsigned long long u64;

constexpr int kMaxWaves = 16;
constexpr int kRowPad = kStreamRowPad;

// (explicitly a pointer to global memory: an address that has been through an integer, as the tile addresses in
// the records have, would otherwise be loaded from with flat instructions, which count in both memory counters
// and force every wait behind them to wait for everything)
typedef __attribute__((address_space(1))) const unsigned char g_bytes;
typedef __attribute__((address_space(1))) const u32x4 g_u32x4;

__device__ inline u32x4 ld_stream(g_bytes *p)
{
    return __builtin_nontemporal_load((g_u32x4 *)p);
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

__device__ inline void store_entry(u64 *p, unsigned tag, unsigned value)
{
    __hip_atomic_store(p, ((u64)tag << 32) | value, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline u64 load_entry(const u64 *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#define TAG_IS(x) ((unsigned)((x) >> 32) == tag)   // an entry that carries this call's number
#ifdef MOE_STREAM_TRACE
__device__ unsigned long long g_layer_timeline[kTimelineGroups][kLayerTimelineWords];
#define MOE_STAMP(var) var = wall_clock64()
// (shader clock: what a wavefront spends in each part of a step, summed over the loop's steps; reading the
// clock waits for the wavefront's LDS operations, so these probes are a build of their own: -DMOE_STREAM_TRACE=2)
#if MOE_STREAM_TRACE > 1
#define MOE_CYC_BEGIN() long long cyc_t = clock64()
#define MOE_CYC(i) do { const long long cyc_n = clock64(); cyc_sum[i] += cyc_n - cyc_t; cyc_t = cyc_n; } while (0)
#else
#define MOE_CYC_BEGIN()
#define MOE_CYC(i)
#endif
#else
#define MOE_STAMP(var)
#define MOE_CYC_BEGIN()
#define MOE_CYC(i)
#endif

// Item classes of a workgroup's list, in the order it walks them:
//   0  gate/up, shared experts   item = (expert, 8 activations): gate rows f..f+7 stacked on up rows f..f+7
//   1  gate/up, routed experts
//   2  down, shared experts      item = (expert, 16 output rows)
//   3  down, routed experts
// An item is one tile per contraction panel (one panel up to 2048 columns).
//
// The loop is bound by how many instructions the sixteen wavefronts of a workgroup issue per tile, not only
// by memory, so everything that can be worked out once is: before the loop the workgroup writes one 32-byte
// record per tile of its list into LDS (thread j writes record j: where the tile's two row groups start in
// memory, which class and panel it is, where its results go), and a step only reads two records, the one
// of the tile it requests and the one of the tile it multiplies.
constexpr int kTabWords = 8;            // words of a tile record
constexpr int kRedStride = 2 * 1024 + 16;   // bytes between the partial results (two 16x16 blocks) of two wavefronts in LDS
constexpr int kOutBytes = 16 * 1024;    // finished values waiting in LDS (a gate/up item: 512 bytes, a down item: 1 or 2 KB)
constexpr int kOutRecs = 32;            // ... of at most this many items
constexpr int kDumpBytes = 2048;        // one KB where pieces that a tile does not have are parked, one KB of zeros

// A workgroup is sixteen wavefronts, each with NPI = 4 one-kilobyte pieces of the tile in flight twice over.
// Nothing is stored to memory inside the loop: stores and loads of a wavefront share one in-order counter, so
// a store between two tile requests makes the next wait for a tile a wait for the store's acknowledgement from
// memory as well (measured: 0.3 us per step, whichever wavefronts store).  Finished values wait in LDS and
// leave in one go when the workgroup passes from its gate/up tiles to its down tiles (the activations, which
// other workgroups wait for), when the buffer is full, and at the end.
template <int NPI, bool ROUTE>
__global__ __launch_bounds__(1024) void layer_kernel(LayerArgs a, RouteArgs ra)
{
    constexpr int kWaves = 16, kThreads = kWaves * 64, kPieces = NPI;
    static_assert(NPI * kWaves >= 64, "a full tile is 64 pieces");
    extern __shared__ __align__(16) unsigned char lds[];
    const int T = a.T, kk = a.k, H = a.H, F = a.F, Fs = a.F_sh, C = a.C, A = T * kk;
    unsigned char *tile_s = lds;
    unsigned char *red_s = lds + a.tile_lds_bytes + kDumpBytes;        // [wavefront] 2 KB of partial results each
    float *out_s = (float *)(red_s + kWaves * kRedStride);   // [kOutBytes / 4] finished values waiting to be stored
    int *ctl_s = (int *)((unsigned char *)out_s + kOutBytes);
    static_assert((kWaves * kRedStride) % 16 == 0, "the arrays behind stay 16-byte aligned");
    int *count_s = ctl_s, *offset_s = ctl_s + C, *active_s = ctl_s + 2 * C, *mask_s = ctl_s + 3 * C;
    int *perm_s = ctl_s + 4 * C;     // token of each entry of the per-slot lists
    int *pos_s = perm_s + A;         // row of each assignment's output, -1 = expert not resident
    int *misc_s = pos_s + A;         // [0] active slots, [1] a bounded wait of this workgroup ran out
    // per class: panels per item, items per expert, first item of this workgroup's share, contraction length,
    // panel width, rows per expert (constants of the launch, looked up on the rare paths)
    // ... rows per item)
    int *orec_s = misc_s + 8;        // [kOutRecs][2]: tile whose item's results wait in out_s, and where
    int *cls_s = orec_s + 2 * kOutRecs;   // [4][8]
    int *geo_s = cls_s + 32;         // [6][4]: tile row bytes, weight row bytes, rows of the six tile layouts
    u64 *clsp_s = (u64 *)(geo_s + 24);   // [4][2]: where the class's weights start (rows 0..7 and 8..15 of a gate/up tile)
    uint32_t *tab_s = (uint32_t *)(ctl_s + ((4 * C + 2 * A + 8 + 2 * kOutRecs + 32 + 24 + 16 + 3) & ~3));   // [tiles + 2][kTabWords]

    const int tid = threadIdx.x, lane = tid & (kWave - 1);
#ifdef MOE_STREAM_TRACE
    unsigned long long tl_start, tl_lists = 0, tl_first = 0, tl_phase = 0, tl_loop = 0;
    long long cyc_sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#endif
    MOE_STAMP(tl_start);
    const int w = __builtin_amdgcn_readfirstlane(tid / kWave);   // wavefront id, known to be uniform
    const int n = lane & 15, g = lane >> 4;
    const int G = gridDim.x, b = blockIdx.x;

    // control block: call number, and the two words with which a test forces the bounded waits to run out
    unsigned *const error_flag = a.ctrl + kCtrlError;
    const unsigned epoch0 = a.ctrl[kCtrlEpoch];
    const unsigned spin_w = a.ctrl[kCtrlSpin], skew = a.ctrl[kCtrlSkew];
    const int spin = spin_w ? (int)spin_w : kSpinLimit;
    const unsigned tag = ROUTE ? epoch0 + 1u : epoch0;   // number of this call
    const unsigned wtag = tag + skew;                    // what this call's entries are stamped with (skew = 0)
    if (ROUTE && b == 0 && tid == 0) check_layout(a.ctrl, ra.layout);
    auto give_up = [&]() __attribute__((always_inline)) {   // never wait for ever: say so in the control block and poison what this workgroup writes
        atomicOr(error_flag, 1u);
        misc_s[1] = 1;
    };
    // a kilobyte that is always there and soon cached: what a wavefront reads for a piece its tile does not have
    // (one of 512 places in the fixed region behind the control block, so that these reads do not all fall on
    // the same cache lines of one memory channel)
    g_bytes *const dummy = (g_bytes *)(uintptr_t)((const unsigned char *)a.ctrl + kCtrlBytes) + (size_t)((b * kWaves + w) & 511) * 1024;

    // A down item is RD rows (16..32: as many as make its tile about as large as a gate/up tile, so that two
    // tiles in flight cover the memory latency in the down part too), the last item of an expert the rest.
    const int RD = a.RD, RDS = a.n_shared ? a.RDS : 16;
    const int tiles_g = F / 8, tiles_gs = a.n_shared ? Fs / 8 : 0;
    const int tiles_d = (H + RD - 1) / RD, tiles_ds = (H + RDS - 1) / RDS;
    const int n_gs = a.n_shared * tiles_gs, n_ds = a.n_shared * tiles_ds;
    const int np_h = H / a.KP_h, np_f = F / a.KP_f, np_fs = a.n_shared ? Fs / a.KP_fs : 1;

    // This workgroup's share of each class: items [sg_start, sg_start + sg_cnt) of the class's list.
    // The shared experts' shares need nothing from the routing step.  (ROUTE: workgroup 0 also ranks the
    // logits and builds the lists, which the others wait for; it takes the last place in the gate/up split.)
    const int rk1 = ROUTE ? (b == 0 ? G - 1 : b - 1) : b;
    const int rk2 = G - 1 - rk1;   // the down part is dealt the other way round: the odd items go elsewhere
    int sg_start0, sg_cnt0, sg_start1 = 0, sg_cnt1 = 0, sg_start2, sg_cnt2, sg_start3 = 0, sg_cnt3 = 0;
    {
        const int per = n_gs / G, rem = n_gs % G;
        sg_cnt0 = per + (rk1 < rem ? 1 : 0);
        sg_start0 = rk1 * per + (rk1 < rem ? rk1 : rem);
        const int per2 = n_ds / G, rem2 = n_ds % G;
        sg_cnt2 = per2 + (rk2 < rem2 ? 1 : 0);
        sg_start2 = rk2 * per2 + (rk2 < rem2 ? rk2 : rem2);
    }
    const int nt0 = sg_cnt0 * np_h;   // tiles of the first class: known at once
    int ntiles = nt0;

    // Record of tile j of this workgroup's list (by thread j):
    //   words 0-1  address of the tile's first row at the tile's panel (16-byte aligned; the four low bits say
    //              how the tile is laid out)
    //   words 2-3  gate/up: address of tile rows 8..15 (the up rows)
    //   word 4     class | first panel << 2 | last panel << 3 | (panel | B operand's identity << 8) << 4
    //   word 5     first row of the item's results (list position of the expert's first token, or expert * T)
    //   word 6     first column of the item's results | rows of the item << 16 | the tile's layout << 24
    //   word 7     tokens of the expert | their bit mask << 8
    auto write_record = [&](int j, int nt1, int nt2) __attribute__((always_inline)) {
        int cls, r = j;
        if (r < nt0) cls = 0;
        else if ((r -= nt0) < nt1) cls = 1;
        else if ((r -= nt1) < nt2) cls = 2;
        else { r -= nt2; cls = 3; }
        const int *cp = cls_s + cls * 8;
        const int npan = cp[0], tl = cp[1], K = cp[3], KP = cp[4], rows = cp[5];
        const int item = r / npan, pan = r - item * npan;
        const int idx = cp[2] + item;
        const int e = idx / tl, rt = idx - e * tl;
        const bool shared = cls == 0 || cls == 2;
        const int c = shared ? e : active_s[e];
        const int rpi = cp[6];   // weight rows of an item per matrix (the last item of an expert may have fewer)
        const size_t eoff = ((size_t)c * rows + (size_t)rt * rpi) * K + (size_t)pan * KP;   // (elements)
        const u64 p0 = clsp_s[cls * 2] + 2 * eoff;
        const u64 p1 = cls < 2 ? clsp_s[cls * 2 + 1] + 2 * eoff : p0;
        const int key = cls < 2 ? 0 : cls == 2 ? 1 + e : 1 + a.n_shared + e;
        int row0 = e * T, mm = T | (((1 << T) - 1) << 8);
        if (!shared) {
            row0 = offset_s[c];
            mm = count_s[c] | (mask_s[c] << 8);
        }
        const bool last_item = cls >= 2 && rt == tl - 1;
        const int item_rows = last_item ? rows - rt * rpi : rpi;
        const int gid = cls < 2 ? 0 : cls - 1 + (last_item ? 2 : 0);
        uint32_t *rec = tab_s + (size_t)j * kTabWords;
        rec[0] = (uint32_t)p0 | (uint32_t)gid; rec[1] = (uint32_t)(p0 >> 32);
        rec[2] = (uint32_t)p1; rec[3] = (uint32_t)(p1 >> 32);
        rec[4] = (uint32_t)cls | (pan == 0 ? 4u : 0u) | (pan == npan - 1 ? 8u : 0u) | ((uint32_t)(pan | key << 8) << 4);
        rec[5] = (uint32_t)row0;
        rec[6] = (uint32_t)(rt * rpi) | ((uint32_t)item_rows << 16) | ((uint32_t)gid << 24);
        rec[7] = (uint32_t)mm;
    };
    auto write_end_records = [&](int nt) __attribute__((always_inline)) {   // two records behind the last tile: nothing to load
        if (tid < 2 * kTabWords) tab_s[(size_t)nt * kTabWords + tid] = (tid & 7) == 0 ? 5u : 0u;
    };

    // Piece i of this wavefront covers bytes [(16i+w) KB, +1 KB) of a tile seen as 16 rows of rs bytes (rs a
    // multiple of 128, so a piece lies wholly in tile rows 0..7 or 8..15 and the choice between the two row
    // pointers is uniform).  A tile of rs-byte rows has rs/64 pieces.  All NPI loads of a tile are issued
    // unconditionally: for a piece beyond the tile the wavefront reads a kilobyte that is always cached and
    // parks it beside the tile.  For each piece this lane keeps its global byte offset from the row group's
    // first row and its LDS byte offset; both depend only on how the tile is laid out and are worked out again
    // when that changes (three times per launch).  Two tiles are in flight per wavefront (st[0], st[1]).
    u32x4 st[2][NPI];
    unsigned goff[NPI];   // layout of the tile being requested
    int loff[NPI];        // layout of the tile being parked
    int p_geo = -1, k_geo = -1;
    unsigned p_hi = 0, p_dm = 0;   // bit i: piece i lies in tile rows 8..15 | is no piece of the tile
    // row << 16 | column of this lane's 16 bytes of piece i in a tile of layout gid; -1: the tile has no such
    // piece; -2: the piece straddles the tile's end and this lane lies beyond it
    auto piece_rc = [&](int i, int rs, int end) __attribute__((always_inline)) {
        const int pc = i * kWaves + w;
        if ((pc << 10) >= end) return -1;
        const int off = (pc << 10) + (lane << 4);
        if (off >= end) return -2;
        const int row = (int)(((float)off + 8.0f) * (1.0f / (float)rs));   // (off + 8 is never within 4 of a multiple of rs)
        return row << 16 | (off - row * rs);
    };
    auto set_pgeo = [&](int gid) __attribute__((always_inline)) {
        p_geo = gid;
        const int rs = __builtin_amdgcn_readfirstlane(geo_s[gid * 4]);
        const int K2 = __builtin_amdgcn_readfirstlane(geo_s[gid * 4 + 1]);
        const int end = __builtin_amdgcn_readfirstlane(geo_s[gid * 4 + 2]) * rs;   // bytes of the tile
        unsigned hi = 0, dm = 0;
#pragma unroll
        for (int i = 0; i < NPI; ++i) {
            const int rc = piece_rc(i, rs, end);
            if (rc >= 0) {
                const int row = rc >> 16, col = rc & 0xffff;
                goff[i] = (unsigned)((gid == 0 ? row & 7 : row) * K2 + col);
            } else if (rc == -2) {   // these lanes read the tile's last 16 bytes again
                goff[i] = (unsigned)((end / rs - 1) * K2 + rs - 16);
            } else {
                goff[i] = (unsigned)(lane << 4);
            }
            const int pc = i * kWaves + w;
            if ((pc << 10) >= end) dm |= 1u << i;
            else if (gid == 0 && (pc << 10) >= 8 * rs) hi |= 1u << i;
        }
        p_hi = hi;
        p_dm = dm;
    };
    auto set_kgeo = [&](int gid) __attribute__((always_inline)) {
        k_geo = gid;
        const int rs = __builtin_amdgcn_readfirstlane(geo_s[gid * 4]);
        const int end = __builtin_amdgcn_readfirstlane(geo_s[gid * 4 + 2]) * rs;
#pragma unroll
        for (int i = 0; i < NPI; ++i) {
            const int rc = piece_rc(i, rs, end);
            loff[i] = rc >= 0 ? (rc >> 16) * (rs + kRowPad) + (rc & 0xffff) : a.tile_lds_bytes + (lane << 4);
        }
    };
    auto issue = [&](int s, int ti) __attribute__((always_inline)) {
        const u32x4 r = *(const u32x4 *)(tab_s + (size_t)ti * kTabWords);
        unsigned p0l = (unsigned)__builtin_amdgcn_readfirstlane((int)r.x);
        const unsigned p0h = (unsigned)__builtin_amdgcn_readfirstlane((int)r.y);
        const unsigned p1l = (unsigned)__builtin_amdgcn_readfirstlane((int)r.z);
        const unsigned p1h = (unsigned)__builtin_amdgcn_readfirstlane((int)r.w);
        const int gid = (int)(p0l & 15u);
        p0l &= ~15u;
        if (gid != p_geo) set_pgeo(gid);
        g_bytes *p0 = (g_bytes *)(uintptr_t)((u64)p0h << 32 | p0l);
        g_bytes *p1 = (g_bytes *)(uintptr_t)((u64)p1h << 32 | p1l);
#pragma unroll
        for (int i = 0; i < NPI; ++i) {
            g_bytes *base = (p_dm >> i) & 1u ? dummy : (p_hi >> i) & 1u ? p1 : p0;   // uniform
            st[s][i] = ld_stream(base + goff[i]);
        }
    };
    auto park = [&](int s, int gid) __attribute__((always_inline)) {   // gid: layout of the tile in register set s
        if (gid != k_geo) set_kgeo(gid);
#pragma unroll
        for (int i = 0; i < NPI; ++i) *(u32x4 *)(tile_s + loff[i]) = st[s][i];
    };

    if (ROUTE) {
        // ---- steps 1-3 inside this launch (Sec. 2.2, 2.3, App. D), as in the routing kernel ----
        // every workgroup: its share of the T*E dot products, one per wavefront, each logit stored with the
        // call's number as one 64-bit word
        const int E = ra.E, TE = T * E;
        const size_t n_pub = list_pub_entries(T, kk, C);
        // (workgroup 0 gives the call its number in the control block, at its end, only when every workgroup
        // has read the old one: each says so with a stamped word of its own)
        u64 *const seen = ra.lists_pub + (size_t)kListReplicas * n_pub;
        if (tid == 0) store_entry(seen + b, tag, 1u);
        int tab_v = -1;
        if (b == 0 && tid < E) tab_v = ra.slot_table[tid];
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
            if (lane == 0) {
                store_entry(ra.tagged_logits + q, wtag, __float_as_uint(dot));
                if (ra.logits_opt) ra.logits_opt[q] = dot;
            }
        }
        if (b == 0) {
            // workgroup 0: one wavefront per token ranks its logits; then histogram, slot lookup, miss list and
            // per-slot lists out of LDS (which nothing else uses yet), every word of the lists published
            PostLds L = carve_lds((int *)lds, E, C, A);
            if (tid < E) {
                L.tab_s[tid] = tab_v;
                L.hist_s[tid] = 0;
            }
            for (int i = tid; i < C * ((T + 31) >> 5); i += kThreads) L.cnt_s[i] = 0;
            lds_f32 *lg = L.lg_s + w * lg_stride(E);
            for (int t = w; t < T; t += kWaves) {
                const u64 *src = ra.tagged_logits + (size_t)t * E;
                for (int e0 = 0; e0 < E; e0 += kWave) {
                    const int e = e0 + lane;
                    u64 v = (u64)tag << 32;
                    int polls = 0;
                    for (;;) {
                        if (e < E) v = load_entry(src + e);
                        if (__ballot(!TAG_IS(v)) == 0ull) break;
                        if (++polls > spin) {
                            if (lane == 0) atomicOr(error_flag, 1u);
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
                // (up to 128 experts here: the ranking of more needs so many registers that the whole
                // kernel would be launched with scratch memory; those batches keep the routing kernel)
                float gate;
                if (E <= kWave)
                    gate = wave_topk_gate_n<1>(E, kk, ra.topk_idx + (size_t)t * kk, L.idx_s + t * kk,
                                               ra.topk_w + (size_t)t * kk, lg);
                else
                    gate = wave_topk_gate_n<2>(E, kk, ra.topk_idx + (size_t)t * kk, L.idx_s + t * kk,
                                               ra.topk_w + (size_t)t * kk, lg);
                // the final sum of every workgroup needs the gate weights: plain stores of this workgroup are
                // not visible to the others inside the launch, so they travel as stamped entries too
                if (lane < kk) {
                    u64 *gw_pub = seen + kMaxGroups;
                    for (int rep = 0; rep < kListReplicas; ++rep)
                        store_entry(gw_pub + (size_t)rep * A + t * kk + lane, wtag, __float_as_uint(gate));
                }
            }
            __syncthreads();
            block_post_small<true>(L.idx_s, L.tab_s, T, kk, E, C, ra, L.hist_s, L.cnt_s, L.scan_s, L.off_s, wtag);
            __syncthreads();   // (the LDS used above is free again)
        }
    }
    if (tid == 0) misc_s[1] = 0;   // (a barrier follows before anything can set it)
    if (tid < 256) ((uint32_t *)(lds + a.tile_lds_bytes + 1024))[tid] = 0u;   // the kilobyte of zeros
    if (tid == 0) {
        int *c0 = cls_s, *c1 = cls_s + 8, *c2 = cls_s + 16, *c3 = cls_s + 24;
        c0[0] = np_h; c0[1] = tiles_gs; c0[2] = sg_start0; c0[3] = H; c0[4] = a.KP_h; c0[5] = Fs;
        c1[0] = np_h; c1[1] = tiles_g; c1[2] = 0; c1[3] = H; c1[4] = a.KP_h; c1[5] = F;
        c2[0] = np_fs; c2[1] = tiles_ds; c2[2] = sg_start2; c2[3] = Fs; c2[4] = a.KP_fs; c2[5] = H; c2[6] = RDS;
        c3[0] = np_f; c3[1] = tiles_d; c3[2] = 0; c3[3] = F; c3[4] = a.KP_f; c3[5] = H; c3[6] = RD;
        c0[6] = 8; c1[6] = 8;
        clsp_s[0] = (u64)(uintptr_t)a.sh_gate; clsp_s[1] = (u64)(uintptr_t)a.sh_up;
        clsp_s[2] = (u64)(uintptr_t)a.w_gate; clsp_s[3] = (u64)(uintptr_t)a.w_up;
        clsp_s[4] = (u64)(uintptr_t)a.sh_down; clsp_s[5] = 0;
        clsp_s[6] = (u64)(uintptr_t)a.w_down; clsp_s[7] = 0;
        // tile layouts: 0 gate/up | 1, 2 down of a shared, a routed expert | 3, 4 the same, last item of an
        // expert (fewer rows) | 5 no tile
        geo_s[0] = 2 * a.KP_h; geo_s[1] = 2 * H; geo_s[2] = 16;
        geo_s[4] = 2 * a.KP_fs; geo_s[5] = 2 * Fs; geo_s[6] = RDS;
        geo_s[8] = 2 * a.KP_f; geo_s[9] = 2 * F; geo_s[10] = RD;
        geo_s[12] = 2 * a.KP_fs; geo_s[13] = 2 * Fs; geo_s[14] = H - (tiles_ds - 1) * RDS;
        geo_s[16] = 2 * a.KP_f; geo_s[17] = 2 * F; geo_s[18] = H - (tiles_d - 1) * RD;
        geo_s[20] = 0; geo_s[21] = 0; geo_s[22] = 0;
    }

    u32x4 bx[kPieces];
    unsigned bx_sig = 0xffffffffu;   // panel | identity << 8 of the B operand that the registers hold
    int c_geo = -1, c_rs = 128;
    bool c_two = false;              // the parked tile has more than 16 rows: two blocks of 16 MFMA rows
    unsigned avalid = 0;             // bit j: this wavefront's j-th column block exists in the parked tile
    int aoff[kPieces];
    auto set_cgeo = [&](int gid) __attribute__((always_inline)) {
        c_geo = gid;
        c_rs = __builtin_amdgcn_readfirstlane(geo_s[gid * 4]);
        c_two = __builtin_amdgcn_readfirstlane(geo_s[gid * 4 + 2]) > 16;
        const int nkb = c_rs / 64;
        avalid = 0;
#pragma unroll
        for (int j = 0; j < kPieces; ++j) {
            const int kb = w + kWaves * j;
            if (kb < nkb) avalid |= 1u << j;
            // (a column block that the tile does not have: zeros from the kilobyte kept for that, so that the
            // multiplication needs no branch and all its LDS reads go out together)
            aoff[j] = kb < nkb ? n * (c_rs + kRowPad) + kb * 64 + g * 16 : a.tile_lds_bytes + 1024 + (lane << 4);
        }
    };
    // B operand of this wavefront's column blocks.  Gate/up part: the hidden states of tokens 0..T-1, token n
    // on column n.  Down part: the activation rows of the expert's list, entry n on column n; they come as
    // stamped entries from whichever workgroups computed them and are polled until they carry this call's number.
    auto load_bx = [&](int cls, int pan, int row0, int m) __attribute__((always_inline)) {
        const int cgid = cls < 2 ? 0 : cls - 1;
        if (cgid != c_geo) set_cgeo(cgid);
        if (cls < 2) {
            const int boff = n < T ? n * H + pan * (c_rs / 2) : -1;
#pragma unroll
            for (int j = 0; j < kPieces; ++j) {
                const int kb = w + kWaves * j;
                bx[j] = (u32x4){0u, 0u, 0u, 0u};
                if (((avalid >> j) & 1u) && boff >= 0) bx[j] = *(const u32x4 *)(a.hidden + (unsigned)(boff + kb * 32 + g * 8));
            }
            // (everything in flight is waited for here, on this rare path, so that behind it the compiler knows
            // the operand to be there and the common path's waits stay exact)
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        } else {
            const u64 *src = cls == 2 ? +a.act_sh : +a.act;
            const int rowlen = (cls == 2 ? +Fs : +F) / 2;
            const bool valid = n < m;
            const u64 *base = src + (size_t)(row0 + (valid ? n : 0)) * rowlen + (size_t)pan * (c_rs / 4) + g * 4;
            int polls = 0;
            for (;;) {
                bool ok = true;
#pragma unroll
                for (int j = 0; j < kPieces; ++j) {
                    const int kb = w + kWaves * j;
                    bx[j] = (u32x4){0u, 0u, 0u, 0u};
                    if (((avalid >> j) & 1u) && valid) {
                        const u64 *p = base + kb * 16;
                        const u64 e0 = load_entry(p), e1 = load_entry(p + 1), e2 = load_entry(p + 2), e3 = load_entry(p + 3);
                        ok = ok && TAG_IS(e0) && TAG_IS(e1) &&
                             TAG_IS(e2) && TAG_IS(e3);
                        bx[j] = (u32x4){(unsigned)e0, (unsigned)e1, (unsigned)e2, (unsigned)e3};
                    }
                }
                if (__ballot(!ok) == 0ull) break;
                if (++polls > spin) {   // cannot happen with the whole grid resident
                    give_up();
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
        }
    };
    auto load_bx_of = [&](int ti) __attribute__((always_inline)) {   // the B operand that tile ti needs
        const uint32_t *rec = tab_s + (size_t)ti * kTabWords;
        const unsigned fl = (unsigned)__builtin_amdgcn_readfirstlane((int)rec[4]);
        const int row0 = __builtin_amdgcn_readfirstlane((int)rec[5]);
        const int m = __builtin_amdgcn_readfirstlane((int)rec[7]) & 0xff;
        load_bx((int)(fl & 3u), (int)((fl >> 4) & 0xffu), row0, m);
        bx_sig = fl >> 4;
    };

    // the shared experts' first tiles need nothing from the routing step: their weights are in flight while
    // the lists are on their way
    int issued = 0;   // tiles requested so far (0, 1 or 2)
    if (nt0 > 0) {
        __syncthreads();   // (the class table)
        for (int j = tid; j < nt0; j += kThreads) write_record(j, 0, 0);
        write_end_records(nt0);
        __syncthreads();
        issue(0, 0);
        issued = 1;
        if (nt0 >= 2) {
            load_bx_of(0);
            issue(1, 1);
            issued = 2;
        }
    }
    int n_act;
    if (ROUTE) {
        // every workgroup: the lists, from one of the published copies.  One lane watches the first word,
        // gently (255 workgroups asking for all words all the time would be a load of its own on the few
        // memory channels the copies live in); once it is there the workgroup reads them all.
        const size_t n_pub = list_pub_entries(T, kk, C);
        const u64 *pub = ra.lists_pub + (size_t)(b % kListReplicas) * n_pub;
        if (tid == 0 && b != 0) {
            int polls = 0;
            while (!TAG_IS(load_entry(pub))) {
                if (++polls > spin) break;   // (the loop below reports it)
                __builtin_amdgcn_s_sleep(16);
            }
        }
        for (int i = tid; i < A; i += kThreads) pos_s[i] = -1;
        __syncthreads();
        for (int i = tid; i < (int)n_pub; i += kThreads) {
            u64 v = 0;
            int polls = 0;
            for (;;) {
                v = load_entry(pub + i);
                if (TAG_IS(v)) break;
                if (++polls > spin) {
                    give_up();
                    v = 0;   // (stay inside every array below)
                    break;
                }
                __builtin_amdgcn_s_sleep(8);
            }
            const int val = (int)(unsigned)v;
            if (i == 0) misc_s[0] = val;
            else if (i <= C) count_s[i - 1] = val < 0 ? 0 : val > T ? T : val;
            else if (i <= 2 * C) offset_s[i - 1 - C] = val < 0 ? 0 : val > A ? A : val;
            else if (i <= 3 * C) active_s[i - 1 - 2 * C] = val < 0 ? 0 : val >= C ? C - 1 : val;
            else {
                const int asg = val < 0 ? -1 : val >= A ? A - 1 : val;   // flat assignment id of list entry i - 1 - 3C
                perm_s[i - 1 - 3 * C] = (asg < 0 ? 0 : asg) / kk;
                if (asg >= 0) pos_s[asg] = i - 1 - 3 * C;
            }
        }
        __syncthreads();
        n_act = misc_s[0];
    } else {
        // one trip to memory for everything the routing step left behind
        for (int i = tid; i < C; i += kThreads) {
            count_s[i] = a.slot_count[i];
            offset_s[i] = a.slot_offset[i];
            active_s[i] = a.active_slots[i];
        }
        for (int i = tid; i < A; i += kThreads) {
            perm_s[i] = a.perm[i] / kk;
            pos_s[i] = a.pos[i];
        }
        n_act = (int)(*a.n_active);
        __syncthreads();
    }
    n_act = n_act < 0 ? 0 : n_act > C ? C : n_act;
    // the tokens of each slot as a bit mask (a token names a slot at most once)
    for (int c = tid; c < C; c += kThreads) {
        int m = 0;
        const int cnt = count_s[c], off = offset_s[c];
        for (int j = 0; j < cnt && off + j < A; ++j) m |= 1 << (perm_s[off + j] & 15);
        mask_s[c] = m;
    }

    // routed shares: equal runs of the gate/up list (items all alike); the down list is cut into runs of equal
    // numbers of TILES (a shared expert's item can have another number of panels than a routed one)
    {
        // (ROUTE: workgroup 0 starts its run a few microseconds late: two items fewer for it)
        const int late = ROUTE && n_act * tiles_g >= 4 * G ? 2 : 0;
        const int total = n_gs + n_act * tiles_g + late;
        const int per = total / G, rem = total % G;
        int cnt = per + (rk1 < rem ? 1 : 0);
        sg_start1 = rk1 * per + (rk1 < rem ? rk1 : rem) - sg_start0;
        if (rk1 == G - 1) cnt -= late;
        sg_cnt1 = cnt - sg_cnt0;
        if (sg_cnt1 < 0) sg_cnt1 = 0;
        // Down part: workgroup of rank x starts at routed item max(0, x * total tiles / G - tiles of the shared
        // items before x) / panels per routed item: never decreasing in x, 0 for x = 0, all for x = G.
        const int n_routed = n_act * tiles_d;
        const long long total2 = (long long)n_ds * np_fs + (long long)n_routed * np_f;
        const int per2 = n_ds / G, rem2 = n_ds % G;
        auto routed_before = [&](int x) __attribute__((always_inline)) {
            const long long sh = (long long)(x * per2 + (x < rem2 ? x : rem2)) * np_fs;
            const long long rt = (long long)x * total2 / G - sh;
            const long long r = rt > 0 ? rt / np_f : 0;
            return (int)(r < n_routed ? r : n_routed);
        };
        sg_start3 = routed_before(rk2);
        sg_cnt3 = routed_before(rk2 + 1) - sg_start3;
    }
    int nt1 = sg_cnt1 * np_h, nt2 = sg_cnt2 * np_fs, nt3 = sg_cnt3 * np_f;
    if (nt0 + nt1 + nt2 + nt3 > a.tab_cap) {   // cannot happen: the host sizes the table for the largest share
        give_up();
        nt3 = 0;
        if (nt0 + nt1 + nt2 > a.tab_cap) nt2 = 0;
        if (nt0 + nt1 > a.tab_cap) nt1 = 0;
    }
    ntiles = nt0 + nt1 + nt2 + nt3;
    if (tid == 0) {
        cls_s[8 + 2] = sg_start1;
        cls_s[24 + 2] = sg_start3;
    }
    __syncthreads();   // (the masks, the class table)
    for (int j = nt0 + tid; j < ntiles; j += kThreads) write_record(j, nt1, nt2);
    write_end_records(ntiles);
    __syncthreads();
    MOE_STAMP(tl_lists);

    // ---- the weighted sum back into token order (Sec. 2.2 last line; the join of App. D when `accumulate`) ----
    auto join = [&]() __attribute__((always_inline)) {
        const int S = kk + a.n_shared, nent = T * 8 * S;
        float *val_s = (float *)tile_s;   // [token][column of the strip][source]; the tile buffer is free by now
        float *gw_s = (float *)red_s;     // gate weights, on their way while the entries are waited for
        if (ROUTE) {
            // (written by workgroup 0 of this launch, long ago; stamped, so that what is read is what was written)
            const size_t n_pub = list_pub_entries(T, kk, C);
            const u64 *gw_pub = ra.lists_pub + (size_t)kListReplicas * n_pub + kMaxGroups + (size_t)(b % kListReplicas) * A;
            for (int i = tid; i < A; i += kThreads) {
                u64 x = 0;
                int polls = 0;
                for (;;) {
                    x = load_entry(gw_pub + i);
                    if (TAG_IS(x)) break;
                    if (++polls > spin) {
                        give_up();
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                gw_s[i] = __uint_as_float((unsigned)x);
            }
        } else {
            for (int i = tid; i < A; i += kThreads) gw_s[i] = a.topk_w[i];
        }
        for (int u = b; u < H / 8; u += G) {
            __syncthreads();
            for (int i = tid; i < nent; i += kThreads) {
                const int tc = i / S, src = i - tc * S, t = tc >> 3, col = u * 8 + (tc & 7);
                const u64 *p = nullptr;
                if (src < kk) {
                    const int row = pos_s[t * kk + src];
                    if (row >= 0) p = a.o + (size_t)row * H + col;
                } else {
                    p = a.o_sh + ((size_t)(src - kk) * T + t) * H + col;
                }
                float v = 0.f;   // an assignment whose expert is not resident adds nothing here
                if (p) {
                    u64 x = 0;
                    int polls = 0;
                    for (;;) {
                        x = load_entry(p);
                        if (TAG_IS(x)) break;
                        if (++polls > spin) {   // cannot happen with the whole grid resident
                            give_up();
                            break;
                        }
                        __builtin_amdgcn_s_sleep(1);
                    }
                    v = __uint_as_float((unsigned)x);
                }
                val_s[i] = v;
            }
            __syncthreads();
            const bool poisoned = misc_s[1] != 0 ||
                                  __hip_atomic_load(error_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
            if (tid < T * 8) {
                const int t = tid >> 3, col = u * 8 + (tid & 7);
                const size_t o = (size_t)t * H + col;
                float acc = 0.f;
                if (a.accumulate)
                    acc = a.out_bf16 ? __uint_as_float((uint32_t)((const uint16_t *)a.out)[o] << 16)
                                     : ((const float *)a.out)[o];
                for (int jj = 0; jj < kk; ++jj) acc += gw_s[t * kk + jj] * val_s[tid * S + jj];
                for (int i = 0; i < a.n_shared; ++i) acc += val_s[tid * S + kk + i];
                if (poisoned) acc = __uint_as_float(0x7fc00000u);   // a wait ran out: not a result
                if (a.out_bf16) ((uint16_t *)a.out)[o] = (uint16_t)f32_to_bf16_rne(acc);
                else ((float *)a.out)[o] = acc;
            }
        }
    };
    auto finish = [&]() __attribute__((always_inline)) {
        join();
        __syncthreads();
        // a wait ran out, here or (the control block says so) anywhere in this call: the call says so in miss_count too
        if (tid == 0 && a.miss_count &&
            (misc_s[1] != 0 || __hip_atomic_load(error_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u))
            __hip_atomic_store(a.miss_count, -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (ROUTE && b == 0) {
            // the call's number goes into the control block once every workgroup has read the old one
            const size_t n_pub = list_pub_entries(T, kk, C);
            const u64 *seen = ra.lists_pub + (size_t)kListReplicas * n_pub;
            for (int i = tid; i < G; i += kThreads) {
                int polls = 0;
                while (!TAG_IS(load_entry(seen + i))) {
                    if (++polls > spin) {
                        atomicOr(error_flag, 1u);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
            __syncthreads();
            if (tid == 0) a.ctrl[kCtrlEpoch] = tag;
        }
    };

    if (ntiles == 0) {
        finish();
        return;
    }
    if (issued == 0) {
        issue(0, 0);
        issued = 1;
    }
    if (issued == 1) {
        // (the first B operand between the first two requests: its wait then covers the first tile only)
        load_bx_of(0);
        issue(1, 1);
    }

    f32x4 acc = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};   // tile rows 0..15 and 16..31

    auto multiply = [&]() __attribute__((always_inline)) {
        u32x4 av[kPieces];
#pragma unroll
        for (int j = 0; j < kPieces; ++j) av[j] = *(const u32x4 *)(tile_s + aoff[j]);
#pragma unroll
        for (int j = 0; j < kPieces; ++j) acc = mfma(av[j], bx[j], acc);
        if (c_two) {
            // (rows beyond the item's last one hold whatever the buffer held: their results are not stored)
            const int blk1 = 16 * (c_rs + kRowPad);
#pragma unroll
            for (int j = 0; j < kPieces; ++j) av[j] = *(const u32x4 *)(tile_s + aoff[j] + ((avalid >> j) & 1u ? blk1 : 0));
#pragma unroll
            for (int j = 0; j < kPieces; ++j) acc1 = mfma(av[j], bx[j], acc1);
        }
    };

    // The sixteen partial results of an item (posted in red_s, barrier passed) are added by wavefronts 0..3 (one
    // per SIMD unit; the others go on to the next tile), in wavefront order: the result does not depend on
    // scheduling.  Element q = lane*4 + j of the MFMA result layout is column (q/4)%16, tile row 4*(q/64) + q%4
    // (+ 16 in the second block); gate rows are tile rows 0..7 (elements 0..127) and the up row of the same
    // activation sits 128 elements further on.  The finished values (SiLU(gate) * up, or the down projection's
    // sums) go to out_s; where they go in memory is worked out when they leave.
    int o_recs = 0, o_used = 0;   // items waiting in out_s, floats used
    auto reduce_item = [&](int ti, unsigned fl) __attribute__((always_inline)) {
        const int cls = (int)(fl & 3u);
        const int n_out = cls < 2 ? 128 : c_two ? 512 : 256;
        if (tid < 256) {
            const unsigned char *p = red_s + tid * 4;
            if (cls < 2) {
                if (tid < 128) {
                    float s0 = 0.f, s1 = 0.f;
#pragma unroll
                    for (int v = 0; v < kWaves; ++v) {
                        s0 += *(const float *)(p + v * kRedStride);
                        s1 += *(const float *)(p + v * kRedStride + 512);
                    }
                    // SiLU(s0) * s1 = s0 / (1 + 2^(-s0 log2 e)) * s1 (hardware exponential and reciprocal: the
                    // result is rounded to bf16 anyway)
                    out_s[o_used + tid] = s0 * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-1.44269504088896f * s0)) * s1;
                }
            } else {
                float s0 = 0.f;
#pragma unroll
                for (int v = 0; v < kWaves; ++v) s0 += *(const float *)(p + v * kRedStride);
                out_s[o_used + tid] = s0;
                if (c_two) {
                    float s1 = 0.f;
#pragma unroll
                    for (int v = 0; v < kWaves; ++v) s1 += *(const float *)(p + v * kRedStride + 1024);
                    out_s[o_used + 256 + tid] = s1;
                }
            }
        }
        if (tid == 0) {
            orec_s[2 * o_recs] = ti;
            orec_s[2 * o_recs + 1] = o_used;
        }
        ++o_recs;
        o_used += n_out;
    };
    // Everything that waits in out_s goes to memory as stamped entries, one wavefront per item at a time.
    auto flush = [&]() __attribute__((always_inline)) {
        __syncthreads();   // (the last reduction's values, by wavefronts 0..3)
        for (int r = w; r < o_recs; r += kWaves) {
            const int ti = __builtin_amdgcn_readfirstlane(orec_s[2 * r]);
            const float *vals = out_s + __builtin_amdgcn_readfirstlane(orec_s[2 * r + 1]);
            const uint32_t *rec = tab_s + (size_t)ti * kTabWords;
            const int cls = __builtin_amdgcn_readfirstlane((int)rec[4]) & 3;
            const int row0 = __builtin_amdgcn_readfirstlane((int)rec[5]);
            const int cr = __builtin_amdgcn_readfirstlane((int)rec[6]);
            const int mm = __builtin_amdgcn_readfirstlane((int)rec[7]);
            const int first_col = cr & 0xffff, item_rows = (cr >> 16) & 0xff, m = mm & 0xff, mask = mm >> 8;
            if (cls < 2) {
                // one 64-bit entry per (token, pair of activations): elements q0, q0 + 1 are rows r, r + 1 of one
                // token; column `col` is token `col`, and the entry of the expert's list that this token is =
                // the number of the expert's tokens below it
                const int q0 = 2 * lane;
                const int col = (q0 >> 2) & 15, row = 4 * (q0 >> 6) + (q0 & 3);
                if ((mask >> col) & 1) {
                    const int li = __popc((unsigned)mask & ((1u << col) - 1u));
                    u64 *dst = (cls == 0 ? a.act_sh : a.act) + (size_t)(row0 + li) * ((cls == 0 ? Fs : F) / 2) +
                               ((first_col + row) >> 1);
                    store_entry(dst, wtag, f32_to_bf16_rne(vals[q0]) | (f32_to_bf16_rne(vals[q0 + 1]) << 16));
                }
            } else {
                u64 *const obase = cls == 2 ? a.o_sh : a.o;
                const int nblk = item_rows > 16 ? 2 : 1;
                for (int i = 0; i < 4 * nblk; ++i) {
                    const int q = lane + 64 * (i & 3);
                    const int col = (q >> 2) & 15, row = 4 * (q >> 6) + (q & 3) + 16 * (i >> 2);
                    // (column `col` is entry `col` of the expert's list)
                    if (col < m && row < item_rows)
                        store_entry(obase + (size_t)(row0 + col) * H + (first_col + row), wtag,
                                    __float_as_uint(vals[(i >> 2) * 256 + q]));
                }
            }
        }
        o_recs = 0;
        o_used = 0;
    };

    // one tile: park it, refresh the B operand if the expert changed, put the tile two steps ahead in flight,
    // multiply, and on the item's last panel add the partial results up
    auto step = [&](int s, int ti) __attribute__((always_inline)) {
        MOE_CYC_BEGIN();
        const u32x4 d = *(const u32x4 *)(tab_s + (size_t)ti * kTabWords + 4);
        const unsigned fl = (unsigned)__builtin_amdgcn_readfirstlane((int)d.x);
        MOE_CYC(7);
#if defined(MOE_STREAM_TRACE) && MOE_STREAM_TRACE > 1
        // (the wait for the tile alone: one register of its last piece is touched before the parking starts)
        asm volatile("" :: "v"(st[s][NPI - 1]));
#endif
        MOE_CYC(0);
        park(s, (__builtin_amdgcn_readfirstlane((int)d.z) >> 24) & 15);
        MOE_CYC(1);
        if ((fl >> 4) != bx_sig) {
            // (what this workgroup computed of the activations that it, or a workgroup that it waits for, waits
            // for here has left: the gate/up results are flushed before the first down tile's step)
            const int row0 = __builtin_amdgcn_readfirstlane((int)d.y);
            const int m = __builtin_amdgcn_readfirstlane((int)d.w) & 0xff;
            load_bx((int)(fl & 3u), (int)((fl >> 4) & 0xffu), row0, m);
            bx_sig = fl >> 4;
        }
        MOE_CYC(2);
        issue(s, ti + 2);
        MOE_CYC(3);
        __syncthreads();
        MOE_CYC(4);
        if (fl & 4u) {
            acc = (f32x4){0.f, 0.f, 0.f, 0.f};
            acc1 = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        multiply();
        if (fl & 8u) {
            *(f32x4 *)(red_s + w * kRedStride + lane * 16) = acc;
            if (c_two) *(f32x4 *)(red_s + w * kRedStride + 1024 + lane * 16) = acc1;
        }
        MOE_CYC(5);
        __syncthreads();   // every wavefront is done with the tile in LDS (and its partial result is posted)
        MOE_CYC(6);
        if (fl & 8u) {
            reduce_item(ti, fl);
            // out they go: before the first down tile (whose B operand may be what waits here), and when the
            // next item might not fit
            const unsigned nfl = (unsigned)__builtin_amdgcn_readfirstlane((int)tab_s[(size_t)(ti + 1) * kTabWords + 4]);
            const bool leaving_gate_up = (fl & 3u) < 2u && ((nfl & 3u) >= 2u || ti + 1 >= ntiles);
            if (leaving_gate_up || o_recs == kOutRecs || o_used + 512 > kOutBytes / 4) flush();
        }
#ifdef MOE_STREAM_TRACE
        if ((fl & 3u) < 2u) MOE_STAMP(tl_phase);   // (the last gate/up tile leaves the stamp)
        if (ti == 0) MOE_STAMP(tl_first);
#endif
    };

    // (tiles alternate between the two register sets, so the loop body is two steps; the first tile is peeled
    // off so that the loop is always entered in the same state: the compiler then counts the loads in flight
    // exactly and each park waits for its own tile only)
    step(0, 0);
    {
        int t = 1;
        for (; t + 1 < ntiles; t += 2) {
            step(1, t);
            step(0, t + 1);
        }
        if (t < ntiles) step(1, t);
    }
    flush();
    MOE_STAMP(tl_loop);
    __syncthreads();   // (the last reduction has read red_s, which the join reuses)
    finish();
#ifdef MOE_STREAM_TRACE
    if (tid == 0 && blockIdx.x < kTimelineGroups) {
        unsigned long long *tl = g_layer_timeline[blockIdx.x];
        tl[0] = tl_start; tl[1] = tl_lists; tl[2] = tl_first; tl[3] = tl_phase; tl[4] = tl_loop; tl[5] = wall_clock64();
        tl[6] = (unsigned long long)(sg_cnt0 + sg_cnt1) << 32 | (unsigned long long)(sg_cnt2 + sg_cnt3);
        tl[7] = (unsigned long long)ntiles;
    }
    if (lane == 0 && (w == 0 || w == kWaves - 1) && blockIdx.x < kTimelineGroups) {
        unsigned long long *tl = g_layer_timeline[blockIdx.x] + (w == 0 ? 8 : 16);
        for (int i = 0; i < 8; ++i) tl[i] = (unsigned long long)cyc_sum[i];
    }
#endif
}



}  // namespace

namespace {


// rows of a down item whose panel is KP columns wide: as many as fit 64 pieces of 1 KB, 16..32
int down_rows(int KP)
{
    int r = 65536 / (2 * KP);
    return r < 16 ? 16 : r > 32 ? 32 : r;
}

struct LayerGeom {
    int KP_h, KP_f, KP_fs, RD, RDS, tile_bytes, npi;
};

LayerGeom layer_geom(int H, int F, int n_shared, int F_shared)
{
    LayerGeom g;
    g.KP_h = stream_panel_width(H);
    g.KP_f = stream_panel_width(F);
    g.KP_fs = n_shared > 0 ? stream_panel_width(F_shared) : 0;
    g.RD = down_rows(g.KP_f);
    g.RDS = n_shared > 0 ? down_rows(g.KP_fs) : 16;
    int tile = 16 * (2 * g.KP_h + kRowPad), pieces = 16 * 2 * g.KP_h / 1024;
    const int t_d = g.RD * (2 * g.KP_f + kRowPad), p_d = (g.RD * 2 * g.KP_f + 1023) / 1024;
    tile = tile > t_d ? tile : t_d;
    pieces = pieces > p_d ? pieces : p_d;
    if (n_shared > 0) {
        const int t_s = g.RDS * (2 * g.KP_fs + kRowPad), p_s = (g.RDS * 2 * g.KP_fs + 1023) / 1024;
        tile = tile > t_s ? tile : t_s;
        pieces = pieces > p_s ? pieces : p_s;
    }
    g.tile_bytes = (tile + 15) & ~15;
    g.npi = (pieces + 15) / 16;   // (at sixteen wavefronts)
    return g;
}

// upper bound of the tiles in one workgroup's list when G workgroups share the layer
int layer_tab_cap(int T, int C, int H, int F, int n_shared, int F_shared, int G)
{
    const LayerGeom g = layer_geom(H, F, n_shared, F_shared);
    const int np_h = H / g.KP_h, np_f = F / g.KP_f;
    const int np_fs = n_shared > 0 ? F_shared / g.KP_fs : 1;
    const long long n_gs = (long long)n_shared * (n_shared > 0 ? F_shared / 8 : 0);
    const long long n_ds = (long long)n_shared * ((H + g.RDS - 1) / g.RDS);
    const long long t0 = (n_gs / G + 1) * np_h;
    const long long t1 = ((n_gs + (long long)C * (F / 8) + 2) / G + 1) * np_h;
    const long long t2 = (n_ds / G + 1) * np_fs;
    const long long t3 = ((n_ds * np_fs + (long long)C * ((H + g.RD - 1) / g.RD) * np_f) / G / np_f + 2) * np_f;
    const long long cap = t0 + t1 + t2 + t3 + 4;
    return cap > (1 << 20) ? (1 << 20) : (int)cap;
}

size_t layer_lds_bytes(int T, int k, int E, int C, int H, int F, int n_shared, int F_shared, bool route, int tab_cap)
{
    const LayerGeom g = layer_geom(H, F, n_shared, F_shared);
    size_t need = (size_t)g.tile_bytes + kDumpBytes + (size_t)kMaxWaves * kRedStride + kOutBytes +
                  (((size_t)4 * C + 2 * (size_t)T * k + 8 + 2 * kOutRecs + 32 + 24 + 16 + 3) & ~(size_t)3) * 4 +
                  ((size_t)tab_cap + 2) * kTabWords * 4;
    if (route) {
        const size_t r = post_lds_bytes(E, C, T * k, true);
        need = need > r ? need : r;
    }
    return need;
}

}  // namespace

bool use_layer_kernel(int T, int k, int E, int C, int H, int F, int n_shared, int F_shared)
{
    if (T > 16 || C < 1 || C > kMaxC || H % 64 != 0 || F % 64 != 0 || (n_shared > 0 && F_shared % 64 != 0)) return false;
    if (!use_stream_kernels(T, k, C, H, F, n_shared, F_shared)) return false;
    const LayerGeom g = layer_geom(H, F, n_shared, F_shared);
    if (g.npi > 4) return false;
    if ((size_t)T * 8 * (k + n_shared) * 4 > (size_t)g.tile_bytes) return false;   // the strip of the final sum sits in the tile buffer
    const int G = device_cus(nullptr);
    if (G <= 0) return false;
    const int cap = layer_tab_cap(T, C, H, F, n_shared, F_shared, G);
    return layer_lds_bytes(T, k, E, C, H, F, n_shared, F_shared, E > 0, cap) <= (size_t)kLdsBytes;
}

hipError_t launch_layer(const LayerArgs &a, const RouteArgs *route, hipStream_t s)
{
    hipError_t e = hipSuccess;
    const int grid = device_cus(&e);
    if (e != hipSuccess) return e;
    const LayerGeom g = layer_geom(a.H, a.F, a.n_shared, a.F_sh);
    LayerArgs args = a;
    args.KP_h = g.KP_h;
    args.KP_f = g.KP_f;
    args.KP_fs = g.KP_fs;
    args.RD = g.RD;
    args.RDS = g.RDS;
    args.tile_lds_bytes = g.tile_bytes;
    args.tab_cap = layer_tab_cap(a.T, a.C, a.H, a.F, a.n_shared, a.F_sh, grid);
    const int E = route ? route->E : 0;
    const size_t lds = layer_lds_bytes(a.T, a.k, E, a.C, a.H, a.F, a.n_shared, a.F_sh, route != nullptr, args.tab_cap);
    if (lds > (size_t)kLdsBytes || g.npi > 4) return hipErrorInvalidValue;
    if (route && (!route->lists_pub || E > 2 * kWave)) return hipErrorInvalidValue;
    // (the routing steps inside the launch use a thread per assignment, slot and expert)
    if (route && (a.T * a.k > 1024 || a.C > 1024 || E > 1024)) return hipErrorInvalidValue;
    static const void *const fns[2] = {(const void *)layer_kernel<4, false>, (const void *)layer_kernel<4, true>};
    const void *fn = fns[route ? 1 : 0];
    e = allow_full_lds(fn);
    if (e != hipSuccess) return e;
    RouteArgs rargs = {};
    if (route) rargs = *route;
    void *params[] = {&args, &rargs};
    hipError_t le = launch_timed(fn, dim3(grid), dim3(1024), params, lds, s, kKindLayer);
    if (le != hipSuccess) return le;
    return hipGetLastError();
}

hipError_t read_layer_timeline(void *dst, size_t bytes)
{
#ifdef MOE_STREAM_TRACE
    if (bytes != sizeof(g_layer_timeline)) return hipErrorInvalidValue;
    return hipMemcpyFromSymbol(dst, HIP_SYMBOL(g_layer_timeline), sizeof(g_layer_timeline));
#else
    (void)dst; (void)bytes;
    return hipErrorNotSupported;
#endif
}

}  // namespace moe
