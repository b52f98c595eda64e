// Expert FFN of the verify-step MoE layer (gfx950): for every resident slot c
// and each token routed to it
//      o = W_down[c] ( silu(W_gate[c] x) * (W_up[c] x) )
// (Sec. 2.2 last line; the gate/up/down matrices and the skip of non-resident
// experts are App. D), followed by the gate-weighted combine into token order.
//
// The work is weight streaming: each bf16 weight is read from HBM exactly
// once per layer call.  One workgroup owns (slot, slice of 128 FFN rows):
//   phase 1  gate/up rows of the slice against all H      -> act[tokens,128] in LDS
//   phase 2  W_down[:, slice] against act                 -> partial o[tokens,H]
// so gate/up/down of an expert stream in one launch, and the slices' partial
// sums are added in a fixed order by the combine kernel (no float atomics:
// the result does not depend on scheduling).
//
// MFMA 16x16x32 bf16 puts 16 weight rows on the M axis and up to 16 tokens on
// the N axis; tokens beyond the routed ones are zero columns that cost
// nothing, because the kernel is bound by the weight bytes.
#include "moe_internal.h"

namespace moe {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWaves = kFfnThreads / kWave;   // 8
constexpr int kStepK = 128;                   // contraction elements per pipeline step (4 MFMAs)
constexpr int kActStride = kSliceF * 2 + 16;  // bytes per act row in LDS (padded)
constexpr int kStages = 4;                    // gate/up steps in flight per wavefront
constexpr int kDownStages = 4;                // down row tiles in flight per wavefront

__device__ inline u32x4 ld_stream(const uint16_t *p)
{
    // weights are read once: keep them out of the way of the activations in cache
    return __builtin_nontemporal_load((const u32x4 *)p);
}

__device__ inline bf16x8 as_bf16(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ inline f32x4 mfma(u32x4 a, bf16x8 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16(a), b, c, 0, 0, 0);
}

// NT = token tiles of 16 processed per pass over the weights.  RAGGED: H or an F is a multiple of 8 only;
// rows and contraction blocks that reach past the end of a matrix are masked lane by lane (loads become
// zeros, stores are skipped), in plain loops without the deep pipelines.
template <int NT, bool RAGGED>
__global__ __launch_bounds__(kFfnThreads) void ffn_kernel(FfnArgs a, int nsl, int nsl_sh, int xs /*bytes per x row in LDS*/)
{
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *x_s = lds;
    unsigned char *act_s = lds + (size_t)NT * 16 * xs;

    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    const int n = lane & 15, g = lane >> 4;
    const int H = a.H;

    // which (expert, slice) is this workgroup?  shared experts come first
    int b = blockIdx.x;
    const bool is_shared = b < a.n_shared * nsl_sh;
    int F, slice, m, base;
    const uint16_t *wg, *wu, *wd;
    float *part;
    if (is_shared) {
        int i = b / nsl_sh;
        slice = b - i * nsl_sh;
        F = a.F_shared;
        size_t off = (size_t)i * F * H;
        wg = (const uint16_t *)a.sh_gate + off;
        wu = (const uint16_t *)a.sh_up + off;
        wd = (const uint16_t *)a.sh_down + off;
        m = a.T;
        base = 0;
        part = a.part_sh + (size_t)(i * nsl_sh + slice) * a.T * H;
    } else {
        b -= a.n_shared * nsl_sh;
        int c = b / nsl;
        slice = b - c * nsl;
        F = a.F;
        m = a.slot_count[c];
        if (m == 0) return;   // no token of this batch uses the slot: nothing to stream
        base = a.slot_offset[c];
        size_t off = (size_t)c * F * H;
        wg = (const uint16_t *)a.w_gate + off;
        wu = (const uint16_t *)a.w_up + off;
        wd = (const uint16_t *)a.w_down + off;
        part = a.part + ((size_t)slice * a.T * a.k + base) * H;
    }
    const int f0 = slice * kSliceF;
    const bool wave_has_rows = f0 + 16 * w < F;      // (not RAGGED: F is a multiple of 32)
    const int nkb_down = (F - f0 + 31) / 32 < 4 ? (F - f0 + 31) / 32 : 4;
    const uint16_t *xg = (const uint16_t *)a.hidden;

    for (int r0 = 0; r0 < m; r0 += NT * 16) {
        // ---- gather the routed tokens' hidden rows into LDS (zero rows beyond m) ----
        const int chunks_per_row = (H + 31) / 32 * 4;   // (zeros up to the next multiple of 32 columns)
        for (int q = tid; q < NT * 16 * chunks_per_row; q += kFfnThreads) {
            int r = q / chunks_per_row, col = q - r * chunks_per_row;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (r0 + r < m && col * 8 < H) {
                int t = is_shared ? (r0 + r) : a.perm[base + r0 + r] / a.k;
                v = *(const u32x4 *)(xg + (size_t)t * H + col * 8);
            }
            *(u32x4 *)(x_s + (size_t)r * xs + col * 16) = v;
        }
        __syncthreads();

        // ---- phase 1: gate/up rows f0+16w .. +16 over the whole of H ----
        f32x4 accg[NT], accu[NT];
#pragma unroll
        for (int tl = 0; tl < NT; ++tl) { accg[tl] = (f32x4){0.f, 0.f, 0.f, 0.f}; accu[tl] = accg[tl]; }
        if (RAGGED && wave_has_rows) {
            const int row = f0 + 16 * w + n;
            const bool row_ok = row < F;
            const size_t roff = (size_t)(row_ok ? row : F - 1) * H;
            const unsigned char *xb = x_s + (size_t)n * xs + g * 16;
            for (int kb = 0; kb < (H + 31) / 32; ++kb) {
                const int col = kb * 32 + g * 8;
                const bool ok = row_ok && col < H;
                const u32x4 zero = {0u, 0u, 0u, 0u};
                const u32x4 tg = ok ? ld_stream(wg + roff + col) : zero;
                const u32x4 tu = ok ? ld_stream(wu + roff + col) : zero;
#pragma unroll
                for (int tl = 0; tl < NT; ++tl) {
                    bf16x8 bx = *(const bf16x8 *)(xb + (size_t)tl * 16 * xs + kb * 64);
                    accg[tl] = mfma(tg, bx, accg[tl]);
                    accu[tl] = mfma(tu, bx, accu[tl]);
                }
            }
        } else if (wave_has_rows) {
            const uint16_t *pg = wg + (size_t)(f0 + 16 * w + n) * H + g * 8;
            const uint16_t *pu = wu + (size_t)(f0 + 16 * w + n) * H + g * 8;
            const unsigned char *xb = x_s + (size_t)n * xs + g * 16;
            const int nks = H / kStepK;
            u32x4 ag[kStages][4], au[kStages][4];
            // one pipeline step = 128 contraction elements = 4 MFMAs per matrix and token tile
            auto load_step = [&](int s) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ag[s][i] = ld_stream(pg + i * 32);
                    au[s][i] = ld_stream(pu + i * 32);
                }
                pg += kStepK;
                pu += kStepK;
            };
            auto compute_step = [&](int s) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
#pragma unroll
                    for (int tl = 0; tl < NT; ++tl) {
                        bf16x8 bx = *(const bf16x8 *)(xb + (size_t)tl * 16 * xs + i * 64);
                        accg[tl] = mfma(ag[s][i], bx, accg[tl]);
                        accu[tl] = mfma(au[s][i], bx, accu[tl]);
                    }
                }
                xb += kStepK * 2;
            };
            if (nks >= kStages && nks % kStages == 0) {
                // steady state: kStages steps (kStages * 8 KB per wavefront) always in flight
#pragma unroll
                for (int s = 0; s < kStages; ++s) load_step(s);
                for (int ks = kStages; ks < nks; ks += kStages) {
#pragma unroll
                    for (int s = 0; s < kStages; ++s) { compute_step(s); load_step(s); }
                }
#pragma unroll
                for (int s = 0; s < kStages; ++s) compute_step(s);
            } else {
                for (int ks = 0; ks < nks; ++ks) { load_step(0); compute_step(0); }
            }
            // ragged end of H (H is a multiple of 32)
            const int rem = (H - nks * kStepK) / 32;
            for (int i = 0; i < rem; ++i) {
                u32x4 tg = ld_stream(pg + i * 32);
                u32x4 tu = ld_stream(pu + i * 32);
#pragma unroll
                for (int tl = 0; tl < NT; ++tl) {
                    bf16x8 bx = *(const bf16x8 *)(xb + (size_t)tl * 16 * xs + i * 64);
                    accg[tl] = mfma(tg, bx, accg[tl]);
                    accu[tl] = mfma(tu, bx, accu[tl]);
                }
            }
        }
        // act = silu(gate) * up, rounded to bf16, to LDS as [token][f within slice]
#pragma unroll
        for (int tl = 0; tl < NT; ++tl) {
            uint32_t pk[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float gt = accg[tl][j], up = accu[tl][j];
                float act = gt / (1.f + expf(-gt)) * up;
                pk[j] = wave_has_rows ? f32_to_bf16_rne(act) : 0u;
            }
            u32x2 v = {pk[0] | (pk[1] << 16), pk[2] | (pk[3] << 16)};
            *(u32x2 *)(act_s + (size_t)(tl * 16 + n) * kActStride + (16 * w + 4 * g) * 2) = v;
        }
        __syncthreads();

        // ---- phase 2: partial down projection over this slice of F ----
        bf16x8 bact[NT][4];
#pragma unroll
        for (int tl = 0; tl < NT; ++tl)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                bact[tl][i] = *(const bf16x8 *)(act_s + (size_t)(tl * 16 + n) * kActStride + (i * 32 + g * 8) * 2);

        const int nrt = (H + 15) / 16;                // output row tiles, dealt round-robin to wavefronts
        const int my_tiles = (nrt - w + kWaves - 1) / kWaves;
        const uint16_t *pd = wd + (size_t)(16 * w + n) * F + f0 + g * 8;
        const size_t tile_step = (size_t)16 * kWaves * F;
        float *po = part + (size_t)(r0 + n) * H + 16 * w + 4 * g;   // this lane's 4 outputs of its first tile
        u32x4 ad[kDownStages][4];
        auto load_tile = [&](int s) {
#pragma unroll
            for (int i = 0; i < 4; ++i) ad[s][i] = ld_stream(pd + i * 32);
            pd += tile_step;
        };
        auto compute_tile = [&](int s) {
#pragma unroll
            for (int tl = 0; tl < NT; ++tl) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < 4; ++i) acc = mfma(ad[s][i], bact[tl][i], acc);
                if (r0 + tl * 16 + n < m) *(f32x4 *)(po + (size_t)tl * 16 * H) = acc;
            }
            po += 16 * kWaves;
        };
        if (RAGGED) {
            const u32x4 zero = {0u, 0u, 0u, 0u};
            for (int it = 0; it < my_tiles; ++it) {
                const int row = 16 * (w + it * kWaves) + n;          // this lane's weight row (an output column)
                const bool row_ok = row < H;
                const uint16_t *prow = wd + (size_t)(row_ok ? row : H - 1) * F;
                const bool store_ok = 16 * (w + it * kWaves) + 4 * g < H;   // the lane's four outputs: all in or all out
#pragma unroll
                for (int tl = 0; tl < NT; ++tl) {
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    for (int i = 0; i < nkb_down; ++i) {
                        const int col = f0 + i * 32 + g * 8;
                        acc = mfma(row_ok && col < F ? ld_stream(prow + col) : zero, bact[tl][i], acc);
                    }
                    if (store_ok && r0 + tl * 16 + n < m) *(f32x4 *)(po + (size_t)tl * 16 * H) = acc;
                }
                po += 16 * kWaves;
            }
        } else if (nkb_down == 4 && my_tiles >= kDownStages && my_tiles % kDownStages == 0) {
#pragma unroll
            for (int s = 0; s < kDownStages; ++s) load_tile(s);
            for (int it = kDownStages; it < my_tiles; it += kDownStages) {
#pragma unroll
                for (int s = 0; s < kDownStages; ++s) { compute_tile(s); load_tile(s); }
            }
#pragma unroll
            for (int s = 0; s < kDownStages; ++s) compute_tile(s);
        } else {
            // short slice (F not a multiple of 128) or a tile count the pipeline does not divide
            for (int it = 0; it < my_tiles; ++it) {
#pragma unroll
                for (int tl = 0; tl < NT; ++tl) {
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
                    for (int i = 0; i < nkb_down; ++i) acc = mfma(ld_stream(pd + i * 32), bact[tl][i], acc);
                    if (r0 + tl * 16 + n < m) *(f32x4 *)(po + (size_t)tl * 16 * H) = acc;
                }
                pd += tile_step;
                po += 16 * kWaves;
            }
        }
        __syncthreads();   // LDS is reused by the next token group
    }
}

// out[t,:] (+)= sum_j w[t,j] * (sum over slices of partial o) + shared experts, in a fixed order.
__global__ __launch_bounds__(256) void combine_kernel(CombineArgs a, int nsl, int nsl_sh)
{
    const int t = blockIdx.y;
    const int h = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (h >= a.H) return;
    const size_t A = (size_t)a.T * a.k;
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
    for (int j = 0; j < a.k; ++j) {
        int p = a.pos[(size_t)t * a.k + j];
        if (p < 0) continue;
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
        for (int sl = 0; sl < nsl; ++sl) s += *(const f32x4 *)(a.part + ((size_t)sl * A + p) * a.H + h);
        acc += a.topk_w[(size_t)t * a.k + j] * s;
    }
    for (int i = 0; i < a.n_shared; ++i)
        for (int sl = 0; sl < nsl_sh; ++sl)
            acc += *(const f32x4 *)(a.part_sh + ((size_t)(i * nsl_sh + sl) * a.T + t) * a.H + h);
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

// (x rows in LDS reach the next multiple of 32 columns, zero-filled)
static int x_row_bytes(int H) { return 2 * ((H + 31) / 32 * 32) + 16; }

size_t ffn_lds_bytes(int H, int nt)
{
    return (size_t)nt * 16 * (size_t)x_row_bytes(H) + (size_t)nt * 16 * kActStride;
}

int ffn_token_tiles(int T, int H)
{
    if (T > 16 && ffn_lds_bytes(H, 2) <= (size_t)kLdsBytes) return 2;
    if (ffn_lds_bytes(H, 1) <= (size_t)kLdsBytes) return 1;
    return 0;
}

hipError_t launch_ffn(const FfnArgs &a, hipStream_t s)
{
    const int nsl = n_slices(a.F), nsl_sh = a.n_shared ? n_slices(a.F_shared) : 0;
    const int blocks = a.C * nsl + a.n_shared * nsl_sh;
    if (blocks == 0) return hipSuccess;
    const int nt = ffn_token_tiles(a.T, a.H);
    if (nt == 0) return hipErrorInvalidValue;
    const size_t lds = ffn_lds_bytes(a.H, nt);
    const int xs = x_row_bytes(a.H);
    const bool ragged = a.H % 32 != 0 || a.F % 32 != 0 || (a.n_shared && a.F_shared % 32 != 0);
    static const void *const fns[2][2] = {{(const void *)ffn_kernel<1, false>, (const void *)ffn_kernel<1, true>},
                                          {(const void *)ffn_kernel<2, false>, (const void *)ffn_kernel<2, true>}};
    const void *fn = fns[nt - 1][ragged ? 1 : 0];
    hipError_t e = allow_full_lds(fn);
    if (e != hipSuccess) return e;
    FfnArgs args = a;
    int nsl_a = nsl, nsl_sh_a = nsl_sh, xs_a = xs;
    void *params[] = {&args, &nsl_a, &nsl_sh_a, &xs_a};
    e = launch_timed(fn, dim3(blocks), dim3(kFfnThreads), params, lds, s, 2);
    return e != hipSuccess ? e : hipGetLastError();
}

hipError_t launch_combine(const CombineArgs &a, hipStream_t s)
{
    const int nsl = n_slices(a.F), nsl_sh = a.n_shared ? n_slices(a.F_shared) : 0;
    dim3 grid((a.H / 4 + 255) / 256, a.T);
    prof_begin(3, s);
    hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, s, a, nsl, nsl_sh);
    prof_end(3, s);
    return hipGetLastError();
}

}  // namespace moe
