// Mixture-of-experts feed-forward of the verification pass on gfx950 (bf16 weights, fp32 accumulation):
// softmax router -> top-k -> renormalised weights; rows bucketed by expert; per expert
// (silu(x Wg^T) * (x Wu^T)) Wd^T; weighted combine.  The paper evaluates such a model (Section 5.3, the
// Qwen3-235B MoE run); the FFN definition itself is the usual one of that model family.
//
// With a few dozen rows per expert the two expert products are bound by streaming the expert weights once
// (1.2 GB a layer at 128 experts of 3 x 2048 x 768), so the kernels are built around that stream: one
// work-group per (expert, strip of output features) pulls its strip of packed weight fragments straight
// from HBM into registers through a ring of loads in flight, while the expert's rows (at most 128 at a time)
// sit in LDS as MFMA operands.  Experts that received no row cost nothing.
#include <hip/hip_runtime.h>

#include "common.h"
#include "kernels.h"

namespace sv {

typedef __attribute__((ext_vector_type(16))) float floatx16;

// ------------------------------------------------------------------ router
// Logits by MFMA (v_mfma_f32_32x32x16_bf16).  A work-group takes 32 rows and one of KQ parts of the reduction;
// each of its four waves covers a quarter of that part for all ET = E/32 expert tiles -- expert rows as the
// first operand straight from the row-major router matrix, the activation fragment straight from the packed
// activations (1 KB contiguous), four slices of loads in flight ahead of the products.  The waves' partial
// logits meet in LDS and leave as one plane [part][row][expert] in global memory.
constexpr int kRouterRows = 32;

template <int ET>
__global__ __launch_bounds__(256) void moe_logits_kernel(MoeArgs a, int KQ) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* logit = reinterpret_cast<float*>(smem);           // [4 waves][32][E + 1]
    const int pitch = a.E + 1, plane = kRouterRows * pitch;
    const int tile = blockIdx.x, kq = blockIdx.y;            // 32-row tile of the packed activations, part of the reduction
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, lg = lane >> 5;
    const int kslices = a.d / 16, nks = kslices / (4 * KQ), ks0 = (kq * 4 + wave) * nks;
    const bf16_t* a_src = a.a + ((int64_t)tile * kslices + ks0) * 512 + lane * 8;
    const bf16_t* w_src = a.w_router + (int64_t)l32 * a.d + ks0 * 16 + 8 * lg;
    constexpr int GS = 4;
    floatx16 acc[ET];
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[et][q] = 0.f;
    u32x4 xa[2][GS], wa[2][GS][ET];
    auto load_group = [&](int g, u32x4 (&x)[GS], u32x4 (&w)[GS][ET]) {
#pragma unroll
        for (int s_ = 0; s_ < GS; ++s_) {
            const int ks = g * GS + s_;
            const bool ok = ks < nks;
            const int kc = ok ? ks : nks - 1;
            const u32x4 xv = *reinterpret_cast<const u32x4*>(a_src + (int64_t)kc * 512);
            x[s_] = ok ? xv : u32x4{0, 0, 0, 0};                // a slice past the end contributes nothing
#pragma unroll
            for (int et = 0; et < ET; ++et) w[s_][et] = *reinterpret_cast<const u32x4*>(w_src + (int64_t)et * 32 * a.d + kc * 16);
        }
    };
    auto mma_group = [&](const u32x4 (&x)[GS], const u32x4 (&w)[GS][ET]) {
#pragma unroll
        for (int s_ = 0; s_ < GS; ++s_)
#pragma unroll
            for (int et = 0; et < ET; ++et)
                acc[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w[s_][et]),
                                                                 __builtin_bit_cast(bf16x8, x[s_]), acc[et], 0, 0, 0);
    };
    const int ngroups = (nks + GS - 1) / GS;
    load_group(0, xa[0], wa[0]);
    for (int g = 0; g < ngroups; g += 2) {
        load_group(g + 1, xa[1], wa[1]);                       // past the end: zero activations
        __builtin_amdgcn_sched_barrier(0);
        mma_group(xa[0], wa[0]);
        __builtin_amdgcn_sched_barrier(0);
        load_group(g + 2, xa[0], wa[0]);
        __builtin_amdgcn_sched_barrier(0);
        mma_group(xa[1], wa[1]);
        __builtin_amdgcn_sched_barrier(0);
    }
    // acc[et][4 q + i] <-> expert et*32 + 8 q + 4 lg + i, row l32
#pragma unroll
    for (int et = 0; et < ET; ++et)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) logit[wave * plane + l32 * pitch + et * 32 + 8 * q + 4 * lg + i] = acc[et][4 * q + i];
    __syncthreads();
    float* dst = a.router_logits + ((int64_t)kq * a.T + (int64_t)tile * 32) * a.E;
    for (int i = threadIdx.x; i < kRouterRows * a.E; i += 256) {
        const int r = i / a.E, e = i % a.E;
        if (tile * 32 + r < a.T)
            dst[(int64_t)r * a.E + e] = (logit[r * pitch + e] + logit[plane + r * pitch + e]) + (logit[2 * plane + r * pitch + e] + logit[3 * plane + r * pitch + e]);
    }
}

// One wave per row: the KQ planes are added in order, softmax over the experts, top_k by repeated arg-max
// (lowest id among equals), renormalisation.
__global__ __launch_bounds__(256) void moe_select_kernel(MoeArgs a, int KQ) {
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= a.T) return;
    constexpr int PER = 4;                                   // experts per lane: E <= 256
    float v[PER];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int e = lane + 64 * i;
        float x = -INFINITY;
        if (e < a.E) {
            x = 0.f;
            for (int kq = 0; kq < KQ; ++kq) x += a.router_logits[((int64_t)kq * a.T + t) * a.E + e];
        }
        v[i] = x;
        mx = fmaxf(mx, x);
    }
    mx = wave_max(mx);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        v[i] = lane + 64 * i < a.E ? expf(v[i] - mx) : -1.f;  // -1 marks "not a candidate"
        sum += v[i] > 0.f ? v[i] : 0.f;
    }
    sum = wave_sum(sum);
    float kept_sum = 0.f, mine = 0.f;
    int mine_id = 0;
    for (int j = 0; j < a.top_k; ++j) {
        float best = -1.f;
        int best_e = 1 << 20;
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (v[i] > best) { best = v[i]; best_e = lane + 64 * i; }     // ascending ids: the first maximum is kept
        const float top = wave_max(best);
        const float cand = best == top ? -(float)best_e : -(float)(1 << 20);
        int win = (int)(-wave_max(cand));                                   // lowest id among the equal maxima
        if (win >= a.E) win = j;                                            // NaN inputs: still a valid expert id
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (lane + 64 * i == win) v[i] = -1.f;
        const float p = top / sum;
        kept_sum += p;
        if (lane == j) { mine = p; mine_id = win; }
    }
    if (lane < a.top_k) {
        a.top_ids[(size_t)t * a.top_k + lane] = mine_id;
        a.top_w[(size_t)t * a.top_k + lane] = mine / kept_sum;
    }
}

// ------------------------------------------------------------------ grouping
// One work-group.  Every (row, expert) assignment sets bit `row` in its expert's bitmap (an OR: the result
// does not depend on the order of the atomics); the rank of a row inside its expert's bucket is the number of
// set bits below it.  Buckets are padded to whole 32-row tiles: bucket e owns padded rows
// 32 * tile_off[e] .. 32 * tile_off[e+1] - 1; perm[padded row] = source row (padding rows name row 0, their
// results are never read), inv[assignment] = padded row.
__global__ __launch_bounds__(1024) void moe_group_kernel(MoeArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int W = (a.T + 31) / 32;
    uint32_t* bm = reinterpret_cast<uint32_t*>(smem);                               // [E][W]
    uint16_t* below = reinterpret_cast<uint16_t*>(smem + (size_t)a.E * W * 4);      // [E][W] set bits in earlier words
    int32_t* offs = reinterpret_cast<int32_t*>(smem + (size_t)a.E * W * 6);          // [E + 1] first tile of a bucket
    int32_t* cnts = offs + a.E + 1;                                                  // [E]
    const int n_asg = a.T * a.top_k;
    for (int i = threadIdx.x; i < a.E * W; i += 1024) bm[i] = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < n_asg; i += 1024) {
        const int e = a.top_ids[i], t = i / a.top_k;
        atomicOr(&bm[e * W + (t >> 5)], 1u << (t & 31));
    }
    __syncthreads();
    for (int e = threadIdx.x; e < a.E; e += 1024) {
        int run = 0;
        for (int w = 0; w < W; ++w) {
            below[e * W + w] = (uint16_t)run;
            run += __popc(bm[e * W + w]);
        }
        cnts[e] = run;
    }
    __syncthreads();
    // first tile of every bucket: exclusive prefix sum of the buckets' tile counts (E <= 256: four waves scan
    // their 64 experts with lane shifts, then add the totals of the waves before them)
    {
        __shared__ int wave_tot[4];
        const int e = threadIdx.x, lane = e & 63;
        const int mine = e < a.E ? (cnts[e] + 31) / 32 : 0;
        int incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        if (e < 256 && lane == 63) wave_tot[e >> 6] = incl;
        __syncthreads();
        if (e < 256) {
            int base = 0;
            for (int w = 0; w < (e >> 6); ++w) base += wave_tot[w];
            if (e < a.E) offs[e] = base + incl - mine;
            if (e == a.E - 1) offs[a.E] = base + incl;
        }
    }
    __syncthreads();
    for (int e = threadIdx.x; e <= a.E; e += 1024) {
        a.tile_off[e] = offs[e];
        if (e < a.E) {
            a.cnt[e] = cnts[e];
            for (int r = cnts[e]; r < (offs[e + 1] - offs[e]) * 32; ++r) a.perm[offs[e] * 32 + r] = 0;
        }
    }
    for (int i = threadIdx.x; i < n_asg; i += 1024) {
        const int e = a.top_ids[i], t = i / a.top_k;
        const int r = below[e * W + (t >> 5)] + __popc(bm[e * W + (t >> 5)] & ((1u << (t & 31)) - 1u));
        const int prow = offs[e] * 32 + r;
        a.inv[i] = prow;
        a.perm[prow] = t;
    }
}

// ------------------------------------------------------------------ rows of a bucket as operand tiles
// The packed activations keep 16 bytes of a row per 1 KB fragment, so a strip that gathered its expert's rows
// itself would pull a whole cache line for every 16 bytes, and every one of the F/64 strips of the expert again
// (measured: 2.7 GB of L2 requests per layer for 0.8 GB of weights).  The gather is done once instead: two
// work-groups copy the 32 rows of one padded tile (half of the slices each) into operand order [tile][d/16][64][8].  The tiles live in
// the buffer of the expert outputs y, which is not written before the first product has read them.
__global__ __launch_bounds__(256) void moe_gather_kernel(MoeArgs a) {
    const int tile = blockIdx.x;
    if (tile >= a.tile_off[a.E]) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kslices = a.d / 16;
    const int t = a.perm[tile * 32 + (lane & 31)];
    const bf16_t* src = a.a + ((int64_t)(t >> 5) * kslices) * 512 + ((t & 31) + 32 * (lane >> 5)) * 8;
    bf16_t* dst = reinterpret_cast<bf16_t*>(a.y) + ((int64_t)tile * kslices) * 512 + lane * 8;
    const int half = kslices / 2;                               // blockIdx.y: which half of the slices
    for (int s0 = blockIdx.y * half + wave * 4; s0 < (blockIdx.y + 1) * half; s0 += 16) {   // four slices in flight per wave
        u32x4 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const u32x4*>(src + (int64_t)(s0 + i) * 512);
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(dst + (int64_t)(s0 + i) * 512) = v[i];
    }
}

// ------------------------------------------------------------------ expert products
// MODE 0: rows = the gathered tiles; waves 0,1 produce 64 gate features, waves 2,3 the 64 up
//         features of the same indices; the epilogue forms silu(gate) * up and writes it, rounded to bf16, as
//         packed MFMA operand tiles for MODE 1.
// MODE 1: rows = those tiles; four waves produce 128 output features; fp32 results go to y[padded row][d].
// A work-group handles the expert's row tiles four at a time (re-streaming its weight strip for experts with
// more than 128 rows).  Products of row tiles beyond the bucket are skipped.
template <int MODE>
__global__ __launch_bounds__(256, 2) void moe_gemm_kernel(MoeArgs a) {
    constexpr int MT = 4, KA = 8, PD = 8;
    __shared__ __attribute__((aligned(16))) unsigned char abuf[2][MT * KA * 1024];
    const int K = MODE == 0 ? a.d : a.F;                    // reduction width
    const int Ntot = MODE == 0 ? 2 * a.F : a.d;             // weight rows per expert
    const int strips = MODE == 0 ? a.F / 64 : a.d / 128;
    // consecutive work-group ids go round the eight XCDs: the strips of an expert are given ids eight apart, so
    // that they share one L2 and the expert's tiles are fetched once (E is a multiple of 8)
    const int grp = blockIdx.x / (8 * strips), in_grp = blockIdx.x % (8 * strips);
    const int e = grp * 8 + (in_grp & 7), p = in_grp >> 3;
    const int tile0 = a.tile_off[e], ntile = a.tile_off[e + 1] - tile0;
    if (ntile == 0) return;
    const int kslices = K / 16, nfill = kslices / KA;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lg = lane >> 5;

    int nt_local;                                           // this wave's 32-feature tile among the expert's rows
    if (MODE == 0) nt_local = wave < 2 ? 2 * p + wave : a.F / 32 + 2 * p + (wave - 2);
    else nt_local = 4 * p + wave;
    const int nt = e * (Ntot / 32) + nt_local;
    const bf16_t* w_src = (MODE == 0 ? a.w_gate_up : a.w_down) + (((int64_t)(nt >> 2) * kslices) * 4 + (nt & 3)) * 512 + lane * 8;
    constexpr int W_STEP = 4 * 512;

    for (int g0 = 0; g0 < ntile; g0 += MT) {
        const int nt_here = ntile - g0 < MT ? ntile - g0 : MT;
        // wave w fills row tile w of the group (all KA slices of a fill); tiles past the bucket repeat its last
        const int my_tile = tile0 + (g0 + wave < ntile ? g0 + wave : ntile - 1);
        const bf16_t* a_src = (MODE == 0 ? reinterpret_cast<const bf16_t*>(a.y) : a.act) + ((int64_t)my_tile * kslices) * 512 + lane * 8;

        floatx16 acc[MT];
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[j][q] = 0.f;

        u32x4 wring[PD];
#pragma unroll
        for (int s = 0; s < PD; ++s)
            wring[s] = *reinterpret_cast<const u32x4*>(w_src + (int64_t)(s < kslices ? s : kslices - 1) * W_STEP);
        u32x4 areg[KA];
#pragma unroll
        for (int i = 0; i < KA; ++i) areg[i] = *reinterpret_cast<const u32x4*>(a_src + (int64_t)i * 512);
#pragma unroll
        for (int i = 0; i < KA; ++i) *reinterpret_cast<u32x4*>(&abuf[0][(wave * KA + i) * 1024 + lane * 16]) = areg[i];

        for (int fill = 0; fill < nfill; ++fill) {
            __builtin_amdgcn_s_waitcnt(0xC07F);             // own LDS writes done
            __builtin_amdgcn_s_barrier();
            const int nxt = fill + 1 < nfill ? fill + 1 : fill;
#pragma unroll
            for (int i = 0; i < KA; ++i) areg[i] = *reinterpret_cast<const u32x4*>(a_src + (int64_t)(nxt * KA + i) * 512);
            const unsigned char* ab = abuf[fill & 1] + lane * 16;
            bf16x8 af[2][MT];
#pragma unroll
            for (int j = 0; j < MT; ++j) af[0][j] = *reinterpret_cast<const bf16x8*>(ab + (j * KA) * 1024);
#pragma unroll
            for (int s = 0; s < KA; ++s) {
                const int slice = fill * KA + s;
                if (s + 1 < KA) {
#pragma unroll
                    for (int j = 0; j < MT; ++j)
                        af[(s + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(ab + (j * KA + s + 1) * 1024);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    if (j < nt_here)      // MODE 1: rows first, so that a half wave stores 128 contiguous bytes of an output row
                        acc[j] = MODE == 0 ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wring[s % PD]),
                                                                                     af[s & 1][j], acc[j], 0, 0, 0)
                                           : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s & 1][j], __builtin_bit_cast(bf16x8, wring[s % PD]),
                                                                                     acc[j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                // refill the slot just consumed (after its readers, so the load lands in place)
                const int ahead = slice + PD < kslices ? slice + PD : kslices - 1;
                wring[s % PD] = *reinterpret_cast<const u32x4*>(w_src + (int64_t)ahead * W_STEP);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < KA; ++i)
                *reinterpret_cast<u32x4*>(&abuf[(fill + 1) & 1][(wave * KA + i) * 1024 + lane * 16]) = areg[i];
        }

        if (MODE == 1) {
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                if (j < nt_here) {
                    // acc[j][4 q + r] <-> padded row 32 (tile0 + g0 + j) + 8 q + 4 lg + r, feature 128 p + 32 wave + l32
                    float* dst = a.y + ((int64_t)(tile0 + g0 + j) * 32 + 4 * lg) * a.d + p * 128 + wave * 32 + l32;
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int r = 0; r < 4; ++r) dst[(int64_t)(8 * q + r) * a.d] = acc[j][4 * q + r];
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();                   // every wave is done with abuf before the next group refills it
        } else {
            // up halves travel through LDS to the waves that hold the gate halves of the same features
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();                   // all reads of abuf are over
            float* xbuf = reinterpret_cast<float*>(&abuf[0][0]);     // [2 waves][MT][16][64] floats = 32 KB
            if (wave >= 2) {
#pragma unroll
                for (int j = 0; j < MT; ++j)
#pragma unroll
                    for (int q = 0; q < 16; ++q) xbuf[(((wave - 2) * MT + j) * 16 + q) * 64 + lane] = acc[j][q];
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();
            if (wave < 2) {
                const int fs = (p * 64 + wave * 32) / 16;     // first 16-wide feature slice of this wave
#pragma unroll
                for (int j = 0; j < MT; ++j) {
                    if (j < nt_here) {
                        bf16_t* dst = a.act + ((int64_t)(tile0 + g0 + j) * (a.F / 16) + fs) * 512;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float r[4];
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float g = acc[j][4 * q + i];
                                const float u = xbuf[((wave * MT + j) * 16 + 4 * q + i) * 64 + lane];
                                r[i] = g / (1.0f + expf(-g)) * u;
                            }
                            // features 8q + 4 lg .. +3 of this wave's 32: slice q/2, half q%2, elements 4 lg ..
                            u32x2 pk = {pack2bf(r[0], r[1]), pack2bf(r[2], r[3])};
                            *reinterpret_cast<u32x2*>(dst + ((q >> 1) * 64 + l32 + 32 * (q & 1)) * 8 + 4 * lg) = pk;
                        }
                    }
                }
            }
            __builtin_amdgcn_s_waitcnt(0xC07F);
            __builtin_amdgcn_s_barrier();                   // xbuf is read before the next group overwrites it
        }
    }
}

// ------------------------------------------------------------------ combine
// out[t][:] = sum over the row's top_k experts, in slot order, of weight * y[padded row of that assignment][:]
__global__ __launch_bounds__(256) void moe_combine_kernel(MoeArgs a) {
    const int t = blockIdx.x;
    for (int c = threadIdx.x * 4; c < a.d; c += 1024) {
        floatx4 s = {0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < a.top_k; ++j) {
            const float w = a.top_w[(size_t)t * a.top_k + j];
            const floatx4 v = *reinterpret_cast<const floatx4*>(a.y + (int64_t)a.inv[(size_t)t * a.top_k + j] * a.d + c);
            s[0] = fmaf(w, v[0], s[0]); s[1] = fmaf(w, v[1], s[1]); s[2] = fmaf(w, v[2], s[2]); s[3] = fmaf(w, v[3], s[3]);
        }
        *reinterpret_cast<floatx4*>(a.out + (int64_t)t * a.d + c) = s;
    }
}

int moe_shape_ok(int T, int d, int E, int top_k, int F) {
    if (T <= 0 || d <= 0 || E <= 0 || top_k <= 0 || F <= 0) return 0;
    if (E % 64 != 0 || E > 256 || top_k > E || top_k > 64) return 0;       // router: 32-expert MFMA tiles, four experts per lane, top_k <= lanes
    if (d % 128 != 0 || F % 128 != 0) return 0;                            // eight 16-wide slices per fill; 128-feature strips
    if (moe_group_lds_bytes(T, E) > 150 * 1024 || (size_t)4 * kRouterRows * (E + 1) * 4 > 150 * 1024) return 0;
    return 1;
}

size_t moe_group_lds_bytes(int T, int E) {
    const size_t W = (T + 31) / 32;
    return (size_t)E * W * 6 + (size_t)(2 * E + 1) * 4 + 16;
}

int moe_max_tiles(int T, int E, int top_k) { return (T * top_k) / 32 + E; }

hipError_t moe_ffn(const MoeArgs& a, hipStream_t st) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(moe_group_kernel),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
        if (e1 != hipSuccess) return e1;
        for (const void* k : {reinterpret_cast<const void*>(moe_logits_kernel<2>), reinterpret_cast<const void*>(moe_logits_kernel<4>),
                              reinterpret_cast<const void*>(moe_logits_kernel<6>), reinterpret_cast<const void*>(moe_logits_kernel<8>)}) {
            hipError_t e2 = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
            if (e2 != hipSuccess) return e2;
        }
        attr_set = true;
    }
    // parts of the router's reduction: as many as leave every wave at least two 16-wide slices, at most four
    const int kslices = a.d / 16;
    int KQ = 4;
    while (KQ > 1 && (kslices % (4 * KQ) != 0 || kslices / (4 * KQ) < 2)) KQ >>= 1;
    const size_t router_lds = (size_t)4 * kRouterRows * (a.E + 1) * 4;
    const dim3 rgrid((a.T + kRouterRows - 1) / kRouterRows, KQ);
    switch (a.E / 32) {
        case 2: hipLaunchKernelGGL(moe_logits_kernel<2>, rgrid, dim3(256), router_lds, st, a, KQ); break;
        case 4: hipLaunchKernelGGL(moe_logits_kernel<4>, rgrid, dim3(256), router_lds, st, a, KQ); break;
        case 6: hipLaunchKernelGGL(moe_logits_kernel<6>, rgrid, dim3(256), router_lds, st, a, KQ); break;
        case 8: hipLaunchKernelGGL(moe_logits_kernel<8>, rgrid, dim3(256), router_lds, st, a, KQ); break;
        default: return hipErrorInvalidValue;
    }
    hipLaunchKernelGGL(moe_select_kernel, dim3((a.T + 3) / 4), dim3(256), 0, st, a, KQ);
    hipLaunchKernelGGL(moe_group_kernel, dim3(1), dim3(1024), moe_group_lds_bytes(a.T, a.E), st, a);
    hipLaunchKernelGGL(moe_gather_kernel, dim3(moe_max_tiles(a.T, a.E, a.top_k), 2), dim3(256), 0, st, a);
    hipLaunchKernelGGL(moe_gemm_kernel<0>, dim3(a.E * (a.F / 64)), dim3(256), 0, st, a);
    hipLaunchKernelGGL(moe_gemm_kernel<1>, dim3(a.E * (a.d / 128)), dim3(256), 0, st, a);
    if (a.out) hipLaunchKernelGGL(moe_combine_kernel, dim3(a.T), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace sv
