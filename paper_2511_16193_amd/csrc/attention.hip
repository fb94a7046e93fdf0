// Verify attention: the n new rows of every request attend that request's paged KV cache plus the
// new rows they are allowed to see.  Every cached byte is read once per step however many rows
// verify against it -- that reuse across the k+1 rows is the saving of parallel verification -- so
// the kernel is bound by HBM bandwidth and is organised around streaming K/V.
//
// bf16 path (head_dim 128).  A work-group owns one (request, kv head, chunk of keys) and R tiles of 16 of the
// G*n query rows that share the kv head (G = q heads per kv head), stacked.  Each of its waves walks its own
// 32-key tiles of the chunk: K (32 x 128) and V^T (128 x 32) of a tile are stored in the page in MFMA operand
// order, S^T = K Q^T is formed with v_mfma_f32_16x16x32_bf16, the online softmax runs in fp32 on the four keys
// per row each lane holds, and P^T (as two or three bf16 terms) goes back as the B operand of O^T += V^T P^T.  The score
// tile's register layout (a lane holds 4 consecutive keys of one row, for two 16-key blocks) is used unchanged as
// the PV operand; the reduction index of that MFMA is only a label, so V^T is simply stored with the same key
// order.  Waves are merged through LDS, chunks by a second small kernel (split-KV).
// Two kernels: up to 48 stacked rows in one work-group, tiles are prefetched into registers and handled one after
// the other; with more rows, tiles travel through an LDS ring and the three stages of consecutive tiles are woven
// into one instruction stream.
//
// Generic path (fp32 models, other head sizes, more than 64 stacked rows): one wave per (row, head),
// plain online softmax; correct for every shape, not tuned.
#include <math.h>
#include <algorithm>
#include <type_traits>
#include "common.h"
#include "kernels.h"

namespace sv {

constexpr int HD = 128;
constexpr int TILE_KEYS = 32;

struct KTile { u32x4 k[2][4]; u32x4 v[8]; };
constexpr int kTileBytes = 2 * TILE_KEYS * HD * 2;     // K and V of one 32-key tile: 16 KB
// Largest of the eight scores a lane holds of one row tile, for the kernel whose time is its instruction count (the
// skewed one below).  Written as the instructions themselves: through fmaxf the compiler first passes every score
// through a v_max_f32 x, x, x of its own (it must assume signalling NaNs in what an MFMA returns), eleven
// instructions where four do.
__device__ __forceinline__ float max8(const floatx4& a, const floatx4& b) {
    float r, t;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a[0]), "v"(a[1]), "v"(a[2]));
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(t) : "v"(a[3]), "v"(b[0]), "v"(b[1]));
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(r), "v"(b[2]), "v"(b[3]));
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(r), "v"(t));
    return r;
}

// ---- Up to three row tiles in one work-group (at most 48 stacked rows) ----
// Four waves per work-group, one work-group per CU (two with a single row tile); each wave has the next tile's
// loads in flight in a second register set while it works on the current one.  Tile after tile per wave: scores,
// online softmax, PV, not skewed.  At these sizes the kernel runs at the rate the cache can be streamed at, and
// inside a verification step it measured 3-14 % faster than the skewed kernel below (which is ahead once the
// products dominate: four row tiles, or several row groups streaming the same keys).
template <int R>
__global__ __launch_bounds__(256, R == 1 ? 2 : 1) void attn_bf16_regs_kernel(AttnArgs a, float scale_log2e) {
    // work item = one piece of one request's keys, cut by the host from its upper bounds of the lengths.
    // Launch order: the kv heads of an item are neighbours, so the list's longest-first order holds chip-wide.
    // With more than 64 stacked rows the row tiles are split over row_groups work-groups that stream the same
    // keys; work-group ids 8 apart run on the same XCD, so the groups of one (item, head) are placed 8 apart
    // and started together: the second reader of a tile finds it in that XCD's L2.
    const int slot = blockIdx.x / (8 * a.row_groups), rem = blockIdx.x % (8 * a.row_groups);
    const int rg = rem >> 3, pair = slot * 8 + (rem & 7);
    const int n_items = a.n_work_dev ? *a.n_work_dev : a.n_work;
    if (pair >= n_items * a.Hkv) return;
    const int hkv = pair % a.Hkv;
    const int4 item = reinterpret_cast<const int4*>(a.work)[pair / a.Hkv];
    const int b = item.x >> 16, chunk = item.x & 0xffff;
    const int seq = item.y;
    const int L = a.seq_len[seq];
    const int total = L + a.n;
    const int kbeg = item.z;
    if (kbeg >= total) return;                            // the live length fell short of the host's bound
    const int kend = min(item.w, total);
    const int row0 = rg * R * 16;                         // first stacked row of this work-group
    const int G = a.Hq / a.Hkv, rows = G * a.n;

    const int tid = threadIdx.x, lane = tid & 63;
    // wave index as a scalar: tile numbers, page-table reads and page addresses stay on the scalar unit
    // (a vector page-table load would have to be waited for with vmcnt(0), draining the K/V prefetch)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    const bf16_t* pool = reinterpret_cast<const bf16_t*>(a.pool);
    const int page_shift = 31 - __builtin_clz(a.geom.page_size), page_mask = a.geom.page_size - 1;
    const int32_t* pages = a.page_table + (int64_t)seq * a.max_pages_per_seq;

    // Q^T operand: lane holds row rt*16 + l16, head_dim slice kk*32 + lg*8 .. +8
    u32x4 qf[R][4];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int r = row0 + rt * 16 + l16;
        const bool ok = r < rows;
        const int j = ok ? r / G : 0, hl = ok ? r % G : 0;
        const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + (((int64_t)b * a.n + j) * a.Hq + hkv * G + hl) * HD;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qf[rt][kk] = ok ? *reinterpret_cast<const u32x4*>(qp + kk * 32 + lg * 8) : u32x4{0, 0, 0, 0};
    }

    // A row sees every cached key, x0 (key L) and the drafts of its own chain up to itself: the keys
    // [vis_lo, vis_hi).  Rows of x0 and padding rows get an empty interval.
    int vis_lo[R], vis_hi[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int r = row0 + rt * 16 + l16;
        const int j = r < rows ? r / G : 0;
        vis_lo[rt] = j > 0 ? L + 1 + row_chain(j, a.k) * a.k : 0;
        vis_hi[rt] = j > 0 ? vis_lo[rt] + row_index_in_chain(j, a.k) : 0;
    }

    floatx4 o[8][R];
    float m_run[R], mc[R], l_run[R];      // reference maximum (raw score), the same times scale*log2(e), partial sum
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        m_run[rt] = -INFINITY;
        mc[rt] = 0.f;
        l_run[rt] = 0.f;
#pragma unroll
        for (int ht = 0; ht < 8; ++ht) o[ht][rt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // The tile's base address is wave-uniform (scalar page number, head, offset): it is kept in scalar registers
    // and every load is "scalar base + lane offset + immediate".  With per-lane 64-bit addresses in vector
    // registers the compiler, short of registers, computed the next tile's address into registers that an
    // in-flight load was still to fill, and had to wait for that load -- and, loads returning in order, for the
    // whole previous tile -- before it could issue the rest: the prefetch never overlapped anything.
    auto uniform = [](int64_t v) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    const int lane_off = lane * 8;
    auto load_tile = [&](int key0, KTile& t) {
        const int page = pages[key0 >> page_shift];
        const int off = key0 & page_mask;
        const int64_t ki = kv_k_index(a.geom, a.layer, page, hkv, off, 0), vi = kv_v_index(a.geom, a.layer, page, hkv, off, 0);
        // one scalar base per 4 KB (the immediate offset of a load reaches 4095 bytes)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const bf16_t* kp = pool + uniform(ki + kb * 2048);
            const bf16_t* vp = pool + uniform(vi + kb * 2048);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                t.k[kb][kk] = *reinterpret_cast<const u32x4*>(kp + kk * 512 + lane_off);
                t.v[kb * 4 + kk] = *reinterpret_cast<const u32x4*>(vp + kk * 512 + lane_off);
            }
        }
    };

    // One 32-key tile: scores, online softmax, PV.  key0 >= kInvalidKey marks a tile past the end of the
    // chunk (its registers hold a re-load of the last tile): every key is masked and nothing changes.
    constexpr int kInvalidKey = 0x3fffffff;
    auto process = [&](const KTile& t, int key0) {
        // S^T = K Q^T (raw dot products): s[kb][rt][i] <-> key key0 + kb*16 + 4*lg + i, row rt*16 + l16
        floatx4 s[2][R];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, t.k[kb][kk]), __builtin_bit_cast(bf16x8, qf[rt][kk]), acc, 0, 0, 0);
                s[kb][rt] = acc;
            }
        if (key0 + TILE_KEYS > L) {   // tile touches the new rows or the end: apply visibility
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int rt = 0; rt < R; ++rt)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int key = key0 + kb * 16 + 4 * lg + i;
                        // bitwise, not short-circuit: this must stay a compare + select chain.  (With
                        // && / || the compiler built branches here and dropped the value of the first
                        // element on the path "beyond L, yet visible".)
                        const bool vis = (key <= L) | ((key >= vis_lo[rt]) & (key < vis_hi[rt]));
                        s[kb][rt][i] = vis ? s[kb][rt][i] : -INFINITY;
                    }
        }
        // Lazy reference maximum.  The softmax reference m_ref of a row is common to the 4 lane groups
        // that share the row (they feed one MFMA accumulator) and is only moved when some score would
        // make 2^(c(s - m_ref)) exceed 2^16 (or on the row's first visible key): fp32 has the range to
        // spare, and the cross-lane reduction + accumulator rescale leave the per-tile path.
        bool trig = false;
        float lmax[R];
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            lmax[rt] = fmaxf(fmaxf(fmaxf(s[0][rt][0], s[0][rt][1]), fmaxf(s[0][rt][2], s[0][rt][3])),
                             fmaxf(fmaxf(s[1][rt][0], s[1][rt][1]), fmaxf(s[1][rt][2], s[1][rt][3])));
            trig |= ((m_run[rt] == -INFINITY) & (lmax[rt] > -INFINITY)) | (fmaf(lmax[rt], scale_log2e, -mc[rt]) > 16.0f);
        }
        if (__any(trig)) {
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                float mx = lmax[rt];
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(m_run[rt], mx);
                const float mc_new = m_new == -INFINITY ? 0.f : m_new * scale_log2e;
                const float alpha = m_run[rt] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mc[rt] - mc_new);
                l_run[rt] *= alpha;
#pragma unroll
                for (int ht = 0; ht < 8; ++ht) o[ht][rt] = o[ht][rt] * alpha;
                m_run[rt] = m_new;
                mc[rt] = mc_new;
            }
        }
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            floatx2 p[4];
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                p[i] = floatx2{__builtin_amdgcn_exp2f(fmaf(s[0][rt][2 * i], scale_log2e, -mc[rt])),
                               __builtin_amdgcn_exp2f(fmaf(s[0][rt][2 * i + 1], scale_log2e, -mc[rt]))};
                p[2 + i] = floatx2{__builtin_amdgcn_exp2f(fmaf(s[1][rt][2 * i], scale_log2e, -mc[rt])),
                                   __builtin_amdgcn_exp2f(fmaf(s[1][rt][2 * i + 1], scale_log2e, -mc[rt]))};
                psum += (p[i].x + p[i].y) + (p[2 + i].x + p[2 + i].y);
            }
            l_run[rt] += psum;
            // P goes to the MFMA as three bf16 terms (24 significant bits in all).  One bf16 term would
            // leave a 2^-9 relative error in the output however many keys there are (V has zero mean, so
            // the output is as small as the error's random walk); two terms leave 2^-17, still enough to
            // move every few-hundredth output across a bf16 rounding boundary.
            u32x4 pf[3];
#pragma unroll
            for (int tm = 0; tm < 3; ++tm)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bf16x2 hb = __builtin_convertvector(p[i], bf16x2);
                    pf[tm][i] = __builtin_bit_cast(uint32_t, hb);
                    if (tm < 2) p[i] = p[i] - __builtin_convertvector(hb, floatx2);
                }
#pragma unroll
            for (int ht = 0; ht < 8; ++ht) {
                const u32x4 vf = t.v[ht];
#pragma unroll
                for (int tm = 2; tm >= 0; --tm)
                    o[ht][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vf),
                                                                        __builtin_bit_cast(bf16x8, pf[tm]), o[ht][rt], 0, 0, 0);
            }
        }
    };

    // Two tiles per trip, ping-pong between two register sets: while one tile is processed the loads of the next
    // are in flight.  (A third set in flight was measured and does not pay: per tile the wave is bound by its own
    // instruction issue -- 96 MFMAs plus the softmax arithmetic at three row tiles -- not by the load latency.)
    // Loads are unconditional (past the end they re-load the last tile) so that the wait before a tile's math
    // only has to cover that tile's loads and the other set stays in flight.
    const int ntiles = (kend - kbeg + TILE_KEYS - 1) / TILE_KEYS;
    const int last = ntiles - 1;
    auto key_of = [&](int it) { return it < ntiles ? kbeg + it * TILE_KEYS : kInvalidKey; };
    {
        KTile ta, tb;
        load_tile(kbeg + min(wave, last) * TILE_KEYS, ta);
        for (int it = wave; it < ntiles; it += 8) {
            // the fences keep a tile's math (and the waits it starts with) behind the issue of the next tile's loads
            load_tile(kbeg + min(it + 4, last) * TILE_KEYS, tb);
            __builtin_amdgcn_sched_barrier(0);
            process(ta, kbeg + it * TILE_KEYS);
            __builtin_amdgcn_sched_barrier(0);
            load_tile(kbeg + min(it + 8, last) * TILE_KEYS, ta);
            __builtin_amdgcn_sched_barrier(0);
            process(tb, key_of(it + 4));
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- merge the four waves of the group through LDS (maxima in log2 units from here on) ----
#pragma unroll
    for (int rt = 0; rt < R; ++rt) m_run[rt] = m_run[rt] == -INFINITY ? -INFINITY : mc[rt];
    constexpr int RP = 16 * R;
    __shared__ float m_sh[4][RP], l_sh[4][RP];
    extern __shared__ __attribute__((aligned(16))) float o_dyn[];          // [4 waves][HD][RP + 1]
    float (*o_sh)[HD][RP + 1] = reinterpret_cast<float (*)[HD][RP + 1]>(o_dyn);
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        float l = l_run[rt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (lg == 0) {
            m_sh[wave][rt * 16 + l16] = m_run[rt];
            l_sh[wave][rt * 16 + l16] = l;
        }
    }
    __syncthreads();
    float fac[R], m_all[R], l_all[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int r = rt * 16 + l16;
        float mm = fmaxf(fmaxf(m_sh[0][r], m_sh[1][r]), fmaxf(m_sh[2][r], m_sh[3][r]));
        const float ms = mm == -INFINITY ? 0.f : mm;
        float ll = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) ll += l_sh[w][r] * exp2f(m_sh[w][r] - ms);
        fac[rt] = exp2f(m_run[rt] - ms);
        m_all[rt] = mm;
        l_all[rt] = ll;
    }
    // every wave lays its rescaled accumulators down in its own LDS plane, all four at once; after one barrier
    // the work-group adds the planes up on the way out (taking turns on a single plane cost four serialised
    // read-modify-write passes, some 10 us per work-group)
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
        for (int ht = 0; ht < 8; ++ht)
#pragma unroll
            for (int i = 0; i < 4; ++i) o_sh[wave][ht * 16 + 4 * lg + i][rt * 16 + l16] = o[ht][rt][i] * fac[rt];
    __syncthreads();
    const int64_t pbase = (((int64_t)b * a.Hkv + hkv) * a.max_chunks + chunk) * a.rows_pad + row0;
    const int rows_here = min(rows - row0, RP);
    for (int e = tid; e < rows_here * HD; e += 256) {
        const int r = e / HD, d = e % HD;
        a.part_o[(pbase + r) * HD + d] = (o_sh[0][d][r] + o_sh[1][d][r]) + (o_sh[2][d][r] + o_sh[3][d][r]);
    }
    if (wave == 0 && lg == 0) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            const int r = rt * 16 + l16;
            if (r < rows_here) {
                a.part_ml[(pbase + r) * 2] = m_all[rt];
                a.part_ml[(pbase + r) * 2 + 1] = l_all[rt];
            }
        }
    }
}

// R row tiles per work-group, W waves, D slots per wave for K and for V in the LDS ring (W * D * 16 KB of LDS).
// Run as W = 2, D = 2: two work-groups share a CU.
// PT: bf16 terms the softmax weights are split into for the PV products.  With four row tiles (or several row
// groups) this kernel is bound by its matrix products and the power they draw, and three quarters of them are PV
// products: it runs with PT = 2 (16 significant bits; the 2^-17 relative it leaves is the size of the fp32
// accumulation error of a few thousand keys, i.e. nothing the result did not carry already), a quarter fewer
// products than with three terms.  The register kernel above is bound by the stream and keeps three.
template <int R, int W, int D, int PT>
__global__ __launch_bounds__(64 * W, 1) void attn_bf16_kernel(AttnArgs a, float scale_log2e) {
    // Work item = one piece of one request's keys, cut by the host from its upper bounds of the lengths.
    // Launch order: the kv heads of an item are neighbours, so the list's longest-first order holds chip-wide.
    // With more stacked rows than one work-group takes, the row tiles are split over row_groups work-groups that
    // stream the same keys; work-group ids 8 apart run on the same XCD, so the groups of one (item, head) are
    // placed 8 apart and started together: the second reader of a tile finds it in that XCD's L2.
    // A work-group is W waves, each alone on its SIMD (the accumulators leave no room for a second), and takes
    // half of the CU's LDS: two work-groups share a CU, so that while one starts an item (three dependent reads:
    // item, page table, first tile) or merges its waves, the other keeps streaming.
    constexpr int RP = 16 * R;
    __shared__ float m_sh[W][RP], l_sh[W][RP];
    const int slot_id = blockIdx.x / (8 * a.row_groups), rem = blockIdx.x % (8 * a.row_groups);
    const int rg = rem >> 3, pair = slot_id * 8 + (rem & 7);
    const int n_items = a.n_work_dev ? *a.n_work_dev : a.n_work;
    if (pair >= n_items * a.Hkv) return;
    const int hkv = pair % a.Hkv;
    const int4 item = reinterpret_cast<const int4*>(a.work)[pair / a.Hkv];
    const int b = item.x >> 16, chunk = item.x & 0xffff;
    const int seq = item.y;
    const int L = a.seq_len[seq];
    const int total = L + a.n;
    const int kbeg = item.z;
    if (kbeg >= total) return;                            // the live length fell short of the host's bound
    const int kend = min(item.w, total);
    const int row0 = rg * R * 16;                         // first stacked row of this work-group
    const int G = a.Hq / a.Hkv, rows = G * a.n;

    const int tid = threadIdx.x, lane = tid & 63;
    // wave index as a scalar: tile numbers, page-table reads and page addresses stay on the scalar unit
    // (a vector page-table load would have to be waited for with vmcnt(0), draining the K/V prefetch)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lg = lane >> 4;
    const bf16_t* pool = reinterpret_cast<const bf16_t*>(a.pool);
    const int page_shift = 31 - __builtin_clz(a.geom.page_size), page_mask = a.geom.page_size - 1;
    // The page table is read through the constant address space: nothing writes it while the kernel runs, and
    // only so do the lookups stay scalar loads once the loop holds direct-to-LDS loads (which the compiler must
    // otherwise assume may alias any global read; a vector lookup would be waited for with vmcnt(0), draining
    // the K/V prefetch).
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
    const_i32_ptr pages = (const_i32_ptr)(a.page_table + (int64_t)seq * a.max_pages_per_seq);

    // Q^T operand: lane holds row rt*16 + l16, head_dim slice kk*32 + lg*8 .. +8
    u32x4 qf[R][4];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int r = row0 + rt * 16 + l16;
        const bool ok = r < rows;
        const int j = ok ? r / G : 0, hl = ok ? r % G : 0;
        const bf16_t* qp = reinterpret_cast<const bf16_t*>(a.q) + (((int64_t)b * a.n + j) * a.Hq + hkv * G + hl) * HD;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qf[rt][kk] = ok ? *reinterpret_cast<const u32x4*>(qp + kk * 32 + lg * 8) : u32x4{0, 0, 0, 0};
    }

    // A row sees every cached key, x0 (key L) and the drafts of its own chain up to itself: the keys
    // [vis_lo, vis_hi).  Rows of x0 and padding rows get an empty interval.
    int vis_lo[R], vis_hi[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int r = row0 + rt * 16 + l16;
        const int j = r < rows ? r / G : 0;
        vis_lo[rt] = j > 0 ? L + 1 + row_chain(j, a.k) * a.k : 0;
        vis_hi[rt] = j > 0 ? vis_lo[rt] + row_index_in_chain(j, a.k) : 0;
    }

    floatx4 o[8][R];
    float m_run[R], mc[R], l_run[R];      // reference maximum (raw score), the same times scale*log2(e), partial sum
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        m_run[rt] = -INFINITY;
        mc[rt] = 0.f;
        l_run[rt] = 0.f;
#pragma unroll
        for (int ht = 0; ht < 8; ++ht) o[ht][rt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }

    // K/V tiles travel HBM -> LDS -> registers.  Each wave owns a ring of D slots for K and D for V (8 KB each)
    // in LDS that it fills with direct-to-LDS loads (16 bytes per lane, 1 KB per instruction, no registers held
    // while in flight) and reads back into one register set: two tiles on their way per wave where a second
    // register set could hold one, and the registers go to the skewed stages instead.  A wave reads only what it
    // loaded itself: no barriers.
    // The tile's base address is wave-uniform (scalar page number, head, offset) and kept in scalar registers.
    auto uniform = [](int64_t v) {
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (int64_t)(((uint64_t)hi << 32) | lo);
    };
    extern __shared__ __attribute__((aligned(16))) unsigned char attn_lds[];
    unsigned char* ring = attn_lds + wave * (D * kTileBytes);          // K slots 0..D-1, then V slots 0..D-1, 8 KB each
    // Tiles start on multiples of 32 keys, where the cache's index functions reduce to
    //   K: layer * layer_elems + page * page_elems + (head * page_size + key_in_page) * 128,   V: the same + v_off
    // (kv_k_index / kv_v_index with tok % 32 == 0, dim == 0); K and V of a tile are 8 KB each, contiguous, and are
    // copied verbatim: 4 loads per 4 KB share one scalar base, one LDS base, and differ in the immediate offset,
    // which the instruction adds to both addresses.
    const int64_t head_base = (int64_t)a.layer * a.geom.layer_elems + (int64_t)hkv * a.geom.page_size * HD;
    const int64_t v_off = (int64_t)a.geom.n_kv_heads * a.geom.page_size * HD;
    const uint32_t lane_bytes = lane * 16;
    // Ring layout per wave: K slots 0,1 then V slots 0,1 (8 KB each).  half = 0 for K, 1 for V.
    auto issue_half = [&](int key0, int half, int slot) __attribute__((always_inline)) {
        const int page = pages[key0 >> page_shift];
        const int off = key0 & page_mask;
        const int64_t ke = uniform(head_base + (int64_t)page * a.geom.page_elems + off * HD + half * v_off);
        unsigned char* dst = ring + (half * D + slot) * 8192;
        const char* src = reinterpret_cast<const char*>(pool + ke) + lane_bytes;
        dma4(src, SV_LDS_PTR(dst));
        dma4(src + 4096, SV_LDS_PTR(dst + 4096));
    };

    // Wave w takes tiles w, w + 4, ... of the piece: its tile t starts at key tile_key(t).
    const int ntiles = (kend - kbeg + TILE_KEYS - 1) / TILE_KEYS;
    const int last = ntiles - 1;
    const int n_my = wave < ntiles ? (ntiles - wave + W - 1) / W : 0;
    auto tile_key = [&](int t) { return kbeg + min(wave + W * t, last) * TILE_KEYS; };   // past the end: a valid tile

    // The three stages of a tile -- scores S^T = K Q^T (MFMA), softmax (vector ALU), O^T += V^T P^T (MFMA) -- depend
    // on each other, and a wave alone on its SIMD issues one instruction at a time: done tile after tile, the
    // matrix unit idles through the softmax and the vector ALU through the products.  So the loop is skewed: trip
    // j forms the scores of tile j + 1, the softmax of tile j and the PV products of tile j - 1, three independent
    // strands that the scheduling directives below weave into one instruction stream (one MFMA, then a few ALU
    // instructions that execute while it runs).  Carried from trip to trip: s_cur (scores of tile j), pf_prev
    // (P^T of tile j - 1 as bf16 terms).  K of tile t is read from the ring in trip t - 1, V in trip t + 1; trip j
    // then refills the two 8 KB slots it has emptied with K of tile j + 3 and V of tile j + 1 (16 loads a trip,
    // always, so that the wait at the top of a trip is a constant: all but the previous trip's loads).
    floatx4 s_cur[2][R], s_next[2][R];
    u32x4 pf_prev[R][PT];
    u32x4 kreg[2][4], vreg[8];
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
        for (int tm = 0; tm < PT; ++tm) pf_prev[rt][tm] = u32x4{0, 0, 0, 0};

    auto pv_products = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt)
#pragma unroll
            for (int ht = 0; ht < 8; ++ht)
#pragma unroll
                for (int tm = PT - 1; tm >= 0; --tm)
                    o[ht][rt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vreg[ht]),
                                                                        __builtin_bit_cast(bf16x8, pf_prev[rt][tm]), o[ht][rt], 0, 0, 0);
    };

    auto trip = [&](auto qk_c, auto sm_c, auto pv_c, auto first_c, int j) __attribute__((always_inline)) {
        constexpr bool QK = decltype(qk_c)::value, SM = decltype(sm_c)::value, PV = decltype(pv_c)::value;
        const int slot = D == 1 ? 0 : (j + 1) & 1;
        if (decltype(first_c)::value) wait_vmcnt<8 * D>(); else wait_vmcnt<16 * (D - 1)>();
        __builtin_amdgcn_sched_barrier(0);
        const unsigned char* src = ring + slot * 8192 + lane * 16;
        if (QK) {
#pragma unroll
            for (int f = 0; f < 8; ++f) kreg[f >> 2][f & 3] = *reinterpret_cast<const u32x4*>(src + f * 1024);
        }
        if (PV) {
#pragma unroll
            for (int f = 0; f < 8; ++f) vreg[f] = *reinterpret_cast<const u32x4*>(src + D * 8192 + f * 1024);
        }
        if (SM) {
            const int key0 = kbeg + (wave + W * j) * TILE_KEYS;
            if (key0 + TILE_KEYS > L) {   // tile touches the new rows or the end: apply visibility
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int rt = 0; rt < R; ++rt)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int key = key0 + kb * 16 + 4 * lg + i;
                            // bitwise, not short-circuit: this must stay a compare + select chain.  (With
                            // && / || the compiler built branches here and dropped the value of the first
                            // element on the path "beyond L, yet visible".)
                            const bool vis = (key <= L) | ((key >= vis_lo[rt]) & (key < vis_hi[rt]));
                            s_cur[kb][rt][i] = vis ? s_cur[kb][rt][i] : -INFINITY;
                        }
            }
        }
        // the slots just read are free once the reads have returned
        __builtin_amdgcn_sched_barrier(0);
        wait_lgkmcnt0();
        issue_half(tile_key(j + 1 + D), 0, slot);
        // (V of tile 0 is requested before the first trip, beside K: the trips whose turn it would be skip it)
        if (!(decltype(first_c)::value || (D == 1 && !PV))) issue_half(tile_key(j - 1 + D), 1, slot);
        __builtin_amdgcn_sched_barrier(0);

        // ---- strand 1: S^T = K Q^T of tile j + 1 (raw dot products):
        //      s[kb][rt][i] <-> key key0 + kb*16 + 4*lg + i, row rt*16 + l16
        if (QK) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int rt = 0; rt < R; ++rt) {
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf16x8, kreg[kb][kk]), __builtin_bit_cast(bf16x8, qf[rt][kk]), acc, 0, 0, 0);
                    s_next[kb][rt] = acc;
                }
        }
        if (SM) {
            // Lazy reference maximum.  The softmax reference m_ref of a row is common to the 4 lane groups
            // that share the row (they feed one MFMA accumulator) and is only moved when some score would
            // make 2^(c(s - m_ref)) exceed 2^16 (or on the row's first visible key): fp32 has the range to
            // spare, and the cross-lane reduction + accumulator rescale leave the per-tile path.
            bool trig = false;
            float lmax[R];
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                lmax[rt] = max8(s_cur[0][rt], s_cur[1][rt]);
                trig |= ((m_run[rt] == -INFINITY) & (lmax[rt] > -INFINITY)) | (fmaf(lmax[rt], scale_log2e, -mc[rt]) > 16.0f);
            }
            if (QK) {
#pragma unroll
                for (int g = 0; g < 8 * R; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);     // two vector ALU instructions
                }
            }
            if (__builtin_expect(__any(trig), 0)) {
                // Move the reference.  It is kept at a whole number of log2 units, so the factor between the old and
                // the new one is a power of two: what was accumulated against the old reference (the sums, the
                // accumulators, and the bf16 terms of P^T whose PV products are still pending) is rescaled exactly.
#pragma unroll
                for (int rt = 0; rt < R; ++rt) {
                    float mx = lmax[rt];
                    mx = fmaxf(mx, __shfl_xor(mx, 16));
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    const float m_new = fmaxf(m_run[rt], mx);
                    const float mc_new = m_new == -INFINITY ? 0.f : ceilf(m_new * scale_log2e);
                    const int shift = (int)fmaxf(mc[rt] - mc_new, -200.f);
                    const float alpha = m_run[rt] == -INFINITY ? 0.f : ldexpf(1.0f, shift);
                    l_run[rt] *= alpha;
#pragma unroll
                    for (int ht = 0; ht < 8; ++ht) {
                        // The accumulators live in the accumulation registers, which arithmetic cannot read.  The empty
                        // statement pins their copy to ordinary registers here, on the rare path (the compiler otherwise
                        // makes those 32 R copies at the head of every trip of the loop, needed or not).
                        floatx4 t = o[ht][rt];
                        asm volatile("" : "+v"(t));
                        o[ht][rt] = t * alpha;
                    }
                    if (PV) {
#pragma unroll
                        for (int tm = 0; tm < PT; ++tm)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const uint32_t w = pf_prev[rt][tm][i];
                                const float lo = __builtin_bit_cast(float, w << 16) * alpha;
                                const float hi = __builtin_bit_cast(float, w & 0xffff0000u) * alpha;
                                pf_prev[rt][tm][i] = (__builtin_bit_cast(uint32_t, lo) >> 16) | (__builtin_bit_cast(uint32_t, hi) & 0xffff0000u);
                            }
                    }
                    m_run[rt] = m_new;
                    mc[rt] = mc_new;
                }
            }
        }
        // ---- strand 2: softmax of tile j;  strand 3: PV products of tile j - 1
        u32x4 pf_cur[R][PT];
        if (SM) {
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                floatx2 p[4];
                float psum = 0.f;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    p[i] = floatx2{__builtin_amdgcn_exp2f(fmaf(s_cur[0][rt][2 * i], scale_log2e, -mc[rt])),
                                   __builtin_amdgcn_exp2f(fmaf(s_cur[0][rt][2 * i + 1], scale_log2e, -mc[rt]))};
                    p[2 + i] = floatx2{__builtin_amdgcn_exp2f(fmaf(s_cur[1][rt][2 * i], scale_log2e, -mc[rt])),
                                       __builtin_amdgcn_exp2f(fmaf(s_cur[1][rt][2 * i + 1], scale_log2e, -mc[rt]))};
                    psum += (p[i].x + p[i].y) + (p[2 + i].x + p[2 + i].y);
                }
                l_run[rt] += psum;
                // P goes to the MFMA as PT bf16 terms (8 significant bits each).  One term would leave a 2^-9
                // relative error in the output however many keys there are (V has zero mean, so the output is
                // as small as the error's random walk): as much as the rounding of the output itself.
#pragma unroll
                for (int tm = 0; tm < PT; ++tm)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bf16x2 hb = __builtin_convertvector(p[i], bf16x2);
                        pf_cur[rt][tm][i] = __builtin_bit_cast(uint32_t, hb);
                        if (tm < PT - 1) p[i] = p[i] - __builtin_convertvector(hb, floatx2);
                    }
            }
        }
        if (PV) pv_products();
        if (SM && PV) {
#pragma unroll
            for (int g = 0; g < 8 * PT * R; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x402, PT == 3 ? 3 : 4, 0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        if (SM) {
#pragma unroll
            for (int rt = 0; rt < R; ++rt)
#pragma unroll
                for (int tm = 0; tm < PT; ++tm) pf_prev[rt][tm] = pf_cur[rt][tm];
        }
        if (QK) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int rt = 0; rt < R; ++rt) s_cur[kb][rt] = s_next[kb][rt];
        }
    };

    {
        constexpr std::true_type yes{};
        constexpr std::false_type no{};
        issue_half(tile_key(0), 0, 0);
        if (D == 2) issue_half(tile_key(1), 0, 1);
        issue_half(tile_key(0), 1, 0);
        if (n_my > 0) {
            trip(yes, no, no, yes, -1);
            if (n_my == 1) {
                trip(no, yes, no, no, 0);
                trip(no, no, yes, no, 1);
            } else {
                trip(yes, yes, no, no, 0);
                for (int j = 1; j <= n_my - 2; ++j) trip(yes, yes, yes, no, j);
                trip(no, yes, yes, no, n_my - 1);
                trip(no, no, yes, no, n_my);
            }
        }
        wait_vmcnt<0>();                                  // the ring is about to be reused for the merge
    }

    // ---- merge the waves of the group through LDS (maxima in log2 units from here on) ----
#pragma unroll
    for (int rt = 0; rt < R; ++rt) m_run[rt] = m_run[rt] == -INFINITY ? -INFINITY : mc[rt];
    float (*o_sh)[HD][RP + 1] = reinterpret_cast<float (*)[HD][RP + 1]>(attn_lds);   // [W waves][HD][RP + 1], over the rings
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        float l = l_run[rt];
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (lg == 0) {
            m_sh[wave][rt * 16 + l16] = m_run[rt];
            l_sh[wave][rt * 16 + l16] = l;
        }
    }
    __syncthreads();
    float fac[R], m_all[R], l_all[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int r = rt * 16 + l16;
        float mm = m_sh[0][r];
#pragma unroll
        for (int w = 1; w < W; ++w) mm = fmaxf(mm, m_sh[w][r]);
        const float ms = mm == -INFINITY ? 0.f : mm;
        float ll = 0.f;
#pragma unroll
        for (int w = 0; w < W; ++w) ll += l_sh[w][r] * exp2f(m_sh[w][r] - ms);
        fac[rt] = exp2f(m_run[rt] - ms);
        m_all[rt] = mm;
        l_all[rt] = ll;
    }
    // every wave lays its rescaled accumulators down in its own LDS plane, all four at once; after one barrier
    // the work-group adds the planes up on the way out (taking turns on a single plane cost four serialised
    // read-modify-write passes, some 10 us per work-group)
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
        for (int ht = 0; ht < 8; ++ht)
#pragma unroll
            for (int i = 0; i < 4; ++i) o_sh[wave][ht * 16 + 4 * lg + i][rt * 16 + l16] = o[ht][rt][i] * fac[rt];
    __syncthreads();
    const int64_t pbase = (((int64_t)b * a.Hkv + hkv) * a.max_chunks + chunk) * a.rows_pad + row0;
    const int rows_here = min(rows - row0, RP);
    for (int e = tid; e < rows_here * HD; e += 64 * W) {
        const int r = e / HD, d = e % HD;
        float acc = o_sh[0][d][r];
#pragma unroll
        for (int w = 1; w < W; ++w) acc += o_sh[w][d][r];
        a.part_o[(pbase + r) * HD + d] = acc;
    }
    if (wave == 0 && lg == 0) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            const int r = rt * 16 + l16;
            if (r < rows_here) {
                a.part_ml[(pbase + r) * 2] = m_all[rt];
                a.part_ml[(pbase + r) * 2 + 1] = l_all[rt];
            }
        }
    }
}

// Combine the chunk partials of one row: out = sum_c 2^(m_c - M) O_c / sum_c 2^(m_c - M) l_c.  A thread
// owns four consecutive dimensions of one q head; a work-group covers 256 / 32 = 8 heads of the row.
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
    const int rows_pad = a.rows_pad;
    const int t = blockIdx.x, h = blockIdx.y * 8 + (threadIdx.x >> 5), d = (threadIdx.x & 31) * 4;
    if (h >= a.Hq) return;
    const int b = t / a.n, j = t % a.n;
    const int G = a.Hq / a.Hkv, hkv = h / G, r = j * G + h % G;
    const int total = a.seq_len[a.batch_seq[b]] + a.n;
    const int clen = a.req_chunk[2 * b];
    const int nch = min(a.req_chunk[2 * b + 1], (total + clen - 1) / clen);   // pieces that start below the live end
    const int64_t base = ((int64_t)b * a.Hkv + hkv) * a.max_chunks;
    float M = -INFINITY;
    for (int c = 0; c < nch; ++c) M = fmaxf(M, a.part_ml[((base + c) * rows_pad + r) * 2]);
    floatx4 num = {0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    for (int c = 0; c < nch; ++c) {
        const int64_t pr = (base + c) * rows_pad + r;
        const floatx2 ml = *reinterpret_cast<const floatx2*>(a.part_ml + pr * 2);
        const float f = exp2f(ml.x - M);
        den += f * ml.y;
        const floatx4 o = *reinterpret_cast<const floatx4*>(a.part_o + pr * HD + d);
        num[0] += f * o[0]; num[1] += f * o[1]; num[2] += f * o[2]; num[3] += f * o[3];
    }
    // four consecutive dimensions stay inside one 8-element piece of either output order
    u32x2 pk = {pack2bf(num[0] / den, num[1] / den), pack2bf(num[2] / den, num[3] / den)};
    *reinterpret_cast<u32x2*>(reinterpret_cast<bf16_t*>(a.out) + act_index(t, h * HD + d, a.Hq * HD, a.out_packed)) = pk;
}

// Generic path: one wave per (new row, q head).  Lane-strided keys, per-lane online softmax with the
// accumulator in registers, wave reduction at the end.
template <typename T, int D>
__global__ __launch_bounds__(64) void attn_generic_kernel(AttnArgs a, float scale) {
    const int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int b = t / a.n, j = t % a.n;
    const int seq = a.batch_seq[b];
    const int L = a.seq_len[seq], total = L + a.n;
    const int hkv = h / (a.Hq / a.Hkv);
    const int32_t* pages = a.page_table + (int64_t)seq * a.max_pages_per_seq;
    const T* pool = reinterpret_cast<const T*>(a.pool);
    __shared__ float q[D];
    for (int d = lane; d < D; d += 64) q[d] = Store<T>::load(reinterpret_cast<const T*>(a.q) + ((int64_t)t * a.Hq + h) * D + d);
    __syncthreads();
    float m = -INFINITY, l = 0.f, acc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    for (int key = lane; key < total; key += 64) {
        if (key >= L && !row_sees(j, key - L, a.k)) continue;
        const int page = pages[key / a.geom.page_size], tok = key % a.geom.page_size;
        float s = 0.f;
#pragma unroll 8
        for (int d = 0; d < D; ++d) s = fmaf(q[d], Store<T>::load(pool + kv_k_index(a.geom, a.layer, page, hkv, tok, d)), s);
        s *= scale;
        const float mn = fmaxf(m, s);
        const float alpha = expf(m - mn), p = expf(s - mn);
        l = l * alpha + p;
#pragma unroll 8
        for (int d = 0; d < D; ++d)
            acc[d] = acc[d] * alpha + p * Store<T>::load(pool + kv_v_index(a.geom, a.layer, page, hkv, tok, d));
        m = mn;
    }
    const float M = wave_max(m);
    const float f = m == -INFINITY ? 0.f : expf(m - M);
    const float den = wave_sum(l * f);
    T* out = reinterpret_cast<T*>(a.out);
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const float v = wave_sum(acc[d] * f);
        if (lane == 0) Store<T>::store(out + act_index(t, h * D + d, a.Hq * D, a.out_packed), v / den);
    }
}

int attn_rows_pad(int n, int group) {
    const int rows = n * group;
    if (rows > 256) return 0;
    return (rows + 15) / 16 * 16;
}

hipError_t attention(const AttnArgs& a, hipStream_t st) {
    const float scale = 1.0f / sqrtf((float)a.hd);
    const int G = a.Hq / a.Hkv;
    const int rp = (!a.force_generic && a.dtype == 1 && a.hd == HD && a.geom.page_size % TILE_KEYS == 0 &&
                    (a.geom.page_size & (a.geom.page_size - 1)) == 0 && a.chunk_keys % 128 == 0)
                       ? attn_rows_pad(a.n, G) : 0;
    if (rp && rp <= a.rows_pad) {
        const float sl2 = scale * 1.44269504088896340736f;
        // up to four 16-row tiles per work-group; more stacked rows are split over row groups
        AttnArgs b = a;
        const int tiles = rp / 16;
        const int cap = std::min(4, std::max(1, a.max_row_tiles));
        b.row_groups = (tiles + cap - 1) / cap;
        const int R = b.row_groups == 1 ? std::max(tiles, a.min_row_tiles) : (tiles + b.row_groups - 1) / b.row_groups;
        const int items = a.grid_items > 0 ? a.grid_items : a.n_work;
        dim3 grid((items * a.Hkv + 7) / 8 * 8 * b.row_groups);
        auto launch = [&](auto kern, int r, int waves, int depth) -> hipError_t {
            const size_t lds = std::max((size_t)waves * HD * (16 * r + 1) * sizeof(float), (size_t)waves * depth * kTileBytes);
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(kern, grid, dim3(64 * waves), lds, st, b, sl2);
            return hipGetLastError();
        };
        auto launch_regs = [&](auto kern, int r) -> hipError_t {
            const size_t lds = (size_t)4 * HD * (16 * r + 1) * sizeof(float);
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, b, sl2);
            return hipGetLastError();
        };
        hipError_t e;
        if (b.row_groups > 1 || R >= 4) {
            switch (R) {
                case 1: e = launch_regs(attn_bf16_regs_kernel<1>, 1); break;
                case 2: e = launch(attn_bf16_kernel<2, 2, 2, 2>, 2, 2, 2); break;
                case 3: e = launch(attn_bf16_kernel<3, 2, 2, 2>, 3, 2, 2); break;
                default: e = launch(attn_bf16_kernel<4, 2, 2, 2>, 4, 2, 2); break;
            }
        } else {
            switch (R) {
                case 1: e = launch_regs(attn_bf16_regs_kernel<1>, 1); break;
                case 2: e = launch_regs(attn_bf16_regs_kernel<2>, 2); break;
                default: e = launch_regs(attn_bf16_regs_kernel<3>, 3); break;
            }
        }
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(attn_merge_kernel, dim3(a.B * a.n, (a.Hq + 7) / 8), dim3(256), 0, st, b);
        return hipGetLastError();
    }
    dim3 grid(a.B * a.n, a.Hq);
    if (a.dtype == 1 && a.hd == 128)
        hipLaunchKernelGGL((attn_generic_kernel<bf16_t, 128>), grid, dim3(64), 0, st, a, scale);
    else if (a.dtype == 1 && a.hd == 64)
        hipLaunchKernelGGL((attn_generic_kernel<bf16_t, 64>), grid, dim3(64), 0, st, a, scale);
    else if (a.dtype == 0 && a.hd == 128)
        hipLaunchKernelGGL((attn_generic_kernel<float, 128>), grid, dim3(64), 0, st, a, scale);
    else if (a.dtype == 0 && a.hd == 64)
        hipLaunchKernelGGL((attn_generic_kernel<float, 64>), grid, dim3(64), 0, st, a, scale);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace sv
