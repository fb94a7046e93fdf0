// Verify attention: the n new rows of every request attend that request's paged KV cache plus the
// new rows they are allowed to see.  Every cached byte is read once per step however many rows
// verify against it -- that reuse across the k+1 rows is the saving of parallel verification -- so
// the kernel is bound by HBM bandwidth and is organised around streaming K/V.
//
// bf16 path (head_dim 128).  A work-group owns one (request, kv head, chunk of keys).  All G*n query
// rows that share the kv head (G = q heads per kv head) are stacked into R tiles of 16 rows.  Each
// of the 4 waves walks its own 32-key tiles of the chunk; per tile it loads K (32 x 128) and V^T
// (128 x 32) straight from the page into MFMA operand registers (the next tile's loads are issued
// before the current tile's math), forms S^T = K Q^T with v_mfma_f32_16x16x32_bf16, runs the online
// softmax in fp32 on the four keys per row each lane holds, and feeds P^T (as three bf16 terms) back
// as the B operand of O^T += V^T P^T.  The score tile's register layout (a lane holds 4 consecutive keys of one row, for
// two 16-key blocks) is used unchanged as the PV operand; the reduction index of that MFMA is only a
// label, so V^T is simply loaded with the same key order.  Waves are merged through LDS, chunks by
// a second small kernel (split-KV).
//
// Generic path (fp32 models, other head sizes, more than 64 stacked rows): one wave per (row, head),
// plain online softmax; correct for every shape, not tuned.
#include <math.h>
#include <algorithm>
#include "common.h"
#include "kernels.h"

namespace sv {

constexpr int HD = 128;
constexpr int TILE_KEYS = 32;

struct KTile { u32x4 k[2][4]; u32x4 v[8]; };

template <int R>
__global__ __launch_bounds__(256, R == 1 ? 2 : 1) void attn_bf16_kernel(AttnArgs a, float scale_log2e) {
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
        auto launch = [&](auto kern, int r) -> hipError_t {
            const size_t lds = (size_t)4 * HD * (16 * r + 1) * sizeof(float);
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, b, sl2);
            return hipGetLastError();
        };
        hipError_t e;
        switch (R) {
            case 1: e = launch(attn_bf16_kernel<1>, 1); break;
            case 2: e = launch(attn_bf16_kernel<2>, 2); break;
            case 3: e = launch(attn_bf16_kernel<3>, 3); break;
            default: e = launch(attn_bf16_kernel<4>, 4); break;
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
