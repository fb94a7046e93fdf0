// Accept / reject over the target logits, the replacement or bonus draw, the choice of the chain to
// keep, and the cache rollback.  Three passes over vocabulary-wide data, all bound by HBM:
//   row_stats   every logits row once: max, sum exp((x - max)/temp), argmax (lowest id on ties)
//   accept      per (request, chain), scalar: walk the drafts; p_i(d_i) from the row statistics and
//               one gathered logit; u_i * q_i(d_i) < p_i(d_i); record the row the final draw uses
//   draw        per (request, chain), one pass over that row (and the draft distribution's row when
//               a draft was rejected): weights w = max(p - q, 0) or p; inverse-CDF or exponential race
// then select (longest chain) and rollback (move the kept chain's K/V next to x0, advance lengths).
#include <math.h>
#include "common.h"
#include "kernels.h"

namespace sv {

constexpr int NT = 1024;

// One logits row is cut into gridDim.y contiguous parts, one work-group each (a row per work-group leaves a
// 150k-wide row to 1024 threads and the launch to a few hundred work-groups: latency-bound at a third of the
// memory rate); part statistics go to `part` [T][parts][4] and row_stats_merge_kernel folds them.
__global__ __launch_bounds__(NT) void row_stats_kernel(const float* __restrict__ logits, float* __restrict__ part,
                                                       int V, float inv_temp) {
    const int t = blockIdx.x;
    const float* row = logits + (int64_t)t * V;
    const int span = ((V + gridDim.y - 1) / gridDim.y + 3) & ~3;          // ids per part, a multiple of 4
    const int vbeg = blockIdx.y * span, vend = min(V, vbeg + span);
    float m = -INFINITY, s = 0.f;
    int am = 0x7fffffff;
    auto take = [&](float x, int v) {
        if (x > m) {
            s = s * expf((m - x) * inv_temp) + 1.0f;
            m = x;
            am = v;
        } else if (x > -INFINITY) {
            s += expf((x - m) * inv_temp);
        }
    };
    if ((V & 3) == 0) {
        // Rows start on 16-byte boundaries: four ids per load, and kAhead loads of a thread in flight before the
        // arithmetic on any of them (one new maximum and one rescale per batch of loads, not per load).  The
        // exponentials are the hardware's base-2 ones on pre-scaled arguments.
        constexpr int kAhead = 5;
        const float c2 = inv_temp * 1.4426950408889634f;
        for (int v0 = vbeg + 4 * threadIdx.x; v0 < vend; v0 += 4 * NT * kAhead) {
            floatx4 x[kAhead];
#pragma unroll
            for (int u = 0; u < kAhead; ++u) {
                const int v = v0 + u * 4 * NT;
                x[u] = v < vend ? *reinterpret_cast<const floatx4*>(row + v) : floatx4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            }
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < kAhead; ++u) mx = fmaxf(mx, fmaxf(fmaxf(x[u][0], x[u][1]), fmaxf(x[u][2], x[u][3])));
            if (mx > m) {                                  // new maximum: its first holder in ascending id order
                s *= __builtin_amdgcn_exp2f((m - mx) * c2);   // (m = -inf: s is 0 and stays 0)
                m = mx;
#pragma unroll
                for (int u = kAhead - 1; u >= 0; --u)
#pragma unroll
                    for (int i = 3; i >= 0; --i)
                        if (x[u][i] == mx) am = v0 + u * 4 * NT + i;
            }
            if (mx > -INFINITY) {
                float add = 0.f;
#pragma unroll
                for (int u = 0; u < kAhead; ++u)
                    add += (__builtin_amdgcn_exp2f((x[u][0] - m) * c2) + __builtin_amdgcn_exp2f((x[u][1] - m) * c2)) +
                           (__builtin_amdgcn_exp2f((x[u][2] - m) * c2) + __builtin_amdgcn_exp2f((x[u][3] - m) * c2));
                s += add;
            }
        }
    } else {
        for (int v = vbeg + threadIdx.x; v < vend; v += NT) take(row[v], v);
    }
    __shared__ float sm[NT / 64], ss[NT / 64];
    __shared__ int sa[NT / 64];
    // wave merge, then group merge: (m, s, am) with ties on m resolved to the lower id
    auto merge = [&](float& m1, float& s1, int& a1, float m2, float s2, int a2) {
        const float mm = fmaxf(m1, m2);
        const float f1 = m1 == -INFINITY ? 0.f : expf((m1 - mm) * inv_temp);
        const float f2 = m2 == -INFINITY ? 0.f : expf((m2 - mm) * inv_temp);
        s1 = s1 * f1 + s2 * f2;
        if (m2 > m1 || (m2 == m1 && a2 < a1)) a1 = a2;
        m1 = mm;
    };
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float m2 = __shfl_xor(m, o), s2 = __shfl_xor(s, o);
        const int a2 = __shfl_xor(am, o);
        merge(m, s, am, m2, s2, a2);
    }
    if ((threadIdx.x & 63) == 0) {
        sm[threadIdx.x >> 6] = m;
        ss[threadIdx.x >> 6] = s;
        sa[threadIdx.x >> 6] = am;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < NT / 64; ++w) merge(m, s, am, sm[w], ss[w], sa[w]);
        float* out = part + ((int64_t)t * gridDim.y + blockIdx.y) * 4;
        out[0] = m;
        out[1] = s;
        out[2] = __int_as_float(am);
        out[3] = 0.f;
    }
}

__global__ void row_stats_merge_kernel(const float* __restrict__ part, float* __restrict__ stat, int T, int parts, float inv_temp) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    float m = -INFINITY, s = 0.f;
    int am = 0x7fffffff;
    for (int i = 0; i < parts; ++i) {                     // ascending ids: on equal maxima the earlier part's id stays
        const float* in = part + ((int64_t)t * parts + i) * 4;
        const float m2 = in[0], s2 = in[1];
        const int a2 = __float_as_int(in[2]);
        const float mm = fmaxf(m, m2);
        const float f1 = m == -INFINITY ? 0.f : expf((m - mm) * inv_temp);
        const float f2 = m2 == -INFINITY ? 0.f : expf((m2 - mm) * inv_temp);
        s = s * f1 + s2 * f2;
        if (m2 > m || (m2 == m && a2 < am)) am = a2;
        m = mm;
    }
    stat[t * 4 + 0] = m;
    stat[t * 4 + 1] = s;
    stat[t * 4 + 2] = __int_as_float(am);
    stat[t * 4 + 3] = 0.f;
}

// Logits row that holds the target distribution of draft slot i (1-based) of chain c of request b.
__device__ __forceinline__ int slot_row(int b, int c, int i, int n, int k) {
    return b * n + (i == 1 ? 0 : 1 + c * k + (i - 2));
}

__global__ void accept_kernel(SampleArgs a) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= a.B * a.N) return;
    const int b = s / a.N, c = s % a.N;
    const int n = 1 + a.N * a.k;
    const int klim = a.draft_lens ? min(a.draft_lens[b], a.k) : a.k;
    const float inv_temp = 1.0f / a.temperature;
    int acc = 0;
    for (int i = 1; i <= klim; ++i) {
        const int row = slot_row(b, c, i, n, a.k);
        const int x = a.drafts[(int64_t)s * a.k + (i - 1)];
        bool ok;
        if ((unsigned)x >= (unsigned)a.V) {
            ok = false;                                   // not a token of this vocabulary: rejected, nothing is read at it
        } else if (a.verify_mode == 0) {
            ok = x == __float_as_int(a.row_stat[row * 4 + 2]);
        } else if (a.verify_mode == 2) {
            ok = x == __float_as_int(a.row_stat[row * 4 + 3]);       // the token drawn for this slot
        } else {
            const float m = a.row_stat[row * 4], sum = a.row_stat[row * 4 + 1];
            const float p = expf((a.logits[(int64_t)row * a.V + x] - m) * inv_temp) / sum;
            const float q = a.draft_probs ? a.draft_probs[((int64_t)s * a.k + (i - 1)) * a.V + x] : 1.0f;
            ok = a.uniforms[(int64_t)s * (a.k + 1) + (i - 1)] * q < p;
        }
        if (!ok) break;
        ++acc;
    }
    a.chain_acc[s] = acc;
    const int row = slot_row(b, c, acc + 1, n, a.k);
    a.chain_row[s] = row;
    if (a.verify_mode == 0) a.chain_tok[s] = __float_as_int(a.row_stat[row * 4 + 2]);
    if (a.verify_mode == 2) a.chain_tok[s] = __float_as_int(a.row_stat[row * 4 + 3]);
}

__device__ __forceinline__ uint64_t splitmix_finalise(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Draw of one token.  ROWS == false (stochastic verification): the final draw of one (request, chain), from the
// residual after a rejection or from the bonus row.  ROWS == true (match verification): the target's own token of
// one logits row, i.e. of one draft slot, from that row's distribution; the randomness is keyed by the request's
// index in the batch and the slot alone (the uniform of chain 0), so every chain of a request is held to the same
// token at the same slot.  The result goes to row_stat[row][3].
template <bool ROWS>
__global__ __launch_bounds__(NT) void draw_kernel(SampleArgs a) {
    const int s = blockIdx.x;                             // (request, chain), or logits row
    const int n = 1 + a.N * a.k;
    const int b = ROWS ? s / n : s / a.N;
    const int klim = a.draft_lens ? min(a.draft_lens[b], a.k) : a.k;
    const int acc = ROWS ? 0 : a.chain_acc[s];
    const bool rejected = ROWS ? false : acc < klim;
    const int row = ROWS ? s : a.chain_row[s];
    const float* lrow = a.logits + (int64_t)row * a.V;
    // a rejected id outside the vocabulary was rejected unread: the replacement comes from p_r itself (q taken as zero)
    const int xraw = rejected ? a.drafts[(int64_t)s * a.k + acc] : -1;
    const int xrej = (unsigned)xraw < (unsigned)a.V ? xraw : -1;
    const float* qrow = (rejected && a.draft_probs && xrej >= 0) ? a.draft_probs + ((int64_t)s * a.k + acc) * a.V : nullptr;
    const float inv_temp = 1.0f / a.temperature;
    const float m = a.row_stat[row * 4], sum = a.row_stat[row * 4 + 1];
    const float log_sum = logf(sum);
    // slot served by row j of a request: row 0 -> slot 1, the row of draft i of any chain -> slot i + 1
    const int j = s % n;
    const int slot = j == 0 ? 1 : (j - 1) % max(a.k, 1) + 2;
    const float u = ROWS ? a.uniforms[(int64_t)b * a.N * (a.k + 1) + (slot - 1)] : a.uniforms[(int64_t)s * (a.k + 1) + a.k];
    const int V = a.V;

    auto prob = [&](int v) { return expf((lrow[v] - m) * inv_temp) / sum; };
    auto resid = [&](int v, float p) {          // weight of id v in the residual distribution
        if (!rejected) return p;
        const float q = qrow ? qrow[v] : (v == xrej ? 1.0f : 0.0f);
        return fmaxf(p - q, 0.0f);
    };

    if (a.sample_mode == 1) {
        // exponential race: argmax_v ln w_v - ln e_v ; track the residual's winner and, for the case that
        // the residual is identically zero, the winner under p as well.
        const uint64_t key = ((uint64_t)(uint32_t)(ROWS ? b : s) << 32) | (uint64_t)__float_as_uint(u);
        float best_r = -INFINITY, best_p = -INFINITY;
        int arg_r = 0x7fffffff, arg_p = 0x7fffffff;
        // the vocabulary is cut into gridDim.y contiguous parts; each work-group finds the winners of its part
        const int part = (V + gridDim.y - 1) / gridDim.y;
        const int vbeg = blockIdx.y * part, vend = min(V, vbeg + part);
        for (int v = vbeg + threadIdx.x; v < vend; v += NT) {
            const uint64_t z = splitmix_finalise(key + (uint64_t)(v + 1) * 0x9E3779B97F4A7C15ull);
            const float U = ((float)(uint32_t)(z >> 32) + 0.5f) * 2.3283064365386963e-10f;
            const float ln_e = logf(-log1pf(-U));
            const float lp = (lrow[v] - m) * inv_temp - log_sum;
            const float sp = lp - ln_e;
            if (sp > best_p) { best_p = sp; arg_p = v; }
            if (rejected) {
                const float w = resid(v, expf(lp));
                if (w > 0.f) {
                    const float sr = logf(w) - ln_e;
                    if (sr > best_r) { best_r = sr; arg_r = v; }
                }
            }
        }
        __shared__ float sh_r[NT / 64], sh_p[NT / 64];
        __shared__ int sh_ar[NT / 64], sh_ap[NT / 64];
        auto take = [](float& bv, int& ba, float ov, int oa) {
            if (ov > bv || (ov == bv && oa < ba)) { bv = ov; ba = oa; }
        };
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            take(best_r, arg_r, __shfl_xor(best_r, o), __shfl_xor(arg_r, o));
            take(best_p, arg_p, __shfl_xor(best_p, o), __shfl_xor(arg_p, o));
        }
        if ((threadIdx.x & 63) == 0) {
            sh_r[threadIdx.x >> 6] = best_r; sh_ar[threadIdx.x >> 6] = arg_r;
            sh_p[threadIdx.x >> 6] = best_p; sh_ap[threadIdx.x >> 6] = arg_p;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < NT / 64; ++w) {
                take(best_r, arg_r, sh_r[w], sh_ar[w]);
                take(best_p, arg_p, sh_p[w], sh_ap[w]);
            }
            float* out = a.draw_part + ((int64_t)s * gridDim.y + blockIdx.y) * 4;
            out[0] = best_r; out[1] = __int_as_float(arg_r); out[2] = best_p; out[3] = __int_as_float(arg_p);
        }
        return;
    }

    // inverse CDF over ascending id.  Thread i owns the contiguous ids [i*seg, (i+1)*seg); sums in double.
    const int seg = (V + NT - 1) / NT;
    const int v0 = threadIdx.x * seg, v1 = min(V, v0 + seg);
    __shared__ double seg_r[NT], seg_p[NT];
    __shared__ int pick_seg, use_p;
    __shared__ double target, before;
    double sr = 0.0, spp = 0.0;
    for (int v = v0; v < v1; ++v) {
        const float p = prob(v);
        spp += (double)p;
        sr += (double)resid(v, p);
    }
    seg_r[threadIdx.x] = sr;
    seg_p[threadIdx.x] = spp;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot_r = 0.0, tot_p = 0.0;
        for (int i = 0; i < NT; ++i) { tot_r += seg_r[i]; tot_p += seg_p[i]; }
        const int up = !(tot_r > 0.0);
        const double* segs = up ? seg_p : seg_r;
        const double tgt = (double)u * (up ? tot_p : tot_r);
        double run = 0.0;
        int pick = -1;
        for (int i = 0; i < NT; ++i) {
            if (run + segs[i] > tgt) { pick = i; break; }
            run += segs[i];
        }
        if (pick < 0) {          // u * total reached the total through rounding: last segment with weight
            run = 0.0;
            for (int i = 0; i < NT; ++i) if (segs[i] > 0.0) pick = i;
            for (int i = 0; i < pick; ++i) run += segs[i];
        }
        pick_seg = pick; use_p = up; target = tgt; before = run;
    }
    __syncthreads();
    if ((int)threadIdx.x == pick_seg) {
        double run = before;
        int tok = -1, last_pos = -1;
        for (int v = v0; v < v1; ++v) {
            const float p = prob(v);
            const float w = use_p ? p : resid(v, p);
            if (w > 0.f) last_pos = v;
            run += (double)w;
            if (run > target) { tok = v; break; }
        }
        const int drawn = tok >= 0 ? tok : last_pos;
        if (ROWS) a.row_stat[row * 4 + 3] = __int_as_float(drawn);
        else a.chain_tok[s] = drawn;
    }
}

__global__ void select_kernel(SampleArgs a) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= a.B) return;
    int best = 0, acc = a.chain_acc[b * a.N];
    for (int c = 1; c < a.N; ++c)
        if (a.chain_acc[b * a.N + c] > acc) { acc = a.chain_acc[b * a.N + c]; best = c; }
    a.accepted_len[b] = acc;
    a.best_chain[b] = best;
    int32_t* out = a.out_tokens + (int64_t)b * (a.k + 1);
    for (int i = 0; i < acc; ++i) out[i] = a.drafts[((int64_t)b * a.N + best) * a.k + i];
    out[acc] = a.chain_tok[b * a.N + best];
    for (int i = acc + 1; i <= a.k; ++i) out[i] = -1;
}

// Move the kept chain's accepted entries to slots L+1 .. L+a (chain 0 already sits there).  One work-group per
// (request, layer).  In the tile layout of the cache a key's K entries of one head are head_dim/8 whole 16-byte
// pieces (one per 8-wide slice of the head), moved as such with one index computation each; its V entries lie
// one element apart per dimension (V is stored transposed, keys innermost) and move one by one.  Source slots
// (>= L+1+k for a chain other than 0) and destination slots (<= L+k) never overlap.
template <typename T>
__global__ __launch_bounds__(256) void compact_kernel(RollbackArgs r) {
    const int b = blockIdx.x, layer = blockIdx.y;
    const int best = r.best_chain[b], acc = r.accepted_len[b];
    if (best <= 0 || best >= r.N || acc <= 0 || acc > r.k) return;
    const int seq = r.batch_seq[b];
    const int L = r.seq_len[seq];
    const int32_t* pages = r.page_table + (int64_t)seq * r.max_pages_per_seq;
    T* pool = reinterpret_cast<T*>(r.pool);
    const int hd = r.geom.head_dim, H = r.geom.n_kv_heads;
    constexpr int EPP = 16 / (int)sizeof(T);              // elements per 16-byte piece
    const int ppk = hd / 8;                               // pieces of 8 consecutive dimensions per (key, head)
    // K: 8 consecutive dimensions of one key are contiguous (16 bytes in bf16, two 16-byte pieces in fp32)
    for (int e = threadIdx.x; e < acc * H * ppk; e += 256) {
        const int i = e / (H * ppk) + 1, rem = e % (H * ppk), h = rem / ppk, d = (rem % ppk) * 8;
        const int src = L + 1 + best * r.k + (i - 1), dst = L + i;
        const int64_t si = kv_k_index(r.geom, layer, pages[src / r.geom.page_size], h, src % r.geom.page_size, d);
        const int64_t di = kv_k_index(r.geom, layer, pages[dst / r.geom.page_size], h, dst % r.geom.page_size, d);
#pragma unroll
        for (int q = 0; q < 8 / EPP; ++q)
            *reinterpret_cast<u32x4*>(pool + di + q * EPP) = *reinterpret_cast<const u32x4*>(pool + si + q * EPP);
    }
    // V: one element per (key, head, dimension)
    for (int e = threadIdx.x; e < acc * H * hd; e += 256) {
        const int i = e / (H * hd) + 1, rem = e % (H * hd), h = rem / hd, d = rem % hd;
        const int src = L + 1 + best * r.k + (i - 1), dst = L + i;
        pool[kv_v_index(r.geom, layer, pages[dst / r.geom.page_size], h, dst % r.geom.page_size, d)] =
            pool[kv_v_index(r.geom, layer, pages[src / r.geom.page_size], h, src % r.geom.page_size, d)];
    }
}

__global__ void commit_len_kernel(RollbackArgs r) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < r.B) r.seq_len[r.batch_seq[b]] += r.accepted_len[b] + 1;
}

// Winner of a chain's (or, ROWS, a row's) exponential race over the parts of the vocabulary (larger score; lower
// id among equals).
template <bool ROWS>
__global__ void draw_reduce_kernel(SampleArgs a, int parts) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= (ROWS ? a.B * (1 + a.N * a.k) : a.B * a.N)) return;
    const int b = ROWS ? 0 : s / a.N;
    const int klim = a.draft_lens ? min(a.draft_lens[b], a.k) : a.k;
    const bool rejected = ROWS ? false : a.chain_acc[s] < klim;
    float best_r = -INFINITY, best_p = -INFINITY;
    int arg_r = 0x7fffffff, arg_p = 0x7fffffff;
    for (int i = 0; i < parts; ++i) {
        const float* in = a.draw_part + ((int64_t)s * parts + i) * 4;
        const float r = in[0], p = in[2];
        const int ar = __float_as_int(in[1]), ap = __float_as_int(in[3]);
        if (r > best_r || (r == best_r && ar < arg_r)) { best_r = r; arg_r = ar; }
        if (p > best_p || (p == best_p && ap < arg_p)) { best_p = p; arg_p = ap; }
    }
    const int drawn = (rejected && best_r > -INFINITY) ? arg_r : arg_p;
    if (ROWS) a.row_stat[s * 4 + 3] = __int_as_float(drawn);
    else a.chain_tok[s] = drawn;
}

hipError_t sample_verify(const SampleArgs& a, hipStream_t st) {
    const int T = a.B * (1 + a.N * a.k), S = a.B * a.N;
    // the race's part buffer is free until the draws: it takes the rows' part statistics first
    hipLaunchKernelGGL(row_stats_kernel, dim3(T, kDrawParts), dim3(NT), 0, st, a.logits, a.draw_part, a.V, 1.0f / a.temperature);
    hipLaunchKernelGGL(row_stats_merge_kernel, dim3((T + 63) / 64), dim3(64), 0, st, a.draw_part, a.row_stat, T, kDrawParts,
                       1.0f / a.temperature);
    if (a.verify_mode == 2) {          // match: the target's token of every slot first, then the comparison
        if (a.sample_mode == 1) {
            hipLaunchKernelGGL(draw_kernel<true>, dim3(T, kDrawParts), dim3(NT), 0, st, a);
            hipLaunchKernelGGL(draw_reduce_kernel<true>, dim3((T + 63) / 64), dim3(64), 0, st, a, kDrawParts);
        } else {
            hipLaunchKernelGGL(draw_kernel<true>, dim3(T), dim3(NT), 0, st, a);
        }
    }
    hipLaunchKernelGGL(accept_kernel, dim3((S + 63) / 64), dim3(64), 0, st, a);
    if (a.verify_mode == 1) {
        if (a.sample_mode == 1) {      // the race's per-id arithmetic dominates: spread every chain over several work-groups
            hipLaunchKernelGGL(draw_kernel<false>, dim3(S, kDrawParts), dim3(NT), 0, st, a);
            hipLaunchKernelGGL(draw_reduce_kernel<false>, dim3((S + 63) / 64), dim3(64), 0, st, a, kDrawParts);
        } else {
            hipLaunchKernelGGL(draw_kernel<false>, dim3(S), dim3(NT), 0, st, a);
        }
    }
    hipLaunchKernelGGL(select_kernel, dim3((a.B + 63) / 64), dim3(64), 0, st, a);
    return hipGetLastError();
}

hipError_t rollback(const RollbackArgs& r, hipStream_t st, bool commit) {
    if (r.N > 1) {
        if (r.dtype == 1)
            hipLaunchKernelGGL(compact_kernel<bf16_t>, dim3(r.B, r.n_layers), dim3(256), 0, st, r);
        else
            hipLaunchKernelGGL(compact_kernel<float>, dim3(r.B, r.n_layers), dim3(256), 0, st, r);
    }
    if (commit) hipLaunchKernelGGL(commit_len_kernel, dim3((r.B + 63) / 64), dim3(64), 0, st, r);
    return hipGetLastError();
}

}  // namespace sv
