// The memory-bound glue of the forward pass: row preparation (positions, cache slots, rotary table),
// embedding gather, residual-add + RMSNorm (which also sums split-K partial products), rotary embedding
// + KV append into the paged cache, SwiGLU, and dense <-> paged KV copies.
#include "common.h"
#include "kernels.h"

namespace sv {

// One group per new row t = b*n + j.  Position = L + index-in-chain, cache slot = L + j.  The rotary
// angle pos * theta^(-2i/hd) is formed in double: at positions of tens of thousands a float angle is
// off by ~1e-3 rad, which is visible after rounding q and k to bf16.
__global__ void prep_rows_kernel(RowPrep p) {
    const int t = blockIdx.x, b = t / p.n, j = t % p.n;
    const int L = p.seq_len[p.batch_seq[b]];
    const int pos = L + row_index_in_chain(j, p.k);
    if (threadIdx.x == 0) {
        int tok;
        if (p.tok_matrix) {
            const int col = min(p.tok_col0 + j, p.tok_len[b] - 1);
            tok = p.tok_matrix[(int64_t)b * p.tok_ld + col];
        } else {
            // (a pass over given residual rows brings no tokens at all)
            tok = !p.last_tokens ? 0 : j == 0 ? p.last_tokens[b] : p.drafts[(int64_t)b * (p.n - 1) + (j - 1)];
        }
        // ids arrive in device memory from another process and cannot be checked on the host: an id outside the
        // vocabulary is embedded as the nearest valid one (the sampler rejects such a draft whatever its row yields)
        p.row_tok[t] = min(max(tok, 0), p.vocab - 1);
        p.row_pos[t] = pos;
        p.row_slot[t] = L + j;
    }
    const int half = p.head_dim / 2;
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
        const double inv_freq = pow((double)p.rope_theta, -2.0 * (double)i / (double)p.head_dim);
        double s, c;
        sincos((double)pos * inv_freq, &s, &c);
        p.rope[((int64_t)t * half + i) * 2 + 0] = (float)c;
        p.rope[((int64_t)t * half + i) * 2 + 1] = (float)s;
    }
}

template <typename T>
__global__ void embed_kernel(const T* __restrict__ embed, const int32_t* __restrict__ row_tok, float* __restrict__ h, int d) {
    const int t = blockIdx.x;
    const T* src = embed + (int64_t)row_tok[t] * d;
    for (int i = threadIdx.x; i < d; i += blockDim.x) h[(int64_t)t * d + i] = Store<T>::load(src + i);
}

// One 256-thread group per row.  Each thread owns up to NV float4 pieces of the row; the loads of the
// residual and of every split-K partial product are issued before the first use, so the row costs a
// few memory round trips rather than one per element.
// With `inv` set the addend is not S planes but the weighted sum of the row's top_k expert outputs
// (part = expert outputs [padded row][d], row of assignment j at inv[t*top_k + j], weight wts[t*top_k + j]),
// accumulated in slot order.
template <typename T, int NV>
__global__ __launch_bounds__(256) void add_rmsnorm_kernel(float* __restrict__ h, const float* __restrict__ part, int S,
                                                          int64_t part_stride, const T* __restrict__ w,
                                                          T* __restrict__ a, int d, float eps, bool packed,
                                                          const int32_t* __restrict__ inv, const float* __restrict__ wts,
                                                          int top_k) {
    __shared__ float red[4];
    const int t = blockIdx.x;
    const int nq = d >> 2;                               // float4 pieces per row
    floatx4* hr = reinterpret_cast<floatx4*>(h + (int64_t)t * d);
    floatx4 x[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int i = threadIdx.x + v * 256;
        x[v] = i < nq ? hr[i] : floatx4{0.f, 0.f, 0.f, 0.f};
    }
    if (inv) {
        floatx4 acc[NV];
#pragma unroll
        for (int v = 0; v < NV; ++v) acc[v] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int j0 = 0; j0 < top_k; j0 += 4) {             // four expert rows in flight at a time
            floatx4 y[4][NV];
            float wj[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int j = j0 + u < top_k ? j0 + u : j0;
                wj[u] = j0 + u < top_k ? wts[(int64_t)t * top_k + j] : 0.f;
                const floatx4* pr = reinterpret_cast<const floatx4*>(part + (int64_t)inv[(int64_t)t * top_k + j] * d);
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int i = threadIdx.x + v * 256;
                    y[u][v] = ((i < nq) & (j0 + u < top_k)) ? pr[i] : floatx4{0.f, 0.f, 0.f, 0.f};
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + u < top_k) {
#pragma unroll
                    for (int v = 0; v < NV; ++v)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[v][e] = fmaf(wj[u], y[u][v][e], acc[v][e]);
                }
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) x[v] = x[v] + acc[v];
    } else {
    // partial planes four at a time: all their loads are in flight together, the additions keep plane order
        for (int s0 = 0; s0 < S; s0 += 4) {
            floatx4 y[4][NV];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const floatx4* pr = reinterpret_cast<const floatx4*>(part + (s0 + u < S ? s0 + u : s0) * part_stride + (int64_t)t * d);
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int i = threadIdx.x + v * 256;
                    y[u][v] = ((i < nq) & (s0 + u < S)) ? pr[i] : floatx4{0.f, 0.f, 0.f, 0.f};
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v) x[v] = x[v] + y[u][v];
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int i = threadIdx.x + v * 256;
        if (i < nq) {
            if (S | (inv != nullptr)) hr[i] = x[v];
            ss = fmaf(x[v][0], x[v][0], ss);
            ss = fmaf(x[v][1], x[v][1], ss);
            ss = fmaf(x[v][2], x[v][2], ss);
            ss = fmaf(x[v][3], x[v][3], ss);
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = red[0] + red[1] + red[2] + red[3];
    const float r = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int i = threadIdx.x + v * 256;
        if (i < nq) {
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = x[v][e] * r * Store<T>::load(w + 4 * i + e);
            // four consecutive columns are contiguous in either output order
            Store<T>::store4(a + act_index(t, 4 * i, d, packed), o);
        }
    }
}

// q and k heads are rotated, k and v heads go to the row's cache slot.  One work-group per row, four consecutive
// dimensions (and their partners half a head away) per thread: 16-byte reads of the partial planes and of the
// rotary table, one 8- or 16-byte store per four q or K values (four consecutive dimensions of a key are contiguous
// in the cache's K tiles); V is stored transposed, one element at a time.  head_dim % 8 == 0 (it is 64 or 128).
template <typename T>
__global__ __launch_bounds__(256) void rope_append_vec_kernel(RopeAppend p) {
    const int t = blockIdx.x, b = t / p.n;
    const int hd = p.hd, half = hd / 2, upq = half / 4;   // units of four pairs per head
    const int nheads = p.Hq + 2 * p.Hkv;
    const int ncol = nheads * hd;
    const int64_t stride = (int64_t)p.T * ncol;
    const int slot = p.row_slot[t];
    const int page = p.page_table[(int64_t)p.batch_seq[b] * p.max_pages_per_seq + slot / p.geom.page_size];
    const int tok = slot % p.geom.page_size;
    T* pool = reinterpret_cast<T*>(p.pool);
    for (int u = threadIdx.x; u < nheads * upq; u += 256) {
        const int head = u / upq, i = (u % upq) * 4;
        const float* src = p.qkv_part + (int64_t)t * ncol + head * hd + i;
        floatx4 x1 = {0.f, 0.f, 0.f, 0.f}, x2 = {0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < p.S; ++s) {
            x1 += *reinterpret_cast<const floatx4*>(src + s * stride);
            x2 += *reinterpret_cast<const floatx4*>(src + s * stride + half);
        }
        if (head < p.Hq + p.Hkv) {
            const floatx4 r0 = *reinterpret_cast<const floatx4*>(p.rope + ((int64_t)t * half + i) * 2);
            const floatx4 r1 = *reinterpret_cast<const floatx4*>(p.rope + ((int64_t)t * half + i) * 2 + 4);
            const float c[4] = {r0[0], r0[2], r1[0], r1[2]}, sn[4] = {r0[1], r0[3], r1[1], r1[3]};
            float o1[4], o2[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o1[e] = x1[e] * c[e] - x2[e] * sn[e];
                o2[e] = x2[e] * c[e] + x1[e] * sn[e];
            }
            if (head < p.Hq) {
                T* q = reinterpret_cast<T*>(p.q_out) + ((int64_t)t * p.Hq + head) * hd;
                Store<T>::store4(q + i, o1);
                Store<T>::store4(q + i + half, o2);
            } else {
                const int kh = head - p.Hq;
                Store<T>::store4(pool + kv_k_index(p.geom, p.layer, page, kh, tok, i), o1);
                Store<T>::store4(pool + kv_k_index(p.geom, p.layer, page, kh, tok, i + half), o2);
            }
        } else {
            const int kh = head - p.Hq - p.Hkv;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                Store<T>::store(pool + kv_v_index(p.geom, p.layer, page, kh, tok, i + e), x1[e]);
                Store<T>::store(pool + kv_v_index(p.geom, p.layer, page, kh, tok, i + half + e), x2[e]);
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void swiglu_kernel(const float* __restrict__ part, int S, int64_t stride,
                                                     T* __restrict__ act, int F, bool packed) {
    const int t = blockIdx.y;
    const int f = blockIdx.x * 256 + threadIdx.x;
    if (f >= F) return;
    const float* src = part + (int64_t)t * 2 * F;
    float g = 0.f, u = 0.f;
    for (int s = 0; s < S; ++s) {
        g += src[s * stride + f];
        u += src[s * stride + F + f];
    }
    const float y = g / (1.0f + expf(-g)) * u;
    Store<T>::store(act + act_index(t, f, F, packed), y);
}

template <typename T>
__global__ void kv_copy_kernel(T* pool, KvGeom g, int layer, const int32_t* __restrict__ pages, int pos0, T* k, T* v,
                               bool to_pool) {
    const int i = blockIdx.x, pos = pos0 + i;
    const int page = pages[pos / g.page_size], tok = pos % g.page_size;
    const int per = g.n_kv_heads * g.head_dim;
    for (int e = threadIdx.x; e < per; e += blockDim.x) {
        const int h = e / g.head_dim, d = e % g.head_dim;
        const int64_t ki = kv_k_index(g, layer, page, h, tok, d), vi = kv_v_index(g, layer, page, h, tok, d);
        if (to_pool) {
            pool[ki] = k[(int64_t)i * per + e];
            pool[vi] = v[(int64_t)i * per + e];
        } else {
            k[(int64_t)i * per + e] = pool[ki];
            v[(int64_t)i * per + e] = pool[vi];
        }
    }
}

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }
__global__ void add_len_kernel(int32_t* seq_len, const int32_t* batch_seq, int B, int delta) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) seq_len[batch_seq[b]] += delta;
}

__global__ void add_len_ragged_kernel(int32_t* seq_len, const int32_t* batch_seq, int B, const int32_t* len, int col0, int width) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) seq_len[batch_seq[b]] += max(0, min(width, len[b] - col0));
}

// ---------------------------------------------------------------- launchers ---

hipError_t prep_rows(const RowPrep& p, hipStream_t st) {
    hipLaunchKernelGGL(prep_rows_kernel, dim3(p.B * p.n), dim3(64), 0, st, p);
    return hipGetLastError();
}

hipError_t embed_rows(const void* embed, int dtype, const int32_t* row_tok, float* h, int T, int d, hipStream_t st) {
    if (dtype == 1)
        hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(T), dim3(256), 0, st, (const bf16_t*)embed, row_tok, h, d);
    else
        hipLaunchKernelGGL(embed_kernel<float>, dim3(T), dim3(256), 0, st, (const float*)embed, row_tok, h, d);
    return hipGetLastError();
}

template <typename T>
static hipError_t add_rmsnorm_t(float* h, const float* part, int S, const T* w, T* a, int T_, int d, float eps, bool packed,
                                const int32_t* inv, const float* wts, int top_k, hipStream_t st) {
    const int64_t stride = (int64_t)T_ * d;
    const int nq = d / 4;
    if (d % 4 != 0 || nq > 256 * 8) return hipErrorInvalidValue;
    if (nq <= 256 * 2)
        hipLaunchKernelGGL((add_rmsnorm_kernel<T, 2>), dim3(T_), dim3(256), 0, st, h, part, S, stride, w, a, d, eps, packed, inv, wts, top_k);
    else if (nq <= 256 * 4)
        hipLaunchKernelGGL((add_rmsnorm_kernel<T, 4>), dim3(T_), dim3(256), 0, st, h, part, S, stride, w, a, d, eps, packed, inv, wts, top_k);
    else
        hipLaunchKernelGGL((add_rmsnorm_kernel<T, 8>), dim3(T_), dim3(256), 0, st, h, part, S, stride, w, a, d, eps, packed, inv, wts, top_k);
    return hipGetLastError();
}

hipError_t add_rmsnorm(float* h, const float* part, int S, const void* w, void* a, int dtype, int T, int d, float eps,
                       bool packed, hipStream_t st) {
    if (dtype == 1) return add_rmsnorm_t<bf16_t>(h, part, S, (const bf16_t*)w, (bf16_t*)a, T, d, eps, packed, nullptr, nullptr, 0, st);
    return add_rmsnorm_t<float>(h, part, S, (const float*)w, (float*)a, T, d, eps, packed, nullptr, nullptr, 0, st);
}

hipError_t add_rmsnorm_experts(float* h, const float* y, const int32_t* inv, const float* wts, int top_k, const void* w, void* a,
                               int T, int d, float eps, bool packed, hipStream_t st) {
    return add_rmsnorm_t<bf16_t>(h, y, 0, (const bf16_t*)w, (bf16_t*)a, T, d, eps, packed, inv, wts, top_k, st);
}

hipError_t rope_append(const RopeAppend& p, hipStream_t st) {
    if (p.hd % 8 != 0) return hipErrorInvalidValue;
    if (p.dtype == 1)
        hipLaunchKernelGGL(rope_append_vec_kernel<bf16_t>, dim3(p.T), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(rope_append_vec_kernel<float>, dim3(p.T), dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t swiglu(const float* gu_part, int S, void* act, int dtype, int T, int F, bool packed, hipStream_t st) {
    const int64_t stride = (int64_t)T * 2 * F;
    dim3 grid((F + 255) / 256, T);
    if (dtype == 1)
        hipLaunchKernelGGL(swiglu_kernel<bf16_t>, grid, dim3(256), 0, st, gu_part, S, stride, (bf16_t*)act, F, packed);
    else
        hipLaunchKernelGGL(swiglu_kernel<float>, grid, dim3(256), 0, st, gu_part, S, stride, (float*)act, F, packed);
    return hipGetLastError();
}

hipError_t kv_copy(void* pool, const KvGeom& geom, int layer, const int32_t* page_table_row, int pos0, int n, void* k,
                   void* v, int dtype, bool to_pool, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (dtype == 1)
        hipLaunchKernelGGL(kv_copy_kernel<bf16_t>, dim3(n), dim3(256), 0, st, (bf16_t*)pool, geom, layer,
                           page_table_row, pos0, (bf16_t*)k, (bf16_t*)v, to_pool);
    else
        hipLaunchKernelGGL(kv_copy_kernel<float>, dim3(n), dim3(256), 0, st, (float*)pool, geom, layer, page_table_row,
                           pos0, (float*)k, (float*)v, to_pool);
    return hipGetLastError();
}

hipError_t set_i32(int32_t* p, int32_t v, hipStream_t st) {
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, st, p, v);
    return hipGetLastError();
}

hipError_t add_len_ragged(int32_t* seq_len, const int32_t* batch_seq, int B, const int32_t* len, int col0, int width, hipStream_t st) {
    hipLaunchKernelGGL(add_len_ragged_kernel, dim3((B + 63) / 64), dim3(64), 0, st, seq_len, batch_seq, B, len, col0, width);
    return hipGetLastError();
}

hipError_t add_len(int32_t* seq_len, const int32_t* batch_seq, int B, int delta, hipStream_t st) {
    hipLaunchKernelGGL(add_len_kernel, dim3((B + 63) / 64), dim3(64), 0, st, seq_len, batch_seq, B, delta);
    return hipGetLastError();
}

}  // namespace sv
