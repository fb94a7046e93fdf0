// Shared device-side definitions for the gfx950 kernels of the verification step.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sv {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kVBlk = 32;          // keys per tile of a KV page

typedef uint16_t bf16_t;           // raw bf16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float floatx2;

// float -> bf16, round to nearest even: gfx950's v_cvt_pk_bf16_f32.
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2{lo, hi}, bf16x2));
}

// Storage-type traits: T is float (fp32 model) or bf16_t (bf16 model).
template <typename T> struct Store;
template <> struct Store<float> {
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
    static __device__ __forceinline__ void store4(float* p, const float* v) {      // p 16-byte aligned
        *reinterpret_cast<floatx4*>(p) = floatx4{v[0], v[1], v[2], v[3]};
    }
};
template <> struct Store<bf16_t> {
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf2f(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f2bf(v); }
    static __device__ __forceinline__ void store4(bf16_t* p, const float* v) {     // p 8-byte aligned
        *reinterpret_cast<u32x2*>(p) = u32x2{pack2bf(v[0], v[1]), pack2bf(v[2], v[3])};
    }
};

// ---- paged KV layout -------------------------------------------------------
// pool[layer][page][K | V][kv_head][tile of 32 keys], each tile stored in the order the 16x16x32 MFMA
// reads its operands, so that a wave fetches one operand fragment (64 lanes x 8 elements) as one
// contiguous, fully used 1 KB (bf16) piece:
//   K tile: fragments [key block kb = 0,1][head_dim slice kk = 0 .. hd/32-1], fragment element
//           (lane = 16*g + r, e) = K[key 16*kb + r][dim 32*kk + 8*g + e]
//   V tile: fragments [ht = 0 .. hd/16-1], fragment element (lane = 16*g + r, j) = V[key][dim 16*ht + r]
//           with key = 4*g + j for j < 4 and 16 + 4*g + (j-4) otherwise -- the order in which the
//           score tile leaves the MFMA (a lane holds 4 consecutive keys of each 16-key block).
struct KvGeom {
    int n_kv_heads, head_dim, page_size;
    int64_t page_elems;    // 2 * n_kv_heads * page_size * head_dim
    int64_t layer_elems;   // num_pages * page_elems
};
__host__ __device__ __forceinline__ int64_t kv_k_index(const KvGeom& g, int layer, int page, int head, int tok, int dim) {
    const int t = tok % kVBlk, kb = t / 16, r = t % 16;
    const int kk = dim / 32, grp = (dim % 32) / 8, e = dim % 8;
    return (int64_t)layer * g.layer_elems + (int64_t)page * g.page_elems +
           ((int64_t)head * g.page_size + (tok / kVBlk) * kVBlk) * g.head_dim +
           ((kb * (g.head_dim / 32) + kk) * 64 + grp * 16 + r) * 8 + e;
}
__host__ __device__ __forceinline__ int64_t kv_v_index(const KvGeom& g, int layer, int page, int head, int tok, int dim) {
    const int t = tok % kVBlk, half = t / 16, grp = (t % 16) / 4, j = half * 4 + t % 4;
    const int ht = dim / 16, r = dim % 16;
    return (int64_t)layer * g.layer_elems + (int64_t)page * g.page_elems +
           (int64_t)g.n_kv_heads * g.page_size * g.head_dim +
           ((int64_t)head * g.page_size + (tok / kVBlk) * kVBlk) * g.head_dim +
           ((ht * 64) + grp * 16 + r) * 8 + j;
}

// Activations that feed a projection, [rows, K]: row-major, or (packed) in the fragment order the
// weight-streaming kernel reads -- [rows/32][K/16][64 lanes][8], lane 32*g + r of a fragment holding row r of
// the 32-row tile, elements 8*g .. 8*g+7 of the 16-wide slice.
__host__ __device__ __forceinline__ int64_t act_index(int row, int col, int K, bool packed) {
    if (!packed) return (int64_t)row * K + col;
    return ((((int64_t)(row >> 5) * (K >> 4) + (col >> 4)) * 64) + ((col >> 3) & 1) * 32 + (row & 31)) * 8 + (col & 7);
}

// Index of new row j (0 = x0, then chain 0's drafts, chain 1's ...) -> chain, index in chain.
__host__ __device__ __forceinline__ int row_chain(int j, int k) { return j == 0 ? -1 : (j - 1) / k; }
__host__ __device__ __forceinline__ int row_index_in_chain(int j, int k) { return j == 0 ? 0 : (j - 1) % k + 1; }
// Does new row i attend new row j?  (x0, and the earlier drafts of its own chain.)
__host__ __device__ __forceinline__ bool row_sees(int i, int j, int k) {
    if (j == 0) return true;
    if (i == 0) return false;
    return (i - 1) / k == (j - 1) / k && j <= i;
}

// ---- waits and direct-to-LDS loads ----
#define SV_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// s_waitcnt immediates (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8; all-ones = no wait)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }

// 4 KB from global memory straight into LDS: four wave-wide loads of 16 bytes per lane.  src is the lane's own
// address (base + 16 * lane), dst the wave's LDS base; lane l's bytes land at dst + 16 * l + the immediate.
__device__ __forceinline__ void dma4(const char* src, __attribute__((address_space(3))) void* dst) {
    __builtin_amdgcn_global_load_lds((const void*)src, dst, 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const void*)src, dst, 16, 1024, 0);
    __builtin_amdgcn_global_load_lds((const void*)src, dst, 16, 2048, 0);
    __builtin_amdgcn_global_load_lds((const void*)src, dst, 16, 3072, 0);
}

template <typename T> __device__ __forceinline__ T wave_max(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) { T w = __shfl_xor(v, o); v = w > v ? w : v; }
    return v;
}
template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

}  // namespace sv
