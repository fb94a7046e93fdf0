// Dense projections of the target's forward pass: out[s][M][N] = A[M, Ks] * W[N, Ks]^T, where the
// reduction dimension may be cut into `splits` contiguous ranges whose partial products are written
// side by side and summed by the consuming kernel (deterministic split-K).
//
// bf16 path: v_mfma_f32_16x16x32_bf16, fp32 accumulate.  A work-group of WM x WN waves computes a
// (16*MT*WM) x (16*NT*WN) tile; the weight tile is the MFMA "A" operand (rows = output features) and the
// activation tile the "B" operand, so a lane ends up with four consecutive output features of one
// token and stores them as one 16-byte word.  Operand tiles are staged through LDS (row pitch 72
// elements: the 16 lanes of a quarter-wave hit 64 distinct banks), double buffered, with the next
// tile's global loads in flight during the MFMAs of the current one.  Work-group ids are remapped so
// that the groups that share one weight panel run on the same XCD (one L2) at about the same time.
#include "common.h"
#include "kernels.h"

namespace sv {

constexpr int BK = 64;
constexpr int LDS_PITCH = BK + 8;

// Work-groups are dealt to the 8 XCDs round-robin by id.  Give XCD x a contiguous range of logical
// ids instead, so that neighbours in logical order share an L2.
__device__ __forceinline__ int xcd_remap(int id, int n) {
    const int q = n >> 3, r = n & 7;
    const int x = id & 7, local = id >> 3;
    return x * q + (x < r ? x : r) + local;
}

template <int MT, int NT, int WM, int WN>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, float* __restrict__ out,
    int M, int N, int K, int k_per_split, int splits, int tiles_m, int tiles_n) {
    constexpr int BM = 16 * MT * WM;       // tokens per group tile
    constexpr int BN = 16 * NT * WN;       // output features per group tile
    constexpr int NTHR = 64 * WM * WN;
    constexpr int A_CH = BM * (BK / 8) / NTHR;   // 16-byte chunks per thread
    constexpr int W_CH = BN * (BK / 8) / NTHR;
    static_assert(BM * (BK / 8) % NTHR == 0 && BN * (BK / 8) % NTHR == 0, "tile/threads mismatch");

    extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
    bf16_t* As = lds;                                  // [2][BM][LDS_PITCH]
    bf16_t* Ws = lds + 2 * BM * LDS_PITCH;             // [2][BN][LDS_PITCH]

    const int nblk = tiles_m * tiles_n * splits;
    int logical = xcd_remap(blockIdx.x, nblk);
    const int tm = logical % tiles_m;
    logical /= tiles_m;
    const int sp = logical % splits;
    const int tn = logical / splits;
    const int m0 = tm * BM, n0 = tn * BN;
    const int kbeg = sp * k_per_split;
    const int nk = k_per_split / BK;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int l16 = lane & 15, lg = lane >> 4;

    u32x4 a_reg[A_CH], w_reg[W_CH];
    auto load_global = [&](int kt) {
        const int k0 = kbeg + kt * BK;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int cid = tid + i * NTHR, row = cid >> 3, ch = cid & 7;
            int gm = m0 + row;
            gm = gm < M ? gm : M - 1;
            a_reg[i] = *reinterpret_cast<const u32x4*>(A + (int64_t)gm * K + k0 + ch * 8);
        }
#pragma unroll
        for (int i = 0; i < W_CH; ++i) {
            const int cid = tid + i * NTHR, row = cid >> 3, ch = cid & 7;
            w_reg[i] = *reinterpret_cast<const u32x4*>(W + (int64_t)(n0 + row) * K + k0 + ch * 8);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            const int cid = tid + i * NTHR, row = cid >> 3, ch = cid & 7;
            *reinterpret_cast<u32x4*>(As + (buf * BM + row) * LDS_PITCH + ch * 8) = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < W_CH; ++i) {
            const int cid = tid + i * NTHR, row = cid >> 3, ch = cid & 7;
            *reinterpret_cast<u32x4*>(Ws + (buf * BN + row) * LDS_PITCH + ch * 8) = w_reg[i];
        }
    };

    floatx4 acc[NT][MT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_global(kt + 1);
#pragma unroll
        for (int kk = 0; kk < BK / 32; ++kk) {
            bf16x8 wf[NT], af[MT];
#pragma unroll
            for (int i = 0; i < NT; ++i)
                wf[i] = *reinterpret_cast<const bf16x8*>(
                    Ws + (buf * BN + (wn * NT + i) * 16 + l16) * LDS_PITCH + kk * 32 + lg * 8);
#pragma unroll
            for (int j = 0; j < MT; ++j)
                af[j] = *reinterpret_cast<const bf16x8*>(
                    As + (buf * BM + (wm * MT + j) * 16 + l16) * LDS_PITCH + kk * 32 + lg * 8);
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[i], af[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_lds(buf ^ 1);
        __syncthreads();
    }

    // lane holds, per (i, j): features n = n0 + (wn*NT+i)*16 + 4*lg + {0..3}, token m = m0 + (wm*MT+j)*16 + l16
    float* dst = out + (int64_t)sp * M * N;
#pragma unroll
    for (int j = 0; j < MT; ++j) {
        const int m = m0 + (wm * MT + j) * 16 + l16;
        if (m < M) {
#pragma unroll
            for (int i = 0; i < NT; ++i) {
                const int n = n0 + (wn * NT + i) * 16 + 4 * lg;
                *reinterpret_cast<floatx4*>(dst + (int64_t)m * N + n) = acc[i][j];
            }
        }
    }
}

// fp32 path (small models only): 32x32 output tile per 256-thread group, 4 outputs per thread, every
// access bounds-checked.  Accumulates in fp32 in ascending k.
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                       float* __restrict__ out, int M, int N, int K) {
    __shared__ float As[32][33], Ws[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // ty 0..7
    const int m0 = blockIdx.y * 32, n0 = blockIdx.x * 32;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < K; k0 += 32) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = ty + 8 * r;
            const int k = k0 + tx;
            As[row][tx] = (m0 + row < M && k < K) ? A[(int64_t)(m0 + row) * K + k] : 0.f;
            Ws[row][tx] = (n0 + row < N && k < K) ? W[(int64_t)(n0 + row) * K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < 32; ++k) {
            const float w = Ws[tx][k];
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = fmaf(As[ty + 8 * r][k], w, acc[r]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int m = m0 + ty + 8 * r, n = n0 + tx;
        if (m < M && n < N) out[(int64_t)m * N + n] = acc[r];
    }
}

template <int MT, int NT, int WM, int WN>
static hipError_t launch_bf16(const bf16_t* A, const bf16_t* W, float* out, int M, int N, int K, int splits,
                              hipStream_t st) {
    constexpr int BM = 16 * MT * WM, BN = 16 * NT * WN;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    const size_t lds = (size_t)2 * (BM + BN) * LDS_PITCH * sizeof(bf16_t);
    auto kern = gemm_bf16_kernel<MT, NT, WM, WN>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n * splits), dim3(64 * WM * WN), lds, st, A, W, out, M, N, K,
                       K / splits, splits, tiles_m, tiles_n);
    return hipGetLastError();
}

int gemm_bf16_shape_ok(int N, int K, int splits) {
    return N > 0 && K > 0 && splits > 0 && N % 128 == 0 && K % (BK * splits) == 0;
}

hipError_t gemm_bf16(const bf16_t* A, const bf16_t* W, float* out, int M, int N, int K, int splits, int variant,
                     hipStream_t st) {
    switch (variant) {
        case 1: return launch_bf16<2, 4, 2, 2>(A, W, out, M, N, K, splits, st);    // 64 x 128
        case 2: return launch_bf16<4, 4, 4, 2>(A, W, out, M, N, K, splits, st);    // 256 x 128, 8 waves
        default: return launch_bf16<4, 4, 2, 2>(A, W, out, M, N, K, splits, st);   // 128 x 128
    }
}

hipError_t gemm_f32(const float* A, const float* W, float* out, int M, int N, int K, hipStream_t st) {
    hipLaunchKernelGGL(gemm_f32_kernel, dim3((N + 31) / 32, (M + 31) / 32), dim3(256), 0, st, A, W, out, M, N, K);
    return hipGetLastError();
}

}  // namespace sv
