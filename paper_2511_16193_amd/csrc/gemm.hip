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

typedef __attribute__((ext_vector_type(16))) float floatx16;

// ---- second bf16 kernel: weight streaming (v_mfma_f32_32x32x16_bf16; one wave per SIMD issuing independent
// 16x16x32 MFMAs reaches 1.34 PFLOP/s over the chip, the 32x32x16 form 2.41: a kernel whose accumulators leave room
// for one wave per SIMD only must use the larger form).  For the few hundred rows of a verification step the
// projections sit on the ridge between HBM and MFMA, and what matters is that the weights stream at
// memory speed.  A wave owns a strip of NT 32-feature tiles and loads ITS weight fragments (packed
// order: one contiguous 1 KB per fragment) straight from global memory into the registers the MFMA
// reads, PD k-slices ahead, with no LDS and no barrier on that path.  Only the activations, which every
// wave needs, go through LDS: KA 16-wide slices of all MT 32-token tiles per fill (packed order too, so
// a fill is a handful of contiguous 1 KB copies), double buffered, one barrier per fill.
template <int MT, int NT, int KA, int PD, bool GLU>
__device__ __forceinline__ void gemm_bf16_ws_body(
    const bf16_t* __restrict__ Ap, const bf16_t* __restrict__ Wp, float* __restrict__ out,
    int M, int N, int K, int k_per_split, int splits, int tiles_m, int tiles_n, int tn0, int block_id) {
    constexpr int BM = 32 * MT, BN = 128 * NT;
    constexpr int AFR = MT * KA;                          // activation fragments per fill
    static_assert(AFR % 4 == 0, "fill must split over 4 waves");
    constexpr int APW = AFR / 4;                          // 1 KB pieces per wave per fill
    __shared__ __attribute__((aligned(16))) unsigned char abuf[2][AFR * 1024];

    const int nblk = tiles_m * tiles_n * splits;
    int logical = xcd_remap(block_id, nblk);
    const int tm = logical % tiles_m;
    logical /= tiles_m;
    const int sp = logical % splits;
    const int tn = tn0 + logical / splits;
    const int m0 = tm * BM, n0 = tn * BN;
    const int ks0 = sp * (k_per_split / 16);              // first 16-wide slice of this split
    const int nfill = k_per_split / (16 * KA);
    const int kslices = K / 16;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, lg = lane >> 5;

    // activations, packed [M/32][K/16][64][8]: piece i of this wave's share of a fill
    const int m_tiles_total = (M + 31) / 32;
    const bf16_t* a_src[APW];
#pragma unroll
    for (int i = 0; i < APW; ++i) {
        const int f = wave * APW + i;                     // fragment of the fill: tile f / KA, slice f % KA
        int mt = m0 / 32 + f / KA;
        mt = mt < m_tiles_total ? mt : m_tiles_total - 1;
        a_src[i] = Ap + ((int64_t)mt * kslices + ks0 + f % KA) * 512 + lane * 8;
    }
    // weights, packed [N/128][K/16][4][64][8]: fragment (tile nt, slice ks)
    const bf16_t* w_src[NT];
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        // gated form (N = 2F weight rows, gate rows first).  NT == 1: work-group tn covers features
        // 64 tn .. 64 tn + 63; waves 0,1 stream their gate rows, waves 2,3 the up rows of the same features.
        // NT == 2: work-group tn covers features 128 tn .. 128 tn + 127; every wave streams the gate rows (i = 0)
        // and the up rows (i = 1) of its own 32 features.
        const int nt = !GLU ? n0 / 32 + wave * NT + i
                     : NT == 1 ? (wave < 2 ? 2 * tn + wave : N / 64 + 2 * tn + (wave - 2))
                               : (i == 0 ? 4 * tn + wave : N / 64 + 4 * tn + wave);
        w_src[i] = Wp + (((int64_t)(nt >> 2) * kslices + ks0) * 4 + (nt & 3)) * 512 + lane * 8;
    }
    constexpr int W_STEP = 4 * 512;                       // elements between consecutive slices of a tile

    floatx16 acc[NT][MT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int total_slices = nfill * KA;
    u32x4 wring[PD][NT];                                  // weight fragments in flight
#pragma unroll
    for (int p = 0; p < PD; ++p)
#pragma unroll
        for (int i = 0; i < NT; ++i)
            wring[p][i] = *reinterpret_cast<const u32x4*>(w_src[i] + (int64_t)(p < total_slices ? p : total_slices - 1) * W_STEP);

    // first fill
    u32x4 areg[APW];
#pragma unroll
    for (int i = 0; i < APW; ++i) areg[i] = *reinterpret_cast<const u32x4*>(a_src[i]);
#pragma unroll
    for (int i = 0; i < APW; ++i) *reinterpret_cast<u32x4*>(&abuf[0][(wave * APW + i) * 1024 + lane * 16]) = areg[i];

    for (int fill = 0; fill < nfill; ++fill) {
        // everyone's share of this fill is in LDS; the other buffer has no reader left
        __builtin_amdgcn_s_waitcnt(0xC07F);               // lgkmcnt(0): own LDS writes done
        __builtin_amdgcn_s_barrier();
        // next fill's activations: loaded unconditionally (the last fill is loaded twice) so that the loop body
        // has no branch and the compiler can count the loads in flight exactly; behind a branch it falls back
        // to waiting for these loads at the first product of the fill
        const int nxt = fill + 1 < nfill ? fill + 1 : fill;
#pragma unroll
        for (int i = 0; i < APW; ++i) areg[i] = *reinterpret_cast<const u32x4*>(a_src[i] + (int64_t)nxt * KA * 512);
        const unsigned char* ab = abuf[fill & 1] + lane * 16;
        static_assert(KA % PD == 0, "ring slots must be static across a fill");
        bf16x8 af[2][MT];                                  // activation fragments: this slice and the next
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
            // keep loads and reads where they are: left alone, the scheduler sinks each one to just before
            // its use and the stream degenerates into load - wait - compute
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int j = 0; j < MT; ++j)
                    // gated form: weights first, so that a lane holds one row and consecutive features (what the
                    // packed output wants); plain form: activations first, so that a lane holds one feature and the
                    // 32 lanes of a half wave write 128 contiguous bytes of an output row
                    acc[i][j] = GLU ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wring[s % PD][i]),
                                                                              af[s & 1][j], acc[i][j], 0, 0, 0)
                                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[s & 1][j], __builtin_bit_cast(bf16x8, wring[s % PD][i]),
                                                                              acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            // refill the ring slot just consumed with the slice PD ahead (clamped at the end: a harmless
            // re-load).  Issued after the products that read the slot, so the slot's registers are dead and
            // the load lands in place: issued before them, every slot needs a copy, and the compiler
            // gathers those copies at the top of the fill, behind a wait for the whole ring.
            const int ahead = slice + PD < total_slices ? slice + PD : total_slices - 1;
#pragma unroll
            for (int i = 0; i < NT; ++i)
                wring[s % PD][i] = *reinterpret_cast<const u32x4*>(w_src[i] + (int64_t)ahead * W_STEP);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < APW; ++i)
            *reinterpret_cast<u32x4*>(&abuf[(fill + 1) & 1][(wave * APW + i) * 1024 + lane * 16]) = areg[i];
    }

    if (GLU && NT == 2) {
        // gate and up of a feature sit in the same lane: silu(gate) * up in registers, rounded to bf16, written as
        // packed operand tiles [M/32][F/16][64][8] of the next projection
        const int F = N / 2;
        bf16_t* act = reinterpret_cast<bf16_t*>(out);
        const int fs = (tn * 128 + wave * 32) / 16;
#pragma unroll
        for (int j = 0; j < MT; ++j) {
            const int mt = m0 / 32 + j;
            if (mt < m_tiles_total) {
                bf16_t* dst = act + ((int64_t)mt * (F / 16) + fs) * 512;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    float r[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float g = acc[0][j][4 * q + i];
                        r[i] = g / (1.0f + expf(-g)) * acc[NT - 1][j][4 * q + i];
                    }
                    u32x2 pk = {pack2bf(r[0], r[1]), pack2bf(r[2], r[3])};
                    *reinterpret_cast<u32x2*>(dst + ((q >> 1) * 64 + l32 + 32 * (q & 1)) * 8 + 4 * lg) = pk;
                }
            }
        }
        return;
    }
    if (GLU) {
        // up halves travel through LDS to the waves that hold the gate halves; those write
        // silu(gate) * up, rounded to bf16, as packed operand tiles [M/32][F/16][64][8] of the next projection
        const int F = N / 2;
        bf16_t* act = reinterpret_cast<bf16_t*>(out);
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();                        // every wave is done reading the activations
        float* xbuf = reinterpret_cast<float*>(&abuf[0][0]); // [2 waves][MT][16][64] floats
        static_assert(2 * MT * 16 * 64 * 4 <= 2 * AFR * 1024, "exchange area");
        if (wave >= 2) {
#pragma unroll
            for (int j = 0; j < MT; ++j)
#pragma unroll
                for (int q = 0; q < 16; ++q) xbuf[(((wave - 2) * MT + j) * 16 + q) * 64 + lane] = acc[0][j][q];
        }
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        if (wave < 2) {
            const int fs = (tn * 64 + wave * 32) / 16;
#pragma unroll
            for (int j = 0; j < MT; ++j) {
                const int mt = m0 / 32 + j;
                if (mt < m_tiles_total) {
                    bf16_t* dst = act + ((int64_t)mt * (F / 16) + fs) * 512;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float r[4];
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float g = acc[0][j][4 * q + i];
                            const float u = xbuf[((wave * MT + j) * 16 + 4 * q + i) * 64 + lane];
                            r[i] = g / (1.0f + expf(-g)) * u;
                        }
                        u32x2 pk = {pack2bf(r[0], r[1]), pack2bf(r[2], r[3])};
                        *reinterpret_cast<u32x2*>(dst + ((q >> 1) * 64 + l32 + 32 * (q & 1)) * 8 + 4 * lg) = pk;
                    }
                }
            }
        }
        return;
    }
    // acc[i][j][4 q + r] <-> row m0 + 32 j + 8 q + 4 lg + r, feature n0 + 32 (wave NT + i) + l32
    float* dst = out + (int64_t)sp * M * N;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const int n = n0 + (wave * NT + i) * 32 + l32;
#pragma unroll
        for (int j = 0; j < MT; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + j * 32 + 8 * q + 4 * lg + r;
                    if (m < M) dst[(int64_t)m * N + n] = acc[i][j][4 * q + r];
                }
    }
}

// Two work-groups share a CU where the accumulator tile leaves room (up to 96 rows x 256 features, or 128-feature
// strips): more, smaller work-groups resident at once, which evens out a launch whose work-group count is not a
// multiple of the 256 CUs.
template <int MT, int NT, int KA, int PD, bool GLU = false>
__global__ __launch_bounds__(256, (NT == 1 || MT <= 3) ? 2 : 1) void gemm_bf16_ws_kernel(
    const bf16_t* __restrict__ Ap, const bf16_t* __restrict__ Wp, float* __restrict__ out,
    int M, int N, int K, int k_per_split, int splits, int tiles_m, int tiles_n, int tn0) {
    gemm_bf16_ws_body<MT, NT, KA, PD, GLU>(Ap, Wp, out, M, N, K, k_per_split, splits, tiles_m, tiles_n, tn0, blockIdx.x);
}

// Gate/up projection with a short last round: the first n_main work-groups are 160-row ones over the 128-feature
// strips [0, strips_main); the rest are 64-row ones over the remaining strips cut in two (64 features each).  One
// launch: the small work-groups start on whichever CUs free up first instead of waiting for the whole main round.
// A small work-group streams the whole reduction depth of its weight rows whatever its share of the products,
// so the last round is bound by how often the strips are re-read from L2: 64 rows x 64 features (five readers of
// 0.9 MB per half strip) take 26 us where 32 rows x 128 features (ten readers of 1.8 MB) took 35 us.
__global__ __launch_bounds__(256, 1) void gemm_bf16_ws_glu_mixed_kernel(
    const bf16_t* __restrict__ Ap, const bf16_t* __restrict__ Wp, float* __restrict__ out, int M, int N, int K,
    int tiles_m, int strips_main, int tiles_m2, int strips_tail) {
    const int n_main = tiles_m * strips_main;
    if ((int)blockIdx.x < n_main)
        gemm_bf16_ws_body<5, 2, 8, 8, true>(Ap, Wp, out, M, N, K, K, 1, tiles_m, strips_main, 0, blockIdx.x);
    else
        gemm_bf16_ws_body<2, 1, 8, 8, true>(Ap, Wp, out, M, N, K, K, 1, tiles_m2, 2 * strips_tail, 2 * strips_main, blockIdx.x - n_main);
}

// ---- third bf16 kernel: 256 rows x 256 features per work-group, both operands through LDS ----
// For a thousand rows and more the weights no longer dominate the traffic and what a work-group pulls through
// the caches per product decides: a 256 x 256 tile asks for (256 + 256) x 32 bytes per 16-wide slice of the
// reduction where the weight-streaming kernel's 160 x 256 asks for (160 + 256) x 32 for 5/8 of the products.
// Four waves, each a 128 x 128 quarter (sixteen 32x32 accumulators); a fill is four slices of both operands,
// 64 KB, copied global -> LDS by direct-to-LDS loads with no register in between (in the packed orders a fill
// is sixteen contiguous 4 KB runs: four slices of one 32-row activation tile, or the four 32-feature tiles of
// one 128-feature strip at one slice), double buffered, one barrier per fill.  Every wave reads its eight
// operand fragments of a slice from LDS as 1 KB pieces, the next slice's between the products of this one.
// Measured alone on MI355X (LM head, 2304 rows): 1.16 (K = 3584) and 1.21 PFLOP/s (K = 5120) against 1.02 and 1.06
// of the weight-streaming kernel and 1.39 and 1.31 of the vendor library; the matrix unit is busy 62 % of the cycles.
// GLU: the tile's features are 128 gate rows and the 128 up rows of the same features; a wave holds both for its
// 64 features and writes silu(gate) * up, rounded to bf16, in the packed order of the next projection.
template <bool GLU>
__global__ __launch_bounds__(256, 1) void gemm_bf16_tile_kernel(
    const bf16_t* __restrict__ Ap, const bf16_t* __restrict__ Wp, float* __restrict__ out,
    int M, int N, int K, int k_per_split, int splits, int tiles_m, int tiles_n) {
    extern __shared__ __attribute__((aligned(16))) unsigned char tile_lds[];   // two fills
    constexpr int KA = 4;                                 // 16-wide slices per fill
    constexpr int FILL = KA * 16 * 1024;                  // KA slices of 8 activation and 8 weight fragments
    constexpr int B_OFF = KA * 8 * 1024;                  // weights behind the activations of a fill
    constexpr int RW = KA / 2;                            // 4 KB weight runs (strip, slice) per wave and fill
    constexpr int LPF = 4 * KA;                           // loads per wave and fill

    const int nblk = tiles_m * tiles_n * splits;
    int logical = xcd_remap(blockIdx.x, nblk);
    const int tm = logical % tiles_m;
    logical /= tiles_m;
    const int sp = logical % splits;
    const int tn = logical / splits;
    const int m0 = tm * 256;
    const int ks0 = sp * (k_per_split / 16);
    const int nfill = k_per_split / (16 * KA);
    const int kslices = K / 16;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lg = lane >> 5;
    const int m_tiles_total = (M + 31) / 32;

    // this wave's share of a fill: activation row tiles 2 wave, 2 wave + 1 (KA slices each, contiguous) and RW of
    // the 2 KA weight runs (strip, slice), 4 KB each
    const char* a_src[2];
    const char* w_src[RW];
    int a_dst[2], w_dst[RW];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int mt = m0 / 32 + 2 * wave + i;
        mt = mt < m_tiles_total ? mt : m_tiles_total - 1;        // rows beyond M: any valid tile, never stored
        a_src[i] = reinterpret_cast<const char*>(Ap + ((int64_t)mt * kslices + ks0) * 512) + lane * 16;
        a_dst[i] = (2 * wave + i) * KA * 1024;
    }
#pragma unroll
    for (int i = 0; i < RW; ++i) {
        const int run = wave * RW + i, strip = run / KA, sl = run % KA;
        const int strip_g = GLU ? (strip == 0 ? tn : N / 256 + tn) : 2 * tn + strip;
        w_src[i] = reinterpret_cast<const char*>(Wp + (((int64_t)strip_g * kslices + ks0 + sl) * 4) * 512) + lane * 16;
        w_dst[i] = B_OFF + (strip * KA + sl) * 4096;
    }
    auto issue_fill = [&](int fill, int buf) __attribute__((always_inline)) {
        unsigned char* base = tile_lds + buf * FILL;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const char* src = a_src[i] + (int64_t)fill * (KA * 1024);
            dma4(src, SV_LDS_PTR(base + a_dst[i]));
        }
#pragma unroll
        for (int i = 0; i < RW; ++i) dma4(w_src[i] + (int64_t)fill * (KA * 4096), SV_LDS_PTR(base + w_dst[i]));
    };
    // fragment offsets of this wave inside a fill, slice 0
    int a_off[4], b_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) a_off[j] = ((wm * 4 + j) * KA) * 1024 + lane * 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int strip = GLU ? (i >> 1) : wn, tile = GLU ? 2 * wn + (i & 1) : i;
        b_off[i] = B_OFF + (strip * KA * 4 + tile) * 1024 + lane * 16;
    }

    floatx16 acc[4][4];                                   // [feature tile i][row tile j]
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // The loop is written out instruction by instruction.  A wave alone on its SIMD issues in order, and the matrix
    // unit runs dry whenever anything else is issued in a block: with the eight LDS reads of a slice and the sixteen
    // loads of a fill issued together it was busy 55 % of the cycles.  So the LDS reads of the next slice and the
    // loads of the fill after next sit between the products, one or two at a time, and execute in their shadow (the
    // last read of a slice early enough for its data to be there when the slice ends).  The reads are
    // hand-placed instructions with hand-counted waits because a direct-to-LDS load in flight makes the compiler
    // wait for every LDS read at once.
    u32x4 af[2][4], wf[2][4];
    const uint32_t lds0 = (uint32_t)(uintptr_t)SV_LDS_PTR(tile_lds);
    uint32_t a_addr[4], b_addr[4];
    auto set_buf = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 4; ++j) a_addr[j] = lds0 + buf * FILL + a_off[j];
#pragma unroll
        for (int i = 0; i < 4; ++i) b_addr[i] = lds0 + buf * FILL + b_off[i];
    };
#define SV_FENCE __builtin_amdgcn_sched_barrier(0)
#define SV_RA(SET, J, S) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(af[SET][J]) : "v"(a_addr[J]), "n"((S) * 1024))
#define SV_RB(SET, I, S) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(wf[SET][I]) : "v"(b_addr[I]), "n"((S) * 4096))
    // gated form: weights first, so that a lane holds one row and consecutive features; plain form: activations first,
    // so that a lane holds one feature and a half wave writes 128 contiguous bytes
#define SV_MF(SET, I, J)                                                                                              \
    acc[I][J] = GLU ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wf[SET][I]),                 \
                                                              __builtin_bit_cast(bf16x8, af[SET][J]), acc[I][J], 0, 0, 0) \
                    : __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af[SET][J]),                 \
                                                              __builtin_bit_cast(bf16x8, wf[SET][I]), acc[I][J], 0, 0, 0)
    // the products of one slice (operands in SET), the reads of slice S into the other set woven into the first half
#define SV_SLICE_HEAD(SET, S)                                                                                         \
    SV_FENCE; SV_MF(SET, 0, 0); SV_MF(SET, 0, 1); SV_FENCE; SV_RA(1 - SET, 0, S); SV_RA(1 - SET, 1, S); SV_FENCE;     \
    SV_MF(SET, 0, 2); SV_MF(SET, 0, 3); SV_FENCE; SV_RA(1 - SET, 2, S); SV_RA(1 - SET, 3, S); SV_FENCE;               \
    SV_MF(SET, 1, 0); SV_MF(SET, 1, 1); SV_FENCE; SV_RB(1 - SET, 0, S); SV_FENCE;                                     \
    SV_MF(SET, 1, 2); SV_MF(SET, 1, 3); SV_FENCE; SV_RB(1 - SET, 1, S); SV_FENCE
#define SV_SLICE_TAIL(SET, S)                                                                                         \
    SV_MF(SET, 2, 0); SV_MF(SET, 2, 1); SV_FENCE; SV_RB(1 - SET, 2, S); SV_FENCE;                                     \
    SV_MF(SET, 2, 2); SV_MF(SET, 2, 3); SV_FENCE; SV_RB(1 - SET, 3, S); SV_FENCE;                                     \
    SV_MF(SET, 3, 0); SV_MF(SET, 3, 1); SV_MF(SET, 3, 2); SV_MF(SET, 3, 3); SV_FENCE

    issue_fill(0, 0);
    issue_fill(nfill > 1 ? 1 : 0, 1);
    wait_vmcnt<LPF>();                                    // the first fill has landed (loads return in order)
    __builtin_amdgcn_s_barrier();
    set_buf(0);
    SV_RA(0, 0, 0); SV_RA(0, 1, 0); SV_RA(0, 2, 0); SV_RA(0, 3, 0);
    SV_RB(0, 0, 0); SV_RB(0, 1, 0); SV_RB(0, 2, 0); SV_RB(0, 3, 0);
    for (int fill = 0; fill < nfill; ++fill) {
        const int buf = fill & 1;
        wait_lgkmcnt0();
        SV_SLICE_HEAD(0, 1); SV_SLICE_TAIL(0, 1);
        wait_lgkmcnt0();
        SV_SLICE_HEAD(1, 2); SV_SLICE_TAIL(1, 2);
        wait_lgkmcnt0();
        SV_SLICE_HEAD(0, 3); SV_SLICE_TAIL(0, 3);
        // This wave holds everything it needs of the buffer; its share of the next fill has landed; after the barrier
        // so has everyone's, and nobody reads this buffer any more.
        wait_lgkmcnt0();
        wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
        set_buf(buf ^ 1);
        // last slice: the first slice of the next fill is read, and the fill after next (past the end: the last one
        // again, so that the loop has no branch) is requested into the buffer just given up
        SV_SLICE_HEAD(1, 0);
        {
            const int ahead = fill + 2 < nfill ? fill + 2 : nfill - 1;
            unsigned char* base = tile_lds + buf * FILL;
            SV_MF(1, 2, 0); SV_MF(1, 2, 1); SV_FENCE; SV_RB(0, 2, 0); SV_FENCE;
            dma4(a_src[0] + (int64_t)ahead * (KA * 1024), SV_LDS_PTR(base + a_dst[0])); SV_FENCE;
            SV_MF(1, 2, 2); SV_MF(1, 2, 3); SV_FENCE; SV_RB(0, 3, 0); SV_FENCE;
            dma4(a_src[1] + (int64_t)ahead * (KA * 1024), SV_LDS_PTR(base + a_dst[1])); SV_FENCE;
            SV_MF(1, 3, 0); SV_MF(1, 3, 1); SV_FENCE;
            dma4(w_src[0] + (int64_t)ahead * (KA * 4096), SV_LDS_PTR(base + w_dst[0])); SV_FENCE;
            SV_MF(1, 3, 2); SV_MF(1, 3, 3); SV_FENCE;
            dma4(w_src[1] + (int64_t)ahead * (KA * 4096), SV_LDS_PTR(base + w_dst[1])); SV_FENCE;
        }
    }
    wait_lgkmcnt0();
#undef SV_FENCE
#undef SV_RA
#undef SV_RB
#undef SV_MF
#undef SV_SLICE_HEAD
#undef SV_SLICE_TAIL
    wait_vmcnt<0>();                                      // nothing of this work-group may land in LDS after it has gone

    if (GLU) {
        const int F = N / 2;
        bf16_t* act = reinterpret_cast<bf16_t*>(out);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int fs = (tn * 128 + (2 * wn + i) * 32) / 16;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int mt = m0 / 32 + wm * 4 + j;
                if (mt < m_tiles_total) {
                    bf16_t* dst = act + ((int64_t)mt * (F / 16) + fs) * 512;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        float r[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float g = acc[i][j][4 * q + e];
                            r[e] = g / (1.0f + expf(-g)) * acc[2 + i][j][4 * q + e];
                        }
                        u32x2 pk = {pack2bf(r[0], r[1]), pack2bf(r[2], r[3])};
                        *reinterpret_cast<u32x2*>(dst + ((q >> 1) * 64 + l32 + 32 * (q & 1)) * 8 + 4 * lg) = pk;
                    }
                }
            }
        }
        return;
    }
    // acc[i][j][4 q + r] <-> row m0 + 32 (4 wm + j) + 8 q + 4 lg + r, feature 256 tn + 32 (4 wn + i) + l32
    float* dst = out + (int64_t)sp * M * N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = tn * 256 + (wn * 4 + i) * 32 + l32;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = m0 + (wm * 4 + j) * 32 + 8 * q + 4 * lg + r;
                    if (m < M) dst[(int64_t)m * N + n] = acc[i][j][4 * q + r];
                }
    }
}

// plain: out [splits][M][N] fp32, N % 256 == 0.  gated: N = 2 F weight rows, out = packed bf16 [ceil(M/32)*32, F],
// F % 128 == 0, splits == 1.  (K / splits) % 64 == 0.
hipError_t gemm_bf16_tile(const bf16_t* Ap, const bf16_t* Wp, float* out, int M, int N, int K, int splits, bool glu, hipStream_t st) {
    if (splits < 1 || K % splits != 0 || (K / splits) % 64 != 0 || N % 256 != 0 || (glu && splits != 1))
        return hipErrorInvalidValue;
    const int tiles_m = (M + 255) / 256, tiles_n = glu ? N / 2 / 128 : N / 256;
    auto launch = [&](auto kern) -> hipError_t {
        const size_t lds = 2 * 4 * 16 * 1024;             // two fills of four slices
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n * splits), dim3(256), lds, st, Ap, Wp, out, M, N, K, K / splits, splits,
                           tiles_m, tiles_n);
        return hipGetLastError();
    };
    return glu ? launch(gemm_bf16_tile_kernel<true>) : launch(gemm_bf16_tile_kernel<false>);
}

// Activations [M, K] row-major -> packed [ceil(M/32)][K/16][64 lanes][8]: lane 32*g + r of a fragment holds
// row 32*tile + r, elements 8*g .. 8*g+7 of the slice; rows beyond M are written as zeros.
__global__ void pack_rows_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int M, int K) {
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)((M + 31) / 32) * 32 * K / 8;
    if (piece >= total) return;
    const int lane = piece & 63;
    const int64_t frag = piece >> 6;
    const int ks = frag % (K / 16), mt = frag / (K / 16);
    const int row = mt * 32 + (lane & 31), col = ks * 16 + (lane >> 5) * 8;
    u32x4 v = {0, 0, 0, 0};
    if (row < M) v = *reinterpret_cast<const u32x4*>(src + (int64_t)row * K + col);
    *reinterpret_cast<u32x4*>(dst + piece * 8) = v;
}

hipError_t pack_rows(const bf16_t* src, bf16_t* dst, int M, int K, hipStream_t st) {
    const int64_t pieces = (int64_t)((M + 31) / 32) * 32 * K / 8;
    hipLaunchKernelGGL(pack_rows_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, src, dst, M, K);
    return hipGetLastError();
}

template <int MT, int NT, int KA, int PD>
static hipError_t launch_ws(const bf16_t* Ap, const bf16_t* Wp, float* out, int M, int N, int K, int splits, hipStream_t st) {
    constexpr int BM = 32 * MT, BN = 128 * NT;
    if (N % BN != 0 || (K / splits) % (16 * KA) != 0) return hipErrorInvalidValue;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = N / BN;
    hipLaunchKernelGGL((gemm_bf16_ws_kernel<MT, NT, KA, PD>), dim3(tiles_m * tiles_n * splits), dim3(256), 0, st, Ap, Wp,
                       out, M, N, K, K / splits, splits, tiles_m, tiles_n, 0);
    return hipGetLastError();
}

// Gate/up projection fused with SwiGLU: Wp packed [2F, K] (gate rows, then up rows); act_out packed
// [ceil(M/32)*32, F] bf16.  F a multiple of 64.
hipError_t gemm_bf16_ws_glu(const bf16_t* Ap, const bf16_t* Wp, bf16_t* act_out, int M, int F, int K, hipStream_t st, int tile_mode) {
    if (F % 64 != 0 || K % 64 != 0) return hipErrorInvalidValue;
    float* out = reinterpret_cast<float*>(act_out);
    if (F % 128 == 0 && tile_mode != 0) {
        // From a thousand rows on the 256-row tiles win where their launch fills its rounds about as well as the
        // 160-row one does: rounds x rows per work-group / the rate a CU reaches with either (TFLOP/s, measured).
        const long long n_ws = (long long)((M + 159) / 160) * (F / 128), n_tile = (long long)((M + 255) / 256) * (F / 128);
        const double t_ws = (double)((n_ws + 255) / 256) * 160.0 / 4.47, t_tile = (double)((n_tile + 255) / 256) * 256.0 / kTileRateGlu;
        if (tile_mode == 1 || (M >= 1024 && t_tile < 0.97 * t_ws)) return gemm_bf16_tile(Ap, Wp, out, M, 2 * F, K, 1, true, st);
    }
    if (F % 128 == 0 && K % 128 == 0) {
        // 128-feature strips, gate and up in one wave.  One work-group per CU: the launch runs in rounds of 256,
        // and a last round that is less than half full would leave most CUs idle for a whole work-group's time.
        // Its strips are then given to 64-row work-groups of half a strip each (five times as many, a fifth of the
        // products) at the end of the same launch.
        const int mt = gemm_bf16_ws_row_tiles(M);
        const int tiles_m = (M + 32 * mt - 1) / (32 * mt), strips = F / 128;
        const int rem = (strips * tiles_m) % 256;
        const int strips_tail = mt == 5 && rem > 0 && rem <= 128 ? (rem + tiles_m - 1) / tiles_m : 0;
        const int strips_main = strips - strips_tail;
        const int tiles_m1 = (M + 31) / 32;
        auto launch = [&](auto kern) {
            hipLaunchKernelGGL(kern, dim3(tiles_m * strips), dim3(256), 0, st, Ap, Wp, out, M, 2 * F, K, K, 1, tiles_m, strips, 0);
        };
        if (strips_tail == 0) {
            switch (mt) {
                case 1: launch(gemm_bf16_ws_kernel<1, 2, 8, 8, true>); break;
                case 2: launch(gemm_bf16_ws_kernel<2, 2, 8, 8, true>); break;
                case 3: launch(gemm_bf16_ws_kernel<3, 2, 8, 8, true>); break;
                case 4: launch(gemm_bf16_ws_kernel<4, 2, 8, 8, true>); break;
                default: launch(gemm_bf16_ws_kernel<5, 2, 8, 8, true>); break;
            }
        } else if (strips_main == 0)
            hipLaunchKernelGGL((gemm_bf16_ws_kernel<1, 2, 8, 8, true>), dim3(tiles_m1 * strips_tail), dim3(256), 0, st, Ap, Wp,
                               out, M, 2 * F, K, K, 1, tiles_m1, strips_tail, 0);
        else {
            const int tiles_m2 = (M + 63) / 64;
            hipLaunchKernelGGL(gemm_bf16_ws_glu_mixed_kernel, dim3(tiles_m * strips_main + tiles_m2 * 2 * strips_tail), dim3(256), 0,
                               st, Ap, Wp, out, M, 2 * F, K, tiles_m, strips_main, tiles_m2, strips_tail);
        }
        return hipGetLastError();
    }
    const int tiles_m = (M + 159) / 160, tiles_n = F / 64;
    if (K % 128 == 0)
        hipLaunchKernelGGL((gemm_bf16_ws_kernel<5, 1, 8, 8, true>), dim3(tiles_m * tiles_n), dim3(256), 0, st, Ap, Wp,
                           out, M, 2 * F, K, K, 1, tiles_m, tiles_n, 0);
    else
        hipLaunchKernelGGL((gemm_bf16_ws_kernel<5, 1, 4, 4, true>), dim3(tiles_m * tiles_n), dim3(256), 0, st, Ap, Wp,
                           out, M, 2 * F, K, K, 1, tiles_m, tiles_n, 0);
    return hipGetLastError();
}

// Weight-streaming projection: packed activations, packed weights.  wide: 256 features per work-group.
// 32-row tiles per work-group for M rows: as few work-groups along the rows as five tiles each allow, then no
// more tiles each than those work-groups need (320 rows: 2 x 5; 512 rows: 4 x 4; 64 rows: 1 x 2).
int gemm_bf16_ws_row_tiles(int M) {
    const int tiles = (M + 31) / 32, groups = (tiles + 4) / 5;
    return (tiles + groups - 1) / groups;
}

hipError_t gemm_bf16_ws(const bf16_t* Ap, const bf16_t* Wp, float* out, int M, int N, int K, int splits, bool wide,
                        hipStream_t st, int row_tiles) {
    if (row_tiles == 8) return gemm_bf16_tile(Ap, Wp, out, M, N, K, splits, false, st);
    const bool long_fill = (K / splits) % 128 == 0;
    const int mt = row_tiles >= 1 && row_tiles <= 5 ? row_tiles : gemm_bf16_ws_row_tiles(M);
    if (!long_fill) {        // short fills (small models; many splits of a deep reduction at a few rows): narrow strips of
                             // one or two row tiles, else the five-tile form
        if (!wide && mt == 1) return launch_ws<1, 1, 4, 4>(Ap, Wp, out, M, N, K, splits, st);
        if (!wide && mt == 2) return launch_ws<2, 1, 4, 4>(Ap, Wp, out, M, N, K, splits, st);
        return wide ? launch_ws<5, 2, 4, 4>(Ap, Wp, out, M, N, K, splits, st) : launch_ws<5, 1, 4, 4>(Ap, Wp, out, M, N, K, splits, st);
    }
    switch (mt * 2 + (wide ? 1 : 0)) {
        case 2: return launch_ws<1, 1, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 3: return launch_ws<1, 2, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 4: return launch_ws<2, 1, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 5: return launch_ws<2, 2, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 6: return launch_ws<3, 1, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 7: return launch_ws<3, 2, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 8: return launch_ws<4, 1, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 9: return launch_ws<4, 2, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        case 10: return launch_ws<5, 1, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
        default: return launch_ws<5, 2, 8, 8>(Ap, Wp, out, M, N, K, splits, st);
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

// dst (packed) <- src [N, K] row-major.  Packed order: [N/128][K/16][4 tiles of 32 rows][64 lanes][8],
// lane 32*g + r of a tile holding row r, elements 8*g .. 8*g+7 of the 16-wide k slice.
__global__ void pack_weight_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N, int K) {
    const int64_t piece = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;          // one 16-byte piece
    const int64_t total = (int64_t)N * K / 8;
    if (piece >= total) return;
    const int lane = piece & 63;
    int64_t frag = piece >> 6;
    const int within = frag & 3;
    frag >>= 2;
    const int ks = frag % (K / 16);
    const int grp = frag / (K / 16);
    const int row = (grp * 4 + within) * 32 + (lane & 31), col = ks * 16 + (lane >> 5) * 8;
    *reinterpret_cast<u32x4*>(dst + piece * 8) = *reinterpret_cast<const u32x4*>(src + (int64_t)row * K + col);
}

hipError_t pack_weight(const bf16_t* src, bf16_t* dst, int N, int K, hipStream_t st) {
    const int64_t pieces = (int64_t)N * K / 8;
    hipLaunchKernelGGL(pack_weight_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, src, dst, N, K);
    return hipGetLastError();
}

int gemm_bf16_variant_ok(int variant, int N) { return variant >= 0 && variant <= 2 && N % 128 == 0; }

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
