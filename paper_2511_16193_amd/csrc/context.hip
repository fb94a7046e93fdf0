// C ABI of the verification step: context, host-side page bookkeeping, and the sequence of kernel
// launches that makes up one parallel verification pass (declared in include/specverify.h).
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <algorithm>
#include <functional>
#include <cmath>
#include <string>
#include <vector>

#include "../../include/specverify.h"
#include "../../include/specverify_ops.h"
#include "kernels.h"

using namespace sv;

namespace {

constexpr int kRing = 8;              // pinned staging slots for per-step host -> device metadata
constexpr int kMaxSplits = 8;
constexpr int kMaxSplitsWs = 16;       // weight-streaming kernel: any divisor of the slice count up to this
constexpr int kChunkKeys = 1024;      // keys per split-KV chunk of the bf16 attention

struct SeqState {
    bool live = false;
    int len_ub = 0;                   // host upper bound of the live length
    std::vector<int32_t> pages;
};

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

int pick_splits(int M, int N, int K) {
    // enough work-groups to cover the 256 CUs about twice; the reduction range stays a multiple of 64
    const int tiles = ((M + 127) / 128) * (N / 128);
    int s = 1;
    while (s < kMaxSplits && tiles * s < 512 && K % (64 * s * 2) == 0) s *= 2;
    return s;
}

// Launch plan of the weight-streaming projection kernel: 32-row tiles per work-group, strip width and reduction
// splits, by an estimate of the run time in microseconds.  The estimate plays the launch through: work-groups are
// dealt to the 256 CUs in rounds (one work-group per CU for the 128- and 160-row x 256-feature tiles, two for the
// smaller ones); a CU works its share off at a rate that grows with the rows it holds (the weight stream is
// shared by more products), no faster than a lone work-group can walk its reduction slices; the chip as a whole
// sustains about 1.2 PFLOP/s on random data (it is power-limited well below the MFMA peak) and 5 TB/s of
// weights; a partial plane costs its bytes, written here and read again by the consumer.  The constants are a
// fit to a sweep of every (tiles, width, splits) over thirty shapes of the benchmark models on MI355X (rows 5 to
// 2304), except the lone work-group's pace, which is taken from whole steps (cold weights); on the sweep the plan
// chosen was within 0.3 % of the best on average and 4.5 % at worst.
struct WsPlan { int splits; bool wide; int row_tiles; };
WsPlan plan_ws(int M, int N, int K, bool allow_split, int tile_mode = -1) {
    const int slices_all = K / 16;
    const int tiles = (M + 31) / 32;
    WsPlan best{1, false, gemm_bf16_ws_row_tiles(M)};
    double best_t = 1e30;
    // up to 160 rows: one work-group along the rows (cutting so few rows only multiplies the readers of a strip)
    const int mt_lo = tiles <= 5 ? tiles : 1, mt_hi = tiles <= 5 ? tiles : 5;
    for (int mt = mt_lo; mt <= mt_hi; ++mt)
        for (int wide = 0; wide < 2; ++wide) {
            if (wide && N % 256 != 0) continue;
            const int cols = wide ? 256 : 128;
            const int tiles_m = (tiles + mt - 1) / mt;
            const int per_cu = (wide && mt >= 4) ? 1 : 2;                     // work-groups resident per CU
            const double base = wide ? 5.19 : 4.14;                           // TFLOP/s of a CU at full tile height
            // us per slice a lone work-group cannot beat: inside a step a layer's weights come cold from HBM (32 KB in
            // flight per work-group against ~1 us of latency), twice what a sweep of one projection in a loop shows
            const double lone = wide ? 0.17 : 0.13;
            // share of that rate a CU reaches with one resp. two work-groups of mt tiles
            static const double kOne[6] = {0, 0.56, 0.97, 0.94, 0.93, 0.98}, kTwo[6] = {0, 0.58, 0.82, 0.90, 0.96, 0.95};
            auto cu_rate = [&](int g) { return base * (g == 1 ? kOne[mt] : kTwo[mt]) * 1e6; };   // flop per microsecond
            for (int s = 1; s <= (allow_split ? kMaxSplitsWs : 1); ++s) {
                if (slices_all % (4 * s) != 0) continue;
                if ((K / s) % 128 != 0 && tiles > 5 && mt != 5) continue;     // short fills exist in the five-tile form only
                const double slices = (double)slices_all / s;
                const double wg_flop = 2.0 * 32 * mt * cols * 16 * slices;
                const long long blocks = (long long)tiles_m * (N / cols) * s;
                auto round_time = [&](long long n) {                          // n work-groups dealt to the 256 CUs at once
                    const int g = (int)((n + 255) / 256);
                    return std::max(g * wg_flop / cu_rate(g), slices * lone * (1.0 + 0.373 * (g - 1)));
                };
                const long long cap = 256LL * per_cu, full = blocks / cap, rem = blocks % cap;
                double t = full * round_time(cap) + (rem ? round_time(rem) : 0.0);
                t = std::max(t, 2.0 * M * (double)N * K / 1198.0e6);          // the chip's sustained rate
                t = std::max(t, (double)N * K * 2.0 / 4.98e6);                // a weight stream cannot beat the memory system
                if (s > 1) t += (double)s * M * N * 4.0 / 5.4e6 + (double)(s - 1) * M * N * 4.0 / 4.0e6;   // planes written here, read by the consumer
                t += 2.3;
                if (t < best_t - 1e-9) { best_t = t; best = WsPlan{s, wide != 0, mt}; }
            }
        }
    // The 256 x 256 kernel (row_tiles 8) from a thousand rows on, where its tiles fill the chip at least four times
    // over (the LM head): measured inside the steps of the 7B shape it takes 8 % off that launch at 1280 and at 2304
    // rows.  Narrower projections (QKV, O, down: fewer tiles than CUs) stay with the weight-streaming kernel.
    if (tile_mode != 0 && N % 256 == 0 && K % 64 == 0) {
        const long long blocks = (long long)((M + 255) / 256) * (N / 256);
        if (tile_mode == 1 || (M >= 1024 && blocks >= 4 * 256)) best = WsPlan{1, true, 8};
    }
    return best;
}

struct Layout {                       // byte offsets into the workspace
    size_t seq_len, page_table, batch_seq, upd, work, req_chunk, row_tok, row_pos, row_slot, chain_acc, chain_tok, chain_row, draw_part;
    size_t rope, row_stat, h, a_norm, q, attn, part, act, logits, part_o, part_ml, total;
    size_t moe_ids, moe_w, moe_cnt, moe_off, moe_perm, moe_inv, moe_act, moe_y, moe_logits;   // mixture-of-experts scratch
    int T, rows_pad, max_chunks;
};

bool make_layout(const sv_model& m, const sv_runtime& r, Layout& L) {
    if (r.max_batch <= 0 || r.max_k < 0 || r.max_chains <= 0 || r.max_seqs <= 0 || r.page_size <= 0 ||
        r.page_size % kVBlk != 0 || r.num_pages <= 0 || r.max_pages_per_seq <= 0 || r.max_batch > 32767 ||
        (size_t)r.max_pages_per_seq * r.page_size / kChunkKeys > 65535)
        return false;
    const size_t es = m.dtype == SV_BF16 ? 2 : 4;
    const int T = r.max_batch * (1 + r.max_chains * r.max_k);
    const int qw = m.n_q_heads * m.head_dim, qkvw = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    const int F = m.n_experts ? m.d_expert : m.d_ff;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
    L.T = T;
    L.seq_len = take(sizeof(int32_t) * r.max_seqs);
    L.page_table = take(sizeof(int32_t) * (size_t)r.max_seqs * r.max_pages_per_seq);
    L.batch_seq = take(sizeof(int32_t) * r.max_batch);
    L.upd = take(sizeof(int32_t) * 3 * (size_t)r.max_batch * 8);
    L.max_chunks = (int)(((size_t)r.max_pages_per_seq * r.page_size + kChunkKeys - 1) / kChunkKeys);
    L.work = take(sizeof(int32_t) * 4 * (size_t)r.max_batch * L.max_chunks);
    L.req_chunk = take(sizeof(int32_t) * (2 * (size_t)r.max_batch + 1));      // + the number of work items
    L.row_tok = take(sizeof(int32_t) * T);
    L.row_pos = take(sizeof(int32_t) * T);
    L.row_slot = take(sizeof(int32_t) * T);
    L.chain_acc = take(sizeof(int32_t) * r.max_batch * r.max_chains);
    L.chain_tok = take(sizeof(int32_t) * r.max_batch * r.max_chains);
    L.chain_row = take(sizeof(int32_t) * r.max_batch * r.max_chains);
    L.draw_part = take(sizeof(float) * 4 * kDrawParts * T);       // per (request, chain); per row in match mode
    L.rope = take(sizeof(float) * (size_t)T * m.head_dim);
    L.row_stat = take(sizeof(float) * 4 * T);
    L.h = take(sizeof(float) * (size_t)T * m.d_model);
    const size_t Tp = (size_t)(T + 31) / 32 * 32;          // packed activations come in 32-row tiles
    L.a_norm = take(es * Tp * m.d_model);
    L.q = take(es * (size_t)T * qw);
    L.attn = take(es * Tp * qw);
    // split-K partial products: the largest splits * rows * features any projection can ask for
    size_t part = 0;
    const int shapes[4][2] = {{qkvw, m.d_model}, {m.d_model, qw}, {2 * F, m.d_model}, {m.d_model, F}};
    for (int tm = 1; tm <= (T + 127) / 128; ++tm) {
        const int M = std::min(tm * 128, T);
        for (auto& sh : shapes)
            part = std::max(part, (size_t)(m.dtype == SV_BF16 ? pick_splits(M, sh[0], sh[1]) : 1) * M * sh[0]);
    }
    if (m.dtype == SV_BF16)                                 // the same for the plans of the weight-streaming kernel
        for (int M = 1; M <= T; ++M)                       // every row count a call can bring (the plan weighs M itself)
            for (auto& sh : shapes)
                if (sh[1] % 64 == 0) part = std::max(part, (size_t)plan_ws(M, sh[0], sh[1], true).splits * M * sh[0]);
    L.part = take(sizeof(float) * part);
    L.act = take(es * Tp * F);
    L.logits = take(sizeof(float) * (size_t)T * m.vocab);
    const int G = m.n_q_heads / std::max(1, m.n_kv_heads);
    // the MFMA attention stacks G * n rows per kv head; its chunk partials are kept for up to 256 of them
    L.rows_pad = std::max(64, std::min(256, (G * (1 + r.max_chains * r.max_k) + 15) / 16 * 16));
    L.part_o = take(sizeof(float) * (size_t)r.max_batch * m.n_kv_heads * L.max_chunks * L.rows_pad * m.head_dim);
    L.part_ml = take(sizeof(float) * (size_t)r.max_batch * m.n_kv_heads * L.max_chunks * L.rows_pad * 2);
    L.moe_ids = L.moe_w = L.moe_cnt = L.moe_off = L.moe_perm = L.moe_inv = L.moe_act = L.moe_y = L.moe_logits = 0;
    if (m.n_experts > 0) {
        const size_t tiles = (size_t)moe_max_tiles(T, m.n_experts, m.top_k);
        L.moe_ids = take(sizeof(int32_t) * (size_t)T * m.top_k);
        L.moe_w = take(sizeof(float) * (size_t)T * m.top_k);
        L.moe_cnt = take(sizeof(int32_t) * m.n_experts);
        L.moe_off = take(sizeof(int32_t) * (m.n_experts + 1));
        L.moe_perm = take(sizeof(int32_t) * 32 * tiles);
        L.moe_inv = take(sizeof(int32_t) * (size_t)T * m.top_k);
        L.moe_act = take(es * 32 * tiles * m.d_expert);
        L.moe_y = take(sizeof(float) * 32 * tiles * m.d_model);
        L.moe_logits = take(sizeof(float) * 4 * (size_t)T * m.n_experts);
    }
    L.total = o;
    return true;
}

bool model_ok(const sv_model& m) {
    return m.n_layers > 0 && m.d_model > 0 && m.n_q_heads > 0 && m.n_kv_heads > 0 && m.head_dim > 0 &&
           m.head_dim % 2 == 0 && m.vocab > 0 && m.n_q_heads % m.n_kv_heads == 0 &&
           (m.dtype == SV_FP32 || m.dtype == SV_BF16) && (m.n_experts > 0 || m.d_ff > 0);
}

__global__ void apply_page_updates_kernel(int32_t* page_table, int mpps, const int32_t* upd, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) page_table[(int64_t)upd[3 * i] * mpps + upd[3 * i + 1]] = upd[3 * i + 2];
}

__global__ void set_lens_kernel(int32_t* seq_len, const int32_t* pairs, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) seq_len[pairs[2 * i]] = pairs[2 * i + 1];
}

}  // namespace

struct sv_ctx {
    sv_model model;
    sv_runtime rt;
    std::vector<const void*> ln1, wqkv, wo, ln2, wgu, wdown, wrouter;
    const void *embed, *lm_head, *final_norm;
    hipStream_t stream;
    Layout lay;
    KvGeom geom;
    char* ws;
    std::vector<SeqState> seqs;
    std::vector<int32_t> free_pages;
    int32_t* staging[kRing];
    hipEvent_t staged[kRing];
    bool staged_valid[kRing];
    int ring_pos;
    int n_work;                                           // attention work items staged for the current batch
    const int32_t* tok_matrix = nullptr;                  // batched prefill: the prompts the next forward pass reads its rows from
    const int32_t* tok_len = nullptr;
    int tok_ld = 0, tok_col0 = 0;
    int gemm_variant;                                     // -1 = choose per shape
    int gemm_tile;                                        // 256 x 256 projection kernel: -1 = where it pays, 0 = never, 1 = wherever the shape allows
    bool packed;                                          // projection weights are in fragment order
    bool attn_generic;
    int attn_min_rt;
    int attn_max_rt;
    bool use_graph;                                       // replay verify_step's device work from captured graphs
    bool graph_launch_shape;                              // launches take shapes that do not depend on the lengths
    struct GraphEntry {
        int B, k, N;
        const void* ptr[9];
        hipGraphExec_t exec;
        unsigned long long used;
    };
    std::vector<GraphEntry> graphs;
    unsigned long long graph_clock;
    int attn_chunk;                                       // keys per split-KV chunk of the staged batch
    int attn_chunk_opt;                                   // 0 = chosen per batch, else fixed by option
    unsigned prof_mask;                                   // kinds of kernels to time with events
    struct ProfRec { int kind; hipEvent_t a, b; };
    std::vector<ProfRec> prof_recs;                       // recorded, not yet read
    std::vector<hipEvent_t> prof_free;                    // event pool
    std::string err;

    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
    int fail(int code, const char* fmt, ...) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        err = buf;
        return code;
    }
    int hip(hipError_t e, const char* what) {
        if (e == hipSuccess) return SV_OK;
        return fail(SV_EHIP, "%s: %s", what, hipGetErrorString(e));
    }
};

// Brackets the launches of one kind with a pair of events on the context's stream when that kind is
// being profiled.
struct ProfScope {
    sv_ctx* c; int kind; bool on; hipEvent_t a;
    ProfScope(sv_ctx* c_, int kind_) : c(c_), kind(kind_), on(((c_->prof_mask >> kind_) & 1u) != 0), a(nullptr) {
        if (!on) return;
        a = take();
        if (a) (void)hipEventRecord(a, c->stream); else on = false;
    }
    ~ProfScope() {
        if (!on) return;
        hipEvent_t b = take();
        if (!b) { c->prof_free.push_back(a); return; }
        (void)hipEventRecord(b, c->stream);
        c->prof_recs.push_back({kind, a, b});
    }
    hipEvent_t take() {
        if (!c->prof_free.empty()) { hipEvent_t e = c->prof_free.back(); c->prof_free.pop_back(); return e; }
        hipEvent_t e = nullptr;
        return hipEventCreate(&e) == hipSuccess ? e : nullptr;
    }
};

#define SV_TRY(expr)                    \
    do {                                \
        int _rc = (expr);               \
        if (_rc != SV_OK) return _rc;   \
    } while (0)
#define SV_HIP(ctx, expr) SV_TRY((ctx)->hip((expr), #expr))

static KvGeom make_geom(const sv_model& m, const sv_runtime& r) {
    KvGeom g;
    g.n_kv_heads = m.n_kv_heads;
    g.head_dim = m.head_dim;
    g.page_size = r.page_size;
    g.page_elems = (int64_t)2 * m.n_kv_heads * r.page_size * m.head_dim;
    g.layer_elems = (int64_t)r.num_pages * g.page_elems;
    return g;
}

extern "C" size_t verify_kv_pool_bytes(const sv_model* m, const sv_runtime* r) {
    if (!m || !r || !model_ok(*m) || r->num_pages <= 0 || r->page_size <= 0) return 0;
    const KvGeom g = make_geom(*m, *r);
    return (size_t)m->n_layers * g.layer_elems * (m->dtype == SV_BF16 ? 2 : 4);
}

extern "C" size_t verify_workspace_bytes(const sv_model* m, const sv_runtime* r) {
    Layout L;
    if (!m || !r || !model_ok(*m) || !make_layout(*m, *r, L)) return 0;
    return L.total;
}

extern "C" int verify_init(const sv_model* m, const sv_weights* w, const sv_runtime* r, void* hip_stream, sv_ctx** out) {
    if (!m || !w || !r || !out) return SV_EINVAL;
    *out = nullptr;
    Layout L;
    if (!model_ok(*m) || !make_layout(*m, *r, L)) return SV_EINVAL;
    if (!r->kv_pool || !r->workspace || r->kv_pool_bytes < verify_kv_pool_bytes(m, r) || r->workspace_bytes < L.total ||
        ((uintptr_t)r->kv_pool & 255) || ((uintptr_t)r->workspace & 255))
        return SV_EINVAL;
    if (!(r->temperature > 0.f) || r->verify_mode < 0 || r->verify_mode > 2 || r->sample_mode < 0 || r->sample_mode > 1)
        return SV_EINVAL;
    if (!w->embed || !w->lm_head || !w->final_norm || !w->ln1 || !w->wqkv || !w->wo || !w->ln2 || !w->w_gate_up || !w->w_down)
        return SV_EINVAL;
    if (m->n_experts > 0) {
        // mixture-of-experts FFN: bf16 with packed weights only, within the expert kernels' shape cover
        if (m->dtype != SV_BF16 || !w->packed || !w->w_router) return SV_EUNSUPPORTED;
        if (!moe_shape_ok(L.T, m->d_model, m->n_experts, m->top_k, m->d_expert)) return SV_EUNSUPPORTED;
    }
    if (w->packed && m->dtype != SV_BF16) return SV_EINVAL;        // only bf16 projections have a packed form
    if (m->head_dim != 64 && m->head_dim != 128) return SV_EUNSUPPORTED;
    if (m->d_model % 4 != 0 || m->d_model > 8192) return SV_EUNSUPPORTED;   // RMSNorm kernel: float4 pieces, <= 8 per thread
    if (m->dtype == SV_BF16) {
        const int qw = m->n_q_heads * m->head_dim, qkvw = (m->n_q_heads + 2 * m->n_kv_heads) * m->head_dim;
        if (!gemm_bf16_shape_ok(qkvw, m->d_model, 1) || !gemm_bf16_shape_ok(m->d_model, qw, 1) ||
            (m->n_experts == 0 && (!gemm_bf16_shape_ok(2 * m->d_ff, m->d_model, 1) || !gemm_bf16_shape_ok(m->d_model, m->d_ff, 1))) ||
            !gemm_bf16_shape_ok(m->vocab, m->d_model, 1))
            return SV_EUNSUPPORTED;                                // GEMM N must be a multiple of 128, K of 64
    }
    sv_ctx* c = new sv_ctx();
    c->model = *m;
    c->rt = *r;
    c->lay = L;
    c->geom = make_geom(*m, *r);
    c->ws = reinterpret_cast<char*>(r->workspace);
    c->stream = reinterpret_cast<hipStream_t>(hip_stream);
    c->embed = w->embed; c->lm_head = w->lm_head; c->final_norm = w->final_norm;
    for (int l = 0; l < m->n_layers; ++l) {
        if (!w->ln1[l] || !w->wqkv[l] || !w->wo[l] || !w->ln2[l] || !w->w_gate_up[l] || !w->w_down[l] ||
            (m->n_experts > 0 && !w->w_router[l])) {
            delete c;
            return SV_EINVAL;
        }
        c->ln1.push_back(w->ln1[l]); c->wqkv.push_back(w->wqkv[l]); c->wo.push_back(w->wo[l]);
        c->ln2.push_back(w->ln2[l]); c->wgu.push_back(w->w_gate_up[l]); c->wdown.push_back(w->w_down[l]);
        c->wrouter.push_back(w->w_router ? w->w_router[l] : nullptr);
    }
    c->seqs.resize(r->max_seqs);
    c->free_pages.resize(r->num_pages);
    for (int i = 0; i < r->num_pages; ++i) c->free_pages[i] = r->num_pages - 1 - i;   // pop_back yields 0,1,2..
    c->ring_pos = 0;
    c->gemm_variant = -1;
    c->gemm_tile = -1;
    c->packed = w->packed != 0;
    c->attn_generic = false;
    c->attn_min_rt = 1;
    c->use_graph = false;
    c->graph_launch_shape = false;
    c->graph_clock = 0;
    c->attn_max_rt = 4;
    c->attn_chunk = kChunkKeys;
    c->attn_chunk_opt = 0;
    c->prof_mask = 0;
    const size_t slot_ints = (size_t)r->max_batch * (1 + 3 * 8 + 4 * L.max_chunks + 2) + 16;
    for (int i = 0; i < kRing; ++i) { c->staging[i] = nullptr; c->staged[i] = nullptr; c->staged_valid[i] = false; }
    for (int i = 0; i < kRing; ++i) {
        if (hipHostMalloc(reinterpret_cast<void**>(&c->staging[i]), slot_ints * sizeof(int32_t), hipHostMallocDefault) != hipSuccess ||
            hipEventCreateWithFlags(&c->staged[i], hipEventDisableTiming) != hipSuccess) {
            verify_destroy(c);
            return SV_EHIP;
        }
    }
    // lengths and page table start at zero; an uninitialised pool could hold NaN patterns, which a
    // masked-out key would still feed into the PV product (0 * NaN), so the pool is cleared once.
    if (hipMemsetAsync(c->ws, 0, L.rope, c->stream) != hipSuccess ||
        hipMemsetAsync(r->kv_pool, 0, verify_kv_pool_bytes(m, r), c->stream) != hipSuccess) {
        verify_destroy(c);
        return SV_EHIP;
    }
    *out = c;
    return SV_OK;
}

static void drop_graphs(sv_ctx* c);

extern "C" void verify_destroy(sv_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    drop_graphs(c);
    for (auto& r : c->prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (hipEvent_t e : c->prof_free) (void)hipEventDestroy(e);
    for (int i = 0; i < kRing; ++i) {
        if (c->staging[i]) (void)hipHostFree(c->staging[i]);
        if (c->staged[i]) (void)hipEventDestroy(c->staged[i]);
    }
    delete c;
}

extern "C" const char* verify_last_error(const sv_ctx* c) { return c ? c->err.c_str() : "null context"; }

// ------------------------------------------------------------ sequences ---

static int pages_for(const sv_ctx* c, int len) { return (len + c->rt.page_size - 1) / c->rt.page_size; }

extern "C" int verify_seq_add(sv_ctx* c, int32_t id, int32_t cached_len) {
    if (!c) return SV_EINVAL;
    if (id < 0 || id >= c->rt.max_seqs) return c->fail(SV_ENOSEQ, "sequence id %d out of range", id);
    if (c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d already live", id);
    const int need = pages_for(c, cached_len);
    if (cached_len < 0 || need > c->rt.max_pages_per_seq)
        return c->fail(SV_EINVAL, "cached_len %d exceeds max_pages_per_seq", cached_len);
    if (need > (int)c->free_pages.size()) return c->fail(SV_ENOPAGES, "need %d pages, %zu free", need, c->free_pages.size());
    SeqState& s = c->seqs[id];
    std::vector<int32_t> pages;
    for (int i = 0; i < need; ++i) { pages.push_back(c->free_pages.back()); c->free_pages.pop_back(); }
    hipError_t e = hipSuccess;
    if (need) e = hipMemcpyAsync(c->at<int32_t>(c->lay.page_table) + (size_t)id * c->rt.max_pages_per_seq, pages.data(),
                                 need * sizeof(int32_t), hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = set_i32(c->at<int32_t>(c->lay.seq_len) + id, cached_len, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);     // `pages` is a temporary
    if (e != hipSuccess) {
        for (int32_t p : pages) c->free_pages.push_back(p);
        return c->hip(e, "verify_seq_add");
    }
    s.live = true; s.len_ub = cached_len; s.pages.swap(pages);
    return SV_OK;
}

extern "C" int verify_seq_remove(sv_ctx* c, int32_t id) {
    if (!c) return SV_EINVAL;
    if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
    SeqState& s = c->seqs[id];
    for (int32_t p : s.pages) c->free_pages.push_back(p);
    s = SeqState();
    return SV_OK;
}

extern "C" int verify_seq_set_len(sv_ctx* c, int32_t id, int32_t len) {
    if (!c) return SV_EINVAL;
    if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
    SeqState& s = c->seqs[id];
    if (len < 0 || len > (int)s.pages.size() * c->rt.page_size)
        return c->fail(SV_EINVAL, "length %d beyond the %zu pages held", len, s.pages.size());
    SV_HIP(c, set_i32(c->at<int32_t>(c->lay.seq_len) + id, len, c->stream));
    s.len_ub = len;
    return SV_OK;
}

extern "C" int verify_seq_len(sv_ctx* c, int32_t id, int32_t* len_out) {
    if (!c || !len_out) return SV_EINVAL;
    if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
    int32_t len = 0;
    SV_HIP(c, hipMemcpyAsync(&len, c->at<int32_t>(c->lay.seq_len) + id, sizeof len, hipMemcpyDeviceToHost, c->stream));
    SV_HIP(c, hipStreamSynchronize(c->stream));
    SeqState& s = c->seqs[id];
    s.len_ub = len;
    const int keep = pages_for(c, len);
    while ((int)s.pages.size() > keep) { c->free_pages.push_back(s.pages.back()); s.pages.pop_back(); }
    *len_out = len;
    return SV_OK;
}

static int kv_io(sv_ctx* c, int32_t id, int32_t layer, int32_t pos0, int32_t n, void* k, void* v, bool to_pool) {
    if (!c || !k || !v) return SV_EINVAL;
    if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
    if (layer < 0 || layer >= c->model.n_layers || pos0 < 0 || n < 0 ||
        pos0 + n > (int)c->seqs[id].pages.size() * c->rt.page_size)
        return c->fail(SV_EINVAL, "kv range [%d,%d) of layer %d outside the pages held", pos0, pos0 + n, layer);
    SV_HIP(c, kv_copy(c->rt.kv_pool, c->geom, layer, c->at<int32_t>(c->lay.page_table) + (size_t)id * c->rt.max_pages_per_seq,
                      pos0, n, k, v, c->model.dtype, to_pool, c->stream));
    return SV_OK;
}
extern "C" int verify_kv_write(sv_ctx* c, int32_t id, int32_t layer, int32_t pos0, int32_t n, const void* k, const void* v) {
    return kv_io(c, id, layer, pos0, n, const_cast<void*>(k), const_cast<void*>(v), true);
}
extern "C" int verify_kv_read(sv_ctx* c, int32_t id, int32_t layer, int32_t pos0, int32_t n, void* k, void* v) {
    return kv_io(c, id, layer, pos0, n, k, v, false);
}

// ---------------------------------------------------------- forward pass ---

// Make sure every listed sequence holds pages for `extra` more entries; push ids and new page-table
// entries to the device.  Nothing changes if the pool cannot cover the whole batch.
static int stage_batch(sv_ctx* c, const int32_t* ids, int B, int extra) {
    int need_total = 0;
    for (int b = 0; b < B; ++b) {
        const int id = ids[b];
        if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
        for (int b2 = 0; b2 < b; ++b2)
            if (ids[b2] == id) return c->fail(SV_ENOSEQ, "sequence id %d appears twice in the batch", id);
        const int need = pages_for(c, c->seqs[id].len_ub + extra);
        if (need > c->rt.max_pages_per_seq) return c->fail(SV_ENOPAGES, "sequence %d would exceed max_pages_per_seq", id);
        need_total += std::max(0, need - (int)c->seqs[id].pages.size());
    }
    if (need_total > (int)c->free_pages.size())
        return c->fail(SV_ENOPAGES, "need %d more pages, %zu free", need_total, c->free_pages.size());
    if (need_total > B * 8) return c->fail(SV_EINVAL, "more than %d new pages in one step", B * 8);

    const int slot = c->ring_pos;
    if (c->staged_valid[slot]) SV_HIP(c, hipEventSynchronize(c->staged[slot]));
    int32_t* st = c->staging[slot];
    int nupd = 0;
    int32_t* upd = st + B;
    for (int b = 0; b < B; ++b) {
        SeqState& s = c->seqs[ids[b]];
        st[b] = ids[b];
        const int need = pages_for(c, s.len_ub + extra);
        while ((int)s.pages.size() < need) {
            const int32_t p = c->free_pages.back();
            c->free_pages.pop_back();
            upd[3 * nupd] = ids[b]; upd[3 * nupd + 1] = (int32_t)s.pages.size(); upd[3 * nupd + 2] = p;
            s.pages.push_back(p);
            ++nupd;
        }
    }
    SV_HIP(c, hipMemcpyAsync(c->at<int32_t>(c->lay.batch_seq), st, B * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    if (nupd) {
        SV_HIP(c, hipMemcpyAsync(c->at<int32_t>(c->lay.upd), upd, 3 * nupd * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
        hipLaunchKernelGGL(apply_page_updates_kernel, dim3((nupd + 63) / 64), dim3(64), 0, c->stream,
                           c->at<int32_t>(c->lay.page_table), c->rt.max_pages_per_seq, c->at<int32_t>(c->lay.upd), nupd);
        SV_HIP(c, hipGetLastError());
    }
    // attention work list: every (request, chunk) that can exist given the upper bounds of the lengths,
    // longest pieces first (the hardware hands work-groups to CUs in order, so this is longest-processing-
    // time-first list scheduling).  Keys per chunk, unless fixed by option: each candidate's launch is
    // simulated -- every piece goes to the CU that frees up first and costs its keys plus a fixed ~300 keys'
    // worth (measured: ~6 us of start-up and merge per work-group against ~46 keys per us per CU) -- and the
    // shortest makespan wins.
    {
        int chunk = c->attn_chunk_opt;
        if (chunk == 0) {
            double best = 1e300;
            std::vector<int> lens;
            std::vector<double> cu(256);
            for (int cand : {1024, 1536, 2048, 3072, 4096, 6144, 8192, 12288, 16384, 24576, 32768}) {
                lens.clear();
                for (int b = 0; b < B; ++b) {
                    const int total = c->seqs[ids[b]].len_ub + extra;
                    const int nch = std::max(1, std::min((total + cand - 1) / cand, c->lay.max_chunks));
                    for (int ch = 0; ch < nch; ++ch) lens.push_back((total + nch - 1) / nch);
                }
                std::sort(lens.begin(), lens.end(), std::greater<int>());
                std::fill(cu.begin(), cu.end(), 0.0);
                for (int len : lens)
                    for (int h = 0; h < c->model.n_kv_heads; ++h) {
                        std::pop_heap(cu.begin(), cu.end(), std::greater<double>());
                        cu.back() += len + 300.0;
                        std::push_heap(cu.begin(), cu.end(), std::greater<double>());
                    }
                const double makespan = *std::max_element(cu.begin(), cu.end());
                if (makespan < best) { best = makespan; chunk = cand; }
            }
        }
        c->attn_chunk = chunk;
        // An item carries all a work-group needs to start streaming -- (request << 16 | chunk), sequence id,
        // first key, end of the piece -- so that its first K/V load is two dependent reads away (item, then
        // page table; the live length is read beside it and only clips the end).  Pieces are cut from the
        // upper bounds of the lengths: equal parts, whole 32-key tiles.
        int32_t* req = upd + 3 * nupd;                   // per request: keys per piece, pieces
        int32_t* work = req + 2 * c->rt.max_batch + 1;
        struct Item { int len, b, ch, seq, kbeg, kend; };
        std::vector<Item> items;
        for (int b = 0; b < B; ++b) {
            const int total = c->seqs[ids[b]].len_ub + extra;
            const int nch = std::max(1, std::min((total + chunk - 1) / chunk, c->lay.max_chunks));
            const int clen = ((total + nch - 1) / nch + 31) / 32 * 32;
            req[2 * b] = clen; req[2 * b + 1] = nch;
            for (int ch = 0; ch < nch && ch * clen < total; ++ch)
                items.push_back({std::min(clen, total - ch * clen), b, ch, ids[b], ch * clen, std::min((ch + 1) * clen, total)});
        }
        std::stable_sort(items.begin(), items.end(), [](const Item& x, const Item& y) { return x.len > y.len; });
        int nw = 0;
        for (auto& t : items) {
            work[4 * nw] = (t.b << 16) | t.ch; work[4 * nw + 1] = t.seq; work[4 * nw + 2] = t.kbeg; work[4 * nw + 3] = t.kend;
            ++nw;
        }
        req[2 * c->rt.max_batch] = nw;                    // read by launches that were captured into a graph
        SV_HIP(c, hipMemcpyAsync(c->at<int32_t>(c->lay.req_chunk), req, (2 * c->rt.max_batch + 1) * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
        SV_HIP(c, hipMemcpyAsync(c->at<int32_t>(c->lay.work), work, 4 * nw * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
        c->n_work = nw;
    }
    SV_HIP(c, hipEventRecord(c->staged[slot], c->stream));
    c->staged_valid[slot] = true;
    c->ring_pos = (slot + 1) % kRing;
    return SV_OK;
}

// Work-group tile of the row-major projection kernel for M rows: 64, 128 or 256 tokens x 128 features.
static int pick_variant(const sv_ctx* c, int M) {
    if (c->gemm_variant >= 0) return c->gemm_variant;
    return M <= 64 ? 1 : M >= 512 ? 2 : 0;
}

static int gemm(sv_ctx* c, const void* A, const void* W, float* out, int M, int N, int K, int* splits_out, bool allow_split = true) {
    ProfScope prof(c, SV_PROF_GEMM);
    if (c->model.dtype == SV_BF16) {
        if (c->packed) {
            // packed weights + packed activations: the weight-streaming kernel
            const WsPlan p = plan_ws(M, N, K, allow_split, c->gemm_tile);
            *splits_out = p.splits;
            SV_HIP(c, gemm_bf16_ws((const bf16_t*)A, (const bf16_t*)W, out, M, N, K, p.splits, p.wide, c->stream, p.row_tiles));
        } else {
            const int s = allow_split ? pick_splits(M, N, K) : 1;
            *splits_out = s;
            SV_HIP(c, gemm_bf16((const bf16_t*)A, (const bf16_t*)W, out, M, N, K, s, pick_variant(c, M), c->stream));
        }
    } else {
        *splits_out = 1;
        SV_HIP(c, gemm_f32((const float*)A, (const float*)W, out, M, N, K, c->stream));
    }
    return SV_OK;
}

// Row preparation of a pass: positions, cache slots, rotary table, token ids of the B * n new rows.
static int prepare_rows(sv_ctx* c, int B, int n, int k, const int32_t* last_tokens, const int32_t* drafts) {
    const sv_model& m = c->model;
    const Layout& L = c->lay;
    RowPrep rp;
    rp.batch_seq = c->at<int32_t>(L.batch_seq); rp.seq_len = c->at<int32_t>(L.seq_len);
    rp.last_tokens = last_tokens; rp.drafts = drafts;
    rp.row_tok = c->at<int32_t>(L.row_tok); rp.row_pos = c->at<int32_t>(L.row_pos); rp.row_slot = c->at<int32_t>(L.row_slot);
    rp.rope = c->at<float>(L.rope);
    rp.B = B; rp.n = n; rp.k = k; rp.head_dim = m.head_dim; rp.vocab = m.vocab; rp.rope_theta = m.rope_theta;
    rp.tok_matrix = c->tok_matrix; rp.tok_len = c->tok_len; rp.tok_ld = c->tok_ld; rp.tok_col0 = c->tok_col0;
    SV_HIP(c, prep_rows(rp, c->stream));
    return SV_OK;
}

// Residual add of what the previous projection left behind, then RMSNorm into the packed operand buffer.
// pending > 0: that many split-K planes in `part`; 0: nothing to add; -1: the expert outputs of a
// mixture-of-experts layer, still to be combined with the routing weights and added.
static int add_norm(sv_ctx* c, int T, int pending, const void* gain) {
    const sv_model& m = c->model;
    const Layout& L = c->lay;
    float* h = c->at<float>(L.h);
    void* a_norm = c->at<void>(L.a_norm);
    if (pending < 0)
        SV_HIP(c, add_rmsnorm_experts(h, c->at<float>(L.moe_y), c->at<int32_t>(L.moe_inv), c->at<float>(L.moe_w), m.top_k, gain, a_norm,
                                      T, m.d_model, m.rms_eps, c->packed, c->stream));
    else
        SV_HIP(c, add_rmsnorm(h, c->at<float>(L.part), pending, gain, a_norm, m.dtype, T, m.d_model, m.rms_eps, c->packed, c->stream));
    return SV_OK;
}

// Row pitch of the split-KV partials for a pass of B requests with n rows each.  The buffers are sized for
// max_batch requests with the rows of a verification step; a pass of fewer requests with more rows each (a prompt
// prefilled in long chunks) may spread over the same memory with a larger pitch, up to the 256 stacked rows the MFMA
// attention takes.
static int attn_partial_pitch(const sv_ctx* c, int B, int n, int max_chunks) {
    const Layout& L = c->lay;
    const int G = c->model.n_q_heads / c->model.n_kv_heads;
    const int need = attn_rows_pad(n, G);                 // padded stacked rows per kv head; 0: more than the kernels take
    if (need == 0 || need <= L.rows_pad) return L.rows_pad;
    const long long room = (long long)c->rt.max_batch * L.max_chunks * L.rows_pad / ((long long)B * std::max(1, max_chunks));
    return room >= need ? need : L.rows_pad;
}

// Rows per request and pass when B prompts are prefilled together: what the workspace holds rows for, at most the 256
// stacked rows per kv head of the MFMA attention, and no more than the split-KV partials have room for.
static int prefill_width(const sv_ctx* c, int B) {
    const Layout& L = c->lay;
    const int G = c->model.n_q_heads / c->model.n_kv_heads;
    int width = std::max(1, std::min(L.T / B, 256 / G));
    while (width > 1 && attn_rows_pad(width, G) > L.rows_pad &&
           (long long)c->rt.max_batch * L.rows_pad / B < attn_rows_pad(width, G))
        --width;                                          // (the pitch is checked against the chunk count of the pass again)
    return width;
}

// One decoder layer over the prepared rows.  On entry the residual stream h lacks `pending` (see add_norm) of
// the previous layer; on exit it lacks this layer's feed-forward output, described by the new `pending`.
static int layer_rows(sv_ctx* c, int l, int B, int n, int k, int max_len_ub, int& pending) {
    const sv_model& m = c->model;
    const Layout& L = c->lay;
    const int T = B * n, d = m.d_model, qw = m.n_q_heads * m.head_dim, qkvw = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    hipStream_t st = c->stream;
    float* h = c->at<float>(L.h);
    float* part = c->at<float>(L.part);
    void* a_norm = c->at<void>(L.a_norm);

    SV_TRY(add_norm(c, T, pending, c->ln1[l]));
    pending = 0;
    int s_qkv = 1;
    SV_TRY(gemm(c, a_norm, c->wqkv[l], part, T, qkvw, d, &s_qkv));
    RopeAppend ra;
    ra.qkv_part = part; ra.S = s_qkv; ra.rope = c->at<float>(L.rope); ra.row_slot = c->at<int32_t>(L.row_slot);
    ra.batch_seq = c->at<int32_t>(L.batch_seq);
    ra.page_table = c->at<int32_t>(L.page_table); ra.max_pages_per_seq = c->rt.max_pages_per_seq;
    ra.q_out = c->at<void>(L.q); ra.pool = c->rt.kv_pool; ra.geom = c->geom; ra.layer = l;
    ra.T = T; ra.n = n; ra.Hq = m.n_q_heads; ra.Hkv = m.n_kv_heads; ra.hd = m.head_dim; ra.dtype = m.dtype;
    SV_HIP(c, rope_append(ra, st));

    AttnArgs aa;
    aa.q = ra.q_out; aa.pool = c->rt.kv_pool; aa.geom = c->geom; aa.layer = l;
    aa.page_table = ra.page_table; aa.max_pages_per_seq = c->rt.max_pages_per_seq;
    aa.batch_seq = ra.batch_seq; aa.seq_len = c->at<int32_t>(L.seq_len); aa.out = c->at<void>(L.attn);
    aa.part_o = c->at<float>(L.part_o); aa.part_ml = c->at<float>(L.part_ml); aa.rows_pad = L.rows_pad; aa.row_groups = 1;
    aa.B = B; aa.n = n; aa.k = k; aa.Hq = m.n_q_heads; aa.Hkv = m.n_kv_heads; aa.hd = m.head_dim; aa.dtype = m.dtype;
    aa.chunk_keys = c->attn_chunk; aa.work = c->at<int32_t>(L.work); aa.n_work = c->n_work; aa.req_chunk = c->at<int32_t>(L.req_chunk);
    aa.out_packed = c->packed;
    aa.force_generic = c->attn_generic; aa.min_row_tiles = c->attn_min_rt; aa.max_row_tiles = c->attn_max_rt;
    aa.max_chunks = std::min(L.max_chunks, (max_len_ub + n + c->attn_chunk - 1) / c->attn_chunk);
    aa.n_work_dev = nullptr; aa.grid_items = 0;
    if (c->graph_launch_shape) {      // nothing in the launch may depend on the lengths
        aa.max_chunks = L.max_chunks;
        aa.n_work_dev = c->at<int32_t>(L.req_chunk) + 2 * c->rt.max_batch;
        aa.grid_items = B * L.max_chunks;
    }
    aa.rows_pad = attn_partial_pitch(c, B, n, aa.max_chunks);
    {
        ProfScope prof(c, SV_PROF_ATTENTION);
        SV_HIP(c, attention(aa, st));
    }

    int s_o = 1;
    SV_TRY(gemm(c, aa.out, c->wo[l], part, T, d, qw, &s_o));
    SV_HIP(c, add_rmsnorm(h, part, s_o, c->ln2[l], a_norm, m.dtype, T, d, m.rms_eps, c->packed, st));
    if (m.n_experts > 0) {
        MoeArgs ma;
        ma.a = (const bf16_t*)a_norm; ma.w_router = (const bf16_t*)c->wrouter[l];
        ma.w_gate_up = (const bf16_t*)c->wgu[l]; ma.w_down = (const bf16_t*)c->wdown[l];
        ma.top_ids = c->at<int32_t>(L.moe_ids); ma.top_w = c->at<float>(L.moe_w); ma.router_logits = c->at<float>(L.moe_logits);
        ma.cnt = c->at<int32_t>(L.moe_cnt); ma.tile_off = c->at<int32_t>(L.moe_off);
        ma.perm = c->at<int32_t>(L.moe_perm); ma.inv = c->at<int32_t>(L.moe_inv);
        ma.act = c->at<bf16_t>(L.moe_act); ma.y = c->at<float>(L.moe_y); ma.out = nullptr;   // combined by the next norm
        ma.T = T; ma.d = d; ma.E = m.n_experts; ma.top_k = m.top_k; ma.F = m.d_expert;
        ProfScope prof(c, SV_PROF_MOE);
        SV_HIP(c, moe_ffn(ma, st));
        pending = -1;
        return SV_OK;
    }
    if (c->packed && m.d_ff % 64 == 0) {
        // gate/up projection with SwiGLU in its epilogue: the [T, 2F] fp32 intermediate never exists
        ProfScope prof(c, SV_PROF_GEMM);
        SV_HIP(c, gemm_bf16_ws_glu((const bf16_t*)a_norm, (const bf16_t*)c->wgu[l], c->at<bf16_t>(L.act), T, m.d_ff, d, st, c->gemm_tile));
    } else {
        int s_gu = 1;
        SV_TRY(gemm(c, a_norm, c->wgu[l], part, T, 2 * m.d_ff, d, &s_gu));
        SV_HIP(c, swiglu(part, s_gu, c->at<void>(L.act), m.dtype, T, m.d_ff, c->packed, st));
    }
    SV_TRY(gemm(c, c->at<void>(L.act), c->wdown[l], part, T, d, m.d_ff, &pending));
    return SV_OK;
}

// Rows are already described by batch_seq / last_tokens / drafts.  Leaves logits in the workspace.
static int forward_rows(sv_ctx* c, int B, int n, int k, const int32_t* last_tokens, const int32_t* drafts, int max_len_ub) {
    const sv_model& m = c->model;
    const Layout& L = c->lay;
    const int T = B * n;
    SV_TRY(prepare_rows(c, B, n, k, last_tokens, drafts));
    SV_HIP(c, embed_rows(c->embed, m.dtype, c->at<int32_t>(L.row_tok), c->at<float>(L.h), T, m.d_model, c->stream));
    int pending = 0;
    for (int l = 0; l < m.n_layers; ++l) SV_TRY(layer_rows(c, l, B, n, k, max_len_ub, pending));
    SV_TRY(add_norm(c, T, pending, c->final_norm));
    int one = 1;
    SV_TRY(gemm(c, c->at<void>(L.a_norm), c->lm_head, c->at<float>(L.logits), T, m.vocab, m.d_model, &one, false));
    return SV_OK;
}

extern "C" int verify_prefill(sv_ctx* c, int32_t id, const int32_t* tokens, int32_t n, float* last_logits) {
    if (!c || !tokens) return SV_EINVAL;
    if (n <= 0) return c->fail(SV_EINVAL, "prefill of %d tokens", n);
    // a batch of one prompt: chunks of as many rows as the kernels take for a single request
    return verify_prefill_batch(c, &id, 1, tokens, n, &n, last_logits);
}

// Prompts of several sequences at once.  Pass p covers tokens p*c .. p*c+c-1 of every prompt that is that long
// (the prompts come longest first, so those are the first B_act of them): B_act * c rows through the same kernels as
// a verification step -- a chunk is x0 plus one chain of c-1 "drafts", causal visibility, every row kept -- with
// c the rows per request the workspace was sized for (1 + max_chains * max_k; at most 256 / G so that the rows of
// a kv head fit the attention kernel's tiles).  Rows past the end of a shorter prompt are padding: they sit
// behind the real rows, which therefore never see them, their cache entries lie beyond the new length, and
// the length advances by the real count.
extern "C" int verify_prefill_batch(sv_ctx* c, const int32_t* seq_ids, int32_t B, const int32_t* tokens, int32_t ld,
                                    const int32_t* n, float* last_logits) {
    if (!c || !seq_ids || !tokens || !n) return SV_EINVAL;
    if (B <= 0 || B > c->rt.max_batch || ld <= 0) return c->fail(SV_EINVAL, "prefill of %d prompts (limit %d), row pitch %d", B, c->rt.max_batch, ld);
    const int width_max = prefill_width(c, B);
    for (int b = 0; b < B; ++b) {
        if (n[b] <= 0 || n[b] > ld) return c->fail(SV_EINVAL, "prompt %d has %d tokens (row pitch %d)", b, n[b], ld);
        if (b && n[b] > n[b - 1]) return c->fail(SV_EINVAL, "prompts must come longest first (prompt %d: %d after %d)", b, n[b], n[b - 1]);
        const int id = seq_ids[b];
        if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
        if (pages_for(c, c->seqs[id].len_ub + n[b] + width_max) > c->rt.max_pages_per_seq)     // the last pass may carry padding rows
            return c->fail(SV_ENOPAGES, "sequence %d would exceed max_pages_per_seq", id);
    }
    int32_t* len_dev = c->at<int32_t>(c->lay.chain_acc);          // free outside a verification step
    {   // the lengths travel through a slot of the pinned staging ring, like a batch's ids
        const int slot = c->ring_pos;
        if (c->staged_valid[slot]) SV_HIP(c, hipEventSynchronize(c->staged[slot]));
        for (int b = 0; b < B; ++b) c->staging[slot][b] = n[b];
        SV_HIP(c, hipMemcpyAsync(len_dev, c->staging[slot], sizeof(int32_t) * B, hipMemcpyHostToDevice, c->stream));
        SV_HIP(c, hipEventRecord(c->staged[slot], c->stream));
        c->staged_valid[slot] = true;
        c->ring_pos = (slot + 1) % kRing;
    }
    for (int col0 = 0; col0 < n[0]; col0 += width_max) {
        int B_act = 0;
        while (B_act < B && n[B_act] > col0) ++B_act;
        const int width = std::min(width_max, n[0] - col0);
        SV_TRY(stage_batch(c, seq_ids, B_act, width));
        int max_ub = 0;
        for (int b = 0; b < B_act; ++b) max_ub = std::max(max_ub, c->seqs[seq_ids[b]].len_ub);
        c->tok_matrix = tokens; c->tok_len = len_dev; c->tok_ld = ld; c->tok_col0 = col0;
        const int rc = forward_rows(c, B_act, width, width - 1, nullptr, nullptr, max_ub);
        c->tok_matrix = nullptr; c->tok_len = nullptr;
        if (rc != SV_OK) return rc;
        SV_HIP(c, add_len_ragged(c->at<int32_t>(c->lay.seq_len), c->at<int32_t>(c->lay.batch_seq), B_act, len_dev, col0, width, c->stream));
        for (int b = 0; b < B_act; ++b) {
            const int real = std::min(width, n[b] - col0);
            c->seqs[seq_ids[b]].len_ub += real;
            if (last_logits && n[b] <= col0 + width)              // this pass holds the prompt's last token
                SV_HIP(c, hipMemcpyAsync(last_logits + (size_t)b * c->model.vocab,
                                         c->at<float>(c->lay.logits) + ((size_t)b * width + real - 1) * c->model.vocab,
                                         sizeof(float) * c->model.vocab, hipMemcpyDeviceToDevice, c->stream));
        }
    }
    return SV_OK;
}

// Everything verify_step enqueues after the batch is staged: forward pass, accept/reject + draw, chain choice,
// rollback, optional copy of the logits.
static int step_device_work(sv_ctx* c, const sv_batch* bt, const int32_t* drafts, const float* draft_probs,
                            const float* uniforms, const sv_out* out, int max_ub) {
    const int B = bt->B, k = bt->k, N = bt->N, n = 1 + N * k;
    SV_TRY(forward_rows(c, B, n, k, bt->last_tokens, drafts, max_ub));

    const Layout& L = c->lay;
    SampleArgs sa;
    sa.logits = c->at<float>(L.logits); sa.drafts = drafts; sa.draft_probs = draft_probs; sa.uniforms = uniforms;
    sa.draft_lens = bt->draft_lens; sa.row_stat = c->at<float>(L.row_stat);
    sa.chain_acc = c->at<int32_t>(L.chain_acc); sa.chain_tok = c->at<int32_t>(L.chain_tok); sa.chain_row = c->at<int32_t>(L.chain_row); sa.draw_part = c->at<float>(L.draw_part);
    sa.accepted_len = out->accepted_len; sa.out_tokens = out->out_tokens; sa.best_chain = out->best_chain;
    sa.B = B; sa.N = N; sa.k = k; sa.V = c->model.vocab; sa.verify_mode = c->rt.verify_mode; sa.sample_mode = c->rt.sample_mode;
    sa.temperature = c->rt.temperature;
    {
        ProfScope prof(c, SV_PROF_SAMPLER);
        SV_HIP(c, sample_verify(sa, c->stream));
    }

    RollbackArgs rb;
    rb.pool = c->rt.kv_pool; rb.geom = c->geom; rb.n_layers = c->model.n_layers; rb.dtype = c->model.dtype;
    rb.page_table = c->at<int32_t>(L.page_table); rb.max_pages_per_seq = c->rt.max_pages_per_seq;
    rb.batch_seq = c->at<int32_t>(L.batch_seq); rb.seq_len = c->at<int32_t>(L.seq_len);
    rb.accepted_len = out->accepted_len; rb.best_chain = out->best_chain; rb.B = B; rb.N = N; rb.k = k;
    {
        ProfScope prof(c, SV_PROF_ROLLBACK);
        SV_HIP(c, rollback(rb, c->stream));
    }
    if (out->logits)
        SV_HIP(c, hipMemcpyAsync(out->logits, sa.logits, sizeof(float) * (size_t)B * n * c->model.vocab,
                                 hipMemcpyDeviceToDevice, c->stream));
    return SV_OK;
}

static void drop_graphs(sv_ctx* c) {
    bool launched = false;
    for (auto& g : c->graphs) launched |= g.exec != nullptr;
    if (launched) (void)hipStreamSynchronize(c->stream);  // an executable graph may still be replaying on the stream
    for (auto& g : c->graphs)
        if (g.exec) (void)hipGraphExecDestroy(g.exec);
    c->graphs.clear();
}

// Graph replay of the step's device work.  A step's launches depend on the batch shape and on the caller's
// buffers only (the lengths reach the kernels through device memory; the attention grid is sized for the most
// work items the shape can have), so one captured graph serves every step with the same shape and buffers.
// The first step of a kind runs as plain launches (one-off set-up calls are not capturable), the second is
// captured, later ones replay.  Returns 1 if the work was enqueued through a graph, 0 if the caller should
// enqueue it itself, < 0 on error.
static int step_through_graph(sv_ctx* c, const sv_batch* bt, const int32_t* drafts, const float* draft_probs,
                              const float* uniforms, const sv_out* out, int max_ub) {
    if (!c->use_graph || c->stream == nullptr || c->prof_mask != 0) return 0;
    const void* ptr[9] = {bt->last_tokens, drafts, draft_probs, uniforms, bt->draft_lens,
                          out->accepted_len, out->out_tokens, out->best_chain, out->logits};
    sv_ctx::GraphEntry* e = nullptr;
    for (auto& g : c->graphs)
        if (g.B == bt->B && g.k == bt->k && g.N == bt->N && memcmp(g.ptr, ptr, sizeof(ptr)) == 0) e = &g;
    if (!e) {
        if (c->graphs.size() >= 8) {                       // forget the least recently used
            size_t old = 0;
            for (size_t i = 1; i < c->graphs.size(); ++i)
                if (c->graphs[i].used < c->graphs[old].used) old = i;
            if (c->graphs[old].exec) {
                (void)hipStreamSynchronize(c->stream);     // it may still be replaying
                (void)hipGraphExecDestroy(c->graphs[old].exec);
            }
            c->graphs.erase(c->graphs.begin() + old);
        }
        sv_ctx::GraphEntry g;
        g.B = bt->B; g.k = bt->k; g.N = bt->N;
        memcpy(g.ptr, ptr, sizeof(ptr));
        g.exec = nullptr;
        g.used = ++c->graph_clock;
        c->graphs.push_back(g);
        return 0;                                           // first step of this kind: plain launches
    }
    e->used = ++c->graph_clock;
    if (!e->exec) {
        hipGraph_t graph = nullptr;
        SV_HIP(c, hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal));
        c->graph_launch_shape = true;
        const int rc = step_device_work(c, bt, drafts, draft_probs, uniforms, out, max_ub);
        c->graph_launch_shape = false;
        const hipError_t ec = hipStreamEndCapture(c->stream, &graph);
        if (rc != SV_OK || ec != hipSuccess || !graph) {
            if (graph) (void)hipGraphDestroy(graph);
            return rc != SV_OK ? rc : c->fail(SV_EHIP, "stream capture failed: %s", hipGetErrorString(ec));
        }
        const hipError_t ei = hipGraphInstantiate(&e->exec, graph, nullptr, nullptr, 0);
        (void)hipGraphDestroy(graph);
        if (ei != hipSuccess) { e->exec = nullptr; return c->fail(SV_EHIP, "graph instantiation failed: %s", hipGetErrorString(ei)); }
    }
    SV_HIP(c, hipGraphLaunch(e->exec, c->stream));
    return 1;
}

extern "C" int verify_step(sv_ctx* c, const sv_batch* bt, const int32_t* drafts, const float* draft_probs,
                           const float* uniforms, const sv_out* out) {
    if (!c || !bt || !out) return SV_EINVAL;
    const int B = bt->B, k = bt->k, N = bt->N;
    if (B <= 0 || B > c->rt.max_batch || k < 0 || k > c->rt.max_k || N <= 0 || N > c->rt.max_chains)
        return c->fail(SV_EINVAL, "batch %d / k %d / chains %d outside the limits given at init", B, k, N);
    if (!bt->seq_ids || !bt->last_tokens || (k > 0 && !drafts) || !out->accepted_len || !out->out_tokens || !out->best_chain)
        return c->fail(SV_EINVAL, "null argument");
    if (c->rt.verify_mode != SV_GREEDY && !uniforms) return c->fail(SV_EINVAL, "stochastic and match verification need uniforms");
    const int n = 1 + N * k;
    SV_TRY(stage_batch(c, bt->seq_ids, B, n));
    int max_ub = 0;
    for (int b = 0; b < B; ++b) max_ub = std::max(max_ub, c->seqs[bt->seq_ids[b]].len_ub);
    const int via_graph = step_through_graph(c, bt, drafts, draft_probs, uniforms, out, max_ub);
    if (via_graph < 0) return via_graph;
    if (via_graph == 0) SV_TRY(step_device_work(c, bt, drafts, draft_probs, uniforms, out, max_ub));
    for (int b = 0; b < B; ++b) c->seqs[bt->seq_ids[b]].len_ub += k + 1;
    return SV_OK;
}

// -------------------------------------------------- single-operation entry points ---

extern "C" int sv_op_gemm_bf16(const void* A, const void* W, float* out, int M, int N, int K, int splits, int variant,
                               void* stream) {
    if (!A || !W || !out || M <= 0 || !gemm_bf16_shape_ok(N, K, splits) || !gemm_bf16_variant_ok(variant, N)) return SV_EINVAL;
    return gemm_bf16((const bf16_t*)A, (const bf16_t*)W, out, M, N, K, splits, variant, (hipStream_t)stream) ==
                   hipSuccess ? SV_OK : SV_EHIP;
}

extern "C" int sv_op_gemm_bf16_ws(const void* Ap, const void* Wp, float* out, int M, int N, int K, int splits, int wide,
                                  int row_tiles, void* stream) {
    if (!Ap || !Wp || !out || M <= 0 || N <= 0 || K <= 0 || splits <= 0 || N % (wide ? 256 : 128) != 0 ||
        K % (64 * splits) != 0 || row_tiles < 0 || (row_tiles > 5 && row_tiles != 8) || (row_tiles == 8 && N % 256 != 0))
        return SV_EINVAL;
    return gemm_bf16_ws((const bf16_t*)Ap, (const bf16_t*)Wp, out, M, N, K, splits, wide != 0, (hipStream_t)stream, row_tiles) == hipSuccess
               ? SV_OK : SV_EHIP;
}

extern "C" int sv_op_gemm_plan(int M, int N, int K, int* splits, int* wide, int* row_tiles) {
    if (!splits || !wide || !row_tiles || M <= 0 || N <= 0 || K <= 0 || N % 128 != 0 || K % 64 != 0) return SV_EINVAL;
    const WsPlan p = plan_ws(M, N, K, true);
    *splits = p.splits; *wide = p.wide ? 1 : 0; *row_tiles = p.row_tiles;
    return SV_OK;
}

extern "C" int sv_op_pack_rows(const void* src, void* dst, int M, int K, void* stream) {
    if (!src || !dst || src == dst || M <= 0 || K <= 0 || K % 16 != 0) return SV_EINVAL;
    return pack_rows((const bf16_t*)src, (bf16_t*)dst, M, K, (hipStream_t)stream) == hipSuccess ? SV_OK : SV_EHIP;
}

extern "C" int sv_op_pack_weight(const void* src, void* dst, int N, int K, void* stream) {
    if (!src || !dst || src == dst || N <= 0 || K <= 0 || N % 128 != 0 || K % 32 != 0) return SV_EINVAL;
    return pack_weight((const bf16_t*)src, (bf16_t*)dst, N, K, (hipStream_t)stream) == hipSuccess ? SV_OK : SV_EHIP;
}

extern "C" int sv_op_sample(const float* logits, const int32_t* drafts, const float* draft_probs, const float* uniforms,
                            const int32_t* draft_lens, int B, int N, int k, int V, int verify_mode, int sample_mode,
                            float temperature, void* scratch, int32_t* accepted_len, int32_t* out_tokens,
                            int32_t* best_chain, void* stream) {
    if (!logits || (k > 0 && !drafts) || !scratch || !accepted_len || !out_tokens || !best_chain || B <= 0 || N <= 0 ||
        k < 0 || V <= 0 || !(temperature > 0.f) || verify_mode < 0 || verify_mode > 2 || (verify_mode != SV_GREEDY && !uniforms))
        return SV_EINVAL;
    const int T = B * (1 + N * k), S = B * N;
    char* p = reinterpret_cast<char*>(scratch);
    SampleArgs sa;
    sa.logits = logits; sa.drafts = drafts; sa.draft_probs = draft_probs; sa.uniforms = uniforms; sa.draft_lens = draft_lens;
    sa.row_stat = reinterpret_cast<float*>(p); p += align_up(sizeof(float) * 4 * T);
    sa.chain_acc = reinterpret_cast<int32_t*>(p); p += align_up(sizeof(int32_t) * S);
    sa.chain_tok = reinterpret_cast<int32_t*>(p); p += align_up(sizeof(int32_t) * S);
    sa.chain_row = reinterpret_cast<int32_t*>(p); p += align_up(sizeof(int32_t) * S);
    sa.draw_part = reinterpret_cast<float*>(p);
    sa.accepted_len = accepted_len; sa.out_tokens = out_tokens; sa.best_chain = best_chain;
    sa.B = B; sa.N = N; sa.k = k; sa.V = V; sa.verify_mode = verify_mode; sa.sample_mode = sample_mode; sa.temperature = temperature;
    return sample_verify(sa, (hipStream_t)stream) == hipSuccess ? SV_OK : SV_EHIP;
}

extern "C" size_t sv_op_sample_scratch_bytes(int B, int N, int k) {
    if (B <= 0 || N <= 0 || k < 0) return 0;
    return align_up(sizeof(float) * 4 * (size_t)B * (1 + N * k)) + 3 * align_up(sizeof(int32_t) * (size_t)B * N) +
           align_up(sizeof(float) * 4 * kDrawParts * (size_t)B * (1 + N * k));      // match mode draws per row
}

struct MoeScratch { size_t ids, w, cnt, off, perm, inv, act, y, logits, total; };
static MoeScratch moe_scratch(int T, int d, int E, int top_k, int F) {
    MoeScratch m;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align_up(bytes); return at; };
    const size_t tiles = (size_t)moe_max_tiles(T, E, top_k);
    m.ids = take(sizeof(int32_t) * (size_t)T * top_k);
    m.w = take(sizeof(float) * (size_t)T * top_k);
    m.cnt = take(sizeof(int32_t) * E);
    m.off = take(sizeof(int32_t) * (E + 1));
    m.perm = take(sizeof(int32_t) * 32 * tiles);
    m.inv = take(sizeof(int32_t) * (size_t)T * top_k);
    m.act = take(sizeof(bf16_t) * 32 * tiles * F);
    m.y = take(sizeof(float) * 32 * tiles * d);
    m.logits = take(sizeof(float) * 4 * (size_t)T * E);
    m.total = o;
    return m;
}

extern "C" size_t sv_op_moe_scratch_bytes(int T, int d, int E, int top_k, int F) {
    if (!moe_shape_ok(T, d, E, top_k, F)) return 0;
    return moe_scratch(T, d, E, top_k, F).total;
}

extern "C" int sv_op_moe_ffn(const void* a_packed, const void* w_router, const void* w_gate_up_packed,
                             const void* w_down_packed, int T, int d, int E, int top_k, int F, void* scratch,
                             size_t scratch_bytes, float* out, int32_t* top_ids, float* top_w, void* stream) {
    if (!a_packed || !w_router || !w_gate_up_packed || !w_down_packed || !scratch || !out) return SV_EINVAL;
    if (!moe_shape_ok(T, d, E, top_k, F)) return SV_EUNSUPPORTED;
    const MoeScratch m = moe_scratch(T, d, E, top_k, F);
    if (scratch_bytes < m.total || ((uintptr_t)scratch & 255)) return SV_EINVAL;
    char* ws = reinterpret_cast<char*>(scratch);
    MoeArgs ma;
    ma.a = (const bf16_t*)a_packed; ma.w_router = (const bf16_t*)w_router;
    ma.w_gate_up = (const bf16_t*)w_gate_up_packed; ma.w_down = (const bf16_t*)w_down_packed;
    ma.top_ids = reinterpret_cast<int32_t*>(ws + m.ids); ma.top_w = reinterpret_cast<float*>(ws + m.w);
    ma.router_logits = reinterpret_cast<float*>(ws + m.logits);
    ma.cnt = reinterpret_cast<int32_t*>(ws + m.cnt); ma.tile_off = reinterpret_cast<int32_t*>(ws + m.off);
    ma.perm = reinterpret_cast<int32_t*>(ws + m.perm); ma.inv = reinterpret_cast<int32_t*>(ws + m.inv);
    ma.act = reinterpret_cast<bf16_t*>(ws + m.act); ma.y = reinterpret_cast<float*>(ws + m.y); ma.out = out;
    ma.T = T; ma.d = d; ma.E = E; ma.top_k = top_k; ma.F = F;
    hipStream_t st = (hipStream_t)stream;
    if (moe_ffn(ma, st) != hipSuccess) return SV_EHIP;
    if (top_ids && hipMemcpyAsync(top_ids, ma.top_ids, sizeof(int32_t) * (size_t)T * top_k, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return SV_EHIP;
    if (top_w && hipMemcpyAsync(top_w, ma.top_w, sizeof(float) * (size_t)T * top_k, hipMemcpyDeviceToDevice, st) != hipSuccess)
        return SV_EHIP;
    return SV_OK;
}

extern "C" int sv_op_attention(sv_ctx* c, const int32_t* seq_ids, int B, int n, int k, int layer, const void* q, void* out) {
    if (!c || !seq_ids || !q || !out) return SV_EINVAL;
    if (B <= 0 || B > c->rt.max_batch || n <= 0 || B * n > c->lay.T || k < 0 || layer < 0 || layer >= c->model.n_layers ||
        (k > 0 && (n - 1) % k != 0) || (k == 0 && n != 1))
        return c->fail(SV_EINVAL, "attention of %d x %d rows (k=%d, layer %d) outside the limits given at init", B, n, k, layer);
    SV_TRY(stage_batch(c, seq_ids, B, n));
    int max_ub = 0;
    for (int b = 0; b < B; ++b) max_ub = std::max(max_ub, c->seqs[seq_ids[b]].len_ub);
    const sv_model& m = c->model;
    AttnArgs aa;
    aa.q = q; aa.pool = c->rt.kv_pool; aa.geom = c->geom; aa.layer = layer;
    aa.page_table = c->at<int32_t>(c->lay.page_table); aa.max_pages_per_seq = c->rt.max_pages_per_seq;
    aa.batch_seq = c->at<int32_t>(c->lay.batch_seq); aa.seq_len = c->at<int32_t>(c->lay.seq_len); aa.out = out;
    aa.part_o = c->at<float>(c->lay.part_o); aa.part_ml = c->at<float>(c->lay.part_ml); aa.rows_pad = c->lay.rows_pad; aa.row_groups = 1;
    aa.B = B; aa.n = n; aa.k = k; aa.Hq = m.n_q_heads; aa.Hkv = m.n_kv_heads; aa.hd = m.head_dim; aa.dtype = m.dtype;
    aa.chunk_keys = c->attn_chunk; aa.work = c->at<int32_t>(c->lay.work); aa.n_work = c->n_work; aa.req_chunk = c->at<int32_t>(c->lay.req_chunk);
    aa.out_packed = false;
    aa.force_generic = c->attn_generic; aa.min_row_tiles = c->attn_min_rt; aa.max_row_tiles = c->attn_max_rt;
    aa.max_chunks = std::min(c->lay.max_chunks, (max_ub + n + c->attn_chunk - 1) / c->attn_chunk);
    aa.n_work_dev = nullptr; aa.grid_items = 0;
    aa.rows_pad = attn_partial_pitch(c, B, n, aa.max_chunks);
    SV_HIP(c, attention(aa, c->stream));
    return SV_OK;
}

extern "C" int sv_op_layer(sv_ctx* c, const int32_t* seq_ids, int B, int n, int k, int layer, const float* h_in,
                           float* h_out, int32_t* top_ids, float* top_w) {
    if (!c || !seq_ids || !h_in || !h_out) return SV_EINVAL;
    if (B <= 0 || B > c->rt.max_batch || n <= 0 || B * n > c->lay.T || k < 0 || layer < 0 || layer >= c->model.n_layers ||
        (k > 0 && (n - 1) % k != 0) || (k == 0 && n != 1))
        return c->fail(SV_EINVAL, "layer %d over %d x %d rows (k=%d) outside the limits given at init", layer, B, n, k);
    SV_TRY(stage_batch(c, seq_ids, B, n));
    int max_ub = 0;
    for (int b = 0; b < B; ++b) max_ub = std::max(max_ub, c->seqs[seq_ids[b]].len_ub);
    const sv_model& m = c->model;
    const Layout& L = c->lay;
    const int T = B * n;
    const size_t bytes = sizeof(float) * (size_t)T * m.d_model;
    SV_TRY(prepare_rows(c, B, n, k, nullptr, nullptr));
    SV_HIP(c, hipMemcpyAsync(c->at<float>(L.h), h_in, bytes, hipMemcpyDeviceToDevice, c->stream));
    int pending = 0;
    SV_TRY(layer_rows(c, layer, B, n, k, max_ub, pending));
    // the feed-forward output is still pending: the residual add that the next layer's (or the final) norm would do
    SV_TRY(add_norm(c, T, pending, c->final_norm));
    SV_HIP(c, hipMemcpyAsync(h_out, c->at<float>(L.h), bytes, hipMemcpyDeviceToDevice, c->stream));
    if (m.n_experts > 0) {
        if (top_ids) SV_HIP(c, hipMemcpyAsync(top_ids, c->at<int32_t>(L.moe_ids), sizeof(int32_t) * (size_t)T * m.top_k, hipMemcpyDeviceToDevice, c->stream));
        if (top_w) SV_HIP(c, hipMemcpyAsync(top_w, c->at<float>(L.moe_w), sizeof(float) * (size_t)T * m.top_k, hipMemcpyDeviceToDevice, c->stream));
    }
    return SV_OK;
}

extern "C" int sv_op_rollback(sv_ctx* c, const int32_t* seq_ids, int B, int N, int k, const int32_t* accepted_len,
                              const int32_t* best_chain, int commit) {
    if (!c || !seq_ids || !accepted_len || !best_chain) return SV_EINVAL;
    if (B <= 0 || B > c->rt.max_batch || k < 0 || k > c->rt.max_k || N <= 0 || N > c->rt.max_chains)
        return c->fail(SV_EINVAL, "batch %d / k %d / chains %d outside the limits given at init", B, k, N);
    SV_TRY(stage_batch(c, seq_ids, B, 1 + N * k));       // the slots of a pass: L .. L + N*k
    RollbackArgs rb;
    rb.pool = c->rt.kv_pool; rb.geom = c->geom; rb.n_layers = c->model.n_layers; rb.dtype = c->model.dtype;
    rb.page_table = c->at<int32_t>(c->lay.page_table); rb.max_pages_per_seq = c->rt.max_pages_per_seq;
    rb.batch_seq = c->at<int32_t>(c->lay.batch_seq); rb.seq_len = c->at<int32_t>(c->lay.seq_len);
    rb.accepted_len = accepted_len; rb.best_chain = best_chain; rb.B = B; rb.N = N; rb.k = k;
    {
        ProfScope prof(c, SV_PROF_ROLLBACK);
        SV_HIP(c, rollback(rb, c->stream, commit != 0));
    }
    if (commit)
        for (int b = 0; b < B; ++b) c->seqs[seq_ids[b]].len_ub += k + 1;
    return SV_OK;
}

extern "C" int sv_profile_enable(sv_ctx* c, unsigned kind_mask) {
    if (!c) return SV_EINVAL;
    c->prof_mask = kind_mask & ((1u << SV_PROF_KINDS) - 1u);
    return SV_OK;
}

extern "C" int sv_profile_read(sv_ctx* c, int kind, double* total_ms, int* launches) {
    if (!c || !total_ms || !launches || kind < 0 || kind >= SV_PROF_KINDS) return SV_EINVAL;
    SV_HIP(c, hipStreamSynchronize(c->stream));
    double tot = 0.0;
    int n = 0;
    std::vector<sv_ctx::ProfRec> keep;
    for (auto& r : c->prof_recs) {
        if (r.kind != kind) { keep.push_back(r); continue; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) { tot += ms; ++n; }
        c->prof_free.push_back(r.a);
        c->prof_free.push_back(r.b);
    }
    c->prof_recs.swap(keep);
    *total_ms = tot;
    *launches = n;
    return SV_OK;
}

extern "C" int sv_seq_set_lens(sv_ctx* c, const int32_t* seq_ids, const int32_t* lens, int n) {
    if (!c || !seq_ids || !lens || n <= 0 || n > c->rt.max_batch) return SV_EINVAL;
    for (int i = 0; i < n; ++i) {
        const int id = seq_ids[i];
        if (id < 0 || id >= c->rt.max_seqs || !c->seqs[id].live) return c->fail(SV_ENOSEQ, "sequence id %d not live", id);
        if (lens[i] < 0 || lens[i] > (int)c->seqs[id].pages.size() * c->rt.page_size)
            return c->fail(SV_EINVAL, "length %d beyond the pages sequence %d holds", lens[i], id);
    }
    const int slot = c->ring_pos;
    if (c->staged_valid[slot]) SV_HIP(c, hipEventSynchronize(c->staged[slot]));
    int32_t* st = c->staging[slot];
    for (int i = 0; i < n; ++i) { st[2 * i] = seq_ids[i]; st[2 * i + 1] = lens[i]; }
    SV_HIP(c, hipMemcpyAsync(c->at<int32_t>(c->lay.upd), st, 2 * n * sizeof(int32_t), hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(set_lens_kernel, dim3((n + 63) / 64), dim3(64), 0, c->stream, c->at<int32_t>(c->lay.seq_len),
                       c->at<int32_t>(c->lay.upd), n);
    SV_HIP(c, hipGetLastError());
    SV_HIP(c, hipEventRecord(c->staged[slot], c->stream));
    c->staged_valid[slot] = true;
    c->ring_pos = (slot + 1) % kRing;
    for (int i = 0; i < n; ++i) c->seqs[seq_ids[i]].len_ub = lens[i];
    return SV_OK;
}

extern "C" int sv_set_option(sv_ctx* c, int option, int value) {
    if (!c) return SV_EINVAL;
    drop_graphs(c);                                       // captured launches carry the options they were made with
    switch (option) {
        case SV_OPT_GEMM_VARIANT:
            if (value < -1 || value > 2)
                return c->fail(SV_EINVAL, "gemm variant %d", value);
            c->gemm_variant = value;
            return SV_OK;
        case SV_OPT_GEMM_TILE:
            if (value < -1 || value > 1) return c->fail(SV_EINVAL, "gemm tile mode %d", value);
            c->gemm_tile = value;
            return SV_OK;
        case SV_OPT_ATTN_GENERIC:
            c->attn_generic = value != 0;
            return SV_OK;
        case SV_OPT_ATTN_CHUNK_KEYS:
            if (value != 0 && (value < kChunkKeys || value % 128 != 0)) return c->fail(SV_EINVAL, "chunk of %d keys", value);
            c->attn_chunk_opt = value;
            return SV_OK;
        case SV_OPT_GRAPH:
            if (value != 0 && c->stream == nullptr) return c->fail(SV_EINVAL, "graph replay needs a stream of its own, not the null stream");
            c->use_graph = value != 0;
            drop_graphs(c);
            return SV_OK;
        case SV_OPT_ATTN_MAX_ROW_TILES:
            if (value < 1 || value > 4) return c->fail(SV_EINVAL, "row tiles %d", value);
            c->attn_max_rt = value;
            return SV_OK;
        case SV_OPT_ATTN_MIN_ROW_TILES:
            if (value < 1 || value > 4) return c->fail(SV_EINVAL, "row tiles %d", value);
            c->attn_min_rt = value;
            return SV_OK;
        default:
            return c->fail(SV_EINVAL, "unknown option %d", option);
    }
}
