// libpo host side: the C ABI of include/po.h, the arena layouts and the forward driver
// (layer loop, token-chunk loop, one HIP stream, no device<->host synchronisation inside
// a request except the final one).
#include "../../include/po.h"
#include "po_internal.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

using namespace po;

namespace {

thread_local char g_dev_err[512] = "";

#define PO_HIP(expr)                                                                           \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) {                                                                \
            snprintf(g_dev_err, sizeof(g_dev_err), "%s: %s (%s:%d)", #expr, hipGetErrorString(e_), \
                     __FILE__, __LINE__);                                                      \
            return PO_ERR_DEVICE;                                                              \
        }                                                                                      \
    } while (0)

constexpr size_t ALIGN = 256;
constexpr int MAX_CAND = 4096;
constexpr int GU_INTERLEAVE_BF16 = 32;   // rows per gate/up block in the packed bf16 weight

inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline bool is_bf16(int dtype) { return dtype == PO_BF16 || dtype == PO_BF16_FP8; }   // bf16 storage and kernels

struct LayerOff {
    size_t attn_norm, wqkv, bqkv, wo, mlp_norm, wgu, wd;
    size_t s_wqkv, s_wo, s_wgu, s_wd;     // PO_BF16_FP8: float32 scale per weight row (the matrices hold codes)
};

struct Layout {
    // weights arena
    size_t embed, final_norm, lm_head;
    std::vector<LayerOff> layers;
    size_t weights_bytes;
    // workspace arena
    size_t tokens, X, Q, K, V, Vt, Xn, H, GU, rope_cos, rope_sin, logits, xn_last, cand, cand_lp;
    size_t attn_redo;   // bf16: one word per 256-row query tile and head (see launch_attention_mfma)
    size_t profile_mark;  // the last 256 bytes: where po_profile's scan leaves its result (not part of what it scans)
    size_t sx;          // PO_BF16_FP8: float32 scale per row of the activation being multiplied
    size_t workspace_bytes;
    int64_t ldv;
    int chunk;          // effective chunk = min(mlp_chunk, max_len)
};

po_status validate_config(const po_model_config* c) {
    if (!c) return PO_ERR_INVALID_ARG;
    if (c->dtype != PO_F32 && c->dtype != PO_BF16 && c->dtype != PO_BF16_FP8) return PO_ERR_INVALID_ARG;
    if (c->qkv_bias != 0 && c->qkv_bias != 1) return PO_ERR_INVALID_ARG;
    if (c->n_layers < 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->ffn_dim <= 0 || c->vocab_size <= 0)
        return PO_ERR_INVALID_ARG;
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return PO_ERR_INVALID_ARG;
    if (c->n_q_heads % c->n_kv_heads != 0) return PO_ERR_BAD_CONFIG;
    if (c->d_model % 8 != 0 || c->ffn_dim % 8 != 0) return PO_ERR_BAD_CONFIG;
    const int hd = c->head_dim;
    if (c->dtype == PO_F32) {
        if (hd != 32 && hd != 64 && hd != 128) return PO_ERR_BAD_CONFIG;
    } else {
        const int qd = c->n_q_heads * hd, kvd = c->n_kv_heads * hd;
        if (!attention_mfma_supported(c->n_q_heads, c->n_kv_heads, hd)) return PO_ERR_BAD_CONFIG;
        if (!gemm_mfma_supported(qd + 2 * kvd, c->d_model)) return PO_ERR_BAD_CONFIG;
        if (!gemm_mfma_supported(c->d_model, qd)) return PO_ERR_BAD_CONFIG;
        if (c->ffn_dim % GU_INTERLEAVE_BF16 != 0) return PO_ERR_BAD_CONFIG;
        if (!gemm_mfma_supported(2 * c->ffn_dim, c->d_model)) return PO_ERR_BAD_CONFIG;
        if (!gemm_mfma_supported(c->d_model, c->ffn_dim)) return PO_ERR_BAD_CONFIG;
        if (c->dtype == PO_BF16_FP8) {
            if (!gemm_fp8_supported(qd + 2 * kvd, c->d_model) || !gemm_fp8_supported(c->d_model, qd) ||
                !gemm_fp8_supported(2 * c->ffn_dim, c->d_model) || !gemm_fp8_supported(c->d_model, c->ffn_dim))
                return PO_ERR_BAD_CONFIG;
            if (!quant_rows_supported(c->d_model) || !quant_rows_supported(qd) || !quant_rows_supported(c->ffn_dim))
                return PO_ERR_BAD_CONFIG;
            // the fused norm keeps a row in registers; the codes of an attention-output chunk borrow the norm buffer
            if (c->d_model > 8192 || qd > 2 * c->d_model) return PO_ERR_BAD_CONFIG;
        }
    }
    return PO_OK;
}

po_status make_layout(const po_model_config* c, int64_t max_len, int32_t mlp_chunk, Layout* L) {
    po_status st = validate_config(c);
    if (st != PO_OK) return st;
    if (max_len <= 0 || mlp_chunk <= 0) return PO_ERR_INVALID_ARG;
    if (max_len > (int64_t)1 << 24) return PO_ERR_TOO_LONG;
    // the bf16 attention addresses one layer of K (and V^T) with 32-bit byte offsets
    if (is_bf16(c->dtype) && (max_len + 64) * c->n_kv_heads * c->head_dim * 2 >= ((int64_t)1 << 32)) return PO_ERR_TOO_LONG;
    const size_t esz = c->dtype == PO_F32 ? 4 : 2;
    const bool fp8 = c->dtype == PO_BF16_FP8;
    const size_t d = c->d_model, F = c->ffn_dim, V = c->vocab_size;
    const size_t qd = (size_t)c->n_q_heads * c->head_dim, kvd = (size_t)c->n_kv_heads * c->head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L->embed = take(V * d * esz);
    L->final_norm = take(d * esz);
    L->lm_head = take(V * d * esz);
    L->layers.resize(c->n_layers);
    for (int l = 0; l < c->n_layers; ++l) {
        LayerOff& o = L->layers[l];
        const size_t wsz = fp8 ? 1 : esz;         // bytes per element of a decoder linear weight
        o.attn_norm = take(d * esz);
        o.wqkv = take((qd + 2 * kvd) * d * wsz);
        o.bqkv = c->qkv_bias ? take((qd + 2 * kvd) * esz) : 0;
        o.wo = take(d * qd * wsz);
        o.mlp_norm = take(d * esz);
        o.wgu = take(2 * F * d * wsz);
        o.wd = take(d * F * wsz);
        o.s_wqkv = fp8 ? take((qd + 2 * kvd) * 4) : 0;
        o.s_wo = fp8 ? take(d * 4) : 0;
        o.s_wgu = fp8 ? take(2 * F * 4) : 0;
        o.s_wd = fp8 ? take(d * 4) : 0;
    }
    L->weights_bytes = off;

    const size_t N = (size_t)max_len;
    const size_t C = (size_t)(mlp_chunk < max_len ? mlp_chunk : max_len);
    L->chunk = (int)C;
    L->ldv = round_up64(max_len, 64);
    off = 0;
    L->tokens = take(N * 4);
    L->X = take(N * d * esz);
    L->Q = take(N * qd * esz);
    L->K = take(N * kvd * esz);
    L->V = c->dtype == PO_F32 ? take(N * kvd * esz) : 0;   // bf16: V lives only as V^T
    L->Vt = is_bf16(c->dtype) ? take(kvd * (size_t)L->ldv * esz) : 0;
    L->Xn = take(C * d * esz);
    L->H = take(C * F * esz);
    L->GU = c->dtype == PO_F32 ? take(C * 2 * F * esz) : 0;
    L->rope_cos = take(N * (c->head_dim / 2) * 4);
    L->rope_sin = take(N * (c->head_dim / 2) * 4);
    L->logits = take(V * 4);
    L->xn_last = take(d * esz);
    L->cand = take(MAX_CAND * 4);
    L->cand_lp = take(MAX_CAND * 4);
    L->attn_redo = is_bf16(c->dtype) ? take(attention_mfma_redo_bytes(max_len, c->n_q_heads)) : 0;
    // one scale per row of a launch: at most the rows of d values the MLP chunk buffer holds
    L->sx = fp8 ? take(std::max(C, C * F / d) * 4) : 0;
    L->profile_mark = take(sizeof(unsigned long long));
    L->workspace_bytes = off;
    return PO_OK;
}

void kv_cache_geometry(const po_model_config* c, int64_t cap, int64_t* ldvc, size_t* v_off, size_t* layer_bytes) {
    const size_t esz = c->dtype == PO_F32 ? 4 : 2;
    const size_t kvd = (size_t)c->n_kv_heads * c->head_dim;
    *ldvc = round_up64(cap, 64);
    *v_off = align_up((size_t)cap * kvd * esz);
    const size_t v_bytes = is_bf16(c->dtype) ? kvd * (size_t)*ldvc * esz : (size_t)cap * kvd * esz;
    *layer_bytes = *v_off + align_up(v_bytes);
}

}  // namespace

struct po_ctx {
    po_model_config cfg;
    int64_t max_len;
    int32_t mlp_chunk;
    Layout lay;
    unsigned char* w;      // weights arena (device)
    unsigned char* ws;     // workspace arena (device)
    hipStream_t stream;
    std::vector<uint32_t> loaded;     // per layer bitmask of tensor kinds; index n_layers = globals
    hipEvent_t ev_start, ev_stop;
    bool phase_timing;
    bool split_few_rows;              // requests of few rows: split reductions for occupancy (not bit-identical)
    bool store_round;                 // float32 contexts: tensors kept between operators are rounded to bf16 values
    bool lazy_last_layer;             // last layer: queries, attention rows and MLP only where the last token needs them
    // prefix K/V cache (caller-provided device memory): per layer K [cap, kvd], then V^T [kvd, ldvc]
    // (bf16) or V [cap, kvd] (fp32); see kv_slots
    unsigned char* kvc;
    int64_t kv_cap, kv_ldv;
    size_t kv_layer_bytes, kv_v_off;
    // the cache is kv_slots.size() slots of n_layers * kv_layer_bytes each; a slot remembers the token ids whose
    // K/V it holds and when it was last used (replacement: least recently used)
    struct KvSlot {
        std::vector<int32_t> tokens;
        uint64_t last_use;
    };
    std::vector<KvSlot> kv_slots;
    uint64_t kv_tick;
    int kv_src, kv_dst;               // slots the running request reads its prefix from / stores its prefix to
    std::vector<hipEvent_t> ev_pool;  // pairs
    std::vector<int> ev_kind;         // per pair: po_kernel_class
    size_t ev_used;
    po_stats stats;
};

namespace {

uint32_t required_layer_mask(const po_model_config& c) {
    uint32_t m = (1u << PO_T_ATTN_NORM) | (1u << PO_T_WQ) | (1u << PO_T_WK) | (1u << PO_T_WV) | (1u << PO_T_WO) |
                 (1u << PO_T_MLP_NORM) | (1u << PO_T_WG) | (1u << PO_T_WU) | (1u << PO_T_WD);
    if (c.qkv_bias) m |= (1u << PO_T_BQ) | (1u << PO_T_BK) | (1u << PO_T_BV);
    return m;
}
constexpr uint32_t GLOBAL_MASK = (1u << PO_T_EMBED) | (1u << PO_T_FINAL_NORM) | (1u << PO_T_LM_HEAD);

// RAII-less helper: records an event pair around a launch when phase timing is on
struct PhaseTimer {
    po_ctx* c;
    bool on;
    size_t idx;
    PhaseTimer(po_ctx* ctx, int kind) : c(ctx), on(ctx->phase_timing), idx(0) {
        if (!on) return;
        if (c->ev_used + 2 > c->ev_pool.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
            c->ev_pool.push_back(a);
            c->ev_pool.push_back(b);
            c->ev_kind.push_back(kind);
        }
        idx = c->ev_used;
        c->ev_kind[idx / 2] = kind;
        c->ev_used += 2;
        (void)hipEventRecord(c->ev_pool[idx], c->stream);
    }
    ~PhaseTimer() {
        if (on) (void)hipEventRecord(c->ev_pool[idx + 1], c->stream);
    }
};

// Rows per launch of a chunk loop.  The MFMA GEMM works in tiles of 256 (or 128) rows x 256 columns, one per CU at a
// time, so a launch costs whole rounds of tiles over the 256 CUs (gemm_mfma_launch_cost): among max_rows and the
// multiples of 256 rows below it this picks the one with the least such cost per row, summed over the GEMMs of the loop (ties:
// the larger).  Results do not depend on the choice (row results are independent of the other rows of a launch);
// only the buffers' capacity (max_rows) binds it.
struct GemmCols {
    int64_t n_cols, k;
};
int64_t pick_chunk_rows(int64_t max_rows, std::initializer_list<GemmCols> gemms) {
    if (max_rows < 512) return max_rows;
    auto cost_per_row = [&](int64_t rows) {
        double cost = 0;
        for (const GemmCols& g : gemms) cost += gemm_mfma_launch_cost(rows, (int)g.n_cols) * (double)g.k;
        return cost / (double)rows;
    };
    int64_t best = max_rows;
    double best_cost = cost_per_row(max_rows);
    for (int64_t m = max_rows / 256; m >= 1; --m) {
        const double cost = cost_per_row(m * 256);
        if (cost < best_cost * (1 - 1e-9)) { best_cost = cost; best = m * 256; }
    }
    return best;
}

// One request inside the token buffer of a run: rows [start, start + len) of X / Q / K / V^T.
struct Seg {
    int64_t start, len;
};
constexpr int64_t SEG_ALIGN = 64;   // packed requests start on a key-tile boundary (16-byte aligned V^T columns)

// One pass of the whole path over a token buffer that holds one request (segs = {{0, len}}) or several
// requests packed one after the other; tokens already validated.  `tokens` holds `total` ids (packed:
// gaps between requests filled with id 0; those rows are computed and never read).  The position-wise
// operators run over all rows at once, attention runs per request, and each request's last row gets the
// final norm, the LM head and the candidate log-probs; out_logits / out_lp receive one row per request.
// Row results of the position-wise kernels do not depend on the other rows in a launch, so every request's
// output is bit-identical to running it alone.
// p_reuse / p_store (single request only): positions [0, p_reuse) are not computed, their K/V of every
// layer come from the prefix cache; afterwards the cache holds the K/V of positions [0, p_store).
po_status run_rows(po_ctx* c, const int32_t* tokens, int64_t total, const std::vector<Seg>& segs,
                   const int32_t* cand, int32_t n_cand, float* out_logits, float* out_lp, int64_t p_reuse = 0,
                   int64_t p_store = 0) {
    const po_model_config& m = c->cfg;
    const Layout& L = c->lay;
    const bool fp8 = m.dtype == PO_BF16_FP8;            // bf16 path with FP8-dynamic linear layers
    const int dt = fp8 ? (int)PO_BF16 : m.dtype;
    const size_t esz = dt == PO_F32 ? 4 : 2;
    const int d = m.d_model, F = m.ffn_dim, hd = m.head_dim;
    const int qd = m.n_q_heads * hd, kvd = m.n_kv_heads * hd;
    hipStream_t s = c->stream;
    unsigned char* ws = c->ws;
    float* sx = (float*)(ws + L.sx);
    int32_t* d_tok = (int32_t*)(ws + L.tokens);
    unsigned char* X = ws + L.X;
    unsigned char* Q = ws + L.Q;
    unsigned char* K = ws + L.K;
    unsigned char* V = ws + L.V;
    unsigned char* Xn = ws + L.Xn;
    unsigned char* H = ws + L.H;
    const float* rc = (const float*)(ws + L.rope_cos);
    const float* rs = (const float*)(ws + L.rope_sin);
    float* d_logits = (float*)(ws + L.logits);
    // rows per launch of the position-wise loops: the chunk buffers' capacity, or less where that wastes
    // fewer CU rounds (bf16 path; e.g. d = 5120 gives 20 column tiles: 12 row tiles fill 240 CUs in one
    // round where 16 would take two)
    // (the plain bf16 path runs the O-projection outside the chunk loop, see below: it does not weigh in there)
    const bool oproj_apart = dt == PO_BF16 && !fp8 && !c->split_few_rows;
    const int C = dt != PO_BF16 ? L.chunk
                  : oproj_apart ? (int)pick_chunk_rows(L.chunk, {{2 * (int64_t)F, d}, {d, F}})
                                : (int)pick_chunk_rows(L.chunk, {{d, qd}, {2 * (int64_t)F, d}, {d, F}});
    const bool packed = segs.size() > 1;
    const int64_t n_seg = (int64_t)segs.size();
    // bf16 path: the QKV epilogue hands the attention kernels Q times the softmax scale (in log2 units), applied in
    // fp32 before Q's one rounding, so that K Q^T is the exponent's argument as it comes out of the matrix pipe
    const float q_scale = attention_q_scale(hd);
    // float32 path, second evaluation mode: every tensor kept between operators takes bf16 values (Section 4.2's
    // claim is about chunking only; this mode measures what bf16 storage alone does at shapes no CPU run reaches)
    const bool sr = dt == PO_F32 && c->store_round;

    c->ev_used = 0;
    PO_HIP(hipMemcpyAsync(d_tok, tokens, (size_t)total * 4, hipMemcpyHostToDevice, s));
    if (n_cand > 0) PO_HIP(hipMemcpyAsync(ws + L.cand, cand, (size_t)n_cand * 4, hipMemcpyHostToDevice, s));
    PO_HIP(hipEventRecord(c->ev_start, s));
    int64_t n_split_launches = 0;
    launch_embed(dt, d_tok + p_reuse, c->w + L.embed, X + (size_t)p_reuse * d * esz, total - p_reuse, d, s);
    // Packed: the sequence position of every buffer row, for the rotary embedding in the QKV epilogue.  The
    // token ids are dead once the embedding has been gathered, so the positions take over their buffer.
    std::vector<int32_t> row_pos;
    const int32_t* d_row_pos = nullptr;
    if (packed) {
        row_pos.assign((size_t)total, 0);
        for (const Seg& g : segs)
            for (int64_t i = 0; i < g.len; ++i) row_pos[(size_t)(g.start + i)] = (int32_t)i;
        PO_HIP(hipMemcpyAsync(d_tok, row_pos.data(), (size_t)total * 4, hipMemcpyHostToDevice, s));
        d_row_pos = d_tok;
    }
    // the last key tile of the attention reads V^T up to the next multiple of 64 positions
    if (dt == PO_BF16) launch_vt_pad_zero((bf16_t*)(ws + L.Vt), kvd, L.ldv, total, s);
    // the attention's give-up words start every request at zero (its second launch leaves them so)
    int* attn_redo = (int*)(ws + L.attn_redo);
    if (dt == PO_BF16) launch_fill_zero32(attn_redo, attention_mfma_redo_bytes(c->max_len, m.n_q_heads) / 4, s);

    for (int l = 0; l < m.n_layers; ++l) {
        const LayerOff& o = L.layers[l];
        const unsigned char* wqkv = c->w + o.wqkv;
        const unsigned char* bqkv = m.qkv_bias ? c->w + o.bqkv : nullptr;
        // ---- position-wise part before attention, chunk by chunk: norm -> QKV projection.
        // Its only intermediate is the normalised chunk, so it borrows the (larger, idle) MLP
        // chunk buffer and runs on up to twice as many tokens per launch: with 256-token
        // tiles that fills whole rounds of the 256 CUs (e.g. 32 x 24 tiles = 3 rounds).
        const int64_t cap_q = (int64_t)L.chunk * F / d;          // rows of d values the MLP chunk buffer holds
        int64_t Cq = L.chunk;
        if (dt == PO_BF16 && cap_q > L.chunk) Cq = pick_chunk_rows(cap_q, {{qd + 2 * (int64_t)kvd, d}});
        else if (cap_q >= 2 * (int64_t)L.chunk) Cq = 2 * (int64_t)L.chunk;
        unsigned char* Xq = (Cq > L.chunk) ? H : Xn;
        const size_t slot_bytes = c->kv_layer_bytes * (size_t)m.n_layers;
        const unsigned char* kc_l = c->kvc ? c->kvc + (size_t)c->kv_src * slot_bytes + (size_t)l * c->kv_layer_bytes : nullptr;
        unsigned char* kd_l = c->kvc ? c->kvc + (size_t)c->kv_dst * slot_bytes + (size_t)l * c->kv_layer_bytes : nullptr;
        // Few-rows mode: the split attention reads whole key tiles of the cached prefix from the cache entry
        // itself, so only the prefix's last, partial tile is copied next to the fresh keys -- unless the prefix
        // is about to be stored into ANOTHER entry, which takes it from the one-layer buffers.
        int64_t p_direct = 0;
        if (p_reuse >= 64 && dt == PO_BF16 && c->split_few_rows && !packed && (c->kv_dst == c->kv_src || p_store == 0)) {
            const int64_t q0 = (c->lazy_last_layer && l == m.n_layers - 1) ? total - 1 : p_reuse;
            if (launch_attention_mfma_split((const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)(ws + L.Vt), L.ldv, (bf16_t*)Q, total,
                                            m.n_q_heads, m.n_kv_heads, hd, q0, (float*)H, (size_t)L.chunk * F * esz, false,
                                            nullptr, nullptr, 0, 0, true, s) > 1)
                p_direct = p_reuse / 64 * 64;
        }
        if (p_reuse > p_direct) {
            // cached prefix of this layer -> rows [p_direct, p_reuse) of the one-layer K / V buffers
            if (dt == PO_BF16) {
                const size_t r0 = (size_t)p_direct, nr = (size_t)(p_reuse - p_direct);
                launch_kv_copy(K + r0 * kvd * esz, kc_l + r0 * kvd * esz, nr * kvd * esz, ws + L.Vt + r0 * esz, (size_t)L.ldv * esz,
                               kc_l + c->kv_v_off + r0 * esz, (size_t)c->kv_ldv * esz, nr * esz, kvd, s);
            } else {
                PO_HIP(hipMemcpyAsync(K, kc_l, (size_t)p_reuse * kvd * esz, hipMemcpyDeviceToDevice, s));
                PO_HIP(hipMemcpyAsync(V, kc_l + c->kv_v_off, (size_t)p_reuse * kvd * esz, hipMemcpyDeviceToDevice, s));
            }
        }
        for (int64_t c0 = p_reuse; c0 < total; c0 += Cq) {
            const int64_t rows = (total - c0 < Cq) ? total - c0 : Cq;
            unsigned char* Xn = Xq;     // (shadows the MLP-phase buffer inside this loop)
            if (fp8)
                launch_rmsnorm_quant((const bf16_t*)(X + (size_t)c0 * d * esz), (const bf16_t*)(c->w + o.attn_norm), Xn, sx,
                                     rows, d, m.rms_eps, s);
            else
                launch_rmsnorm(dt, X + (size_t)c0 * d * esz, c->w + o.attn_norm, Xn, rows, d, m.rms_eps, s);
            if (sr) launch_round_bf16_f32((float*)Xn, rows * d, s);
            PhaseTimer pt(c, PO_K_QKV);
            if (fp8) {
                const size_t h_bytes = (size_t)L.chunk * F * esz;
                const size_t h_used = (Xn == H) ? (((size_t)rows * d) + ALIGN - 1) / ALIGN * ALIGN : 0;   // codes: one byte each
                if (c->split_few_rows && h_used < h_bytes &&
                    launch_gemm_fp8_qkv_rope_splitk(Xn, d, sx, wqkv, d, (const float*)(c->w + o.s_wqkv), (const bf16_t*)bqkv,
                                                    (bf16_t*)(Q + (size_t)c0 * qd * esz), (bf16_t*)(K + (size_t)c0 * kvd * esz),
                                                    (bf16_t*)(ws + L.Vt), L.ldv, rc, rs, c0, d_row_pos, rows, qd, kvd, hd, d,
                                                    q_scale, (float*)(H + h_used), h_bytes - h_used, s) > 1)
                    ++n_split_launches;
                else
                    launch_gemm_fp8_qkv_rope(Xn, d, sx, wqkv, d, (const float*)(c->w + o.s_wqkv), (const bf16_t*)bqkv,
                                             (bf16_t*)(Q + (size_t)c0 * qd * esz), (bf16_t*)(K + (size_t)c0 * kvd * esz),
                                             (bf16_t*)(ws + L.Vt), L.ldv, rc, rs, c0, d_row_pos, rows, qd, kvd, hd, d, q_scale, s);
            } else if (dt == PO_BF16) {
                // one GEMM: RoPE applied to Q and K in the epilogue, V written as V^T (few rows: split over K,
                // partials in the chunk buffer H behind the norm output if that sits there)
                const size_t h_bytes = (size_t)L.chunk * F * esz;
                const size_t h_used = (Xn == H) ? (((size_t)rows * d * esz) + ALIGN - 1) / ALIGN * ALIGN : 0;
                if (c->split_few_rows && h_used < h_bytes &&
                    launch_gemm_qkv_rope_splitk((const bf16_t*)Xn, d, (const bf16_t*)wqkv, d, (const bf16_t*)bqkv,
                                                  (bf16_t*)(Q + (size_t)c0 * qd * esz), (bf16_t*)(K + (size_t)c0 * kvd * esz),
                                                  (bf16_t*)(ws + L.Vt), L.ldv, rc, rs, c0, d_row_pos, rows, qd, kvd, hd, d,
                                                q_scale, (float*)(H + h_used), h_bytes - h_used, true, s) > 1)
                    ++n_split_launches;
                else
                    launch_gemm_qkv_rope((const bf16_t*)Xn, d, (const bf16_t*)wqkv, d, (const bf16_t*)bqkv,
                                         (bf16_t*)(Q + (size_t)c0 * qd * esz), (bf16_t*)(K + (size_t)c0 * kvd * esz),
                                         (bf16_t*)(ws + L.Vt), L.ldv, rc, rs, c0, d_row_pos, rows, qd, kvd, hd, d, q_scale, s);
            } else {
                launch_gemm_basic(dt, Xn, d, wqkv, d, Q + (size_t)c0 * qd * esz, qd, bqkv, nullptr, 0, rows, qd, d, s);
                launch_gemm_basic(dt, Xn, d, wqkv + (size_t)qd * d * esz, d, K + (size_t)c0 * kvd * esz, kvd,
                                  bqkv ? bqkv + (size_t)qd * esz : nullptr, nullptr, 0, rows, kvd, d, s);
                launch_gemm_basic(dt, Xn, d, wqkv + (size_t)(qd + kvd) * d * esz, d, V + (size_t)c0 * kvd * esz, kvd,
                                  bqkv ? bqkv + (size_t)(qd + kvd) * esz : nullptr, nullptr, 0, rows, kvd, d, s);
                if (sr) launch_round_bf16_f32((float*)(V + (size_t)c0 * kvd * esz), rows * kvd, s);
            }
        }
        if (dt == PO_F32) {
            // every request restarts at position 0 (rows below p_reuse came rotated out of the prefix cache)
            for (const Seg& g : segs) {
                const int64_t r0 = g.start + p_reuse, nr = g.len - p_reuse;
                const size_t t0 = (size_t)p_reuse * (hd / 2);
                launch_rope(dt, Q + (size_t)r0 * qd * esz, qd, rc + t0, rs + t0, nr, m.n_q_heads, hd, s);
                launch_rope(dt, K + (size_t)r0 * kvd * esz, kvd, rc + t0, rs + t0, nr, m.n_kv_heads, hd, s);
                if (sr) {
                    launch_round_bf16_f32((float*)(Q + (size_t)r0 * qd * esz), nr * qd, s);
                    launch_round_bf16_f32((float*)(K + (size_t)r0 * kvd * esz), nr * kvd, s);
                }
            }
        }
        // Section 5.1: keep the K/V of the prefix, discard the suffix's with the layer.  Into the slot the
        // prefix came from only the new rows go; another slot receives the whole prefix (the reused rows
        // sit in the one-layer buffers by now).
        const int64_t st0 = (c->kv_dst == c->kv_src) ? p_reuse : 0;
        if (p_store > st0) {
            const size_t r0 = (size_t)st0, nr = (size_t)(p_store - st0);
            if (dt == PO_BF16) {
                launch_kv_copy(kd_l + r0 * kvd * esz, K + r0 * kvd * esz, nr * kvd * esz, kd_l + c->kv_v_off + r0 * esz,
                               (size_t)c->kv_ldv * esz, ws + L.Vt + r0 * esz, (size_t)L.ldv * esz, nr * esz, kvd, s);
            } else {
                PO_HIP(hipMemcpyAsync(kd_l + r0 * kvd * esz, K + r0 * kvd * esz, nr * kvd * esz, hipMemcpyDeviceToDevice, s));
                PO_HIP(hipMemcpyAsync(kd_l + c->kv_v_off + r0 * kvd * esz, V + r0 * kvd * esz, nr * kvd * esz,
                                      hipMemcpyDeviceToDevice, s));
            }
        }
        // Nothing reads the last layer's output except the last position (one output token, Section 1):
        // there the keys and values of every position are still needed, but attention, O-projection and
        // MLP only for the row block / the row that holds a request's last position.  Row results do not
        // depend on which other rows are computed, so the logits are bit-identical with and without this.
        const bool last_only = c->lazy_last_layer && l == m.n_layers - 1;
        // ---- attention over each request's whole sequence in one call; O overwrites Q
        for (const Seg& g : segs) {
            PhaseTimer pt(c, PO_K_ATTENTION);
            const int64_t q_row0 = last_only ? g.len - 1 : p_reuse;
            unsigned char* Qg = Q + (size_t)g.start * qd * esz;
            if (dt == PO_BF16) {
                // few query rows against many keys: key tiles split between workgroups (scratch: the chunk
                // buffer H, idle during attention)
                if (c->split_few_rows &&
                    launch_attention_mfma_split((const bf16_t*)Qg, (const bf16_t*)(K + (size_t)g.start * kvd * esz),
                                                (const bf16_t*)(ws + L.Vt) + g.start, L.ldv, (bf16_t*)Qg, g.len,
                                                m.n_q_heads, m.n_kv_heads, hd, q_row0, (float*)H,
                                                (size_t)L.chunk * F * esz, true, p_direct ? (const bf16_t*)kc_l : nullptr,
                                                p_direct ? (const bf16_t*)(kc_l + c->kv_v_off) : nullptr, c->kv_ldv, p_direct,
                                                true, s) > 1)
                    ++n_split_launches;
                else
                    launch_attention_mfma((const bf16_t*)Qg, (const bf16_t*)(K + (size_t)g.start * kvd * esz),
                                          (const bf16_t*)(ws + L.Vt) + g.start, L.ldv, (bf16_t*)Qg, g.len, m.n_q_heads,
                                          m.n_kv_heads, hd, q_row0, attn_redo, true, s);
            } else {
                launch_attention_basic(dt, Qg, K + (size_t)g.start * kvd * esz, V + (size_t)g.start * kvd * esz, Qg,
                                       g.len, m.n_q_heads, m.n_kv_heads, hd, q_row0, s);
                if (sr) launch_round_bf16_f32((float*)Qg, g.len * qd, s);     // (rows below q_row0 hold rounded Q: unchanged)
            }
        }
        // ---- position-wise part after attention, chunk by chunk, residual stream in place
        int64_t pw0 = p_reuse, pw1 = total;
        if (last_only) {
            if (!packed) {
                pw0 = total - 1;
            } else {
                // the requests' last rows, gathered into rows 0 .. n_seg-1 (whose own contents nothing reads
                // any more; request j's last row is at or beyond row j, so ascending order overwrites no source)
                for (int64_t j = 0; j < n_seg; ++j) {
                    const int64_t r = segs[j].start + segs[j].len - 1;
                    if (r == j) continue;
                    PO_HIP(hipMemcpyAsync(X + (size_t)j * d * esz, X + (size_t)r * d * esz, (size_t)d * esz,
                                          hipMemcpyDeviceToDevice, s));
                    PO_HIP(hipMemcpyAsync(Q + (size_t)j * qd * esz, Q + (size_t)r * qd * esz, (size_t)qd * esz,
                                          hipMemcpyDeviceToDevice, s));
                }
                pw0 = 0;
                pw1 = n_seg;
            }
        }
        // bf16 path: the O-projection has no intermediate of its own (it reads the attention output, which lies in the
        // Q buffer, and adds into the residual stream in place), so it needs no chunking to stay small; it runs over all
        // rows in one launch.  Same bits (a row's result does not depend on the launch it is in); what it saves is the
        // end of eight one-round launches per layer, where every tile reads its residual rows and writes its output at
        // the same moment.
        const bool oproj_whole = oproj_apart && pw1 - pw0 > C;
        if (oproj_whole) {
            PhaseTimer pt(c, PO_K_RESIDUAL);
            unsigned char* Xa = X + (size_t)pw0 * d * esz;
            launch_gemm_mfma(EPI_RESIDUAL, (const bf16_t*)(Q + (size_t)pw0 * qd * esz), qd, (const bf16_t*)(c->w + o.wo), qd,
                             (bf16_t*)Xa, d, nullptr, (const bf16_t*)Xa, d, pw1 - pw0, d, qd, s);
        }
        for (int64_t c0 = pw0; c0 < pw1; c0 += C) {
            const int64_t rows = (pw1 - c0 < C) ? pw1 - c0 : C;
            unsigned char* Xc = X + (size_t)c0 * d * esz;
            const unsigned char* Oc = Q + (size_t)c0 * qd * esz;
            if (fp8) {
                // few rows: the same split over K as on the bf16 path; scratch = H behind this chunk's rows
                const size_t h_bytes = (size_t)L.chunk * F * esz;
                const size_t h_used = (((size_t)rows * F * esz) + ALIGN - 1) / ALIGN * ALIGN;
                const bool split = c->split_few_rows && h_used < h_bytes;
                float* part = (float*)(H + h_used);
                // attention output -> codes (into the norm buffer), O-projection + residual
                launch_quant_rows((const bf16_t*)Oc, qd, Xn, qd, sx, rows, qd, 0, 0, 0, s);
                {
                    PhaseTimer pt(c, PO_K_RESIDUAL);
                    if (split && launch_gemm_fp8_splitk(EPI_RESIDUAL, Xn, qd, sx, c->w + o.wo, qd, (const float*)(c->w + o.s_wo),
                                                        (bf16_t*)Xc, d, (const bf16_t*)Xc, d, rows, d, qd, part, h_bytes - h_used, s) > 1)
                        ++n_split_launches;
                    else
                        launch_gemm_fp8(EPI_RESIDUAL, Xn, qd, sx, c->w + o.wo, qd, (const float*)(c->w + o.s_wo), (bf16_t*)Xc, d,
                                        nullptr, (const bf16_t*)Xc, d, rows, d, qd, s);
                }
                launch_rmsnorm_quant((const bf16_t*)Xc, (const bf16_t*)(c->w + o.mlp_norm), Xn, sx, rows, d, m.rms_eps, s);
                {
                    PhaseTimer pt(c, PO_K_GATE_UP);
                    if (split && launch_gemm_fp8_splitk(EPI_SILU_MUL, Xn, d, sx, c->w + o.wgu, d, (const float*)(c->w + o.s_wgu),
                                                        (bf16_t*)H, F, nullptr, 0, rows, 2 * F, d, part, h_bytes - h_used, s) > 1)
                        ++n_split_launches;
                    else
                        launch_gemm_fp8(EPI_SILU_MUL, Xn, d, sx, c->w + o.wgu, d, (const float*)(c->w + o.s_wgu), (bf16_t*)H, F,
                                        nullptr, nullptr, 0, rows, 2 * F, d, s);
                }
                // the gated intermediate -> codes in place (a row's codes take the first half of the row)
                launch_quant_rows((const bf16_t*)H, F, H, 2 * (int64_t)F, sx, rows, F, 0, 0, 0, s);
                PhaseTimer pt(c, PO_K_RESIDUAL);
                if (split && launch_gemm_fp8_splitk(EPI_RESIDUAL, H, 2 * (int64_t)F, sx, c->w + o.wd, F, (const float*)(c->w + o.s_wd),
                                                    (bf16_t*)Xc, d, (const bf16_t*)Xc, d, rows, d, F, part, h_bytes - h_used, s) > 1)
                    ++n_split_launches;
                else
                    launch_gemm_fp8(EPI_RESIDUAL, H, 2 * (int64_t)F, sx, c->w + o.wd, F, (const float*)(c->w + o.s_wd), (bf16_t*)Xc, d,
                                    nullptr, (const bf16_t*)Xc, d, rows, d, F, s);
            } else if (dt == PO_BF16) {
                // few rows (a short request, or the suffix behind a long cached prefix): the two GEMMs with
                // only d output columns split their reduction over K so that the whole chip streams the
                // weights; scratch = the part of the chunk buffer H that this chunk's rows leave free
                const size_t h_bytes = (size_t)L.chunk * F * esz;
                if (!oproj_whole) {
                    PhaseTimer pt(c, PO_K_RESIDUAL);
                    if (c->split_few_rows &&
                        launch_gemm_mfma_splitk_residual((const bf16_t*)Oc, qd, (const bf16_t*)(c->w + o.wo), qd, (bf16_t*)Xc, d,
                                                         (const bf16_t*)Xc, d, rows, d, qd, (float*)H, h_bytes, true, s) > 1)
                        ++n_split_launches;
                    else
                        launch_gemm_mfma(EPI_RESIDUAL, (const bf16_t*)Oc, qd, (const bf16_t*)(c->w + o.wo), qd,
                                         (bf16_t*)Xc, d, nullptr, (const bf16_t*)Xc, d, rows, d, qd, s);
                }
                launch_rmsnorm(dt, Xc, c->w + o.mlp_norm, Xn, rows, d, m.rms_eps, s);
                const size_t h_used = (((size_t)rows * F * esz) + ALIGN - 1) / ALIGN * ALIGN;
                {
                    PhaseTimer pt(c, PO_K_GATE_UP);
                    if (c->split_few_rows && h_used < h_bytes &&
                        launch_gemm_mfma_splitk_silu((const bf16_t*)Xn, d, (const bf16_t*)(c->w + o.wgu), d, (bf16_t*)H, F, rows,
                                                     2 * F, d, (float*)(H + h_used), h_bytes - h_used, true, s) > 1)
                        ++n_split_launches;
                    else
                        launch_gemm_mfma(EPI_SILU_MUL, (const bf16_t*)Xn, d, (const bf16_t*)(c->w + o.wgu), d, (bf16_t*)H, F,
                                         nullptr, nullptr, 0, rows, 2 * F, d, s);
                }
                PhaseTimer pt(c, PO_K_RESIDUAL);
                if (c->split_few_rows && h_used < h_bytes &&
                    launch_gemm_mfma_splitk_residual((const bf16_t*)H, F, (const bf16_t*)(c->w + o.wd), F, (bf16_t*)Xc, d,
                                                     (const bf16_t*)Xc, d, rows, d, F, (float*)(H + h_used), h_bytes - h_used,
                                                     true, s) > 1)
                    ++n_split_launches;
                else
                    launch_gemm_mfma(EPI_RESIDUAL, (const bf16_t*)H, F, (const bf16_t*)(c->w + o.wd), F, (bf16_t*)Xc, d,
                                     nullptr, (const bf16_t*)Xc, d, rows, d, F, s);
            } else {
                unsigned char* GU = ws + L.GU;
                {
                    PhaseTimer pt(c, PO_K_RESIDUAL);
                    launch_gemm_basic(dt, Oc, qd, c->w + o.wo, qd, Xc, d, nullptr, Xc, d, rows, d, qd, s);
                }
                if (sr) launch_round_bf16_f32((float*)Xc, rows * d, s);
                launch_rmsnorm(dt, Xc, c->w + o.mlp_norm, Xn, rows, d, m.rms_eps, s);
                if (sr) launch_round_bf16_f32((float*)Xn, rows * d, s);
                {
                    PhaseTimer pt(c, PO_K_GATE_UP);
                    launch_gemm_basic(dt, Xn, d, c->w + o.wgu, d, GU, 2 * F, nullptr, nullptr, 0, rows, 2 * F, d, s);
                    launch_silu_mul(dt, GU, H, rows, F, s);
                    if (sr) launch_round_bf16_f32((float*)H, rows * F, s);
                }
                PhaseTimer pt(c, PO_K_RESIDUAL);
                launch_gemm_basic(dt, H, F, c->w + o.wd, F, Xc, d, nullptr, Xc, d, rows, d, F, s);
                if (sr) launch_round_bf16_f32((float*)Xc, rows * d, s);
            }
        }
    }
    // ---- each request's last position only: final norm, LM head, candidate log-probs
    const bool gathered = packed && c->lazy_last_layer && m.n_layers > 0;
    for (int64_t j = 0; j < n_seg; ++j) {
        const int64_t r = gathered ? j : segs[j].start + segs[j].len - 1;
        launch_rmsnorm(dt, X + (size_t)r * d * esz, c->w + L.final_norm, ws + L.xn_last, 1, d, m.rms_eps, s);
        if (sr) launch_round_bf16_f32((float*)(ws + L.xn_last), d, s);
        // nobody asked for the whole distribution: only the acceptable tokens' rows of the LM head
        const bool cand_only = !out_logits && n_cand > 0;
        launch_lm_head(dt, ws + L.xn_last, c->w + L.lm_head, d_logits, m.vocab_size, d,
                       cand_only ? (const int32_t*)(ws + L.cand) : nullptr, cand_only ? n_cand : 0, s);
        if (n_cand > 0)
            launch_cand_logprobs(d_logits, (const int32_t*)(ws + L.cand), n_cand, (float*)(ws + L.cand_lp), s);
        if (j == n_seg - 1) {
            PO_HIP(hipEventRecord(c->ev_stop, s));
            PO_HIP(hipGetLastError());
        }
        // (stream-ordered: the copies finish before the next request's LM head overwrites the buffers)
        if (out_logits)
            PO_HIP(hipMemcpyAsync(out_logits + (size_t)j * m.vocab_size, d_logits, (size_t)m.vocab_size * 4,
                                  hipMemcpyDeviceToHost, s));
        if (out_lp && n_cand > 0)
            PO_HIP(hipMemcpyAsync(out_lp + (size_t)j * n_cand, ws + L.cand_lp, (size_t)n_cand * 4, hipMemcpyDeviceToHost, s));
    }
    PO_HIP(hipStreamSynchronize(s));
    float ms = 0.f;
    PO_HIP(hipEventElapsedTime(&ms, c->ev_start, c->ev_stop));
    c->stats.last_prefill_ms = ms;
    c->stats.last_len = total;
    c->stats.split_launches = n_split_launches;
    for (int kc = 0; kc < PO_K_COUNT; ++kc) { c->stats.kernel_ms[kc] = 0; c->stats.kernel_launches[kc] = 0; }
    for (size_t i = 0; i + 1 < c->ev_used; i += 2) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, c->ev_pool[i], c->ev_pool[i + 1]) == hipSuccess) {
            c->stats.kernel_ms[c->ev_kind[i / 2]] += t;
            c->stats.kernel_launches[c->ev_kind[i / 2]] += 1;
        }
    }
    return PO_OK;
}

// one request on the device
po_status run_prefill(po_ctx* c, const int32_t* tokens, int64_t len, const int32_t* cand, int32_t n_cand,
                      float* out_logits, float* out_lp, int64_t p_reuse = 0, int64_t p_store = 0) {
    return run_rows(c, tokens, len, std::vector<Seg>{{0, len}}, cand, n_cand, out_logits, out_lp, p_reuse, p_store);
}

po_status validate_request(const po_ctx* c, const int32_t* tokens, int64_t len, const int32_t* cand, int32_t n_cand) {
    if (!tokens || len <= 0 || n_cand < 0 || (n_cand > 0 && !cand) || n_cand > MAX_CAND) return PO_ERR_INVALID_ARG;
    if (len > c->max_len) return PO_ERR_TOO_LONG;
    const int32_t V = c->cfg.vocab_size;
    for (int64_t i = 0; i < len; ++i)
        if (tokens[i] < 0 || tokens[i] >= V) return PO_ERR_TOKEN_RANGE;
    for (int32_t i = 0; i < n_cand; ++i)
        if (cand[i] < 0 || cand[i] >= V) return PO_ERR_TOKEN_RANGE;
    return PO_OK;
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

po_status po_workspace_bytes(const po_model_config* cfg, int64_t max_input_len, int32_t mlp_chunk,
                             size_t* weights_bytes, size_t* workspace_bytes) {
    if (!cfg || !weights_bytes || !workspace_bytes) return PO_ERR_INVALID_ARG;
    Layout L;
    po_status st = make_layout(cfg, max_input_len, mlp_chunk, &L);
    if (st != PO_OK) return st;
    *weights_bytes = L.weights_bytes;
    *workspace_bytes = L.workspace_bytes;
    return PO_OK;
}

po_status po_max_input_len(const po_model_config* cfg, int32_t mlp_chunk, size_t hbm_budget_bytes,
                           int64_t* max_len) {
    if (!cfg || !max_len) return PO_ERR_INVALID_ARG;
    Layout L;
    po_status st = make_layout(cfg, 1, mlp_chunk, &L);
    if (st != PO_OK) return st;
    if (L.weights_bytes + L.workspace_bytes > hbm_budget_bytes) return PO_ERR_OOM;
    // longest length the kernels address (make_layout accepts every length up to it and none beyond)
    int64_t ok = 1, bad = ((int64_t)1 << 24) + 1;
    while (bad - ok > 1) {
        const int64_t mid = ok + (bad - ok) / 2;
        if (make_layout(cfg, mid, mlp_chunk, &L) == PO_OK) ok = mid; else bad = mid;
    }
    // the footprint is non-decreasing in the length: bisect on [1, ok]
    int64_t lo = 1, hi = ok;
    st = make_layout(cfg, hi, mlp_chunk, &L);
    if (st == PO_OK && L.weights_bytes + L.workspace_bytes <= hbm_budget_bytes) { *max_len = hi; return PO_OK; }
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        st = make_layout(cfg, mid, mlp_chunk, &L);
        if (st == PO_OK && L.weights_bytes + L.workspace_bytes <= hbm_budget_bytes) lo = mid; else hi = mid;
    }
    *max_len = lo;
    return PO_OK;
}

po_status po_create(const po_model_config* cfg, int64_t max_input_len, int32_t mlp_chunk, void* dev_weights,
                    size_t weights_bytes, void* dev_workspace, size_t workspace_bytes, void* hip_stream,
                    po_ctx** out) {
    if (!cfg || !out || !dev_weights || !dev_workspace) return PO_ERR_INVALID_ARG;
    if (((uintptr_t)dev_weights % ALIGN) || ((uintptr_t)dev_workspace % ALIGN)) return PO_ERR_INVALID_ARG;
    po_ctx* c = new (std::nothrow) po_ctx();
    if (!c) return PO_ERR_OOM;
    po_status st = make_layout(cfg, max_input_len, mlp_chunk, &c->lay);
    if (st != PO_OK) { delete c; return st; }
    if (weights_bytes < c->lay.weights_bytes || workspace_bytes < c->lay.workspace_bytes) {
        delete c;
        return PO_ERR_WORKSPACE_TOO_SMALL;
    }
    c->cfg = *cfg;
    c->max_len = max_input_len;
    c->mlp_chunk = mlp_chunk;
    c->w = (unsigned char*)dev_weights;
    c->ws = (unsigned char*)dev_workspace;
    c->stream = (hipStream_t)hip_stream;
    c->loaded.assign(cfg->n_layers + 1, 0u);
    c->phase_timing = false;
    c->lazy_last_layer = true;
    c->kvc = nullptr;
    c->kv_cap = c->kv_ldv = 0;
    c->kv_layer_bytes = c->kv_v_off = 0;
    c->kv_tick = 0;
    c->kv_src = c->kv_dst = 0;
    c->split_few_rows = false;
    c->store_round = false;
    c->ev_used = 0;
    memset(&c->stats, 0, sizeof(c->stats));
    c->stats.weights_bytes = c->lay.weights_bytes;
    c->stats.workspace_bytes = c->lay.workspace_bytes;
    c->ev_start = c->ev_stop = nullptr;
    hipError_t ee = hipEventCreate(&c->ev_start);
    if (ee == hipSuccess) ee = hipEventCreate(&c->ev_stop);
    if (ee != hipSuccess) {
        snprintf(g_dev_err, sizeof(g_dev_err), "hipEventCreate: %s", hipGetErrorString(ee));
        if (c->ev_start) (void)hipEventDestroy(c->ev_start);
        delete c;
        return PO_ERR_DEVICE;
    }
    // rotary table for every position up to max_input_len (angles in fp64 on the device)
    launch_rope_table((float*)(c->ws + c->lay.rope_cos), (float*)(c->ws + c->lay.rope_sin), max_input_len,
                      cfg->head_dim, cfg->rope_theta, c->stream);
    hipError_t e = hipStreamSynchronize(c->stream);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        snprintf(g_dev_err, sizeof(g_dev_err), "rope table: %s", hipGetErrorString(e));
        po_destroy(c);
        return PO_ERR_DEVICE;
    }
    *out = c;
    return PO_OK;
}

po_status po_load_tensor(po_ctx* c, int32_t kind, int32_t layer, const void* host, size_t bytes) {
    if (!c || !host || kind < 0 || kind >= PO_T_COUNT) return PO_ERR_INVALID_ARG;
    const po_model_config& m = c->cfg;
    const bool is_global = kind == PO_T_EMBED || kind == PO_T_FINAL_NORM || kind == PO_T_LM_HEAD;
    if (is_global ? layer != -1 : (layer < 0 || layer >= m.n_layers)) return PO_ERR_INVALID_ARG;
    if (!m.qkv_bias && (kind == PO_T_BQ || kind == PO_T_BK || kind == PO_T_BV)) return PO_ERR_INVALID_ARG;
    const size_t esz = m.dtype == PO_F32 ? 4 : 2;
    const size_t d = m.d_model, F = m.ffn_dim, V = m.vocab_size;
    const size_t qd = (size_t)m.n_q_heads * m.head_dim, kvd = (size_t)m.n_kv_heads * m.head_dim;
    const Layout& L = c->lay;
    size_t want = 0, off = 0;
    const LayerOff* o = is_global ? nullptr : &L.layers[layer];
    switch (kind) {
        case PO_T_EMBED: want = V * d; off = L.embed; break;
        case PO_T_FINAL_NORM: want = d; off = L.final_norm; break;
        case PO_T_LM_HEAD: want = V * d; off = L.lm_head; break;
        case PO_T_ATTN_NORM: want = d; off = o->attn_norm; break;
        case PO_T_MLP_NORM: want = d; off = o->mlp_norm; break;
        case PO_T_WQ: want = qd * d; off = o->wqkv; break;
        case PO_T_WK: want = kvd * d; off = o->wqkv + qd * d * esz; break;
        case PO_T_WV: want = kvd * d; off = o->wqkv + (qd + kvd) * d * esz; break;
        case PO_T_BQ: want = qd; off = o->bqkv; break;
        case PO_T_BK: want = kvd; off = o->bqkv + qd * esz; break;
        case PO_T_BV: want = kvd; off = o->bqkv + (qd + kvd) * esz; break;
        case PO_T_WO: want = d * qd; off = o->wo; break;
        case PO_T_WG: want = F * d; off = o->wgu; break;
        case PO_T_WU: want = F * d; off = o->wgu; break;
        case PO_T_WD: want = d * F; off = o->wd; break;
        default: return PO_ERR_INVALID_ARG;
    }
    if (bytes != want * esz) return PO_ERR_INVALID_ARG;
    const bool is_linear = kind == PO_T_WQ || kind == PO_T_WK || kind == PO_T_WV || kind == PO_T_WO || kind == PO_T_WG ||
                           kind == PO_T_WU || kind == PO_T_WD;
    if (m.dtype == PO_BF16_FP8 && is_linear) {
        // FP8-dynamic: the bf16 rows go to a temporary device buffer and are quantised per output channel
        // straight into their final (packed) row positions; the scales take the same positions
        const size_t k_in = (kind == PO_T_WO) ? qd : (kind == PO_T_WD ? F : d);
        const size_t rows = want / k_in;
        size_t row0 = 0;                       // first destination row inside the matrix
        size_t s_off = 0;
        int blk = 0;
        int64_t blk_stride = 0, dst_off = 0;
        switch (kind) {
            case PO_T_WQ: off = o->wqkv; s_off = o->s_wqkv; row0 = 0; break;
            case PO_T_WK: off = o->wqkv; s_off = o->s_wqkv; row0 = qd; break;
            case PO_T_WV: off = o->wqkv; s_off = o->s_wqkv; row0 = qd + kvd; break;
            case PO_T_WO: off = o->wo; s_off = o->s_wo; break;
            case PO_T_WD: off = o->wd; s_off = o->s_wd; break;
            default:      // gate / up: interleaved in blocks of GU_INTERLEAVE_BF16 rows
                off = o->wgu; s_off = o->s_wgu; blk = GU_INTERLEAVE_BF16; blk_stride = 2 * GU_INTERLEAVE_BF16;
                dst_off = kind == PO_T_WU ? GU_INTERLEAVE_BF16 : 0;
                break;
        }
        // Staging area: the per-request buffers at the head of the activation arena (residual stream up to the
        // chunk buffers; nothing in them outlives a request, and no request runs during a load), so loading
        // allocates nothing and the footprint stays what po_workspace_bytes reports.  It holds at least one row
        // of any of these matrices (the chunk buffer alone holds ffn_dim values); larger tensors go row block
        // by row block.
        unsigned char* stage = c->ws + L.X;
        const size_t stage_bytes = L.rope_cos - L.X;
        const size_t row_bytes = k_in * 2;
        const size_t fit = stage_bytes / row_bytes;
        if (fit == 0) return PO_ERR_WORKSPACE_TOO_SMALL;
        unsigned char* codes = c->w + off + row0 * k_in;
        float* scales = (float*)(c->w + s_off) + row0;
        hipError_t e = hipSuccess;
        for (size_t r0 = 0; r0 < rows && e == hipSuccess;) {
            size_t n;
            int blk_c = 0;
            int64_t stride_c = 0, dst_c;
            unsigned char* codes_c = codes;
            float* scales_c = scales;
            if (blk == 0) {
                n = std::min(fit, rows - r0);
                dst_c = (int64_t)r0;
            } else if (fit >= (size_t)blk && r0 % (size_t)blk == 0) {
                // whole interleave blocks: the destination base moves by whole block strides
                n = std::min(fit / (size_t)blk * (size_t)blk, rows - r0);
                codes_c = codes + (r0 / (size_t)blk) * (size_t)blk_stride * k_in;
                scales_c = scales + (r0 / (size_t)blk) * (size_t)blk_stride;
                blk_c = blk; stride_c = blk_stride; dst_c = dst_off;
            } else {
                // fewer rows than one interleave block fit: a run of rows inside one block, kept in order
                n = std::min(std::min(fit, (size_t)blk - r0 % (size_t)blk), rows - r0);
                dst_c = (int64_t)((r0 / (size_t)blk) * (size_t)blk_stride + r0 % (size_t)blk) + dst_off;
            }
            e = hipMemcpyAsync(stage, (const unsigned char*)host + r0 * row_bytes, n * row_bytes, hipMemcpyHostToDevice, c->stream);
            if (e != hipSuccess) break;
            launch_quant_rows((const bf16_t*)stage, (int64_t)k_in, codes_c, (int64_t)k_in, scales_c, (int64_t)n, (int)k_in, blk_c,
                              stride_c, dst_c, c->stream);
            // (the host buffer is pageable: the copy has left it when the call returns, and the next block's copy
            // is ordered behind this block's kernel on the stream)
            r0 += n;
        }
        if (e == hipSuccess) {
            if (kind == PO_T_WQ || kind == PO_T_WK) {
                // the rotary row order of the bf16 path, applied to the rows of codes (k_in bytes = k_in / 2
                // two-byte units) and to their scales (4 bytes = 2 units)
                const int heads = kind == PO_T_WQ ? m.n_q_heads : m.n_kv_heads;
                launch_pack_rope_rows((bf16_t*)codes, heads, m.head_dim, (int64_t)(k_in / 2), c->stream);
                launch_pack_rope_rows((bf16_t*)scales, heads, m.head_dim, 2, c->stream);
            }
            e = hipStreamSynchronize(c->stream);
            if (e == hipSuccess) e = hipGetLastError();
        }
        if (e != hipSuccess) {
            snprintf(g_dev_err, sizeof(g_dev_err), "po_load_tensor: %s", hipGetErrorString(e));
            return PO_ERR_DEVICE;
        }
    } else if (kind == PO_T_WG || kind == PO_T_WU) {
        // gate and up rows are interleaved in blocks of `il` rows so that one GEMM tile
        // holds a feature's gate and up values together (fp32 path: il = F, i.e. [Wg; Wu])
        const size_t il = is_bf16(m.dtype) ? GU_INTERLEAVE_BF16 : F;
        const size_t blk = il * d * esz;
        unsigned char* dst = c->w + off + (kind == PO_T_WU ? blk : 0);
        PO_HIP(hipMemcpy2D(dst, 2 * blk, host, blk, blk, F / il, hipMemcpyHostToDevice));
    } else {
        PO_HIP(hipMemcpy(c->w + off, host, bytes, hipMemcpyHostToDevice));
        if (is_bf16(m.dtype) && (kind == PO_T_WQ || kind == PO_T_WK || kind == PO_T_BQ || kind == PO_T_BK)) {
            // rotary partners (i, i + head_dim/2) are brought into one 64-row group so that the
            // QKV GEMM can rotate them in its epilogue (see launch_pack_rope_rows)
            const bool is_bias = kind == PO_T_BQ || kind == PO_T_BK;
            const int heads = (kind == PO_T_WQ || kind == PO_T_BQ) ? m.n_q_heads : m.n_kv_heads;
            launch_pack_rope_rows((bf16_t*)(c->w + off), heads, m.head_dim, is_bias ? 1 : (int64_t)d, c->stream);
            PO_HIP(hipStreamSynchronize(c->stream));
            PO_HIP(hipGetLastError());
        }
    }
    c->loaded[is_global ? m.n_layers : layer] |= 1u << kind;
    return PO_OK;
}

po_status po_load_weights(po_ctx* c, const po_host_weights* w) {
    if (!c || !w) return PO_ERR_INVALID_ARG;
    const po_model_config& m = c->cfg;
    const size_t esz = m.dtype == PO_F32 ? 4 : 2;
    const size_t d = m.d_model, F = m.ffn_dim, V = m.vocab_size;
    const size_t qd = (size_t)m.n_q_heads * m.head_dim, kvd = (size_t)m.n_kv_heads * m.head_dim;
    const size_t elems[PO_T_COUNT] = {V * d, d, qd * d, kvd * d, kvd * d, qd, kvd, kvd, d * qd, d, F * d, F * d, d * F, d, V * d};
    for (int kind = 0; kind < PO_T_COUNT; ++kind) {
        const bool is_global = kind == PO_T_EMBED || kind == PO_T_FINAL_NORM || kind == PO_T_LM_HEAD;
        const bool is_bias = kind == PO_T_BQ || kind == PO_T_BK || kind == PO_T_BV;
        if (is_bias && !m.qkv_bias) continue;
        if (!w->tensor[kind]) return PO_ERR_INVALID_ARG;
        if (is_global) {
            po_status st = po_load_tensor(c, kind, -1, w->tensor[kind], elems[kind] * esz);
            if (st != PO_OK) return st;
            continue;
        }
        const void* const* per_layer = (const void* const*)w->tensor[kind];
        for (int l = 0; l < m.n_layers; ++l) {
            if (!per_layer[l]) return PO_ERR_INVALID_ARG;
            po_status st = po_load_tensor(c, kind, l, per_layer[l], elems[kind] * esz);
            if (st != PO_OK) return st;
        }
    }
    return PO_OK;
}

int32_t po_is_loaded(const po_ctx* c) {
    if (!c) return 0;
    const uint32_t need = required_layer_mask(c->cfg);
    for (int l = 0; l < c->cfg.n_layers; ++l)
        if ((c->loaded[l] & need) != need) return 0;
    return (c->loaded[c->cfg.n_layers] & GLOBAL_MASK) == GLOBAL_MASK ? 1 : 0;
}

po_status po_prefill(po_ctx* c, const int32_t* tokens, int64_t len, const int32_t* cand_ids, int32_t n_cand,
                     float* out_logits, float* out_cand_logprobs) {
    if (!c) return PO_ERR_INVALID_ARG;
    po_status st = validate_request(c, tokens, len, cand_ids, n_cand);
    if (st != PO_OK) return st;
    if (!po_is_loaded(c)) return PO_ERR_NOT_LOADED;
    return run_prefill(c, tokens, len, cand_ids, n_cand, out_logits, out_cand_logprobs);
}

po_status po_prefill_batch(po_ctx* c, const int32_t* tokens_concat, const int64_t* lens, int32_t n_req,
                           const int32_t* cand_ids, int32_t n_cand, float* out_logits, float* out_cand_logprobs) {
    if (!c || !tokens_concat || !lens || n_req <= 0) return PO_ERR_INVALID_ARG;
    // validate everything before the first launch: no partial output on error
    int64_t off = 0;
    for (int32_t r = 0; r < n_req; ++r) {
        if (lens[r] <= 0) return PO_ERR_INVALID_ARG;
        po_status st = validate_request(c, tokens_concat + off, lens[r], cand_ids, n_cand);
        if (st != PO_OK) return st;
        off += lens[r];
    }
    if (!po_is_loaded(c)) return PO_ERR_NOT_LOADED;
    off = 0;
    double total_ms = 0, k_ms[PO_K_COUNT] = {0, 0, 0, 0};
    int64_t k_n[PO_K_COUNT] = {0, 0, 0, 0};
    for (int32_t r = 0; r < n_req; ++r) {
        po_status st = run_prefill(c, tokens_concat + off, lens[r], cand_ids, n_cand,
                                   out_logits ? out_logits + (size_t)r * c->cfg.vocab_size : nullptr,
                                   out_cand_logprobs ? out_cand_logprobs + (size_t)r * n_cand : nullptr);
        if (st != PO_OK) return st;
        total_ms += c->stats.last_prefill_ms;
        for (int kc = 0; kc < PO_K_COUNT; ++kc) { k_ms[kc] += c->stats.kernel_ms[kc]; k_n[kc] += c->stats.kernel_launches[kc]; }
        off += lens[r];
    }
    c->stats.last_prefill_ms = total_ms;
    for (int kc = 0; kc < PO_K_COUNT; ++kc) { c->stats.kernel_ms[kc] = k_ms[kc]; c->stats.kernel_launches[kc] = k_n[kc]; }
    c->stats.last_len = off;
    return PO_OK;
}

po_status po_prefill_packed(po_ctx* c, const int32_t* tokens_concat, const int64_t* lens, int32_t n_req,
                            const int32_t* cand_ids, int32_t n_cand, float* out_logits, float* out_cand_logprobs) {
    if (!c || !tokens_concat || !lens || n_req <= 0) return PO_ERR_INVALID_ARG;
    int64_t off = 0;
    for (int32_t r = 0; r < n_req; ++r) {
        if (lens[r] <= 0) return PO_ERR_INVALID_ARG;
        po_status st = validate_request(c, tokens_concat + off, lens[r], cand_ids, n_cand);
        if (st != PO_OK) return st;
        off += lens[r];
    }
    if (!po_is_loaded(c)) return PO_ERR_NOT_LOADED;
    double total_ms = 0, k_ms[PO_K_COUNT] = {0, 0, 0, 0};
    int64_t k_n[PO_K_COUNT] = {0, 0, 0, 0};
    std::vector<Seg> segs;
    std::vector<int32_t> buf;
    off = 0;
    int32_t r = 0;
    while (r < n_req) {
        // the next group: consecutive requests, each starting on a multiple of SEG_ALIGN rows, as many as
        // the buffers (sized for max_input_len rows) hold
        segs.clear();
        const int32_t r_first = r;
        int64_t end = 0;
        while (r < n_req) {
            const int64_t start = (end + SEG_ALIGN - 1) / SEG_ALIGN * SEG_ALIGN;
            if (!segs.empty() && start + lens[r] > c->max_len) break;
            segs.push_back(Seg{start, lens[r]});
            end = start + lens[r];
            ++r;
        }
        buf.assign((size_t)end, 0);
        int64_t src = off;
        for (const Seg& g : segs) {
            memcpy(buf.data() + g.start, tokens_concat + src, (size_t)g.len * 4);
            src += g.len;
        }
        po_status st = run_rows(c, buf.data(), end, segs, cand_ids, n_cand,
                                out_logits ? out_logits + (size_t)r_first * c->cfg.vocab_size : nullptr,
                                out_cand_logprobs ? out_cand_logprobs + (size_t)r_first * n_cand : nullptr);
        if (st != PO_OK) return st;
        total_ms += c->stats.last_prefill_ms;
        for (int kc = 0; kc < PO_K_COUNT; ++kc) { k_ms[kc] += c->stats.kernel_ms[kc]; k_n[kc] += c->stats.kernel_launches[kc]; }
        off = src;
    }
    c->stats.last_prefill_ms = total_ms;
    for (int kc = 0; kc < PO_K_COUNT; ++kc) { c->stats.kernel_ms[kc] = k_ms[kc]; c->stats.kernel_launches[kc] = k_n[kc]; }
    c->stats.last_len = off;
    return PO_OK;
}

po_status po_profile(po_ctx* c, int64_t len, double* elapsed_ms, size_t* touched_bytes) {
    if (!c || len <= 0) return PO_ERR_INVALID_ARG;
    if (len > c->max_len) return PO_ERR_TOO_LONG;
    if (!po_is_loaded(c)) return PO_ERR_NOT_LOADED;
    // everything in front of the mark word is filled and scanned; the word itself is the arena's last 256 bytes
    const size_t ws_bytes = c->lay.profile_mark;
    unsigned long long* d_mark = (unsigned long long*)(c->ws + c->lay.profile_mark);
    std::vector<int32_t> tokens((size_t)len, 0);
    const int32_t cand[2] = {0, c->cfg.vocab_size - 1};
    float lp[2];
    po_status st = PO_ERR_DEVICE;
    if (hipMemsetAsync(c->ws, 0xA5, ws_bytes, c->stream) == hipSuccess &&
        hipMemsetAsync(d_mark, 0, sizeof(unsigned long long), c->stream) == hipSuccess) {
        // the rotary table is the one thing in the arena that outlives a request: rebuild it
        launch_rope_table((float*)(c->ws + c->lay.rope_cos), (float*)(c->ws + c->lay.rope_sin), c->max_len,
                          c->cfg.head_dim, c->cfg.rope_theta, c->stream);
        st = run_prefill(c, tokens.data(), len, cand, 2, nullptr, lp);
        if (st == PO_OK) {
            launch_high_water(c->ws, ws_bytes, 0xA5A5A5A5u, d_mark, c->stream);
            unsigned long long mark = 0;
            if (hipMemcpyAsync(&mark, d_mark, sizeof(mark), hipMemcpyDeviceToHost, c->stream) == hipSuccess &&
                hipStreamSynchronize(c->stream) == hipSuccess) {
                if (elapsed_ms) *elapsed_ms = c->stats.last_prefill_ms;
                if (touched_bytes) *touched_bytes = (size_t)mark * 4;
            } else {
                st = PO_ERR_DEVICE;
            }
        }
    }
    return st;
}

po_status po_kv_cache_bytes(const po_model_config* cfg, int64_t prefix_capacity, size_t* bytes) {
    if (!cfg || !bytes) return PO_ERR_INVALID_ARG;
    po_status st = validate_config(cfg);
    if (st != PO_OK) return st;
    if (prefix_capacity <= 0) return PO_ERR_INVALID_ARG;
    int64_t ldvc;
    size_t v_off, layer_bytes;
    kv_cache_geometry(cfg, prefix_capacity, &ldvc, &v_off, &layer_bytes);
    *bytes = layer_bytes * (size_t)cfg->n_layers;
    return PO_OK;
}

po_status po_attach_kv_cache_slots(po_ctx* c, void* dev_cache, size_t bytes, int64_t prefix_capacity, int32_t n_slots) {
    if (!c) return PO_ERR_INVALID_ARG;
    if (!dev_cache) {               // detach
        c->kvc = nullptr;
        c->kv_cap = 0;
        c->kv_slots.clear();
        return PO_OK;
    }
    if (prefix_capacity <= 0 || n_slots <= 0 || ((uintptr_t)dev_cache % ALIGN)) return PO_ERR_INVALID_ARG;
    if (prefix_capacity > c->max_len) return PO_ERR_TOO_LONG;
    size_t need = 0;
    po_status st = po_kv_cache_bytes(&c->cfg, prefix_capacity, &need);
    if (st != PO_OK) return st;
    if (bytes / (size_t)n_slots < need) return PO_ERR_WORKSPACE_TOO_SMALL;
    c->kvc = (unsigned char*)dev_cache;
    c->kv_cap = prefix_capacity;
    kv_cache_geometry(&c->cfg, prefix_capacity, &c->kv_ldv, &c->kv_v_off, &c->kv_layer_bytes);
    c->kv_slots.assign((size_t)n_slots, po_ctx::KvSlot{{}, 0});
    c->kv_tick = 0;
    c->kv_src = c->kv_dst = 0;
    return PO_OK;
}

po_status po_attach_kv_cache(po_ctx* c, void* dev_cache, size_t bytes, int64_t prefix_capacity) {
    return po_attach_kv_cache_slots(c, dev_cache, bytes, prefix_capacity, 1);
}

namespace {
// slot with the longest common prefix with tokens[0, len) (ties: the most recently used), and that length
int best_slot(const po_ctx* c, const int32_t* tokens, int64_t len, int64_t* match) {
    int best = 0;
    int64_t best_m = -1;
    for (size_t i = 0; i < c->kv_slots.size(); ++i) {
        const std::vector<int32_t>& t = c->kv_slots[i].tokens;
        const int64_t lim = std::min<int64_t>((int64_t)t.size(), len);
        int64_t mm = 0;
        while (mm + 64 <= lim && memcmp(t.data() + mm, tokens + mm, 64 * sizeof(int32_t)) == 0) mm += 64;   // whole blocks first
        while (mm < lim && t[(size_t)mm] == tokens[mm]) ++mm;
        if (mm > best_m || (mm == best_m && c->kv_slots[i].last_use > c->kv_slots[(size_t)best].last_use)) {
            best_m = mm;
            best = (int)i;
        }
    }
    *match = best_m < 0 ? 0 : best_m;
    return best;
}
}  // namespace

po_status po_kv_cache_match(const po_ctx* c, const int32_t* tokens, int64_t len, int64_t* cached_len) {
    if (!c || !tokens || len <= 0 || !cached_len) return PO_ERR_INVALID_ARG;
    int64_t mm = 0;
    if (c->kvc) (void)best_slot(c, tokens, len, &mm);
    *cached_len = std::min<int64_t>(mm, len - 1);          // one position is always computed
    return PO_OK;
}

po_status po_kv_cache_slot(const po_ctx* c, int32_t slot, int32_t* tokens_out, int64_t capacity, int64_t* n_tokens) {
    if (!c || !n_tokens || slot < 0) return PO_ERR_INVALID_ARG;
    if ((size_t)slot >= c->kv_slots.size()) return PO_ERR_INVALID_ARG;
    const std::vector<int32_t>& t = c->kv_slots[(size_t)slot].tokens;
    *n_tokens = (int64_t)t.size();
    if (tokens_out) {
        if (capacity < (int64_t)t.size()) return PO_ERR_INVALID_ARG;
        if (!t.empty()) memcpy(tokens_out, t.data(), t.size() * sizeof(int32_t));
    }
    return PO_OK;
}

po_status po_prefill_prefix(po_ctx* c, const int32_t* tokens, int64_t len, int64_t keep_prefix,
                            const int32_t* cand_ids, int32_t n_cand, float* out_logits, float* out_cand_logprobs,
                            int64_t* reused_prefix_len) {
    if (!c || (keep_prefix < 0 && keep_prefix != PO_KEEP_ALL)) return PO_ERR_INVALID_ARG;
    po_status st = validate_request(c, tokens, len, cand_ids, n_cand);
    if (st != PO_OK) return st;
    if (!c->kvc) return PO_ERR_INVALID_ARG;
    if (keep_prefix == PO_KEEP_ALL) keep_prefix = std::min<int64_t>(len, c->kv_cap);
    if (keep_prefix > len || keep_prefix > c->kv_cap) return PO_ERR_TOO_LONG;
    if (!po_is_loaded(c)) return PO_ERR_NOT_LOADED;
    // the slot with the longest common prefix; at least one position is always computed
    int64_t shared = 0;
    const int src = best_slot(c, tokens, len, &shared);
    const int64_t stored = (int64_t)c->kv_slots[(size_t)src].tokens.size();
    const int64_t m = std::min<int64_t>(shared, len - 1);
    // Where the prefix to keep goes.  Already inside the entry: nothing is stored and the entry stays as
    // long as it is.  The request shares all the entry holds, or at least half of it: the entry is cut to
    // the shared part and grows in place (a sequence of requests that differ in their tails keeps ONE entry
    // and rewrites only the tail).  Otherwise (a hit on less than half, or none) the prefix replaces the
    // least recently used of the other entries, so that a short partial hit does not destroy a long entry;
    // with one entry it replaces that one.
    int dst = src;
    int64_t store = keep_prefix;
    if (keep_prefix <= shared) {
        store = 0;
    } else if (shared < stored && c->kv_slots.size() > 1 && shared * 2 < stored) {
        uint64_t oldest = ~0ull;
        for (size_t i = 0; i < c->kv_slots.size(); ++i)
            if ((int)i != src || shared == 0) {
                const uint64_t u = c->kv_slots[i].tokens.empty() ? 0 : c->kv_slots[i].last_use;
                if (u < oldest) { oldest = u; dst = (int)i; }
            }
    }
    c->kv_src = src;
    c->kv_dst = dst;
    st = run_prefill(c, tokens, len, cand_ids, n_cand, out_logits, out_cand_logprobs, m, store);
    if (st != PO_OK) {              // the destination may be half written: forget it
        if (store > 0) c->kv_slots[(size_t)dst].tokens.clear();
        return st;
    }
    ++c->kv_tick;
    if (m > 0 || (keep_prefix > 0 && store == 0)) c->kv_slots[(size_t)src].last_use = c->kv_tick;
    if (store > 0) {
        c->kv_slots[(size_t)dst].tokens.assign(tokens, tokens + store);
        c->kv_slots[(size_t)dst].last_use = c->kv_tick;
    }
    if (reused_prefix_len) *reused_prefix_len = m;
    return PO_OK;
}

po_status po_profile_jct(po_ctx* c, int64_t max_len, int64_t step, int64_t* n_input_out, int64_t* n_cached_out,
                         double* jct_ms_out, int32_t capacity, int32_t* n_samples) {
    if (!c || max_len <= 0 || step <= 0 || !n_samples || capacity < 0) return PO_ERR_INVALID_ARG;
    if (max_len > c->max_len) return PO_ERR_TOO_LONG;
    if (!c->kvc) return PO_ERR_INVALID_ARG;
    if (!po_is_loaded(c)) return PO_ERR_NOT_LOADED;
    const int32_t V = c->cfg.vocab_size;
    if (V < 2) return PO_ERR_BAD_CONFIG;
    // the grid: n_input = step, 2 step, ... and max_len itself; n_cached = 0, step, ... below n_input and
    // within what the cache can hold
    std::vector<int64_t> n_in;
    for (int64_t n = step; n < max_len; n += step) n_in.push_back(n);
    n_in.push_back(max_len);
    int64_t p_max = 0, count = 0;
    for (int64_t n : n_in)
        for (int64_t p = 0; p < n && p <= c->kv_cap; p += step) {
            p_max = std::max(p_max, p);
            ++count;
        }
    if (count > INT32_MAX) return PO_ERR_INVALID_ARG;
    *n_samples = (int32_t)count;
    if (!n_input_out && !n_cached_out && !jct_ms_out) return PO_OK;          // size query
    if (!n_input_out || !n_cached_out || !jct_ms_out || capacity < count) return PO_ERR_INVALID_ARG;
    // two fake token sequences that differ at every position, so that a request made of the first p ids of
    // one and the rest of the other shares exactly p positions with the cached one.  Pseudo-random ids:
    // a run on constant data draws less power and clocks higher than a real request does.
    std::vector<int32_t> base((size_t)max_len), req((size_t)max_len);
    uint64_t x = 0x9E3779B97F4A7C15ull;
    for (int64_t i = 0; i < max_len; ++i) {
        x = x * 6364136223846793005ull + 1442695040888963407ull;
        base[(size_t)i] = (int32_t)((x >> 33) % (uint64_t)V);
    }
    const int32_t cand[2] = {0, V - 1};
    float lp[2];
    for (auto& sl : c->kv_slots) sl.tokens.clear();
    c->kv_src = c->kv_dst = 0;
    po_status st = PO_OK;
    if (p_max > 0) {                                                         // fills entry 0; also the warm-up
        st = run_prefill(c, base.data(), p_max, cand, 2, nullptr, lp, 0, p_max);
    } else {
        st = run_prefill(c, base.data(), n_in[0], cand, 2, nullptr, lp);
    }
    int32_t k = 0;
    for (size_t a = 0; st == PO_OK && a < n_in.size(); ++a) {
        const int64_t n = n_in[a];
        for (int64_t p = 0; st == PO_OK && p < n && p <= c->kv_cap; p += step) {
            for (int64_t i = 0; i < n; ++i) req[(size_t)i] = i < p ? base[(size_t)i] : (base[(size_t)i] + 1) % V;
            st = run_prefill(c, req.data(), n, cand, 2, nullptr, lp, p, 0);
            n_input_out[k] = n;
            n_cached_out[k] = p;
            jct_ms_out[k] = c->stats.last_prefill_ms;
            ++k;
        }
    }
    for (auto& sl : c->kv_slots) sl.tokens.clear();                          // the fake prefix serves nobody
    return st;
}

po_status po_set_storage_rounding(po_ctx* c, int32_t on) {
    if (!c) return PO_ERR_INVALID_ARG;
    if (c->cfg.dtype != PO_F32) return PO_ERR_BAD_CONFIG;
    c->store_round = on != 0;
    return PO_OK;
}

po_status po_set_few_rows_split(po_ctx* c, int32_t on) {
    if (!c) return PO_ERR_INVALID_ARG;
    c->split_few_rows = on != 0;
    return PO_OK;
}

po_status po_set_lazy_last_layer(po_ctx* c, int32_t on) {
    if (!c) return PO_ERR_INVALID_ARG;
    c->lazy_last_layer = on != 0;
    return PO_OK;
}

po_status po_set_phase_timing(po_ctx* c, int32_t on) {
    if (!c) return PO_ERR_INVALID_ARG;
    c->phase_timing = on != 0;
    return PO_OK;
}

po_status po_get_stats(const po_ctx* c, po_stats* out) {
    if (!c || !out) return PO_ERR_INVALID_ARG;
    *out = c->stats;
    return PO_OK;
}

void po_destroy(po_ctx* c) {
    if (!c) return;
    if (c->ev_start) (void)hipEventDestroy(c->ev_start);
    if (c->ev_stop) (void)hipEventDestroy(c->ev_stop);
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    delete c;
}

const char* po_strerror(po_status s) {
    switch (s) {
        case PO_OK: return "ok";
        case PO_ERR_INVALID_ARG: return "invalid argument";
        case PO_ERR_BAD_CONFIG: return "model configuration not supported by the kernels";
        case PO_ERR_NOT_LOADED: return "weights not fully loaded";
        case PO_ERR_TOO_LONG: return "input longer than max_input_len";
        case PO_ERR_TOKEN_RANGE: return "token or candidate id outside [0, vocab_size)";
        case PO_ERR_WORKSPACE_TOO_SMALL: return "device arena smaller than po_workspace_bytes reports";
        case PO_ERR_OOM: return "host allocation failed";
        case PO_ERR_DEVICE: return "HIP call failed";
    }
    return "unknown status";
}

const char* po_last_device_error(void) { return g_dev_err; }

// ------------------------------------------------------------------ single-kernel entry points

static inline bool bad_dtype(int32_t dt) { return dt != PO_F32 && dt != PO_BF16; }

po_status po_op_rmsnorm(int32_t dtype, const void* x, const void* g, void* y, int64_t rows, int32_t d, float eps,
                        void* stream) {
    if (bad_dtype(dtype) || !x || !g || !y || rows <= 0 || d <= 0 || d % 8) return PO_ERR_INVALID_ARG;
    launch_rmsnorm(dtype, x, g, y, rows, d, eps, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_linear(int32_t dtype, const void* a, const void* w, void* cc, const void* residual, int64_t M,
                       int32_t N, int32_t K, void* stream) {
    if (bad_dtype(dtype) || !a || !w || !cc || M <= 0 || N <= 0 || K <= 0) return PO_ERR_INVALID_ARG;
    if (dtype == PO_BF16) {
        if (!gemm_mfma_supported(N, K)) return PO_ERR_BAD_CONFIG;
        launch_gemm_mfma(residual ? EPI_RESIDUAL : EPI_STORE, (const bf16_t*)a, K, (const bf16_t*)w, K, (bf16_t*)cc, N,
                         nullptr, (const bf16_t*)residual, N, M, N, K, (hipStream_t)stream);
    } else {
        launch_gemm_basic(dtype, a, K, w, K, cc, N, nullptr, residual, N, M, N, K, (hipStream_t)stream);
    }
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_linear_split(const void* a, const void* w, void* cc, const void* residual, void* scratch,
                             size_t scratch_bytes, int64_t M, int32_t N, int32_t K, void* stream, int32_t* splits_used) {
    if (!a || !w || !cc || !residual || !scratch || !splits_used || M <= 0 || N <= 0 || K <= 0) return PO_ERR_INVALID_ARG;
    if (!gemm_mfma_supported(N, K)) return PO_ERR_BAD_CONFIG;
    *splits_used = launch_gemm_mfma_splitk_residual((const bf16_t*)a, K, (const bf16_t*)w, K, (bf16_t*)cc, N,
                                                    (const bf16_t*)residual, N, M, N, K, (float*)scratch, scratch_bytes, true,
                                                    (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_gate_up_silu(int32_t dtype, const void* a, const void* wgu, void* h, void* scratch, int64_t M,
                             int32_t F, int32_t K, void* stream) {
    if (bad_dtype(dtype) || !a || !wgu || !h || M <= 0 || F <= 0 || K <= 0) return PO_ERR_INVALID_ARG;
    if (dtype == PO_BF16) {
        if (F % GU_INTERLEAVE_BF16 || !gemm_mfma_supported(2 * F, K)) return PO_ERR_BAD_CONFIG;
        launch_gemm_mfma(EPI_SILU_MUL, (const bf16_t*)a, K, (const bf16_t*)wgu, K, (bf16_t*)h, F, nullptr, nullptr, 0, M,
                         2 * F, K, (hipStream_t)stream);
    } else {
        if (!scratch) return PO_ERR_INVALID_ARG;
        launch_gemm_basic(dtype, a, K, wgu, K, scratch, 2 * F, nullptr, nullptr, 0, M, 2 * F, K, (hipStream_t)stream);
        launch_silu_mul(dtype, scratch, h, M, F, (hipStream_t)stream);
    }
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_pack_gate_up(int32_t dtype, const void* wg, const void* wu, void* wgu, int32_t F, int32_t K,
                             void* stream) {
    if (bad_dtype(dtype) || !wg || !wu || !wgu || F <= 0 || K <= 0 || K % 8) return PO_ERR_INVALID_ARG;
    if (dtype == PO_BF16 && F % GU_INTERLEAVE_BF16) return PO_ERR_BAD_CONFIG;
    launch_pack_gate_up(dtype, wg, wu, wgu, F, K, dtype == PO_BF16 ? GU_INTERLEAVE_BF16 : F, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_attention(int32_t dtype, const void* q, const void* k, const void* v, void* o, void* scratch,
                          int64_t N, int32_t Hq, int32_t Hkv, int32_t hd, int32_t q_prescaled, void* stream) {
    if (bad_dtype(dtype) || !q || !k || !v || !o || N <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv) return PO_ERR_INVALID_ARG;
    if ((q_prescaled != 0 && q_prescaled != 1) || (q_prescaled && dtype != PO_BF16)) return PO_ERR_INVALID_ARG;
    if (N > (int64_t)1 << 24) return PO_ERR_TOO_LONG;
    if (dtype == PO_BF16) {
        if (!attention_mfma_supported(Hq, Hkv, hd)) return PO_ERR_BAD_CONFIG;
        if (!scratch) return PO_ERR_INVALID_ARG;
        if ((N + 64) * Hkv * hd * 2 >= ((int64_t)1 << 32)) return PO_ERR_TOO_LONG;
        const int64_t ldv = round_up64(N, 64);
        // scratch: V^T, then (256-byte aligned) the give-up words of the attention kernel
        int* redo = (int*)((unsigned char*)scratch + align_up((size_t)Hkv * hd * (size_t)ldv * 2));
        launch_fill_zero32(redo, attention_mfma_redo_bytes(N, Hq) / 4, (hipStream_t)stream);
        launch_v_transpose((const bf16_t*)v, (bf16_t*)scratch, N, Hkv * hd, ldv, (hipStream_t)stream);
        launch_attention_mfma((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)scratch, ldv, (bf16_t*)o, N, Hq, Hkv,
                              hd, 0, redo, q_prescaled != 0, (hipStream_t)stream);
    } else {
        if (hd != 32 && hd != 64 && hd != 128) return PO_ERR_BAD_CONFIG;
        launch_attention_basic(dtype, q, k, v, o, N, Hq, Hkv, hd, 0, (hipStream_t)stream);
    }
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_attention_split(const void* q, const void* k, const void* v, void* o, void* scratch_vt, void* scratch_part,
                                size_t part_bytes, int64_t N, int32_t Hq, int32_t Hkv, int32_t hd, int64_t q_row0,
                                void* stream, int32_t* splits_used) {
    if (!q || !k || !v || !o || !scratch_vt || !scratch_part || !splits_used || N <= 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv ||
        q_row0 < 0 || q_row0 >= N)
        return PO_ERR_INVALID_ARG;
    if (!attention_mfma_supported(Hq, Hkv, hd)) return PO_ERR_BAD_CONFIG;
    if (N > (int64_t)1 << 24 || (N + 64) * Hkv * hd * 2 >= ((int64_t)1 << 32)) return PO_ERR_TOO_LONG;
    const int64_t ldv = round_up64(N, 64);
    launch_v_transpose((const bf16_t*)v, (bf16_t*)scratch_vt, N, Hkv * hd, ldv, (hipStream_t)stream);
    *splits_used = launch_attention_mfma_split((const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)scratch_vt, ldv, (bf16_t*)o, N,
                                               Hq, Hkv, hd, q_row0, (float*)scratch_part, part_bytes, true, nullptr, nullptr, 0,
                                               0, false, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_rope(int32_t dtype, void* x, int64_t N, int32_t H, int32_t hd, float theta, void* stream) {
    if (bad_dtype(dtype) || !x || N <= 0 || H <= 0 || hd <= 0 || hd % 2 || !(theta > 0.f)) return PO_ERR_INVALID_ARG;
    float* tab = nullptr;
    const size_t half_bytes = (size_t)N * (hd / 2) * 4;
    PO_HIP(hipMalloc((void**)&tab, 2 * half_bytes));
    launch_rope_table(tab, tab + (size_t)N * (hd / 2), N, hd, theta, (hipStream_t)stream);
    launch_rope(dtype, x, (int64_t)H * hd, tab, tab + (size_t)N * (hd / 2), N, H, hd, (hipStream_t)stream);
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    (void)hipFree(tab);
    PO_HIP(e);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

// ---- po_op_rope for callers that cannot allocate: its rotary table sits in a file-scope device array
// instead of a hipMalloc'd buffer.  Every GPU the library runs on holds its own copy of the array, at its own
// address, until the process ends; in host code the array's NAME is only a stand-in (not a device address), so
// the address is looked up once per device with hipGetSymbolAddress and kept, and only that pointer is ever
// handed to a kernel.
constexpr size_t PO_STATIC_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char po_static_scratch[PO_STATIC_SCRATCH_BYTES];
constexpr int PO_MAX_DEVICES = 64;
static void* g_static_scratch_ptr[PO_MAX_DEVICES];       // per device; null until looked up
static std::mutex g_static_scratch_mu;

// device address of po_static_scratch on the CURRENT device (looked up on first use there)
static po_status static_scratch_ptr(void** out) {
    int dev = -1;
    PO_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= PO_MAX_DEVICES) return PO_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_static_scratch_mu);
    if (!g_static_scratch_ptr[dev]) {
        void* ptr = nullptr;
        PO_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(po_static_scratch)));
        if (!ptr) return PO_ERR_DEVICE;
        g_static_scratch_ptr[dev] = ptr;
    }
    *out = g_static_scratch_ptr[dev];
    return PO_OK;
}

po_status po_op_rope_static(int32_t dtype, void* x, int64_t N, int32_t H, int32_t hd, float theta, void* stream) {
    if (bad_dtype(dtype) || !x || N <= 0 || H <= 0 || hd <= 0 || hd % 2 || !(theta > 0.f)) return PO_ERR_INVALID_ARG;
    // cos and sin tables [N, hd/2] of float32 each
    if ((uint64_t)N * (uint64_t)hd * 4 > PO_STATIC_SCRATCH_BYTES) return PO_ERR_WORKSPACE_TOO_SMALL;
    void* ptr = nullptr;
    po_status st = static_scratch_ptr(&ptr);
    if (st != PO_OK) return st;
    // the table kernel writes every entry the rotation reads, so nothing of an earlier call's contents is seen
    float* tab = (float*)ptr;
    launch_rope_table(tab, tab + (size_t)N * (hd / 2), N, hd, theta, (hipStream_t)stream);
    launch_rope(dtype, x, (int64_t)H * hd, tab, tab + (size_t)N * (hd / 2), N, H, hd, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_rope_table(float* cos_t, float* sin_t, int64_t n, int32_t hd, float theta, void* stream) {
    if (!cos_t || !sin_t || n <= 0 || hd <= 0 || hd % 2 || !(theta > 0.f)) return PO_ERR_INVALID_ARG;
    launch_rope_table(cos_t, sin_t, n, hd, theta, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_pack_qkv(const void* wq, const void* wk, const void* wv, void* wqkv, const void* bq, const void* bk,
                         const void* bv, void* bqkv, int32_t Hq, int32_t Hkv, int32_t hd, int32_t K, void* stream) {
    if (!wq || !wk || !wv || !wqkv || Hq <= 0 || Hkv <= 0 || K <= 0) return PO_ERR_INVALID_ARG;
    if (hd != 64 && hd != 128) return PO_ERR_BAD_CONFIG;
    const bool has_bias = bq || bk || bv;
    if (has_bias && !(bq && bk && bv && bqkv)) return PO_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    const size_t qd = (size_t)Hq * hd, kvd = (size_t)Hkv * hd, rb = (size_t)K * 2;
    unsigned char* w = (unsigned char*)wqkv;
    PO_HIP(hipMemcpyAsync(w, wq, qd * rb, hipMemcpyDeviceToDevice, s));
    PO_HIP(hipMemcpyAsync(w + qd * rb, wk, kvd * rb, hipMemcpyDeviceToDevice, s));
    PO_HIP(hipMemcpyAsync(w + (qd + kvd) * rb, wv, kvd * rb, hipMemcpyDeviceToDevice, s));
    launch_pack_rope_rows((bf16_t*)w, Hq, hd, K, s);
    launch_pack_rope_rows((bf16_t*)(w + qd * rb), Hkv, hd, K, s);
    if (has_bias) {
        unsigned char* b = (unsigned char*)bqkv;
        PO_HIP(hipMemcpyAsync(b, bq, qd * 2, hipMemcpyDeviceToDevice, s));
        PO_HIP(hipMemcpyAsync(b + qd * 2, bk, kvd * 2, hipMemcpyDeviceToDevice, s));
        PO_HIP(hipMemcpyAsync(b + (qd + kvd) * 2, bv, kvd * 2, hipMemcpyDeviceToDevice, s));
        launch_pack_rope_rows((bf16_t*)b, Hq, hd, 1, s);
        launch_pack_rope_rows((bf16_t*)(b + qd * 2), Hkv, hd, 1, s);
    }
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_qkv_rope(const void* a, const void* wqkv, const void* bqkv, void* q, void* k, void* vt, int64_t ldv,
                         const float* cos_t, const float* sin_t, int64_t pos0, int64_t M, int32_t Hq, int32_t Hkv,
                         int32_t hd, int32_t K, float q_scale, void* stream) {
    if (!a || !wqkv || !q || !k || !vt || !cos_t || !sin_t || M <= 0 || pos0 < 0 || Hq <= 0 || Hkv <= 0 || K <= 0 ||
        !(q_scale > 0.f))
        return PO_ERR_INVALID_ARG;
    if ((hd != 64 && hd != 128) || !gemm_mfma_supported((Hq + 2 * Hkv) * hd, K)) return PO_ERR_BAD_CONFIG;
    if (ldv < pos0 + M || ldv % 8) return PO_ERR_INVALID_ARG;
    launch_gemm_qkv_rope((const bf16_t*)a, K, (const bf16_t*)wqkv, K, (const bf16_t*)bqkv, (bf16_t*)q, (bf16_t*)k,
                         (bf16_t*)vt, ldv, cos_t, sin_t, pos0, nullptr, M, Hq * hd, Hkv * hd, hd, K, q_scale,
                         (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_quantize_rows(const void* x, void* codes, float* scales, int64_t M, int32_t K, void* stream) {
    if (!x || !codes || !scales || M <= 0 || K <= 0) return PO_ERR_INVALID_ARG;
    if (!quant_rows_supported(K)) return PO_ERR_BAD_CONFIG;
    // in place: a row's codes start where the row starts (pitch 2K bytes); otherwise dense rows of K bytes
    launch_quant_rows((const bf16_t*)x, K, (unsigned char*)codes, codes == x ? 2 * (int64_t)K : K, scales, M, K, 0, 0, 0,
                      (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_rmsnorm_quantize(const void* x, const void* g, void* codes, float* scales, int64_t rows, int32_t d,
                                 float eps, void* stream) {
    if (!x || !g || !codes || !scales || rows <= 0 || d <= 0) return PO_ERR_INVALID_ARG;
    if (d % 8 || d > 8192) return PO_ERR_BAD_CONFIG;
    launch_rmsnorm_quant((const bf16_t*)x, (const bf16_t*)g, (unsigned char*)codes, scales, rows, d, eps, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_linear_fp8(int32_t epilogue, const void* a_codes, const float* a_scales, const void* w_codes,
                           const float* w_scales, void* cc, const void* residual, int64_t M, int32_t N, int32_t K,
                           void* stream) {
    if (!a_codes || !a_scales || !w_codes || !w_scales || !cc || M <= 0 || N <= 0 || K <= 0) return PO_ERR_INVALID_ARG;
    if (epilogue != EPI_STORE && epilogue != EPI_RESIDUAL && epilogue != EPI_SILU_MUL) return PO_ERR_INVALID_ARG;
    if (epilogue == EPI_RESIDUAL && !residual) return PO_ERR_INVALID_ARG;
    if (!gemm_fp8_supported(N, K) || (epilogue == EPI_SILU_MUL && N % (2 * GU_INTERLEAVE_BF16))) return PO_ERR_BAD_CONFIG;
    const int64_t ldc = epilogue == EPI_SILU_MUL ? N / 2 : N;
    launch_gemm_fp8(epilogue, (const unsigned char*)a_codes, K, a_scales, (const unsigned char*)w_codes, K, w_scales,
                    (bf16_t*)cc, ldc, nullptr, (const bf16_t*)residual, N, M, N, K, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_qkv_rope_fp8(const void* a_codes, const float* a_scales, const void* w_codes, const float* w_scales,
                             const void* bqkv, void* q, void* k, void* vt, int64_t ldv, const float* cos_t,
                             const float* sin_t, int64_t pos0, int64_t M, int32_t Hq, int32_t Hkv, int32_t hd, int32_t K,
                             float q_scale, void* stream) {
    if (!a_codes || !a_scales || !w_codes || !w_scales || !q || !k || !vt || !cos_t || !sin_t || M <= 0 || pos0 < 0 ||
        Hq <= 0 || Hkv <= 0 || K <= 0 || !(q_scale > 0.f))
        return PO_ERR_INVALID_ARG;
    if ((hd != 64 && hd != 128) || !gemm_fp8_supported((Hq + 2 * Hkv) * hd, K)) return PO_ERR_BAD_CONFIG;
    if (ldv < pos0 + M || ldv % 8) return PO_ERR_INVALID_ARG;
    launch_gemm_fp8_qkv_rope((const unsigned char*)a_codes, K, a_scales, (const unsigned char*)w_codes, K, w_scales,
                             (const bf16_t*)bqkv, (bf16_t*)q, (bf16_t*)k, (bf16_t*)vt, ldv, cos_t, sin_t, pos0, nullptr, M,
                             Hq * hd, Hkv * hd, hd, K, q_scale, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_mfma_peak(int32_t kind, int32_t waves_per_simd, int32_t iters, const void* operands, size_t operand_bytes,
                          void* sink, void* stream, double* flop) {
    if (!operands || !sink || !flop) return PO_ERR_INVALID_ARG;
    const double f = launch_mfma_peak(kind, waves_per_simd, iters, operands, operand_bytes, (float*)sink, (hipStream_t)stream);
    if (f == 0.0) return PO_ERR_INVALID_ARG;
    *flop = f;
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_stream_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || bytes == 0 || bytes % 16) return PO_ERR_INVALID_ARG;
    launch_stream_copy(src, dst, bytes, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

po_status po_op_lm_head(int32_t dtype, const void* x, const void* w, float* logits, int32_t V, int32_t d,
                        void* stream) {
    if (bad_dtype(dtype) || !x || !w || !logits || V <= 0 || d <= 0 || d % 8) return PO_ERR_INVALID_ARG;
    launch_lm_head(dtype, x, w, logits, V, d, nullptr, 0, (hipStream_t)stream);
    PO_HIP(hipGetLastError());
    return PO_OK;
}

}  // extern "C"
#pragma GCC visibility pop
