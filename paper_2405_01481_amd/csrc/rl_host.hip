// Host side of librollout: context, workspace layout, page allocator, the
// generation / scoring step sequences, and the C ABI declared in include/rollout.h.
#include "rl_common.h"
#include "rl_gemm.h"
#include "rl_attn.h"
#include "../../include/rollout.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <unordered_map>
#include <vector>

// ---------------------------------------------------------------- errors
static thread_local char g_err[512] = "";
static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
#define HIP_TRY(expr)                                                                            \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) return fail(RL_EHIP, "%s: %s", #expr, hipGetErrorString(e_));      \
    } while (0)

// ---------------------------------------------------------------- workspace layout
struct Layout {
    size_t x, h, h_keep, qkv, q, kbuf, vbuf, attn, ffn, logits, rope, block_table;
    size_t last_tok, seq_len, gen_count, finished, cur_tok, step_count;
    size_t tok_ids, tok_pos, tok_slot, tok_tgt;
    size_t seq_first, row_start, row_len, full_len, row_slot, d_seq_len, d_prompt_len, errflag;
    size_t out_row, seq_id, gen_limit;   // queue mode: per-slot output row, sequence id, token limit
    size_t splitk, attn_part, attn_ml, lse_part, z_tgt, blocks;
    size_t total;
    int rows, logit_rows, mpps, nqkv, vt_cap, max_blocks;
};

static size_t esz_of(int dtype) { return dtype == RL_FP32 ? 4 : 2; }

static const int kLogitRowsScore = 512;    // rows of logits materialised at a time by the plain scoring path
static const int kMaxSplitK = 16;
static const int kMaxAttnSplits = 16;
// bf16 configurations: the first layers can carry their activations (GEMM inputs, q, k, v, softmax
// probabilities, attention output, FFN activation, and their part of the KV cache) as fp16 pairs
// (value = hi + lo, about 22 significant bits) instead of single fp16 values.  Rounding in the FIRST layer
// accounts for about nine tenths of the log-prob error variance of the fp16 path against an unrounded
// evaluation (measured per rounding point and per layer on the 1B, 8B and 70B shapes): every later layer adds
// to a residual stream that the first layer's output dominates.  The pool and the workspace are sized for
// kMaxPreciseLayers such layers; kDefaultPreciseLayers are used unless rollout_set_precise_layers says otherwise.
static const int kMaxPreciseLayers = 2;
static const int kDefaultPreciseLayers = 1;
static int precise_cap(const rl_model_cfg& c) { return c.dtype == RL_BF16 ? std::min(kMaxPreciseLayers, c.n_layers) : 0; }

static Layout make_layout(const rl_model_cfg& c) {
    Layout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += (bytes + 255) / 256 * 256;
        return o;
    };
    const size_t e = esz_of(c.dtype);
    const size_t pw = precise_cap(c) > 0 ? 2 : 1;   // activation rows hold fp16 pairs in the precise layers
    // token rows of one pass; sequences are packed at multiples of 32 rows on the tuned path
    const int rows = (std::max(c.max_chunk_tokens, c.max_batch) + 31) / 32 * 32 + 32;
    const int nqkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const int qd = c.n_q_heads * c.head_dim, kd = c.n_kv_heads * c.head_dim;
    L.rows = rows;
    L.nqkv = nqkv;
    L.mpps = (c.max_seq + c.page_tokens - 1) / c.page_tokens;
    L.logit_rows = std::max(c.max_batch, std::min(rows, kLogitRowsScore));
    L.x = take((size_t)rows * c.d_model * 4);
    L.h = take((size_t)rows * c.d_model * e * pw);
    L.h_keep = take((size_t)rows * c.d_model * e);   // the policy's final hidden states while the reference runs (exact KL)
    L.qkv = take((size_t)rows * nqkv * 4);
    L.q = take((size_t)rows * qd * e * pw);
    L.kbuf = take((size_t)rows * kd * e * pw);
    L.vt_cap = rows;
    L.vbuf = take((size_t)rows * kd * e * pw);
    L.attn = take((size_t)rows * qd * e * pw);
    L.ffn = take((size_t)rows * c.d_ffn * e * pw);
    L.logits = take((size_t)L.logit_rows * c.vocab * 4);
    L.rope = take((size_t)c.max_seq * (c.head_dim / 2) * sizeof(float2));
    L.block_table = take((size_t)c.max_batch * L.mpps * 4);
    L.last_tok = take((size_t)c.max_batch * 4);
    L.seq_len = take((size_t)c.max_batch * 4);
    L.gen_count = take((size_t)c.max_batch * 4);
    L.finished = take((size_t)c.max_batch * 4);
    L.cur_tok = take((size_t)c.max_batch * 4);
    L.step_count = take((size_t)c.max_batch * 4);
    L.tok_ids = take((size_t)rows * 4);
    L.tok_pos = take((size_t)rows * 4);
    L.tok_slot = take((size_t)rows * 4);
    L.tok_tgt = take((size_t)rows * 4);
    L.seq_first = take((size_t)c.max_batch * 4);
    L.row_start = take((size_t)c.max_batch * 4);
    L.row_len = take((size_t)c.max_batch * 4);
    L.full_len = take((size_t)c.max_batch * 4);
    L.row_slot = take((size_t)c.max_batch * 4);
    L.out_row = take((size_t)c.max_batch * 4);
    L.seq_id = take((size_t)c.max_batch * 4);
    L.gen_limit = take((size_t)c.max_batch * 4);
    L.d_seq_len = take((size_t)c.max_batch * 4);
    L.d_prompt_len = take((size_t)c.max_batch * 4);
    L.errflag = take(256);
    // decode-path partial buffers: split-K partial sums and split-KV attention partials
    const int maxn = std::max(std::max(nqkv, c.d_model), 1);
    L.splitk = take((size_t)kMaxSplitK * 128 * ((c.max_batch + 127) / 128) * maxn * 4);
    L.attn_part = take((size_t)c.max_batch * c.n_q_heads * kMaxAttnSplits * c.head_dim * 4);
    L.attn_ml = take((size_t)c.max_batch * c.n_q_heads * kMaxAttnSplits * 2 * 4);
    L.lse_part = take((size_t)rows * ((c.vocab + 63) / 64) * sizeof(float2));
    L.z_tgt = take((size_t)rows * 4);
    L.max_blocks = rows / 32 + c.max_batch;
    L.blocks = take((size_t)L.max_blocks * sizeof(int4));
    L.total = off;
    return L;
}

static int validate_cfg(const rl_model_cfg* c) {
    if (!c) return fail(RL_EINVAL, "cfg is NULL");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 || c->vocab < 2)
        return fail(RL_EINVAL, "non-positive model dimension");
    if (c->n_q_heads % c->n_kv_heads != 0) return fail(RL_EINVAL, "n_q_heads %% n_kv_heads != 0");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(RL_EINVAL, "head_dim must be 64 or 128");
    if (c->d_model % 64 != 0 || c->d_ffn % 64 != 0) return fail(RL_EINVAL, "d_model and d_ffn must be multiples of 64");
    if (c->dtype != RL_FP32 && c->dtype != RL_BF16) return fail(RL_EINVAL, "dtype must be RL_FP32 or RL_BF16");
    if (c->page_tokens != 16) return fail(RL_EINVAL, "page_tokens must be 16");
    if (c->max_batch < 1 || c->max_batch > 4096) return fail(RL_EINVAL, "max_batch out of range [1, 4096]");
    if (c->max_seq < 2 || c->max_seq > 65536) return fail(RL_EINVAL, "max_seq out of range [2, 65536]");
    if (c->max_chunk_tokens < c->max_seq) return fail(RL_EINVAL, "max_chunk_tokens < max_seq");
    if (c->n_pages < 1) return fail(RL_EINVAL, "n_pages < 1");
    if (!(c->rope_base > 1.0f) || !(c->rms_eps >= 0.0f)) return fail(RL_EINVAL, "bad rope_base / rms_eps");
    return RL_OK;
}

// ---------------------------------------------------------------- context
struct WeightsHost {
    const void *tok_embed = nullptr, *final_norm = nullptr, *lm_head = nullptr;
    std::vector<const void*> attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down;
    int location = 0;            // 0: device pointers; 1: host pointers, streamed through `staging`
    char* staging = nullptr;     // dev
    size_t staging_bytes = 0;
    char* fp16_copy = nullptr;   // dev, optional (policy only)
    size_t fp16_copy_bytes = 0;
};

static int copy_weights(const rl_model_cfg& c, const rl_weights* w, WeightsHost& out, const char* what,
                        bool allow_host = false) {
    if (!w) return fail(RL_EINVAL, "%s weights are NULL", what);
    if (w->location != 0 && !(allow_host && w->location == 1))
        return fail(RL_EINVAL, "%s weights: location %d not supported here (0 = device%s)", what, w->location,
                    allow_host ? ", 1 = host, streamed" : "; host-resident weights only in score_logprobs_kl");
    out.location = w->location;
    out.staging = (char*)w->staging;
    out.staging_bytes = w->staging_bytes;
    out.fp16_copy = (char*)w->fp16_copy;
    out.fp16_copy_bytes = w->fp16_copy_bytes;
    if (!w->tok_embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
        !w->w_gate_up || !w->w_down)
        return fail(RL_EINVAL, "%s weights: NULL member", what);
    out.tok_embed = w->tok_embed;
    out.final_norm = w->final_norm;
    out.lm_head = w->lm_head;
    auto cp = [&](std::vector<const void*>& v, const void* const* src) {
        v.assign(src, src + c.n_layers);
        for (auto p : v)
            if (!p) return false;
        return true;
    };
    if (!cp(out.attn_norm, w->attn_norm) || !cp(out.wqkv, w->wqkv) || !cp(out.wo, w->wo) ||
        !cp(out.ffn_norm, w->ffn_norm) || !cp(out.w_gate_up, w->w_gate_up) || !cp(out.w_down, w->w_down))
        return fail(RL_EINVAL, "%s weights: NULL layer pointer", what);
    return RL_OK;
}

struct ProfRec { hipEvent_t a, b; };
static const size_t kProfCap = 8192;

struct rl_ctx {
    rl_model_cfg cfg;
    Layout L;
    char* ws = nullptr;
    void* pool = nullptr;
    WeightsHost policy;
    KvGeom geo;
    int impl = 0;
    int precise = 0;                 // layers [0, precise) carry fp16-pair activations (tuned path only)
    int big_mode = 1;                // GemmArgs::big_mode of every tuned GEMM
    // optional fp16 copy of the policy's matrices for the decode GEMMs (caller's buffer): bf16 pointer -> copy
    std::unordered_map<const void*, const void*> shadow_of;
    // fp16 copy of one more weight set (the frozen reference): built when a set with rl_weights.fp16_copy is first
    // scored, kept while the same set (its first matrix) and the same buffer come back
    std::unordered_map<const void*, const void*> other_shadow_of;
    const void* other_key = nullptr;
    const void* other_buf = nullptr;
    // host-resident weight sets (scoring only): copies run on a stream of the library's own
    hipStream_t copy_stream = nullptr;
    hipEvent_t ev_begin = nullptr, ev_glob_copied = nullptr, ev_glob_free = nullptr;
    hipEvent_t ev_copied[2] = {nullptr, nullptr}, ev_free[2] = {nullptr, nullptr};
    // a policy uploaded from host memory by rollout_set_policy: its copies (and the rebuild of the fp16 copy) run on
    // copy_stream; every call that reads the policy first makes its stream wait for ev_policy
    hipEvent_t ev_policy = nullptr;
    bool policy_pending = false;
    // sequences
    int B = 0;                       // live sequences (0 = no prefill yet)
    std::vector<int> cached;         // tokens in the KV cache per slot (host mirror of seq_len; an upper bound in queue mode)
    std::vector<int> cap;            // queue mode: most tokens slot b's cache will ever hold (0 = classic mode: max_seq, checked)
    std::vector<char> parked;        // queue mode: slot is free or known to have finished: no pages, no growth
    std::vector<std::vector<int>> pages;
    std::vector<int> free_pages;
    // captured decode step (rollout_generate on a non-default stream, tuned kernels)
    struct GraphKey {
        int B, G, impl, eos;
        const void *out_ids, *out_logp;
        uint64_t seed;
        int64_t base;
        float temp;
        hipStream_t s;
        const void* out_len = nullptr;   // non-null: queue mode (per-slot output rows, ids, limits)
        bool operator==(const GraphKey& o) const {
            return B == o.B && G == o.G && impl == o.impl && eos == o.eos && out_ids == o.out_ids &&
                   out_logp == o.out_logp && seed == o.seed && base == o.base && temp == o.temp && s == o.s &&
                   out_len == o.out_len;
        }
    } gkey{};
    hipGraphExec_t gexec = nullptr;
    bool use_graph = true;
    bool fused_sample = true;        // decode LM head emits block statistics instead of logits (tuned path)
    bool fused_qkv = true;           // decode attention sums, rotates and appends the QKV projection's partial rows itself
    // captured steps that may still be running when the policy is swapped without waiting: destroyed once the
    // event recorded behind their last launch has completed
    struct Retired { hipGraphExec_t g; hipEvent_t ev; };
    std::vector<Retired> retired;
    // profiling
    int prof_on[RL_K_COUNT] = {};       // 0 off, n >= 1: time every n-th launch
    uint64_t prof_seen[RL_K_COUNT] = {};
    std::vector<ProfRec> prof[RL_K_COUNT];
    size_t prof_used[RL_K_COUNT] = {};

    template <typename T> T* at(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

struct ProfScope {
    rl_ctx* c; int k; hipStream_t s; ProfRec* r = nullptr;
    ProfScope(rl_ctx* c_, int k_, hipStream_t s_) : c(c_), k(k_), s(s_) {
        if (!c->prof_on[k]) return;
        if ((c->prof_seen[k]++ % (uint64_t)c->prof_on[k]) != 0 || c->prof_used[k] >= kProfCap) return;
        if (c->prof_used[k] >= c->prof[k].size()) {
            ProfRec nr;
            if (hipEventCreate(&nr.a) != hipSuccess) return;
            if (hipEventCreate(&nr.b) != hipSuccess) { (void)hipEventDestroy(nr.a); return; }
            c->prof[k].push_back(nr);
        }
        r = &c->prof[k][c->prof_used[k]++];
        (void)hipEventRecord(r->a, s);
    }
    ~ProfScope() { if (r) (void)hipEventRecord(r->b, s); }
};

// ---------------------------------------------------------------- page allocator (host)
static void release_all_pages(rl_ctx* c) {
    c->free_pages.clear();
    for (int64_t p = c->cfg.n_pages - 1; p >= 0; --p) c->free_pages.push_back((int)p);
    for (auto& v : c->pages) v.clear();
    std::fill(c->cached.begin(), c->cached.end(), 0);
    std::fill(c->cap.begin(), c->cap.end(), 0);
    std::fill(c->parked.begin(), c->parked.end(), 0);
}

static void release_slot_pages(rl_ctx* c, int b) {
    for (int p : c->pages[b]) c->free_pages.push_back(p);
    c->pages[b].clear();
    c->cached[b] = 0;
}

// Make sure every live slot b can hold need[b] tokens; new block-table entries are pushed to the device.
static int ensure_pages(rl_ctx* c, const std::vector<int>& need, hipStream_t s) {
    const int PT = c->cfg.page_tokens;
    size_t want = 0;
    for (int b = 0; b < (int)need.size(); ++b) {
        size_t np = (size_t)(need[b] + PT - 1) / PT;
        if (np > c->pages[b].size()) want += np - c->pages[b].size();
    }
    if (want == 0) return RL_OK;
    if (want > c->free_pages.size())
        return fail(RL_ENOMEM_PAGES, "KV page pool exhausted: need %zu more pages, %zu free", want, c->free_pages.size());
    std::vector<int> triples;
    triples.reserve(want * 3);
    for (int b = 0; b < (int)need.size(); ++b) {
        size_t np = (size_t)(need[b] + PT - 1) / PT;
        while (c->pages[b].size() < np) {
            int p = c->free_pages.back();
            c->free_pages.pop_back();
            triples.push_back(b);
            triples.push_back((int)c->pages[b].size());
            triples.push_back(p);
            c->pages[b].push_back(p);
        }
    }
    k_set_pages(c->at<int>(c->L.block_table), c->L.mpps, triples.data(), (int)triples.size() / 3, s);
    return RL_OK;
}

// ---------------------------------------------------------------- GEMM dispatch
static void gemm(rl_ctx* c, int cls, int epi, const void* A, int lda, const void* W, const void* W2, int M, int N, int K,
                 float* outF, void* outT, int ldc, hipStream_t s) {
    ProfScope ps(c, cls, s);
    k_gemm_simple(c->cfg.dtype, epi, A, lda, W, W2, M, N, K, outF, outT, ldc, s);
}

// ---------------------------------------------------------------- decoder layers on n packed tokens
// Inputs: x (fp32 residual stream) filled by the embedding, tok_pos / tok_slot descriptors.
// paged = attention reads the paged cache (decode); else the chunk's own contiguous K/V.
// write_pages = append K/V of these tokens to the paged cache.
// Returns true when h already holds RMSNorm(x; final_norm) (the tuned decode path fuses it).
// qkv_part (decode, tuned kernels, plain layers): the QKV projection's split-K partial rows, which the attention
// kernel then consumes itself instead of reading rotated queries and an already appended cache.
static void attention(rl_ctx* c, int l, int n, bool paged, int max_ctx, int nblocks, hipStream_t s,
                      const float* qkv_part = nullptr, int qkv_nsplit = 0, int64_t qkv_split_stride = 0) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    ProfScope ps(c, paged ? RL_K_ATTN_DECODE : RL_K_ATTN_PREFILL, s);
    const int sp = c->impl == 1 && l < c->precise;
    if (paged && c->impl == 1) {
        DecodeAttnArgs a;
        a.q = c->at<f16_t>(L.q); a.pool = (const f16_t*)c->pool; a.block_table = c->at<int>(L.block_table);
        a.tok_pos = c->at<int>(L.tok_pos); a.out = c->at<f16_t>(L.attn); a.part_o = c->at<float>(L.attn_part);
        a.part_ml = c->at<float>(L.attn_ml); a.mpps = L.mpps; a.layer = l; a.Hq = m.n_q_heads; a.Hkv = m.n_kv_heads;
        a.scale = 1.0f / sqrtf((float)m.head_dim); a.geo = c->geo;
        a.split = sp; a.layer_lo = m.n_layers + l;
        if (qkv_part) {
            a.qkv_part = qkv_part; a.qkv_nsplit = qkv_nsplit; a.qkv_split_stride = qkv_split_stride;
            a.rope = c->at<float2>(L.rope); a.pool_w = (f16_t*)c->pool;
        }
        // the split count is a property of the context (most sequences, longest sequence), never of the live batch:
        // a row's reduction order, and with it its bits, must not depend on its batch-mates
        int nsplit = (1024 + m.max_batch * m.n_kv_heads - 1) / (m.max_batch * m.n_kv_heads);
        nsplit = std::max(1, std::min(std::min(nsplit, kMaxAttnSplits), std::max(1, L.mpps / 8)));
        k_attn_decode(a, n, nsplit, s);
        return;
    }
    if (!paged && c->impl == 1) {
        PrefillAttnArgs a;
        a.q = c->at<f16_t>(L.q); a.k = c->at<f16_t>(L.kbuf); a.vT = c->at<f16_t>(L.vbuf); a.out = c->at<f16_t>(L.attn);
        a.blocks = c->at<int4>(L.blocks); a.Hq = m.n_q_heads; a.Hkv = m.n_kv_heads; a.hd = m.head_dim;
        a.vt_cap = L.vt_cap; a.scale = 1.0f / sqrtf((float)m.head_dim);
        a.split = sp;
        k_attn_prefill(a, nblocks, s);
        return;
    }
    k_attn_simple(m.dtype, c->at<char>(L.q), paged ? nullptr : c->at<char>(L.kbuf), paged ? nullptr : c->at<char>(L.vbuf),
                  paged ? c->pool : nullptr, l, c->geo, c->at<int>(L.block_table), L.mpps, c->at<int>(L.tok_pos),
                  c->at<int>(L.tok_slot), c->at<char>(L.attn), n, m.n_q_heads, max_ctx, s);
}

static bool run_layers_plain(rl_ctx* c, const WeightsHost& W, int n, bool paged, bool write_pages, int max_ctx,
                             int nblocks, hipStream_t s, float* x, int l0, int l1) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    const int dt = m.dtype;
    const size_t e = esz_of(dt);
    const int qd = m.n_q_heads * m.head_dim;
    void* h = c->at<char>(L.h);
    float* qkv = c->at<float>(L.qkv);
    void* q = c->at<char>(L.q);
    void* kb = c->at<char>(L.kbuf);
    void* vb = c->at<char>(L.vbuf);
    void* att = c->at<char>(L.attn);
    void* ffn = c->at<char>(L.ffn);
    const int* tpos = c->at<int>(L.tok_pos);
    const int* tslot = c->at<int>(L.tok_slot);
    const int* bt = c->at<int>(L.block_table);
    const float2* rope = c->at<float2>(L.rope);
    const int gcls = paged ? RL_K_GEMM_DECODE : RL_K_GEMM_PREFILL;
    for (int l = l0; l < l1; ++l) {
        k_rmsnorm(dt, x, W.attn_norm[l], h, n, m.d_model, m.rms_eps, s);
        gemm(c, gcls, EPI_STORE_F32, h, m.d_model, W.wqkv[l], nullptr, n, L.nqkv, m.d_model, qkv, nullptr, L.nqkv, s);
        k_rope_append(dt, qkv, 1, 0, n, tpos, tslot, rope, q, paged ? nullptr : kb, paged ? nullptr : vb,
                      write_pages ? c->pool : nullptr, l, c->geo, bt, L.mpps, m.n_q_heads, s);
        attention(c, l, n, paged, max_ctx, nblocks, s);
        gemm(c, gcls, EPI_RESID, att, qd, W.wo[l], nullptr, n, m.d_model, qd, x, nullptr, m.d_model, s);
        k_rmsnorm(dt, x, W.ffn_norm[l], h, n, m.d_model, m.rms_eps, s);
        const char* wg = (const char*)W.w_gate_up[l];
        gemm(c, gcls, EPI_SWIGLU, h, m.d_model, wg, wg + (size_t)m.d_ffn * m.d_model * e, n, m.d_ffn, m.d_model,
             nullptr, ffn, m.d_ffn, s);
        gemm(c, gcls, EPI_RESID, ffn, m.d_ffn, W.w_down[l], nullptr, n, m.d_model, m.d_ffn, x, nullptr, m.d_model, s);
    }
    return false;
}

static void mfma(rl_ctx* c, int cls, int epi, const GemmArgs& a0, int splits, hipStream_t s) {
    ProfScope ps(c, cls, s);
    GemmArgs a = a0;
    a.big_mode = c->big_mode;
    auto copy_of = [&](const void* w) -> const void* {
        auto it = c->shadow_of.find(w);
        if (it != c->shadow_of.end()) return it->second;
        it = c->other_shadow_of.find(w);
        return it != c->other_shadow_of.end() ? it->second : nullptr;
    };
    if (cls == RL_K_GEMM_DECODE && a.M <= 128 && (epi == MG_STORE_F32 || epi == MG_SWIGLU || epi == MG_SAMPLE) &&
        k_gemm_decode_supported(epi, a.N, a.K)) {
        if (const void* h = copy_of((const void*)a.W)) { a.W = (const bf16_t*)h; a.w_f16 = 1; }
        k_gemm_decode(epi, a, splits, s);
    } else {
        if (k_gemm_mfma_reads_f16_copy(epi, a, splits))
            if (const void* h = copy_of((const void*)a.W)) { a.W = (const bf16_t*)h; a.w_f16 = 1; }
        k_gemm_mfma(epi, a, splits, s);
    }
}

// Split count for a decode GEMM of n rows with N output columns: one 8-wave workgroup per CU and 128-column
// tiles, so aim for as many workgroups as fit in one round of 256 CUs.  Returns the number of partial
// buffers the kernel that mfma() picks for this shape will actually write.
static int decode_splits(int n, int N, int K) {
    int want = std::max(1, 256 / std::max(1, N / 128));
    want = std::min(want, kMaxSplitK);
    if (n <= 128 && k_gemm_decode_supported(MG_STORE_F32, N, K)) return k_gemm_decode_splits_used(K, want);
    return k_gemm_mfma_splits_used(K, want);
}

// bf16 weights / fp16 activations on the MFMA kernels.
static bool run_layers_fast(rl_ctx* c, const WeightsHost& W, int n, bool paged, bool write_pages, int max_ctx,
                            int nblocks, hipStream_t s, float* x, int l0, int l1) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    const int qd = m.n_q_heads * m.head_dim;
    f16_t* h = c->at<f16_t>(L.h);
    f16_t* q = c->at<f16_t>(L.q);
    f16_t* kb = c->at<f16_t>(L.kbuf);
    f16_t* vb = c->at<f16_t>(L.vbuf);
    f16_t* att = c->at<f16_t>(L.attn);
    f16_t* ffn = c->at<f16_t>(L.ffn);
    float* part = c->at<float>(L.splitk);
    const int* tpos = c->at<int>(L.tok_pos);
    const int* tslot = c->at<int>(L.tok_slot);
    const int* bt = c->at<int>(L.block_table);
    const float2* rope = c->at<float2>(L.rope);
    const int gcls = paged ? RL_K_GEMM_DECODE : RL_K_GEMM_PREFILL;
    // A precise layer (index below c->precise) reads and writes its activations as fp16 pairs: the GEMMs see
    // [hi | lo] rows of twice the width whose k index wraps on the weights' side, the fp16-producing epilogues
    // and the norm kernels write pairs, and attention works on pairs (the lo planes of the cache are layer
    // n_layers + l of the pool).
    auto pair_in = [](GemmArgs& g, int width, int sp) {   // A operand of `width` columns, pairs if sp
        g.lda = sp ? 2 * width : width;
        g.K = g.lda;
        g.Kw = width;
    };
    if (paged) k_rmsnorm(1, x, W.attn_norm[l0], h, n, m.d_model, m.rms_eps, s, l0 < c->precise);
    for (int l = l0; l < l1; ++l) {
        const int sp = l < c->precise, sp_next = l + 1 < c->precise && l + 1 < m.n_layers;
        GemmArgs g;
        g.M = n;
        if (paged) {
            // weight-streaming GEMMs, split over K; consumers reduce the partial sums
            g.A = h; pair_in(g, m.d_model, sp); g.W = (const bf16_t*)W.wqkv[l]; g.N = L.nqkv;
            g.outF = part; g.ldc = L.nqkv; g.split_stride = (int64_t)n * L.nqkv;
            int ks = decode_splits(n, L.nqkv, g.K);
            mfma(c, gcls, MG_STORE_F32, g, ks, s);
            // plain layers on the tuned kernels: attention is the consumer of the partial sums (a decode row's cache
            // slot is its row index, which is what that kernel assumes)
            const bool fuse = c->fused_qkv && c->impl == 1 && !sp &&
                              k_attn_decode_consumes_qkv(m.n_q_heads, m.n_kv_heads, m.head_dim);
            if (!fuse)
                k_rope_append_split(1, part, ks, g.split_stride, n, tpos, tslot, rope, q, c->pool, l, c->geo, bt, L.mpps,
                                    m.n_q_heads, s, sp, m.n_layers + l);
            attention(c, l, n, true, max_ctx, 0, s, fuse ? part : nullptr, ks, g.split_stride);
            g = GemmArgs();
            g.M = n; g.A = att; pair_in(g, qd, sp); g.W = (const bf16_t*)W.wo[l]; g.N = m.d_model;
            g.outF = part; g.ldc = m.d_model; g.split_stride = (int64_t)n * m.d_model;
            ks = decode_splits(n, m.d_model, g.K);
            mfma(c, gcls, MG_STORE_F32, g, ks, s);
            k_resid_norm(1, x, part, ks, g.split_stride, W.ffn_norm[l], h, n, m.d_model, m.rms_eps, s, sp);
            g = GemmArgs();
            g.M = n; g.A = h; pair_in(g, m.d_model, sp); g.W = (const bf16_t*)W.w_gate_up[l]; g.N = m.d_ffn;
            g.up_offset = m.d_ffn; g.outH = ffn; g.ldc = sp ? 2 * m.d_ffn : m.d_ffn; g.split_out = sp;
            mfma(c, gcls, MG_SWIGLU, g, 1, s);
            g = GemmArgs();
            g.M = n; g.A = ffn; pair_in(g, m.d_ffn, sp); g.W = (const bf16_t*)W.w_down[l]; g.N = m.d_model;
            g.outF = part; g.ldc = m.d_model; g.split_stride = (int64_t)n * m.d_model;
            ks = decode_splits(n, m.d_model, g.K);
            mfma(c, gcls, MG_STORE_F32, g, ks, s);
            const void* next = (l + 1 < m.n_layers) ? W.attn_norm[l + 1] : W.final_norm;
            k_resid_norm(1, x, part, ks, g.split_stride, next, h, n, m.d_model, m.rms_eps, s, sp_next);
        } else {
            k_rmsnorm(1, x, W.attn_norm[l], h, n, m.d_model, m.rms_eps, s, sp);
            g.A = h; pair_in(g, m.d_model, sp); g.W = (const bf16_t*)W.wqkv[l]; g.N = L.nqkv;
            g.tok_pos = tpos; g.tok_slot = tslot; g.rope = rope; g.q_out = q; g.k_out = kb; g.v_out = vb;
            g.pool = write_pages ? (f16_t*)c->pool : nullptr; g.block_table = bt; g.mpps = L.mpps; g.layer = l;
            g.Hq = m.n_q_heads; g.Hkv = m.n_kv_heads; g.hd = m.head_dim; g.geo = c->geo; g.vt_cap = L.vt_cap;
            g.split_out = sp; g.layer_lo = m.n_layers + l;
            mfma(c, gcls, MG_QKV, g, 1, s);
            attention(c, l, n, false, max_ctx, nblocks, s);
            g = GemmArgs();
            g.M = n; g.A = att; pair_in(g, qd, sp); g.W = (const bf16_t*)W.wo[l]; g.N = m.d_model;
            g.outF = x; g.ldc = m.d_model;
            mfma(c, gcls, MG_RESID, g, 1, s);
            k_rmsnorm(1, x, W.ffn_norm[l], h, n, m.d_model, m.rms_eps, s, sp);
            g = GemmArgs();
            g.M = n; g.A = h; pair_in(g, m.d_model, sp); g.W = (const bf16_t*)W.w_gate_up[l]; g.N = m.d_ffn;
            g.up_offset = m.d_ffn; g.outH = ffn; g.ldc = sp ? 2 * m.d_ffn : m.d_ffn; g.split_out = sp;
            mfma(c, gcls, MG_SWIGLU, g, 1, s);
            g = GemmArgs();
            g.M = n; g.A = ffn; pair_in(g, m.d_ffn, sp); g.W = (const bf16_t*)W.w_down[l]; g.N = m.d_model;
            g.outF = x; g.ldc = m.d_model;
            mfma(c, gcls, MG_RESID, g, 1, s);
        }
    }
    return paged;
}

// Layers [l0, l1) (default: all) on the n packed rows whose residual stream is x (default: the workspace's).
static bool run_layers(rl_ctx* c, const WeightsHost& W, int n, bool paged, bool write_pages, int max_ctx,
                       int nblocks, hipStream_t s, float* x = nullptr, int l0 = 0, int l1 = -1) {
    if (!x) x = c->at<float>(c->L.x);
    if (l1 < 0) l1 = c->cfg.n_layers;
    if (c->impl == 1) return run_layers_fast(c, W, n, paged, write_pages, max_ctx, nblocks, s, x, l0, l1);
    return run_layers_plain(c, W, n, paged, write_pages, max_ctx, nblocks, s, x, l0, l1);
}

// LM head on rows [0, nr) of h: logits fp32 [nr, V]
static void lm_head_logits(rl_ctx* c, int cls, const WeightsHost& W, const void* hrows, int nr, hipStream_t s) {
    const rl_model_cfg& m = c->cfg;
    if (c->impl == 1) {
        GemmArgs g;
        g.M = nr; g.A = (const f16_t*)hrows; g.lda = m.d_model; g.W = (const bf16_t*)W.lm_head; g.N = m.vocab;
        g.K = m.d_model; g.outF = c->at<float>(c->L.logits); g.ldc = m.vocab;
        mfma(c, cls, MG_STORE_F32, g, 1, s);
    } else {
        gemm(c, cls, EPI_STORE_F32, hrows, m.d_model, W.lm_head, nullptr, nr, m.vocab, m.d_model,
             c->at<float>(c->L.logits), nullptr, m.vocab, s);
    }
}

static bool fast_path_supported(const rl_model_cfg& m) {
    if (m.dtype != RL_BF16 || m.d_model > 8192 || m.n_q_heads / m.n_kv_heads > 8) return false;
    const int nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim, qd = m.n_q_heads * m.head_dim;
    return k_gemm_mfma_supported(MG_QKV, nqkv, m.d_model, m.head_dim) &&
           k_gemm_mfma_supported(MG_STORE_F32, m.d_model, qd, m.head_dim) &&
           k_gemm_mfma_supported(MG_SWIGLU, m.d_ffn, m.d_model, m.head_dim) &&
           k_gemm_mfma_supported(MG_STORE_F32, m.d_model, m.d_ffn, m.head_dim) &&
           k_gemm_mfma_supported(MG_STORE_F32, m.vocab, m.d_model, m.head_dim);
}

// A pass works on whole sequences packed into one token list.  On the tuned path every sequence
// starts at a multiple of 32 rows (the MFMA attention walks 32-key blocks) and the padding rows
// are marked; the plain path packs densely.
struct Chunk {
    std::vector<int> rows_b, starts, lens, full;
    std::vector<int> slots;   // cache slot of each row; empty = the row index itself
    int n = 0;          // rows in the list, padding included
    int max_ctx = 1;
    int nblocks = 0;    // 32-query blocks (tuned path)
};
static int pack_align(const rl_ctx* c) { return c->impl == 1 ? 32 : 1; }

// Take sequences b0.. while they fit; returns the first sequence not taken.
static int chunk_take(const rl_ctx* c, const std::vector<int>& len_of, int b0, int B, Chunk& ch) {
    const int al = pack_align(c);
    int b1 = b0;
    while (b1 < B) {
        int alen = (len_of[b1] + al - 1) / al * al;
        if (ch.n + alen > c->cfg.max_chunk_tokens && ch.n > 0) break;
        ch.rows_b.push_back(b1);
        ch.starts.push_back(ch.n);
        ch.lens.push_back(len_of[b1]);
        ch.full.push_back(len_of[b1]);
        ch.n += alen;
        ch.max_ctx = std::max(ch.max_ctx, len_of[b1]);
        ++b1;
    }
    return b1;
}

// Upload a chunk's row descriptors and build the packed token arrays on the device.
static int pack_chunk(rl_ctx* c, const int* ids, int ld_ids, Chunk& ch, bool targets, hipStream_t s) {
    const Layout& L = c->L;
    const size_t nb = ch.rows_b.size() * sizeof(int);
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.seq_first), ch.rows_b.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.row_start), ch.starts.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.row_len), ch.lens.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.full_len), ch.full.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.row_slot), (ch.slots.empty() ? ch.rows_b : ch.slots).data(), nb,
                           hipMemcpyHostToDevice, s));
    std::vector<int4> blocks;
    if (c->impl == 1) {
        // one workgroup per 32-query block; long (late) blocks first so the tail of the grid is short work
        int maxqb = 0;
        for (int len : ch.lens) maxqb = std::max(maxqb, (len + 31) / 32);
        for (int qb = maxqb - 1; qb >= 0; --qb)
            for (size_t r = 0; r < ch.lens.size(); ++r)
                if (qb < (ch.lens[r] + 31) / 32) blocks.push_back(make_int4(ch.starts[r], ch.lens[r], qb, 0));
        ch.nblocks = (int)blocks.size();
        if (ch.nblocks > L.max_blocks) return fail(RL_EINVAL, "internal: attention block list overflow");
        if (ch.nblocks)
            HIP_TRY(hipMemcpyAsync(c->at<int4>(L.blocks), blocks.data(), blocks.size() * sizeof(int4),
                                   hipMemcpyHostToDevice, s));
    }
    // the host vectors may be reused by the caller right after this returns
    HIP_TRY(hipStreamSynchronize(s));
    k_pack_tokens(ids, ld_ids, c->at<int>(L.seq_first), c->at<int>(L.row_slot), c->at<int>(L.row_start),
                  c->at<int>(L.row_len), c->at<int>(L.full_len), pack_align(c), c->at<int>(L.tok_ids), c->at<int>(L.tok_pos),
                  c->at<int>(L.tok_slot), targets ? c->at<int>(L.tok_tgt) : nullptr, (int)ch.rows_b.size(), s);
    return RL_OK;
}

// ---------------------------------------------------------------- fp16 copy of the policy for the decode GEMMs
// The decode GEMMs are bound by how fast a CU can pull weights, and the bf16 -> fp16 conversion they do next
// to the MFMAs costs them about a tenth of that rate (30 % on the LM head).  With a caller-provided buffer of
// the policy's size the conversion is done once per weight update instead of once per token.
static size_t shadow_bytes_of(const rl_model_cfg& c) {
    if (c.dtype != RL_BF16) return 0;
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    const size_t d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim;
    const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const size_t layer = al(nqkv * d * 2) + al(d * qd * 2) + al(2 * (size_t)c.d_ffn * d * 2) + al(d * (size_t)c.d_ffn * 2);
    return layer * c.n_layers + al((size_t)c.vocab * d * 2);
}

// (Re)builds the copy from the current values of c->policy on stream s.  No-op without a buffer.
static int build_shadow(rl_ctx* c, hipStream_t s) {
    c->shadow_of.clear();
    const rl_model_cfg& m = c->cfg;
    const WeightsHost& W = c->policy;
    if (!W.fp16_copy || m.dtype != RL_BF16 || W.location != 0) return RL_OK;
    if (W.fp16_copy_bytes < shadow_bytes_of(m))
        return fail(RL_ENOSPACE, "policy fp16 copy: %zu bytes given, %zu needed", W.fp16_copy_bytes, shadow_bytes_of(m));
    if (((uintptr_t)W.fp16_copy & 255) != 0) return fail(RL_EINVAL, "policy fp16 copy buffer must be 256-byte aligned");
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    const size_t d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim;
    const size_t nqkv = (size_t)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    char* p = W.fp16_copy;
    auto put = [&](const void* src, size_t elems) {
        k_bf16_to_f16(src, p, (int64_t)elems, s);
        c->shadow_of[src] = p;
        p += al(elems * 2);
    };
    for (int l = 0; l < m.n_layers; ++l) {
        put(W.wqkv[l], nqkv * d);
        put(W.wo[l], d * qd);
        put(W.w_gate_up[l], 2 * (size_t)m.d_ffn * d);
        put(W.w_down[l], d * (size_t)m.d_ffn);
    }
    put(W.lm_head, (size_t)m.vocab * d);
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

// The same for a weight set that is not the context's policy (the reference of a scoring call), on the caller's
// stream, once per (set, buffer) pair.
static int ensure_other_shadow(rl_ctx* c, const WeightsHost& W, hipStream_t s) {
    const rl_model_cfg& m = c->cfg;
    if (!W.fp16_copy || m.dtype != RL_BF16 || W.location != 0 || c->impl != 1) return RL_OK;
    if (!W.wqkv.empty() && c->shadow_of.count(W.wqkv[0])) return RL_OK;      // this is the context's policy: it has its copy
    if (c->other_key == W.wqkv[0] && c->other_buf == W.fp16_copy) return RL_OK;
    if (W.fp16_copy_bytes < shadow_bytes_of(m))
        return fail(RL_ENOSPACE, "fp16 copy: %zu bytes given, %zu needed", W.fp16_copy_bytes, shadow_bytes_of(m));
    if (((uintptr_t)W.fp16_copy & 255) != 0) return fail(RL_EINVAL, "fp16 copy buffer must be 256-byte aligned");
    c->other_shadow_of.clear();
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    const size_t d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim;
    const size_t nqkv = (size_t)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
    char* p = W.fp16_copy;
    auto put = [&](const void* src, size_t elems) {
        k_bf16_to_f16(src, p, (int64_t)elems, s);
        c->other_shadow_of[src] = p;
        p += al(elems * 2);
    };
    for (int l = 0; l < m.n_layers; ++l) {
        put(W.wqkv[l], nqkv * d);
        put(W.wo[l], d * qd);
        put(W.w_gate_up[l], 2 * (size_t)m.d_ffn * d);
        put(W.w_down[l], d * (size_t)m.d_ffn);
    }
    put(W.lm_head, (size_t)m.vocab * d);
    HIP_TRY(hipGetLastError());
    c->other_key = W.wqkv[0];
    c->other_buf = W.fp16_copy;
    return RL_OK;
}

static int ensure_copy_stream(rl_ctx* c);

// Put the captured decode step aside (its launches may still be in flight on the stream it was captured on).
static void retire_graph(rl_ctx* c) {
    if (!c->gexec) return;
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) == hipSuccess && hipEventRecord(ev, c->gkey.s) == hipSuccess) {
        c->retired.push_back({c->gexec, ev});
    } else {
        if (ev) (void)hipEventDestroy(ev);
        (void)hipStreamSynchronize(c->gkey.s);
        (void)hipGraphExecDestroy(c->gexec);
    }
    c->gexec = nullptr;
}
// Destroy the retired steps whose work has completed (all of them, after waiting, with force).
static void reap_graphs(rl_ctx* c, bool force) {
    for (size_t i = 0; i < c->retired.size();) {
        if (force) (void)hipEventSynchronize(c->retired[i].ev);
        if (force || hipEventQuery(c->retired[i].ev) == hipSuccess) {
            (void)hipGraphExecDestroy(c->retired[i].g);
            (void)hipEventDestroy(c->retired[i].ev);
            c->retired.erase(c->retired.begin() + i);
        } else {
            (void)hipGetLastError();
            ++i;
        }
    }
}

// Bytes of a device-resident copy of a whole weight set (every tensor 256-byte aligned).
static size_t resident_bytes_of(const rl_model_cfg& c) {
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    const size_t e = esz_of(c.dtype), d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim;
    const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    const size_t layer = 2 * al(d * e) + al(nqkv * d * e) + al(d * qd * e) + al(2 * (size_t)c.d_ffn * d * e) +
                         al(d * (size_t)c.d_ffn * e);
    return 2 * al((size_t)c.vocab * d * e) + al(d * e) + layer * c.n_layers;
}

// Make stream s wait for a policy upload that may still be running on the copy stream.
static int wait_policy(rl_ctx* c, hipStream_t s) {
    if (!c->policy_pending) return RL_OK;
    if (hipEventQuery(c->ev_policy) == hipSuccess) { c->policy_pending = false; return RL_OK; }
    (void)hipGetLastError();   // hipErrorNotReady is not an error
    HIP_TRY(hipStreamWaitEvent(s, c->ev_policy, 0));
    return RL_OK;
}

// ---------------------------------------------------------------- C ABI
extern "C" {

const char* rollout_last_error(void) { return g_err; }

size_t rollout_workspace_bytes(const rl_model_cfg* cfg) {
    if (validate_cfg(cfg) != RL_OK) return 0;
    return make_layout(*cfg).total;
}

size_t rollout_weight_shadow_bytes(const rl_model_cfg* cfg) {
    if (validate_cfg(cfg) != RL_OK) return 0;
    return shadow_bytes_of(*cfg);
}

size_t rollout_weight_resident_bytes(const rl_model_cfg* cfg) {
    if (validate_cfg(cfg) != RL_OK) return 0;
    return resident_bytes_of(*cfg);
}

size_t rollout_kv_pool_bytes(const rl_model_cfg* cfg) {
    if (validate_cfg(cfg) != RL_OK) return 0;
    // the precise layers keep a second plane (the lo halves of their fp16 pairs) as layers n_layers, n_layers + 1, ...
    return (size_t)(cfg->n_layers + precise_cap(*cfg)) * 2 * (size_t)cfg->n_pages * cfg->n_kv_heads *
           cfg->page_tokens * cfg->head_dim * esz_of(cfg->dtype);
}

int rollout_init(const rl_model_cfg* cfg, const rl_weights* policy, void* workspace, size_t workspace_bytes,
                 void* kv_pool, size_t kv_pool_bytes, rl_ctx** out) {
    if (!out) return fail(RL_EINVAL, "out is NULL");
    *out = nullptr;
    int rc = validate_cfg(cfg);
    if (rc) return rc;
    if (!workspace || !kv_pool) return fail(RL_EINVAL, "workspace / kv_pool is NULL");
    if (((uintptr_t)workspace & 255) || ((uintptr_t)kv_pool & 255))
        return fail(RL_EINVAL, "workspace / kv_pool must be 256-byte aligned");
    Layout L = make_layout(*cfg);
    if (workspace_bytes < L.total)
        return fail(RL_ENOSPACE, "workspace too small: %zu < %zu bytes", workspace_bytes, L.total);
    if (kv_pool_bytes < rollout_kv_pool_bytes(cfg))
        return fail(RL_ENOSPACE, "kv_pool too small: %zu < %zu bytes", kv_pool_bytes, rollout_kv_pool_bytes(cfg));
    rl_ctx* c = new (std::nothrow) rl_ctx();
    if (!c) return fail(RL_EINVAL, "out of host memory");
    c->cfg = *cfg;
    c->L = L;
    c->ws = (char*)workspace;
    c->pool = kv_pool;
    rc = copy_weights(*cfg, policy, c->policy, "policy");
    if (rc) { delete c; return rc; }
    c->geo = KvGeom{cfg->n_kv_heads, cfg->head_dim, cfg->page_tokens, cfg->n_pages};
    c->impl = fast_path_supported(*cfg) ? 1 : 0;
    c->precise = c->impl == 1 ? std::min(kDefaultPreciseLayers, precise_cap(*cfg)) : 0;
    c->cached.assign(cfg->max_batch, 0);
    c->cap.assign(cfg->max_batch, 0);
    c->parked.assign(cfg->max_batch, 0);
    c->pages.assign(cfg->max_batch, {});
    release_all_pages(c);
    hipStream_t s = nullptr;
    k_rope_table(c->at<float2>(L.rope), cfg->max_seq, cfg->head_dim, cfg->rope_base, s);
    k_fill_i32(c->at<int>(L.block_table), 0, (int64_t)cfg->max_batch * L.mpps, s);
    k_fill_i32(c->at<int>(L.errflag), 0, 64, s);
    k_fill_i32(c->at<int>(L.seq_len), 0, cfg->max_batch, s);
    k_fill_i32(c->at<int>(L.last_tok), 0, cfg->max_batch, s);
    k_fill_i32(c->at<int>(L.gen_count), 0, cfg->max_batch, s);
    k_fill_i32(c->at<int>(L.finished), 0, cfg->max_batch, s);
    k_fill_i32(c->at<int>(L.step_count), 0, cfg->max_batch, s);
    rc = build_shadow(c, s);
    if (rc) { delete c; return rc; }
    hipError_t e = hipStreamSynchronize(s);
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) {
        delete c;
        return fail(RL_EHIP, "rollout_init: %s", hipGetErrorString(e));
    }
    *out = c;
    return RL_OK;
}

void rollout_destroy(rl_ctx* c) {
    if (!c) return;
    reap_graphs(c, true);
    if (c->gexec) (void)hipGraphExecDestroy(c->gexec);
    if (c->copy_stream) {
        (void)hipStreamSynchronize(c->copy_stream);
        (void)hipStreamDestroy(c->copy_stream);
        for (hipEvent_t e : {c->ev_begin, c->ev_glob_copied, c->ev_glob_free, c->ev_copied[0], c->ev_copied[1],
                             c->ev_free[0], c->ev_free[1], c->ev_policy})
            if (e) (void)hipEventDestroy(e);
    }
    for (int k = 0; k < RL_K_COUNT; ++k)
        for (auto& r : c->prof[k]) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    delete c;
}

int rollout_reset(rl_ctx* c) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    c->B = 0;
    release_all_pages(c);
    return RL_OK;
}

int rollout_set_policy(rl_ctx* c, const rl_weights* policy) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    WeightsHost w;
    int rc = copy_weights(c->cfg, policy, w, "policy", true);
    if (rc) return rc;
    if (w.location == 1) {
        // Host-resident set: every tensor is copied into the caller's device buffer on the library's copy stream
        // (so the upload overlaps with whatever the caller's streams are still running on the old policy, whose
        // memory is not touched), and the context switches to the device copies.  Calls that read the policy make
        // their stream wait for the upload.
        const rl_model_cfg& m = c->cfg;
        if (!w.staging) return fail(RL_EINVAL, "host-resident policy needs a device buffer (rl_weights.staging)");
        if (((uintptr_t)w.staging & 255) != 0) return fail(RL_EINVAL, "policy buffer must be 256-byte aligned");
        if (w.staging_bytes < resident_bytes_of(m))
            return fail(RL_ENOSPACE, "policy buffer: %zu bytes given, %zu needed", w.staging_bytes, resident_bytes_of(m));
        if ((rc = ensure_copy_stream(c))) return rc;
        if (c->policy_pending) HIP_TRY(hipEventSynchronize(c->ev_policy));   // one upload at a time
        auto al = [](size_t b) { return (b + 255) / 256 * 256; };
        const size_t e = esz_of(m.dtype), d = m.d_model, qd = (size_t)m.n_q_heads * m.head_dim;
        const size_t nqkv = (size_t)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim;
        char* p = w.staging;
        hipStream_t cs = c->copy_stream;
        hipError_t err = hipSuccess;
        auto up = [&](const void*& ptr, size_t bytes) {
            if (err == hipSuccess) err = hipMemcpyAsync(p, ptr, bytes, hipMemcpyHostToDevice, cs);
            ptr = p;
            p += al(bytes);
        };
        up(w.tok_embed, (size_t)m.vocab * d * e);
        up(w.lm_head, (size_t)m.vocab * d * e);
        up(w.final_norm, d * e);
        for (int l = 0; l < m.n_layers; ++l) {
            up(w.attn_norm[l], d * e);
            up(w.wqkv[l], nqkv * d * e);
            up(w.wo[l], d * qd * e);
            up(w.ffn_norm[l], d * e);
            up(w.w_gate_up[l], 2 * (size_t)m.d_ffn * d * e);
            up(w.w_down[l], d * (size_t)m.d_ffn * e);
        }
        if (err != hipSuccess) return fail(RL_EHIP, "policy upload: %s", hipGetErrorString(err));
        w.location = 0;
        w.staging = nullptr;
        w.staging_bytes = 0;
        c->policy = w;
        reap_graphs(c, false);
        retire_graph(c);   // the old policy's captured step may still be replaying on the caller's stream
        rc = build_shadow(c, cs);
        if (rc) return rc;
        HIP_TRY(hipEventRecord(c->ev_policy, cs));
        c->policy_pending = true;
        return rollout_reset(c);
    }
    if (c->policy_pending) { HIP_TRY(hipEventSynchronize(c->ev_policy)); c->policy_pending = false; }
    c->policy = w;
    // the captured decode step holds the old pointers; caches built with the old weights are void
    if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
    rc = build_shadow(c, nullptr);
    if (rc) return rc;
    HIP_TRY(hipStreamSynchronize(nullptr));
    return rollout_reset(c);
}

int rollout_refresh_policy(rl_ctx* c, void* stream) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    int rcw = wait_policy(c, (hipStream_t)stream);
    if (rcw) return rcw;
    // same addresses, new values: only the fp16 copy (if there is one) has to follow; the captured step stays valid
    int rc = build_shadow(c, (hipStream_t)stream);
    if (rc) return rc;
    return rollout_reset(c);
}

int rollout_set_impl(rl_ctx* c, int32_t impl) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    if (impl < 0 || impl > 2) return fail(RL_EINVAL, "impl must be 0, 1 or 2");
    if (impl >= 1 && !fast_path_supported(c->cfg))
        return fail(RL_EINVAL, "impl 1 / 2 need bf16 weights and GEMM widths that are multiples of 128 (K of 64)");
    c->impl = impl >= 1 ? 1 : 0;
    c->big_mode = impl == 2 ? 2 : 1;
    c->precise = c->impl == 1 ? std::min(kDefaultPreciseLayers, precise_cap(c->cfg)) : 0;
    if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
    return rollout_reset(c);
}

int rollout_set_decode_tile_rows(int32_t rows) {
    k_gemm_decode_tile_above(rows);
    return RL_OK;
}

int rollout_set_large_gemm_copy(int32_t on) {
    k_gemm_big_reads_copy(on != 0);
    return RL_OK;
}

int rollout_set_precise_layers(rl_ctx* c, int32_t n) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    if (n < 0 || n > precise_cap(c->cfg))
        return fail(RL_EINVAL, "precise layers: %d outside [0, %d] for this configuration", n, precise_cap(c->cfg));
    if (n > 0 && c->impl != 1) return fail(RL_EINVAL, "precise layers need the tuned kernels (impl 1 or 2)");
    c->precise = n;
    if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
    return rollout_reset(c);
}

int rollout_set_fused_sampling(rl_ctx* c, int32_t on) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    c->fused_sample = on != 0;
    if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
    return RL_OK;
}

int rollout_set_fused_qkv_consumer(rl_ctx* c, int32_t on) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    c->fused_qkv = on != 0;
    if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
    return RL_OK;
}

int rollout_forget_fp16_copies(rl_ctx* c) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    c->other_shadow_of.clear();
    c->other_key = c->other_buf = nullptr;
    return RL_OK;
}

int rollout_check(rl_ctx* c, void* stream) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    hipStream_t s = (hipStream_t)stream;
    int flag = 0;
    HIP_TRY(hipMemcpyAsync(&flag, c->at<int>(c->L.errflag), sizeof(int), hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    HIP_TRY(hipGetLastError());
    if (flag) {
        k_fill_i32(c->at<int>(c->L.errflag), 0, 1, s);
        return fail(RL_EINVAL, "token id outside [0, vocab) was seen (clamped)");
    }
    return RL_OK;
}

int rollout_prefill(rl_ctx* c, const int32_t* prompt_ids, const int32_t* prompt_len, int32_t B, int32_t Pmax,
                    void* stream) {
    if (!c || !prompt_ids || !prompt_len) return fail(RL_EINVAL, "NULL argument");
    const rl_model_cfg& m = c->cfg;
    if (B < 1 || B > m.max_batch) return fail(RL_EINVAL, "B=%d outside [1, max_batch=%d]", B, m.max_batch);
    if (Pmax < 1) return fail(RL_EINVAL, "Pmax < 1");
    for (int b = 0; b < B; ++b)
        if (prompt_len[b] < 1 || prompt_len[b] > Pmax || prompt_len[b] > m.max_seq)
            return fail(RL_EINVAL, "prompt_len[%d]=%d outside [1, min(Pmax, max_seq)]", b, prompt_len[b]);
    hipStream_t s = (hipStream_t)stream;
    const Layout& L = c->L;
    c->B = 0;
    release_all_pages(c);
    int rcw = wait_policy(c, s);
    if (rcw) return rcw;
    std::vector<int> need(B);
    for (int b = 0; b < B; ++b) need[b] = prompt_len[b] - 1;
    int rc = ensure_pages(c, need, s);
    if (rc) { release_all_pages(c); return rc; }
    // chunks of whole sequences, at most max_chunk_tokens tokens each
    int b0 = 0;
    while (b0 < B) {
        Chunk ch;
        b0 = chunk_take(c, need, b0, B, ch);
        if (ch.n > 0) {
            rc = pack_chunk(c, prompt_ids, Pmax, ch, false, s);
            if (rc) return rc;
            k_embed(m.dtype, c->at<int>(L.tok_ids), ch.n, c->policy.tok_embed, m.d_model, m.vocab, c->at<float>(L.x),
                    c->at<int>(L.errflag), s);
            run_layers(c, c->policy, ch.n, false, true, ch.max_ctx, ch.nblocks, s);
        }
    }
    // prompt lengths to the device for the state kernel
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.d_prompt_len), prompt_len, (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    k_prefill_state(prompt_ids, Pmax, c->at<int>(L.d_prompt_len), c->at<int>(L.last_tok), c->at<int>(L.seq_len),
                    c->at<int>(L.gen_count), c->at<int>(L.finished), c->at<int>(L.step_count), B, s);
    for (int b = 0; b < B; ++b) c->cached[b] = need[b];
    c->B = B;
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

static int decode_step_impl(rl_ctx* c, const rl_sample_cfg* sample, const int32_t* tok_in, int32_t* tok_out,
                            float* logp_out, int32_t* out_ids, float* out_logp, int out_stride, hipStream_t s,
                            int32_t* queue_out_len = nullptr) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    const int B = c->B;
    std::vector<int> need(B);
    int max_ctx = 1;
    for (int b = 0; b < B; ++b) {
        if (c->parked[b]) { need[b] = c->cached[b]; continue; }
        if (c->cap[b] > 0) {
            // queue mode: the host's count is an upper bound (a row may have finished unseen); never past the row's cap
            need[b] = std::min(c->cached[b] + 1, c->cap[b]);
        } else {
            if (c->cached[b] + 1 > m.max_seq) return fail(RL_EINVAL, "sequence %d would exceed max_seq=%d", b, m.max_seq);
            need[b] = c->cached[b] + 1;
        }
        max_ctx = std::max(max_ctx, need[b]);
    }
    int rc = ensure_pages(c, need, s);
    if (rc) return rc;
    k_step_begin(tok_in, c->at<int>(L.last_tok), c->at<int>(L.seq_len), c->at<int>(L.finished), c->at<int>(L.cur_tok),
                 c->at<int>(L.tok_pos), c->at<int>(L.tok_slot), B, s);
    k_embed(m.dtype, c->at<int>(L.cur_tok), B, c->policy.tok_embed, m.d_model, m.vocab, c->at<float>(L.x),
            c->at<int>(L.errflag), s);
    if (!run_layers(c, c->policy, B, true, true, max_ctx, 0, s))
        k_rmsnorm(m.dtype, c->at<float>(L.x), c->policy.final_norm, c->at<char>(L.h), B, m.d_model, m.rms_eps, s);
    SampleArgs a{sample->seed, sample->seq_id_base, sample->temperature, sample->eos_id};
    if (queue_out_len) {
        a.out_row = c->at<int>(L.out_row);
        a.seq_id = c->at<int>(L.seq_id);
        a.gen_limit = c->at<int>(L.gen_limit);
        a.out_len = queue_out_len;
    }
    // The LM head either writes fp32 logits [B, V] for the sampler to read, or -- tuned path, decode GEMM shapes --
    // only per-block statistics (16 bytes per row and 32 columns, in the same buffer), from which the sampler draws
    // and re-derives the 32 logits of the one block it lands in: the step's logits never reach memory.
    const bool fused = c->impl == 1 && c->fused_sample && B <= 128 && m.vocab % 128 == 0 && m.d_model % 8 == 0 &&
                       k_gemm_decode_supported(MG_SAMPLE, m.vocab, m.d_model) &&
                       (size_t)B * (m.vocab / 32) * sizeof(float4) <= (size_t)L.logit_rows * m.vocab * 4;
    if (fused) {
        GemmArgs g;
        g.M = B; g.A = c->at<f16_t>(L.h); g.lda = m.d_model; g.W = (const bf16_t*)c->policy.lm_head; g.N = m.vocab;
        g.K = m.d_model; g.samp_part = c->at<float4>(L.logits);
        g.inv_temp = sample->temperature > 0.f ? 1.0f / sample->temperature : 1.0f;
        mfma(c, RL_K_GEMM_DECODE, MG_SAMPLE, g, 1, s);
        k_sample_blocks(c->at<float4>(L.logits), m.vocab, c->at<char>(L.h), m.d_model, c->policy.lm_head, m.d_model, B, a,
                        c->at<int>(L.last_tok), c->at<int>(L.seq_len), c->at<int>(L.gen_count), c->at<int>(L.finished),
                        c->at<int>(L.step_count), tok_out, logp_out, out_ids, out_logp, out_stride, s);
    } else {
        lm_head_logits(c, RL_K_GEMM_DECODE, c->policy, c->at<char>(L.h), B, s);
        k_sample(c->at<float>(L.logits), m.vocab, m.vocab, B, a, c->at<int>(L.last_tok), c->at<int>(L.seq_len),
                 c->at<int>(L.gen_count), c->at<int>(L.finished), c->at<int>(L.step_count), tok_out, logp_out, out_ids,
                 out_logp, out_stride, s);
    }
    for (int b = 0; b < B; ++b) c->cached[b] = need[b];
    return RL_OK;
}

static int check_sample(const rl_sample_cfg* sample) {
    if (!sample) return fail(RL_EINVAL, "sample cfg is NULL");
    if (!(sample->temperature >= 0.0f)) return fail(RL_EINVAL, "temperature must be >= 0");
    return RL_OK;
}

int rollout_decode_step(rl_ctx* c, const rl_sample_cfg* sample, const int32_t* tok_in, int32_t* tok_out,
                        float* logp_out, void* stream) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    int rc = check_sample(sample);
    if (rc) return rc;
    if (c->B < 1) return fail(RL_ESTATE, "rollout_decode_step before rollout_prefill");
    if ((rc = wait_policy(c, (hipStream_t)stream))) return rc;
    rc = decode_step_impl(c, sample, tok_in, tok_out, logp_out, nullptr, nullptr, 0, (hipStream_t)stream);
    if (rc) return rc;
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

int rollout_generate(rl_ctx* c, const rl_sample_cfg* sample, const int32_t* prompt_ids, const int32_t* prompt_len,
                     int32_t B, int32_t Pmax, int32_t G, int32_t* out_ids, int32_t* out_len, float* out_logp,
                     void* stream) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    int rc = check_sample(sample);
    if (rc) return rc;
    if (!out_ids) return fail(RL_EINVAL, "out_ids is NULL");
    if (G < 1) return fail(RL_EINVAL, "G < 1");
    if (!prompt_len) return fail(RL_EINVAL, "NULL argument");
    for (int b = 0; b < B && b < c->cfg.max_batch; ++b)
        if (prompt_len[b] >= 1 && prompt_len[b] - 1 + G > c->cfg.max_seq)
            return fail(RL_EINVAL, "prompt_len[%d] - 1 + G = %d exceeds max_seq=%d", b, prompt_len[b] - 1 + G,
                        c->cfg.max_seq);
    hipStream_t s = (hipStream_t)stream;
    rc = rollout_prefill(c, prompt_ids, prompt_len, B, Pmax, stream);
    if (rc) return rc;
    // reserve every page the rollout will need up front: no allocation inside the loop
    std::vector<int> need(B);
    for (int b = 0; b < B; ++b) need[b] = prompt_len[b] - 1 + G;
    rc = ensure_pages(c, need, s);
    if (rc) return rc;
    bool profiling = false;
    for (int k = 0; k < RL_K_COUNT; ++k) profiling = profiling || c->prof_on[k] != 0;
    if (c->impl == 1 && s != nullptr && c->use_graph && !profiling) {
        // The step is identical from one token to the next (positions, step counters and page
        // tables live on the device), so it is captured once and replayed G times.
        rl_ctx::GraphKey key{B, G, c->impl, sample->eos_id, out_ids, out_logp, sample->seed, sample->seq_id_base,
                             sample->temperature, s};
        if (!c->gexec || !(key == c->gkey)) {
            if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
            std::vector<int> saved = c->cached;
            HIP_TRY(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
            rc = decode_step_impl(c, sample, nullptr, nullptr, nullptr, out_ids, out_logp, G, s);
            hipGraph_t graph = nullptr;
            hipError_t e = hipStreamEndCapture(s, &graph);
            c->cached = saved;
            if (rc) { if (graph) (void)hipGraphDestroy(graph); return rc; }
            if (e != hipSuccess) return fail(RL_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
            e = hipGraphInstantiate(&c->gexec, graph, nullptr, nullptr, 0);
            (void)hipGraphDestroy(graph);
            if (e != hipSuccess) { c->gexec = nullptr; return fail(RL_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e)); }
            c->gkey = key;
        }
        for (int n = 0; n < G; ++n) HIP_TRY(hipGraphLaunch(c->gexec, s));
        for (int b = 0; b < B; ++b) c->cached[b] += G;
    } else {
        for (int n = 0; n < G; ++n) {
            rc = decode_step_impl(c, sample, nullptr, nullptr, nullptr, out_ids, out_logp, G, s);
            if (rc) return rc;
        }
    }
    if (out_len) k_out_len(c->at<int>(c->L.gen_count), out_len, B, s);
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

// ---- queue mode: more prompts than slots, per-prompt token limits, early stops (Section 3.2: generation
// lengths vary widely, so work is handed out dynamically instead of in fixed batches).
//
// Prefill the prompts `rows` (rows of the [*, Pmax] id matrix) into the cache slots `slots` while the other
// slots keep their state: cache tokens [0, P-1), then set the slot's state (last prompt token as next
// input, counters zero, output row / sequence id = the prompt's row, its token limit).
static int prefill_rows(rl_ctx* c, const int32_t* ids, int Pmax, const int32_t* plen, const int32_t* limit,
                        const std::vector<int>& rows, const std::vector<int>& slots, hipStream_t s) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    const int n = (int)rows.size();
    if (n == 0) return RL_OK;
    std::vector<int> need(m.max_batch);
    for (int b = 0; b < m.max_batch; ++b) need[b] = c->cached[b];
    for (int i = 0; i < n; ++i) need[slots[i]] = plen[rows[i]] - 1;
    int rc = ensure_pages(c, need, s);
    if (rc) return rc;
    const int al = pack_align(c);
    for (int i0 = 0; i0 < n;) {
        Chunk ch;
        int i1 = i0;
        while (i1 < n) {
            const int len = plen[rows[i1]] - 1, alen = (len + al - 1) / al * al;
            if (ch.n + alen > m.max_chunk_tokens && ch.n > 0) break;
            ch.rows_b.push_back(rows[i1]);
            ch.slots.push_back(slots[i1]);
            ch.starts.push_back(ch.n);
            ch.lens.push_back(len);
            ch.full.push_back(len);
            ch.n += alen;
            ch.max_ctx = std::max(ch.max_ctx, len);
            ++i1;
        }
        i0 = i1;
        if (ch.n > 0) {
            if ((rc = pack_chunk(c, ids, Pmax, ch, false, s))) return rc;
            k_embed(m.dtype, c->at<int>(L.tok_ids), ch.n, c->policy.tok_embed, m.d_model, m.vocab, c->at<float>(L.x),
                    c->at<int>(L.errflag), s);
            run_layers(c, c->policy, ch.n, false, true, ch.max_ctx, ch.nblocks, s);
        }
    }
    std::vector<int> pl(n), lim(n);
    for (int i = 0; i < n; ++i) { pl[i] = plen[rows[i]]; lim[i] = limit[rows[i]]; }
    const size_t nb = (size_t)n * sizeof(int);
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.seq_first), rows.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.row_slot), slots.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.row_len), pl.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.full_len), lim.data(), nb, hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));   // the host vectors go out of scope
    k_prefill_state_slots(ids, Pmax, n, c->at<int>(L.seq_first), c->at<int>(L.row_slot), c->at<int>(L.row_len),
                          c->at<int>(L.full_len), c->at<int>(L.last_tok), c->at<int>(L.seq_len), c->at<int>(L.gen_count),
                          c->at<int>(L.finished), c->at<int>(L.step_count), c->at<int>(L.out_row), c->at<int>(L.seq_id),
                          c->at<int>(L.gen_limit), s);
    for (int i = 0; i < n; ++i) {
        const int b = slots[i];
        c->cached[b] = plen[rows[i]] - 1;
        c->cap[b] = plen[rows[i]] - 1 + limit[rows[i]];
        c->parked[b] = 0;
    }
    return RL_OK;
}

static const int kQueueBurst = 8;       // decode steps between two looks at the finished flags
static const int kQueueRefillMin = 16;  // free slots to collect before a refill (fewer if fewer prompts wait)

int rollout_generate_queue(rl_ctx* c, const rl_sample_cfg* sample, const int32_t* prompt_ids, const int32_t* prompt_len,
                           const int32_t* gen_limit, int32_t Q, int32_t Pmax, int32_t Gmax, int32_t* out_ids,
                           int32_t* out_len, float* out_logp, void* stream) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    int rc = check_sample(sample);
    if (rc) return rc;
    if (!prompt_ids || !prompt_len || !gen_limit || !out_ids || !out_len) return fail(RL_EINVAL, "NULL argument");
    const rl_model_cfg& m = c->cfg;
    if (Q < 1 || Pmax < 1 || Gmax < 1) return fail(RL_EINVAL, "Q, Pmax and Gmax must be >= 1");
    for (int q = 0; q < Q; ++q) {
        if (prompt_len[q] < 1 || prompt_len[q] > Pmax)
            return fail(RL_EINVAL, "prompt_len[%d]=%d outside [1, Pmax]", q, prompt_len[q]);
        if (gen_limit[q] < 1 || gen_limit[q] > Gmax)
            return fail(RL_EINVAL, "gen_limit[%d]=%d outside [1, Gmax]", q, gen_limit[q]);
        if (prompt_len[q] - 1 + gen_limit[q] > m.max_seq)
            return fail(RL_EINVAL, "prompt_len[%d] - 1 + gen_limit = %d exceeds max_seq=%d", q,
                        prompt_len[q] - 1 + gen_limit[q], m.max_seq);
    }
    hipStream_t s = (hipStream_t)stream;
    const Layout& L = c->L;
    if ((rc = wait_policy(c, s))) return rc;
    // entries past a row's length read eos_id (-1 when there is none) / log-prob 0
    k_fill_i32(out_ids, sample->eos_id, (int64_t)Q * Gmax, s);
    k_fill_i32(out_len, 0, Q, s);
    if (out_logp) k_fill_f32(out_logp, 0.f, (int64_t)Q * Gmax, s);
    c->B = 0;
    release_all_pages(c);
    const int nslots = std::min<int>(Q, m.max_batch);
    std::vector<int> slot_row(nslots, -1), rows, slots, free_slots;
    int next = 0, live = 0;
    for (int b = 0; b < nslots; ++b) { rows.push_back(next); slots.push_back(b); slot_row[b] = next++; }
    if ((rc = prefill_rows(c, prompt_ids, Pmax, prompt_len, gen_limit, rows, slots, s))) { rollout_reset(c); return rc; }
    live = nslots;
    c->B = nslots;
    bool profiling = false;
    for (int k = 0; k < RL_K_COUNT; ++k) profiling = profiling || c->prof_on[k] != 0;
    const bool graph = c->impl == 1 && s != nullptr && c->use_graph && !profiling;
    std::vector<int> fin(nslots), slen(nslots), need(nslots);
    while (live > 0) {
        // reserve the burst's pages up front: nothing is allocated between two looks at the flags
        for (int b = 0; b < nslots; ++b)
            need[b] = c->parked[b] ? c->cached[b] : std::min(c->cached[b] + kQueueBurst, c->cap[b]);
        if ((rc = ensure_pages(c, need, s))) { rollout_reset(c); return rc; }
        if (graph) {
            rl_ctx::GraphKey key{nslots, Gmax, c->impl, sample->eos_id, out_ids, out_logp, sample->seed,
                                 sample->seq_id_base, sample->temperature, s, out_len};
            if (!c->gexec || !(key == c->gkey)) {
                if (c->gexec) { (void)hipGraphExecDestroy(c->gexec); c->gexec = nullptr; }
                std::vector<int> saved = c->cached;
                HIP_TRY(hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
                rc = decode_step_impl(c, sample, nullptr, nullptr, nullptr, out_ids, out_logp, Gmax, s, out_len);
                hipGraph_t g = nullptr;
                hipError_t e = hipStreamEndCapture(s, &g);
                c->cached = saved;
                if (rc) { if (g) (void)hipGraphDestroy(g); rollout_reset(c); return rc; }
                if (e != hipSuccess) { rollout_reset(c); return fail(RL_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e)); }
                e = hipGraphInstantiate(&c->gexec, g, nullptr, nullptr, 0);
                (void)hipGraphDestroy(g);
                if (e != hipSuccess) { c->gexec = nullptr; rollout_reset(c); return fail(RL_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e)); }
                c->gkey = key;
            }
            for (int n = 0; n < kQueueBurst; ++n) HIP_TRY(hipGraphLaunch(c->gexec, s));
            for (int b = 0; b < nslots; ++b) c->cached[b] = need[b];
        } else {
            for (int n = 0; n < kQueueBurst; ++n)
                if ((rc = decode_step_impl(c, sample, nullptr, nullptr, nullptr, out_ids, out_logp, Gmax, s, out_len))) {
                    rollout_reset(c);
                    return rc;
                }
        }
        // which slots have finished, and how long the others' caches really are
        HIP_TRY(hipMemcpyAsync(fin.data(), c->at<int>(L.finished), (size_t)nslots * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipMemcpyAsync(slen.data(), c->at<int>(L.seq_len), (size_t)nslots * 4, hipMemcpyDeviceToHost, s));
        HIP_TRY(hipStreamSynchronize(s));
        for (int b = 0; b < nslots; ++b) {
            if (slot_row[b] < 0) continue;
            if (!fin[b]) { c->cached[b] = slen[b]; continue; }
            // finished: its pages go back to the pool and the slot waits, parked, for a queued prompt
            release_slot_pages(c, b);
            c->parked[b] = 1;
            slot_row[b] = -1;
            --live;
            free_slots.push_back(b);
        }
        // Refill in groups: a prefill of one or two prompts runs the large-M kernels far below their rate,
        // while an idle slot costs only its share of a decode step that streams the weights anyway.
        const int waiting = Q - next;
        if (waiting > 0 && ((int)free_slots.size() >= std::min(kQueueRefillMin, waiting) || live == 0)) {
            rows.clear();
            slots.clear();
            while (next < Q && !free_slots.empty()) {
                const int b = free_slots.back();
                free_slots.pop_back();
                rows.push_back(next);
                slots.push_back(b);
                slot_row[b] = next++;
                ++live;
            }
            if ((rc = prefill_rows(c, prompt_ids, Pmax, prompt_len, gen_limit, rows, slots, s))) { rollout_reset(c); return rc; }
        }
    }
    rollout_reset(c);   // nothing stays live after a queue run
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

// Final norm, LM head and log-prob of every target token for the n packed rows whose residual stream is x.
static void score_head(rl_ctx* c, const WeightsHost& W, float* x, int n, float* logp_out, int Lmax, hipStream_t s) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    k_rmsnorm(m.dtype, x, W.final_norm, c->at<char>(L.h), n, m.d_model, m.rms_eps, s);
    if (c->impl == 1) {
        // LM head with the log-sum-exp and the target gather in its epilogue: no logits in memory
        GemmArgs g;
        g.M = n; g.A = c->at<f16_t>(L.h); g.lda = m.d_model; g.W = (const bf16_t*)W.lm_head; g.N = m.vocab;
        g.K = m.d_model; g.tgt = c->at<int>(L.tok_tgt); g.lse_part = c->at<float2>(L.lse_part);
        g.z_tgt = c->at<float>(L.z_tgt);
        mfma(c, RL_K_LMHEAD_SCORE, MG_LSE, g, 1, s);
        k_lse_reduce(c->at<float2>(L.lse_part), k_gemm_mfma_lse_parts(n, m.vocab, m.d_model, c->big_mode),
                     c->at<float>(L.z_tgt), n, c->at<int>(L.tok_tgt), c->at<int>(L.tok_slot), c->at<int>(L.tok_pos),
                     logp_out, Lmax, s);
        return;
    }
    const size_t e = esz_of(m.dtype);
    for (int r0 = 0; r0 < n; r0 += L.logit_rows) {
        int nr = std::min(L.logit_rows, n - r0);
        lm_head_logits(c, RL_K_LMHEAD_SCORE, W, c->at<char>(L.h) + (size_t)r0 * m.d_model * e, nr, s);
        k_lse_gather(c->at<float>(L.logits), m.vocab, m.vocab, nr, c->at<int>(L.tok_tgt) + r0,
                     c->at<int>(L.tok_slot) + r0, c->at<int>(L.tok_pos) + r0, logp_out, Lmax, s);
    }
}

// One teacher-forced pass of one device-resident weight set over all sequences; writes logp_out [B, Lmax].
// The head applied to the final residual stream of n packed rows: the LM head with log-sum-exp and target
// gather (log-probs), or, with value_head != nullptr, a [d] -> 1 head (critic values / reward-model scores).
static void apply_head(rl_ctx* c, const WeightsHost& W, const void* value_head, float* x, int n, float* out, int Lmax,
                       hipStream_t s) {
    if (!value_head) { score_head(c, W, x, n, out, Lmax, s); return; }
    const rl_model_cfg& m = c->cfg;
    k_value_head(m.dtype, x, W.final_norm, value_head, n, m.d_model, m.rms_eps, c->at<int>(c->L.tok_slot),
                 c->at<int>(c->L.tok_pos), out, Lmax, s);
}

static int score_pass(rl_ctx* c, const WeightsHost& W, const int32_t* ids, const int32_t* seq_len, int B, int Lmax,
                      float* logp_out, hipStream_t s, const void* value_head = nullptr) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    k_fill_f32(logp_out, 0.f, (int64_t)B * Lmax, s);
    std::vector<int> len_of(seq_len, seq_len + B);
    int b0 = 0;
    while (b0 < B) {
        Chunk ch;
        b0 = chunk_take(c, len_of, b0, B, ch);
        int rc = pack_chunk(c, ids, Lmax, ch, true, s);
        if (rc) return rc;
        k_embed(m.dtype, c->at<int>(L.tok_ids), ch.n, W.tok_embed, m.d_model, m.vocab, c->at<float>(L.x),
                c->at<int>(L.errflag), s);
        run_layers(c, W, ch.n, false, false, ch.max_ctx, ch.nblocks, s);
        apply_head(c, W, value_head, c->at<float>(L.x), ch.n, logp_out, Lmax, s);
    }
    return RL_OK;
}

// ---- host-resident weight sets (the reference model of a PPO step that does not fit next to the policy;
// Section 3.1: the reference shares the actor's architecture, and its weights are swapped in for the
// reference-policy inference step).  The weights are streamed layer by layer into a two-slot device
// staging buffer on a copy stream while the previous layer computes.  To pay for each layer's transfer
// once per pass, the loop order is layer-major: the residual stream of ALL tokens stays on the device
// (x_all) and every chunk runs layer l before any runs layer l+1.
struct StageLayout {
    size_t attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down, layer_bytes;   // offsets inside a slot
    size_t slot[2], globals, final_norm, x_all, total;
    size_t b_norm, b_wqkv, b_wo, b_gate_up, b_down, b_globals;              // tensor sizes in bytes
    int64_t x_rows;
};

static StageLayout make_stage_layout(const rl_model_cfg& c) {
    StageLayout S{};
    const size_t e = esz_of(c.dtype);
    const size_t d = c.d_model, qd = (size_t)c.n_q_heads * c.head_dim;
    const size_t nqkv = (size_t)(c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim;
    auto al = [](size_t b) { return (b + 255) / 256 * 256; };
    S.b_norm = d * e; S.b_wqkv = nqkv * d * e; S.b_wo = d * qd * e;
    S.b_gate_up = 2 * (size_t)c.d_ffn * d * e; S.b_down = d * (size_t)c.d_ffn * e;
    S.b_globals = (size_t)c.vocab * d * e;
    size_t o = 0;
    S.attn_norm = o; o += al(S.b_norm);
    S.wqkv = o; o += al(S.b_wqkv);
    S.wo = o; o += al(S.b_wo);
    S.ffn_norm = o; o += al(S.b_norm);
    S.w_gate_up = o; o += al(S.b_gate_up);
    S.w_down = o; o += al(S.b_down);
    S.layer_bytes = o;
    size_t t = 0;
    S.slot[0] = t; t += S.layer_bytes;
    S.slot[1] = t; t += S.layer_bytes;
    S.globals = t; t += al(S.b_globals);          // embedding table first, LM head afterwards
    S.final_norm = t; t += al(S.b_norm);
    // every sequence occupies a multiple of 32 rows on the tuned path
    S.x_rows = (int64_t)c.max_batch * ((c.max_seq + 31) / 32 * 32);
    S.x_all = t; t += al((size_t)S.x_rows * d * sizeof(float));
    S.total = t;
    return S;
}

static int ensure_copy_stream(rl_ctx* c) {
    if (c->copy_stream) return RL_OK;
    HIP_TRY(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
    for (hipEvent_t* e : {&c->ev_begin, &c->ev_glob_copied, &c->ev_glob_free, &c->ev_copied[0], &c->ev_copied[1],
                          &c->ev_free[0], &c->ev_free[1], &c->ev_policy})
        HIP_TRY(hipEventCreateWithFlags(e, hipEventDisableTiming));
    return RL_OK;
}

static int score_pass_streamed(rl_ctx* c, const WeightsHost& W, const int32_t* ids, const int32_t* seq_len, int B,
                               int Lmax, float* logp_out, hipStream_t s, const void* value_head = nullptr) {
    const rl_model_cfg& m = c->cfg;
    const Layout& L = c->L;
    const StageLayout S = make_stage_layout(m);
    if (!W.staging) return fail(RL_EINVAL, "host-resident weights need a device staging buffer (rl_weights.staging)");
    if (((uintptr_t)W.staging & 255) != 0) return fail(RL_EINVAL, "staging buffer must be 256-byte aligned");
    if (W.staging_bytes < S.total)
        return fail(RL_ENOSPACE, "staging buffer: %zu bytes given, %zu needed", W.staging_bytes, S.total);
    int rc = ensure_copy_stream(c);
    if (rc) return rc;
    hipStream_t cs = c->copy_stream;
    char* st = W.staging;
    float* x_all = reinterpret_cast<float*>(st + S.x_all);

    // chunks and their first rows in x_all
    std::vector<int> len_of(seq_len, seq_len + B);
    std::vector<Chunk> chunks;
    std::vector<int64_t> first;
    int64_t rows = 0;
    for (int b0 = 0; b0 < B;) {
        chunks.emplace_back();
        b0 = chunk_take(c, len_of, b0, B, chunks.back());
        first.push_back(rows);
        rows += chunks.back().n;
    }
    if (rows > S.x_rows) return fail(RL_EINVAL, "internal: %lld packed rows exceed the staging rows", (long long)rows);

    // device-pointer view of the staged weights: layer l lives in slot l % 2
    WeightsHost D;
    D.tok_embed = st + S.globals;
    D.lm_head = st + S.globals;
    D.final_norm = st + S.final_norm;
    auto fill = [&](std::vector<const void*>& v, size_t off) {
        v.resize(m.n_layers);
        for (int l = 0; l < m.n_layers; ++l) v[l] = st + S.slot[l & 1] + off;
    };
    fill(D.attn_norm, S.attn_norm); fill(D.wqkv, S.wqkv); fill(D.wo, S.wo);
    fill(D.ffn_norm, S.ffn_norm); fill(D.w_gate_up, S.w_gate_up); fill(D.w_down, S.w_down);
    auto copy_layer = [&](int l) -> int {
        char* slot = st + S.slot[l & 1];
        HIP_TRY(hipMemcpyAsync(slot + S.attn_norm, W.attn_norm[l], S.b_norm, hipMemcpyHostToDevice, cs));
        HIP_TRY(hipMemcpyAsync(slot + S.wqkv, W.wqkv[l], S.b_wqkv, hipMemcpyHostToDevice, cs));
        HIP_TRY(hipMemcpyAsync(slot + S.wo, W.wo[l], S.b_wo, hipMemcpyHostToDevice, cs));
        HIP_TRY(hipMemcpyAsync(slot + S.ffn_norm, W.ffn_norm[l], S.b_norm, hipMemcpyHostToDevice, cs));
        HIP_TRY(hipMemcpyAsync(slot + S.w_gate_up, W.w_gate_up[l], S.b_gate_up, hipMemcpyHostToDevice, cs));
        HIP_TRY(hipMemcpyAsync(slot + S.w_down, W.w_down[l], S.b_down, hipMemcpyHostToDevice, cs));
        HIP_TRY(hipEventRecord(c->ev_copied[l & 1], cs));
        return RL_OK;
    };

    k_fill_f32(logp_out, 0.f, (int64_t)B * Lmax, s);
    // the staging buffer may still be read by work queued earlier on s
    HIP_TRY(hipEventRecord(c->ev_begin, s));
    HIP_TRY(hipStreamWaitEvent(cs, c->ev_begin, 0));
    HIP_TRY(hipMemcpyAsync(st + S.globals, W.tok_embed, S.b_globals, hipMemcpyHostToDevice, cs));
    HIP_TRY(hipMemcpyAsync(st + S.final_norm, W.final_norm, S.b_norm, hipMemcpyHostToDevice, cs));
    HIP_TRY(hipEventRecord(c->ev_glob_copied, cs));
    for (int l = 0; l < std::min(2, m.n_layers); ++l)
        if ((rc = copy_layer(l))) return rc;

    // embedding of every chunk into x_all
    HIP_TRY(hipStreamWaitEvent(s, c->ev_glob_copied, 0));
    for (size_t k = 0; k < chunks.size(); ++k) {
        if ((rc = pack_chunk(c, ids, Lmax, chunks[k], true, s))) return rc;
        k_embed(m.dtype, c->at<int>(L.tok_ids), chunks[k].n, D.tok_embed, m.d_model, m.vocab,
                x_all + first[k] * m.d_model, c->at<int>(L.errflag), s);
    }
    // the LM head takes the embedding table's place once the gathers are done
    HIP_TRY(hipEventRecord(c->ev_glob_free, s));
    HIP_TRY(hipStreamWaitEvent(cs, c->ev_glob_free, 0));
    if (!value_head) HIP_TRY(hipMemcpyAsync(st + S.globals, W.lm_head, S.b_globals, hipMemcpyHostToDevice, cs));
    HIP_TRY(hipEventRecord(c->ev_glob_copied, cs));

    for (int l = 0; l < m.n_layers; ++l) {
        HIP_TRY(hipStreamWaitEvent(s, c->ev_copied[l & 1], 0));
        for (size_t k = 0; k < chunks.size(); ++k) {
            if ((rc = pack_chunk(c, ids, Lmax, chunks[k], true, s))) return rc;
            run_layers(c, D, chunks[k].n, false, false, chunks[k].max_ctx, chunks[k].nblocks, s,
                       x_all + first[k] * m.d_model, l, l + 1);
        }
        if (l + 2 < m.n_layers) {   // slot l % 2 is free once layer l has run on every chunk
            HIP_TRY(hipEventRecord(c->ev_free[l & 1], s));
            HIP_TRY(hipStreamWaitEvent(cs, c->ev_free[l & 1], 0));
            if ((rc = copy_layer(l + 2))) return rc;
        }
    }
    HIP_TRY(hipStreamWaitEvent(s, c->ev_glob_copied, 0));
    for (size_t k = 0; k < chunks.size(); ++k) {
        if ((rc = pack_chunk(c, ids, Lmax, chunks[k], true, s))) return rc;
        apply_head(c, D, value_head, x_all + first[k] * m.d_model, chunks[k].n, logp_out, Lmax, s);
    }
    return RL_OK;
}

size_t rollout_weight_staging_bytes(const rl_model_cfg* cfg) {
    if (validate_cfg(cfg) != RL_OK) return 0;
    return make_stage_layout(*cfg).total;
}

int score_logprobs_kl(rl_ctx* c, const rl_weights* policy, const rl_weights* reference, const int32_t* ids,
                      const int32_t* seq_len, const int32_t* prompt_len, int32_t B, int32_t Lmax, float kl_coef,
                      float* logp_policy, float* logp_ref, float* kl, float* kl_penalty, void* stream) {
    if (!c || !ids || !seq_len || !prompt_len) return fail(RL_EINVAL, "NULL argument");
    const rl_model_cfg& m = c->cfg;
    if (B < 1 || B > m.max_batch) return fail(RL_EINVAL, "B=%d outside [1, max_batch=%d]", B, m.max_batch);
    if (Lmax < 1) return fail(RL_EINVAL, "Lmax < 1");
    for (int b = 0; b < B; ++b) {
        if (seq_len[b] < 1 || seq_len[b] > Lmax || seq_len[b] > m.max_seq)
            return fail(RL_EINVAL, "seq_len[%d]=%d outside [1, min(Lmax, max_seq)]", b, seq_len[b]);
        if (prompt_len[b] < 0 || prompt_len[b] > seq_len[b])
            return fail(RL_EINVAL, "prompt_len[%d]=%d outside [0, seq_len]", b, prompt_len[b]);
    }
    if (!reference && (logp_ref || kl || kl_penalty))
        return fail(RL_EINVAL, "reference is NULL but a reference-dependent output was requested");
    if ((kl || kl_penalty) && (!logp_policy || !logp_ref))
        return fail(RL_EINVAL, "kl outputs need logp_policy and logp_ref buffers");
    hipStream_t s = (hipStream_t)stream;
    WeightsHost wp, wr;
    int rc = RL_OK;
    if (policy) rc = copy_weights(m, policy, wp, "policy", true);
    else { wp = c->policy; rc = wait_policy(c, s); }   // the set the context generates with
    if (rc) return rc;
    if (reference) {
        rc = copy_weights(m, reference, wr, "reference", true);
        if (rc) return rc;
        if ((rc = ensure_other_shadow(c, wr, s))) return rc;
    }
    if (logp_policy) {
        rc = wp.location == 1 ? score_pass_streamed(c, wp, ids, seq_len, B, Lmax, logp_policy, s)
                              : score_pass(c, wp, ids, seq_len, B, Lmax, logp_policy, s);
        if (rc) return rc;
    }
    if (reference && logp_ref) {
        rc = wr.location == 1 ? score_pass_streamed(c, wr, ids, seq_len, B, Lmax, logp_ref, s)
                              : score_pass(c, wr, ids, seq_len, B, Lmax, logp_ref, s);
        if (rc) return rc;
    }
    if (kl || kl_penalty) {
        const Layout& L = c->L;
        HIP_TRY(hipMemcpyAsync(c->at<int>(L.d_seq_len), seq_len, (size_t)B * 4, hipMemcpyHostToDevice, s));
        HIP_TRY(hipMemcpyAsync(c->at<int>(L.d_prompt_len), prompt_len, (size_t)B * 4, hipMemcpyHostToDevice, s));
        HIP_TRY(hipStreamSynchronize(s));
        k_kl(logp_policy, logp_ref, c->at<int>(L.d_seq_len), c->at<int>(L.d_prompt_len), B, Lmax, kl_coef, kl,
             kl_penalty, s);
    }
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

int score_kl_exact(rl_ctx* c, const rl_weights* policy, const rl_weights* reference, const int32_t* ids,
                   const int32_t* seq_len, const int32_t* prompt_len, int32_t B, int32_t Lmax, float* kl_out,
                   void* stream) {
    if (!c || !ids || !seq_len || !prompt_len || !kl_out) return fail(RL_EINVAL, "NULL argument");
    const rl_model_cfg& m = c->cfg;
    if (B < 1 || B > m.max_batch) return fail(RL_EINVAL, "B=%d outside [1, max_batch=%d]", B, m.max_batch);
    if (Lmax < 1) return fail(RL_EINVAL, "Lmax < 1");
    for (int b = 0; b < B; ++b) {
        if (seq_len[b] < 1 || seq_len[b] > Lmax || seq_len[b] > m.max_seq)
            return fail(RL_EINVAL, "seq_len[%d]=%d outside [1, min(Lmax, max_seq)]", b, seq_len[b]);
        if (prompt_len[b] < 0 || prompt_len[b] > seq_len[b])
            return fail(RL_EINVAL, "prompt_len[%d]=%d outside [0, seq_len]", b, prompt_len[b]);
    }
    WeightsHost wp, wr;
    int rc = copy_weights(m, policy, wp, "policy");
    if (rc) return rc;
    if ((rc = copy_weights(m, reference, wr, "reference"))) return rc;
    if ((rc = ensure_other_shadow(c, wr, (hipStream_t)stream))) return rc;
    hipStream_t s = (hipStream_t)stream;
    const Layout& L = c->L;
    const size_t e = esz_of(m.dtype);
    const bool fused = c->impl == 1 && k_gemm_mfma_supported(MG_KLFULL, m.vocab, m.d_model, m.head_dim);
    k_fill_f32(kl_out, 0.f, (int64_t)B * Lmax, s);
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.d_prompt_len), prompt_len, (size_t)B * 4, hipMemcpyHostToDevice, s));
    std::vector<int> len_of(seq_len, seq_len + B);
    // rows per dual-head launch: the partials (5 floats per row and 64 columns) share the buffer of the
    // log-sum-exp partials (2 floats); the plain path holds two logit blocks in the logits buffer
    const int nparts = m.vocab / 64;
    int kl_rows = fused ? (int)((size_t)L.rows * ((m.vocab + 63) / 64) * 2 / ((size_t)nparts * 5)) : L.logit_rows / 2;
    if (kl_rows < 1) return fail(RL_ENOSPACE, "workspace too small for the exact-KL head");
    int b0 = 0;
    while (b0 < B) {
        Chunk ch;
        b0 = chunk_take(c, len_of, b0, B, ch);
        const int n = ch.n;
        if ((rc = pack_chunk(c, ids, Lmax, ch, true, s))) return rc;
        // policy body, final norm; keep its hidden states while the reference body runs on the same rows
        k_embed(m.dtype, c->at<int>(L.tok_ids), n, wp.tok_embed, m.d_model, m.vocab, c->at<float>(L.x),
                c->at<int>(L.errflag), s);
        run_layers(c, wp, n, false, false, ch.max_ctx, ch.nblocks, s);
        k_rmsnorm(m.dtype, c->at<float>(L.x), wp.final_norm, c->at<char>(L.h_keep), n, m.d_model, m.rms_eps, s);
        k_embed(m.dtype, c->at<int>(L.tok_ids), n, wr.tok_embed, m.d_model, m.vocab, c->at<float>(L.x),
                c->at<int>(L.errflag), s);
        run_layers(c, wr, n, false, false, ch.max_ctx, ch.nblocks, s);
        k_rmsnorm(m.dtype, c->at<float>(L.x), wr.final_norm, c->at<char>(L.h), n, m.d_model, m.rms_eps, s);
        for (int r0 = 0; r0 < n; r0 += kl_rows) {
            const int nr = std::min(kl_rows, n - r0);
            const char* hp = c->at<char>(L.h_keep) + (size_t)r0 * m.d_model * e;
            const char* hr = c->at<char>(L.h) + (size_t)r0 * m.d_model * e;
            if (fused) {
                // both LM heads in one tile kernel; neither model's logits reach memory
                GemmArgs g;
                g.M = nr; g.N = m.vocab; g.K = m.d_model;
                g.A = (const f16_t*)hp; g.lda = m.d_model; g.W = (const bf16_t*)wp.lm_head;
                g.A2 = (const f16_t*)hr; g.lda2 = m.d_model; g.W2 = (const bf16_t*)wr.lm_head;
                g.kl_part = c->at<float>(L.lse_part);
                mfma(c, RL_K_LMHEAD_SCORE, MG_KLFULL, g, 1, s);
                k_kl_full_reduce(c->at<float>(L.lse_part), nparts, nr, c->at<int>(L.tok_tgt) + r0,
                                 c->at<int>(L.tok_slot) + r0, c->at<int>(L.tok_pos) + r0, c->at<int>(L.d_prompt_len),
                                 kl_out, Lmax, s);
            } else {
                float* zp = c->at<float>(L.logits);
                float* zr = zp + (size_t)kl_rows * m.vocab;
                gemm(c, RL_K_LMHEAD_SCORE, EPI_STORE_F32, hp, m.d_model, wp.lm_head, nullptr, nr, m.vocab, m.d_model, zp,
                     nullptr, m.vocab, s);
                gemm(c, RL_K_LMHEAD_SCORE, EPI_STORE_F32, hr, m.d_model, wr.lm_head, nullptr, nr, m.vocab, m.d_model, zr,
                     nullptr, m.vocab, s);
                k_kl_full_rows(zp, zr, m.vocab, m.vocab, nr, c->at<int>(L.tok_tgt) + r0, c->at<int>(L.tok_slot) + r0,
                               c->at<int>(L.tok_pos) + r0, c->at<int>(L.d_prompt_len), kl_out, Lmax, s);
            }
        }
    }
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

int score_values(rl_ctx* c, const rl_weights* model, const void* value_head, const int32_t* ids,
                 const int32_t* seq_len, int32_t B, int32_t Lmax, float* values, void* stream) {
    if (!c || !model || !ids || !seq_len || !value_head || !values) return fail(RL_EINVAL, "NULL argument");
    const rl_model_cfg& m = c->cfg;
    if (B < 1 || B > m.max_batch) return fail(RL_EINVAL, "B=%d outside [1, max_batch=%d]", B, m.max_batch);
    if (Lmax < 1) return fail(RL_EINVAL, "Lmax < 1");
    for (int b = 0; b < B; ++b)
        if (seq_len[b] < 1 || seq_len[b] > Lmax || seq_len[b] > m.max_seq)
            return fail(RL_EINVAL, "seq_len[%d]=%d outside [1, min(Lmax, max_seq)]", b, seq_len[b]);
    // the body's LM head is not used; a weight set without one is accepted
    rl_weights w = *model;
    if (!w.lm_head) w.lm_head = w.tok_embed;
    WeightsHost wh;
    int rc = copy_weights(m, &w, wh, "critic / reward model", true);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    rc = wh.location == 1 ? score_pass_streamed(c, wh, ids, seq_len, B, Lmax, values, s, value_head)
                          : score_pass(c, wh, ids, seq_len, B, Lmax, values, s, value_head);
    if (rc) return rc;
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

int ppo_rewards(rl_ctx* c, const float* kl, const float* seq_reward, const int32_t* seq_len, const int32_t* prompt_len,
                int32_t B, int32_t Lmax, float kl_coef, float* rewards, void* stream) {
    if (!c || !kl || !seq_reward || !seq_len || !prompt_len || !rewards) return fail(RL_EINVAL, "NULL argument");
    if (B < 1 || B > c->cfg.max_batch) return fail(RL_EINVAL, "B=%d outside [1, max_batch=%d]", B, c->cfg.max_batch);
    if (Lmax < 1) return fail(RL_EINVAL, "Lmax < 1");
    for (int b = 0; b < B; ++b)
        if (seq_len[b] < 1 || seq_len[b] > Lmax || prompt_len[b] < 0 || prompt_len[b] > seq_len[b])
            return fail(RL_EINVAL, "row %d: need 1 <= seq_len <= Lmax and 0 <= prompt_len <= seq_len", b);
    hipStream_t s = (hipStream_t)stream;
    const Layout& L = c->L;
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.d_seq_len), seq_len, (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipMemcpyAsync(c->at<int>(L.d_prompt_len), prompt_len, (size_t)B * 4, hipMemcpyHostToDevice, s));
    HIP_TRY(hipStreamSynchronize(s));
    k_ppo_reward(kl, seq_reward, c->at<int>(L.d_seq_len), c->at<int>(L.d_prompt_len), B, Lmax, kl_coef, rewards, s);
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

// ---- ppo_rewards for callers that cannot allocate.  The per-sequence lengths have to be device arrays for the
// kernel; ppo_rewards keeps them in the context's workspace and copies them there with the runtime.  Here they
// live in a fixed array of the library's own and are written by kernels that take them as arguments, so the call
// needs no context, no workspace and no copy: nothing in it allocates, and it can be recorded into a graph.
static const int kNoAllocMaxB = 4096;                                    // sequences per call
static __device__ __align__(256) int scratch[2 * kNoAllocMaxB];          // [seq_len | prompt_len], 32 KB per GPU
static const int kMaxDevices = 64;
static int* g_scratch_ptr[kMaxDevices];                                  // device address of `scratch`, per device
static std::mutex g_scratch_mu;

int ppo_rewards_noalloc(const float* kl, const float* seq_reward, const int32_t* seq_len, const int32_t* prompt_len,
                        int32_t B, int32_t Lmax, float kl_coef, float* rewards, void* stream) {
    if (!kl || !seq_reward || !seq_len || !prompt_len || !rewards) return fail(RL_EINVAL, "NULL argument");
    if (B < 1 || B > kNoAllocMaxB) return fail(RL_EINVAL, "B=%d outside [1, %d]", B, kNoAllocMaxB);
    if (Lmax < 1) return fail(RL_EINVAL, "Lmax < 1");
    for (int b = 0; b < B; ++b)
        if (seq_len[b] < 1 || seq_len[b] > Lmax || prompt_len[b] < 0 || prompt_len[b] > seq_len[b])
            return fail(RL_EINVAL, "row %d: need 1 <= seq_len <= Lmax and 0 <= prompt_len <= seq_len", b);
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(RL_EINVAL, "device %d outside [0, %d)", dev, kMaxDevices);
    int* ptr = nullptr;
    {
        // every GPU holds its own copy of the array at its own address: looked up once per device, with that
        // device current
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            g_scratch_ptr[dev] = static_cast<int*>(p);
        }
        ptr = g_scratch_ptr[dev];
    }
    hipStream_t s = (hipStream_t)stream;
    // the array keeps the previous call's lengths: every entry this call reads is rewritten first
    k_put_i32(ptr, seq_len, B, s);
    k_put_i32(ptr + kNoAllocMaxB, prompt_len, B, s);
    k_ppo_reward(kl, seq_reward, ptr, ptr + kNoAllocMaxB, B, Lmax, kl_coef, rewards, s);
    HIP_TRY(hipGetLastError());
    return RL_OK;
}

int rollout_profile_enable(rl_ctx* c, int32_t k, int32_t on) {
    if (!c) return fail(RL_EINVAL, "ctx is NULL");
    if (k < 0 || k >= RL_K_COUNT) return fail(RL_EINVAL, "kernel_class out of range");
    c->prof_on[k] = on < 0 ? 0 : on;
    c->prof_seen[k] = 0;
    return RL_OK;
}

int rollout_profile_read(rl_ctx* c, int32_t k, double* total_ms, int64_t* launches) {
    if (!c || !total_ms || !launches) return fail(RL_EINVAL, "NULL argument");
    if (k < 0 || k >= RL_K_COUNT) return fail(RL_EINVAL, "kernel_class out of range");
    double tot = 0.0;
    for (size_t i = 0; i < c->prof_used[k]; ++i) {
        HIP_TRY(hipEventSynchronize(c->prof[k][i].b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, c->prof[k][i].a, c->prof[k][i].b));
        tot += ms;
    }
    *total_ms = tot;
    *launches = (int64_t)c->prof_used[k];
    c->prof_used[k] = 0;
    return RL_OK;
}

int rollout_profile_event_overhead(rl_ctx* c, int32_t pairs, double* overhead_ms, void* stream) {
    if (!c || !overhead_ms) return fail(RL_EINVAL, "NULL argument");
    if (pairs < 1 || pairs > 4096) return fail(RL_EINVAL, "pairs must be in 1 .. 4096");
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t a = nullptr, b = nullptr;
    HIP_TRY(hipEventCreate(&a));
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return fail(RL_EHIP, "hipEventCreate failed"); }
    double tot = 0.0;
    int rc = RL_OK;
    for (int i = 0; i < pairs && rc == RL_OK; ++i) {
        // a kernel in front, as in a timed pass: the first event then waits for real work instead of an idle queue
        k_fill_f32(c->at<float>(c->L.x), 0.f, 64, s);
        if (hipEventRecord(a, s) != hipSuccess || hipEventRecord(b, s) != hipSuccess || hipEventSynchronize(b) != hipSuccess) {
            rc = fail(RL_EHIP, "event record failed");
            break;
        }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, a, b) != hipSuccess) { rc = fail(RL_EHIP, "hipEventElapsedTime failed"); break; }
        tot += ms;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (rc == RL_OK) *overhead_ms = tot / pairs;
    return rc;
}

int rollout_probe_mfma_rate(rl_ctx* c, int32_t random_operands, double* tflops, void* stream) {
    if (!c || !tflops) return fail(RL_EINVAL, "NULL argument");
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, n_cu = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    if (n_cu < 1 || n_cu > 1024) return fail(RL_EHIP, "unexpected compute-unit count %d", n_cu);
    // the fp32 logits area of the workspace is free between calls (at least 512 rows of vocab floats)
    if ((size_t)c->L.logit_rows * c->cfg.vocab * 4 < 65536 + (size_t)n_cu * 1024)
        return fail(RL_ENOSPACE, "workspace too small for the probe");
    void* scratch = c->at<char>(c->L.logits);
    hipEvent_t a = nullptr, b = nullptr;
    HIP_TRY(hipEventCreate(&a));
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return fail(RL_EHIP, "hipEventCreate failed"); }
    const int iters = 100000;                      // about 0.1 s: long enough for the clock to settle
    k_mfma_rate(scratch, n_cu, iters, random_operands != 0, s);   // warm
    int rc = RL_OK;
    float ms = 0.f;
    if (hipEventRecord(a, s) != hipSuccess) rc = fail(RL_EHIP, "event record failed");
    k_mfma_rate(scratch, n_cu, iters, random_operands != 0, s);
    if (rc == RL_OK && (hipEventRecord(b, s) != hipSuccess || hipEventSynchronize(b) != hipSuccess ||
                        hipEventElapsedTime(&ms, a, b) != hipSuccess))
        rc = fail(RL_EHIP, "event timing failed");
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (rc == RL_OK) *tflops = (double)n_cu * 4 * iters * 64 * 16384.0 / (ms * 1e-3) / 1e12;   // 64 MFMAs of 16 x 16 x 32 per wave and trip
    return rc;
}

}  // extern "C"
