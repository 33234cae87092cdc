// C ABI of libjq: argument validation, planning (wave counts, workspace layout) and the launch
// sequences.  Everything here runs on the host; no HIP call is made before validation succeeds.
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>

#include "jq_common.h"

namespace jq {

static Knobs read_knobs() {
    Knobs k{};
    auto chunk = [](const char* name) {
        const char* env = std::getenv(name);
        const long v = env ? std::atol(env) : 0;
        return (int32_t)((v >= kKeyTile && v <= 8192 && v % kKeyTile == 0) ? v : 0);
    };
    auto depth = [](const char* name) {
        const char* env = std::getenv(name);
        return (int32_t)(env && (env[0] == '1' || env[0] == '2') && env[1] == 0 ? env[0] - '0' : 1);
    };
    k.chunk_keys = chunk("JQ_CHUNK_KEYS");
    k.chunk_keys2 = chunk("JQ_CHUNK_KEYS_2");
    if (!std::getenv("JQ_CHUNK_KEYS_2")) k.chunk_keys2 = k.chunk_keys;
    k.depth1 = depth("JQ_DEPTH_1");
    k.depth2 = depth("JQ_DEPTH_2");
    k.log = std::getenv("JQ_LOG") != nullptr;
    return k;
}
static Knobs& knobs_storage() {
    static Knobs k = read_knobs();  // first use, thread-safe
    return k;
}
const Knobs& knobs() { return knobs_storage(); }

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// Validates `shape` and derives the plan.  `need_budgets`: the entry point uses budgets.
int make_plan(const jq_shape* sh, bool need_budgets, Plan* out) {
    if (!sh || !sh->cu_seqlens) return JQ_ERR_NULL;
    if (need_budgets && !sh->budgets) return JQ_ERR_NULL;
    if (sh->n_layers < 1 || sh->n_seq < 1 || sh->n_q < 1 || sh->h_q < 1 || sh->h_kv < 1 || sh->d < 1) return JQ_ERR_SHAPE;
    if (sh->h_q % sh->h_kv != 0) return JQ_ERR_SHAPE;
    if (sh->pool_k < 1 || sh->pool_k % 2 == 0) return JQ_ERR_SHAPE;
    if (!std::isfinite(sh->scale) || sh->scale < 0.0f) return JQ_ERR_SHAPE;
    if (sh->keep_first < 0 || sh->keep_last < 0) return JQ_ERR_SHAPE;
    if (sh->window != 0 && sh->window != 1) return JQ_ERR_SHAPE;
    if (sh->n_seq > JQ_MAX_SEQ) return JQ_ERR_UNSUPPORTED;
    if (sh->d != kHeadDim) return JQ_ERR_UNSUPPORTED;
    if (sh->n_layers > 65535 || sh->h_kv > 256) return JQ_ERR_UNSUPPORTED;  // grid dimensions
    if (sh->cu_seqlens[0] != 0) return JQ_ERR_SHAPE;
    for (int s = 0; s < sh->n_seq; ++s)
        if (sh->cu_seqlens[s + 1] <= sh->cu_seqlens[s]) return JQ_ERR_SHAPE;

    Plan p{};
    p.n_layers = sh->n_layers; p.n_seq = sh->n_seq; p.n_q = sh->n_q; p.h_q = sh->h_q; p.h_kv = sh->h_kv;
    p.d = sh->d; p.group = sh->h_q / sh->h_kv; p.pool_k = sh->pool_k;
    p.keep_first = sh->keep_first; p.keep_last = sh->keep_last;
    p.window = sh->window;
    p.layer_budgets = sh->layer_budgets;
    if (p.layer_budgets && misaligned(p.layer_budgets, 4)) return JQ_ERR_UNSUPPORTED;
    if (p.window) {  // the window's own positions are always kept
        if (p.keep_last < sh->n_q) p.keep_last = sh->n_q;
        for (int s = 0; s < sh->n_seq; ++s)
            if (sh->cu_seqlens[s + 1] - sh->cu_seqlens[s] < sh->n_q) return JQ_ERR_SHAPE;
    }
    p.scale = sh->scale > 0.0f ? sh->scale : (float)(1.0 / std::sqrt((double)sh->d));
    const int64_t rows = (int64_t)p.n_q * p.group;
    if (rows > (1 << 20)) return JQ_ERR_UNSUPPORTED;
    p.rows = (int32_t)rows;
    p.row_tiles = (p.rows + kRowTile - 1) / kRowTile;
    p.row_groups = (p.row_tiles + kMaxRowTiles - 1) / kMaxRowTiles;
    p.T = sh->cu_seqlens[sh->n_seq];
    p.tab.n_seq = sh->n_seq;
    int64_t tb = 0;
    for (int s = 0; s <= sh->n_seq; ++s) p.tab.cu_seq[s] = sh->cu_seqlens[s];
    p.tab.cu_bud[0] = 0;
    for (int s = 0; s < sh->n_seq; ++s) {
        // the score kernels address one head's rows of a sequence through a 32-bit buffer offset
        if ((int64_t)(sh->cu_seqlens[s + 1] - sh->cu_seqlens[s]) * p.h_kv * kHeadDim * 2 > (int64_t)UINT32_MAX) return JQ_ERR_UNSUPPORTED;
        int32_t b = 1;
        if (sh->budgets) {
            b = sh->budgets[s];
            const int32_t L = sh->cu_seqlens[s + 1] - sh->cu_seqlens[s];
            if (need_budgets && (b < 1 || b > L || (int64_t)p.keep_first + p.keep_last > b)) return JQ_ERR_BUDGET;
            if (b < 1 || b > L) b = 1;  // entry points that ignore budgets still get a sane table
        }
        tb += b;
        if (tb > INT32_MAX) return JQ_ERR_UNSUPPORTED;
        p.tab.cu_bud[s + 1] = (int32_t)tb;
    }
    p.TB = tb;

    // A sequence of L keys is worked on by ceil(L / chunk_keys) waves per head (which share its 32-key tiles
    // round-robin).  Small calls aim at one wave per SIMD (256 CUs x 4) in the pass that reads K cold (the
    // first pass, or the only one when the normalisers are supplied): one wave with two tiles in flight keeps
    // its SIMD busy and the window of K in flight stays small.  The second pass finds part of K in the
    // Infinity Cache and has more arithmetic per tile; it does better with two waves per SIMD.  The cap makes
    // big calls run in several rounds.
    const int64_t keys = (int64_t)p.n_layers * p.h_kv * p.T;
    auto plan_waves = [&](int64_t target_waves, int32_t knob, int32_t* cu_chunk, int32_t* cu_cgrp, int32_t* chunk_keys,
                          int32_t* n_chunks) {
        int64_t chunk = (keys + target_waves - 1) / target_waves;
        chunk = (chunk + kKeyTile - 1) / kKeyTile * kKeyTile;
        if (chunk < 64) chunk = 64;
        if (chunk > 1024) chunk = 1024;
        if (knob) chunk = knob;  // ablation knob
        int64_t nc = 0, ng = 0;
        cu_chunk[0] = 0;
        cu_cgrp[0] = 0;
        for (int s = 0; s < sh->n_seq; ++s) {
            const int64_t L = sh->cu_seqlens[s + 1] - sh->cu_seqlens[s];
            const int64_t waves = (L + chunk - 1) / chunk;
            nc += waves;
            ng += (waves + kScoreWaves - 1) / kScoreWaves;
            cu_chunk[s + 1] = (int32_t)nc;
            cu_cgrp[s + 1] = (int32_t)ng;
        }
        *chunk_keys = (int32_t)chunk;
        *n_chunks = (int32_t)nc;
        return ng;
    };
    const int64_t ng = plan_waves(1024, knobs().chunk_keys, p.tab.cu_chunk, p.tab.cu_cgrp, &p.chunk_keys, &p.n_chunks);
    const int64_t ng2 = plan_waves(2048, knobs().chunk_keys2, p.cu_chunk2, p.cu_cgrp2, &p.chunk_keys2, &p.n_chunks2);
    if ((int64_t)p.n_layers * (ng > ng2 ? ng : ng2) * p.h_kv >= INT32_MAX) return JQ_ERR_UNSUPPORTED;
    if ((int64_t)p.n_layers * p.n_seq * p.h_kv * p.row_tiles >= INT32_MAX) return JQ_ERR_UNSUPPORTED;

    // pooling workgroups (= segments of the selection's lists): whole sequences in pieces of kSegLen positions
    p.cu_seg[0] = 0;
    for (int s = 0; s < sh->n_seq; ++s) {
        const int64_t L = sh->cu_seqlens[s + 1] - sh->cu_seqlens[s];
        p.cu_seg[s + 1] = p.cu_seg[s] + (int32_t)((L + kSegLen - 1) / kSegLen);
    }
    p.n_seg = p.cu_seg[sh->n_seq];
    // Entries a segment keeps: eight times what a block of kSegLen scores contributes to the kept set on average
    // (densest sequence of the call), as a power of two in 128..kSegLen; blocks that hold more are re-read from
    // the scores by the selection.
    {
        double dens = 0.0;  // kept positions per score
        for (int s = 0; s < sh->n_seq; ++s) {
            const double L = sh->cu_seqlens[s + 1] - sh->cu_seqlens[s];
            const double B = p.tab.cu_bud[s + 1] - p.tab.cu_bud[s];
            if (B / L > dens) dens = B / L;
        }
        int head = 128;
        while (head < kSegLen && head < 8.0 * dens * kSegLen) head *= 2;
        p.seg_head = head;
    }

    const size_t RP = (size_t)p.row_tiles * kRowTile;
    size_t off = 0;
    p.off_stats = off;  off += align_up((size_t)p.n_layers * ng * p.h_kv * RP * sizeof(float2));  // one per pass-1 workgroup
    p.off_aug = off;    off += align_up((size_t)p.n_layers * p.n_seq * p.h_kv * RP * sizeof(uint2));
    p.off_hist = off;   off += align_up((size_t)p.n_layers * p.n_seq * p.h_kv * kHistStride * sizeof(uint32_t));
    p.off_scores = off; off += align_up((size_t)p.n_layers * p.h_kv * p.T * sizeof(float));
    p.off_pooled = off; off += align_up((size_t)p.n_layers * p.h_kv * p.T * sizeof(float));
    p.off_idx = off;    off += align_up((size_t)p.n_layers * p.h_kv * p.TB * sizeof(int32_t));
    p.off_seg = off;    off += align_up((size_t)p.n_layers * p.h_kv * p.n_seg * p.seg_head * sizeof(uint2));
    p.off_seghdr = off; off += align_up((size_t)p.n_layers * p.h_kv * p.n_seg * sizeof(uint4));
    p.ws_bytes = off;
    *out = p;
    return JQ_OK;
}

// Validates a paged-cache description against the plan and records it there.
int apply_pages(const jq_pages* pg, Plan* p) {
    if (!pg || !pg->block_table) return JQ_ERR_NULL;
    if (pg->page_size < kKeyTile || pg->page_size > 65536 || (pg->page_size & (pg->page_size - 1)) != 0) return JQ_ERR_SHAPE;
    if (pg->n_pages < 1 || pg->max_pages_per_seq < 1) return JQ_ERR_SHAPE;
    for (int s = 0; s < p->n_seq; ++s) {
        const int64_t L = p->tab.cu_seq[s + 1] - p->tab.cu_seq[s];
        if ((L + pg->page_size - 1) / pg->page_size > pg->max_pages_per_seq) return JQ_ERR_SHAPE;
    }
    // the score kernels address a layer's whole pool through one 32-bit buffer offset
    if ((int64_t)pg->n_pages * pg->page_size * p->h_kv * kHeadDim * 2 > (int64_t)UINT32_MAX) return JQ_ERR_UNSUPPORTED;
    if (misaligned(pg->block_table, 4)) return JQ_ERR_UNSUPPORTED;
    p->block_table = pg->block_table;
    p->page_shift = 0;
    while ((1 << p->page_shift) < pg->page_size) ++p->page_shift;
    p->n_pages = pg->n_pages;
    p->max_pages = pg->max_pages_per_seq;
    return JQ_OK;
}

// The same for the description of a paged output (no tile or 32-bit-offset constraint there).
int apply_out_pages(const jq_pages* pg, Plan* p) {
    if (!pg || !pg->block_table) return JQ_ERR_NULL;
    if (pg->page_size < 1 || pg->page_size > 65536 || (pg->page_size & (pg->page_size - 1)) != 0) return JQ_ERR_SHAPE;
    if (pg->n_pages < 1 || pg->max_pages_per_seq < 1) return JQ_ERR_SHAPE;
    for (int s = 0; s < p->n_seq; ++s) {
        const int64_t b = p->tab.cu_bud[s + 1] - p->tab.cu_bud[s];
        if ((b + pg->page_size - 1) / pg->page_size > pg->max_pages_per_seq) return JQ_ERR_SHAPE;
    }
    if (misaligned(pg->block_table, 4)) return JQ_ERR_UNSUPPORTED;
    p->out_map.block_table = pg->block_table;
    p->out_map.page_shift = 0;
    while ((1 << p->out_map.page_shift) < pg->page_size) ++p->out_map.page_shift;
    p->out_map.n_pages = pg->n_pages;
    p->out_map.max_pages = pg->max_pages_per_seq;
    return JQ_OK;
}

int check_ws(const Plan& p, const void* ws, size_t ws_bytes) {
    if (!ws) return JQ_ERR_NULL;
    if (misaligned(ws, 16) || ws_bytes < p.ws_bytes) return JQ_ERR_WORKSPACE;
    return JQ_OK;
}

size_t kv_bytes(const Plan& p) {  // bytes of K (or V) as the caller holds it: dense rows, or the pools of all layers
    const size_t rows = p.block_table ? ((size_t)p.n_pages << p.page_shift) : (size_t)p.T;
    return (size_t)p.n_layers * rows * p.h_kv * p.d * 2;
}
size_t lb_bytes(const Plan& p) { return p.layer_budgets ? (size_t)p.n_layers * p.n_seq * 4 : 0; }
size_t table_bytes(const Plan& p) { return p.block_table ? (size_t)p.n_seq * p.max_pages * 4 : 0; }
size_t kv_out_bytes(const Plan& p) {  // bytes of K_out (or V_out): dense kept rows, or the output pools of all layers
    const size_t rows = p.out_map.block_table ? ((size_t)p.out_map.n_pages << p.out_map.page_shift) : (size_t)p.TB;
    return (size_t)p.n_layers * rows * p.h_kv * p.d * 2;
}
size_t out_table_bytes(const Plan& p) { return p.out_map.block_table ? (size_t)p.n_seq * p.out_map.max_pages * 4 : 0; }
size_t q_bytes(const Plan& p) { return (size_t)p.n_layers * p.n_seq * p.n_q * p.h_q * p.d * 2; }
size_t score_bytes(const Plan& p) { return (size_t)p.n_layers * p.h_kv * p.T * 4; }
size_t idx_bytes(const Plan& p) { return (size_t)p.n_layers * p.h_kv * p.TB * 4; }
size_t lse_bytes(const Plan& p) { return (size_t)p.n_layers * p.n_seq * p.n_q * p.h_q * 4; }
size_t tail_bytes(const Plan& p) { return (size_t)p.n_layers * p.n_seq * p.n_q * p.h_kv * p.d * 2; }

inline int launch_status(hipError_t e) {
    if (e == hipSuccess) return JQ_OK;
    if (knobs().log) std::fprintf(stderr, "libjq: launch failed: %s\n", hipGetErrorString(e));
    return JQ_ERR_LAUNCH;
}

}  // namespace
}  // namespace jq

using namespace jq;

extern "C" {

int jq_workspace_bytes(const jq_shape* shape, size_t* bytes) {
    if (!bytes) return JQ_ERR_NULL;
    Plan p;
    const int rc = make_plan(shape, shape && shape->budgets, &p);
    if (rc != JQ_OK) return rc;
    *bytes = p.ws_bytes;
    return JQ_OK;
}

// `extra` is the variant's additional input: normalisers (lse) or the soft tokens' keys (k_tail), at most one.
static int score_impl(const jq_shape* shape, const void* Q, const void* K, const float* lse, const void* k_tail,
                      bool want_extra, float* scores, void* ws, size_t ws_bytes, void* stream,
                      const jq_pages* pages = nullptr, bool paged = false) {
    Plan p;
    int rc = make_plan(shape, false, &p);
    if (rc != JQ_OK) return rc;
    if (paged && (rc = apply_pages(pages, &p)) != JQ_OK) return rc;
    const void* extra = lse ? (const void*)lse : k_tail;
    if (p.window && k_tail) return JQ_ERR_SHAPE;  // the window's keys are part of K already
    if (!Q || !K || !scores || (want_extra && !extra)) return JQ_ERR_NULL;
    if ((rc = check_ws(p, ws, ws_bytes)) != JQ_OK) return rc;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(scores, 4) || (lse && misaligned(lse, 4)) ||
        (k_tail && misaligned(k_tail, 16)))
        return JQ_ERR_UNSUPPORTED;
    const size_t extra_bytes = lse ? lse_bytes(p) : tail_bytes(p);
    if (overlaps(scores, score_bytes(p), K, kv_bytes(p)) || overlaps(scores, score_bytes(p), Q, q_bytes(p)) ||
        overlaps(scores, score_bytes(p), ws, p.ws_bytes) || overlaps(ws, p.ws_bytes, Q, q_bytes(p)) ||
        overlaps(ws, p.ws_bytes, K, kv_bytes(p)) ||
        (extra && (overlaps(scores, score_bytes(p), extra, extra_bytes) || overlaps(ws, p.ws_bytes, extra, extra_bytes))) ||
        (paged && (overlaps(scores, score_bytes(p), p.block_table, table_bytes(p)) ||
                   overlaps(ws, p.ws_bytes, p.block_table, table_bytes(p)))))
        return JQ_ERR_ALIAS;
    return launch_status(launch_score(p, Q, K, scores, (char*)ws, (hipStream_t)stream, nullptr, 0, lse, k_tail));
}

int jq_score(const jq_shape* shape, const void* Q, const void* K, float* scores, void* ws, size_t ws_bytes,
             void* stream) {
    return score_impl(shape, Q, K, nullptr, nullptr, false, scores, ws, ws_bytes, stream);
}

int jq_score_lse(const jq_shape* shape, const void* Q, const void* K, const float* lse, float* scores, void* ws,
                 size_t ws_bytes, void* stream) {
    return score_impl(shape, Q, K, lse, nullptr, true, scores, ws, ws_bytes, stream);
}

int jq_score_tail(const jq_shape* shape, const void* Q, const void* K, const void* K_tail, float* scores, void* ws,
                  size_t ws_bytes, void* stream) {
    return score_impl(shape, Q, K, nullptr, K_tail, true, scores, ws, ws_bytes, stream);
}

int jq_pool(const jq_shape* shape, const float* scores, float* pooled, void* stream) {
    Plan p;
    const int rc = make_plan(shape, false, &p);
    if (rc != JQ_OK) return rc;
    if (!scores || !pooled) return JQ_ERR_NULL;
    if (misaligned(scores, 4) || misaligned(pooled, 4)) return JQ_ERR_UNSUPPORTED;
    if (overlaps(scores, score_bytes(p), pooled, score_bytes(p))) return JQ_ERR_ALIAS;
    return launch_status(launch_pool(p, scores, pooled, nullptr, nullptr, (hipStream_t)stream));
}

int jq_select_topk(const jq_shape* shape, const float* pooled, int32_t* idx, void* ws, size_t ws_bytes,
                   void* stream) {
    Plan p;
    int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (!pooled || !idx) return JQ_ERR_NULL;
    if ((rc = check_ws(p, ws, ws_bytes)) != JQ_OK) return rc;
    if (misaligned(pooled, 4) || misaligned(idx, 4)) return JQ_ERR_UNSUPPORTED;
    if (overlaps(idx, idx_bytes(p), pooled, score_bytes(p)) || overlaps(idx, idx_bytes(p), ws, p.ws_bytes) ||
        overlaps(pooled, score_bytes(p), ws, p.ws_bytes) ||
        (p.layer_budgets && (overlaps(idx, idx_bytes(p), p.layer_budgets, lb_bytes(p)) ||
                             overlaps(ws, p.ws_bytes, p.layer_budgets, lb_bytes(p)))))
        return JQ_ERR_ALIAS;
    hipStream_t st = (hipStream_t)stream;
    uint32_t* hist = (uint32_t*)((char*)ws + p.off_hist);
    hipError_t e = launch_fill_u32(hist, (size_t)p.n_layers * p.n_seq * p.h_kv * kHistStride, 0u, st);
    if (e == hipSuccess) e = launch_hist(p, pooled, hist, (char*)ws, st);
    if (e == hipSuccess) e = launch_select(p, pooled, hist, (char*)ws, idx, st);
    return launch_status(e);
}

int jq_compact(const jq_shape* shape, const void* K, const void* V, const int32_t* idx, void* K_out, void* V_out,
               void* stream) {
    Plan p;
    const int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (!K || !V || !idx || !K_out || !V_out) return JQ_ERR_NULL;
    if (misaligned(K, 16) || misaligned(V, 16) || misaligned(K_out, 16) || misaligned(V_out, 16) || misaligned(idx, 4))
        return JQ_ERR_UNSUPPORTED;
    const size_t nin = kv_bytes(p), nout = kv_out_bytes(p);
    if (overlaps(K_out, nout, K, nin) || overlaps(K_out, nout, V, nin) || overlaps(V_out, nout, K, nin) ||
        overlaps(V_out, nout, V, nin) || overlaps(K_out, nout, V_out, nout) || overlaps(K_out, nout, idx, idx_bytes(p)) ||
        overlaps(V_out, nout, idx, idx_bytes(p)) ||
        (p.layer_budgets && (overlaps(K_out, nout, p.layer_budgets, lb_bytes(p)) || overlaps(V_out, nout, p.layer_budgets, lb_bytes(p)))))
        return JQ_ERR_ALIAS;
    return launch_status(launch_compact(p, K, V, idx, K_out, V_out, (hipStream_t)stream));
}

int jq_compact_inplace_workspace_bytes(const jq_shape* shape, size_t* bytes) {
    if (!bytes) return JQ_ERR_NULL;
    Plan p;
    const int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    *bytes = align_up(2 * kv_out_bytes(p));
    return JQ_OK;
}

int jq_compact_inplace(const jq_shape* shape, void* K, void* V, const int32_t* idx, void* ws, size_t ws_bytes,
                       void* stream) {
    Plan p;
    const int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (!K || !V || !idx || !ws) return JQ_ERR_NULL;
    if (misaligned(K, 16) || misaligned(V, 16) || misaligned(idx, 4)) return JQ_ERR_UNSUPPORTED;
    const size_t need = 2 * kv_out_bytes(p);
    if (misaligned(ws, 16) || ws_bytes < need) return JQ_ERR_WORKSPACE;
    const size_t nin = kv_bytes(p);
    if (overlaps(K, nin, V, nin) || overlaps(ws, need, K, nin) || overlaps(ws, need, V, nin) ||
        overlaps(idx, idx_bytes(p), K, nin) || overlaps(idx, idx_bytes(p), V, nin) || overlaps(idx, idx_bytes(p), ws, need) ||
        (p.layer_budgets && (overlaps(K, nin, p.layer_budgets, lb_bytes(p)) || overlaps(V, nin, p.layer_budgets, lb_bytes(p)) ||
                             overlaps(ws, need, p.layer_budgets, lb_bytes(p)))))
        return JQ_ERR_ALIAS;
    return launch_status(launch_compact_inplace(p, K, V, idx, ws, (hipStream_t)stream));
}

static int evict_impl(const jq_shape* shape, const void* Q, const void* K, const void* V, const float* lse,
                      const void* k_tail, void* K_out, void* V_out, int32_t* idx_out, float* scores_out, void* ws,
                      size_t ws_bytes, void* stream, void* const* marks, const jq_pages* pages = nullptr,
                      bool paged = false, const jq_pages* out_pages = nullptr, const int32_t* pos_in = nullptr,
                      int32_t* pos_out = nullptr) {
    Plan p;
    int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (paged && (rc = apply_pages(pages, &p)) != JQ_OK) return rc;
    if (out_pages && (rc = apply_out_pages(out_pages, &p)) != JQ_OK) return rc;
    if (p.window && k_tail) return JQ_ERR_SHAPE;  // the window's keys are part of K already
    if (!Q || !K || !V || !K_out || !V_out) return JQ_ERR_NULL;
    if ((rc = check_ws(p, ws, ws_bytes)) != JQ_OK) return rc;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || misaligned(K_out, 16) || misaligned(V_out, 16) ||
        (idx_out && misaligned(idx_out, 4)) || (scores_out && misaligned(scores_out, 4)) || (lse && misaligned(lse, 4)) ||
        (k_tail && misaligned(k_tail, 16)))
        return JQ_ERR_UNSUPPORTED;
    const size_t nin = kv_bytes(p), nout = kv_out_bytes(p);
    if ((pos_in && misaligned(pos_in, 4)) || (pos_out && misaligned(pos_out, 4))) return JQ_ERR_UNSUPPORTED;
    const void* ins[8] = {Q, K, V, lse ? (const void*)lse : k_tail, p.block_table, p.out_map.block_table, p.layer_budgets, pos_in};
    const size_t in_bytes[8] = {q_bytes(p), nin, nin, lse ? lse_bytes(p) : tail_bytes(p), table_bytes(p), out_table_bytes(p),
                                lb_bytes(p), score_bytes(p)};
    const void* outs[6] = {K_out, V_out, idx_out, scores_out, ws, pos_out};
    const size_t out_bytes[6] = {nout, nout, idx_bytes(p), score_bytes(p), p.ws_bytes, idx_bytes(p)};
    for (int o = 0; o < 6; ++o) {
        if (!outs[o]) continue;
        for (int i = 0; i < 8; ++i)
            if (ins[i] && overlaps(outs[o], out_bytes[o], ins[i], in_bytes[i])) return JQ_ERR_ALIAS;
        for (int o2 = o + 1; o2 < 6; ++o2)
            if (outs[o2] && overlaps(outs[o], out_bytes[o], outs[o2], out_bytes[o2])) return JQ_ERR_ALIAS;
    }

    hipStream_t st = (hipStream_t)stream;
    char* w = (char*)ws;
    uint32_t* hist = (uint32_t*)(w + p.off_hist);
    float* raw = (float*)(w + p.off_scores);
    float* pooled = scores_out ? scores_out : (float*)(w + p.off_pooled);
    int32_t* idx = idx_out ? idx_out : (int32_t*)(w + p.off_idx);
    p.marks = marks;
    const size_t zero_words = (size_t)p.n_layers * p.n_seq * p.h_kv * kHistStride;
    hipError_t e = launch_score(p, Q, K, raw, w, st, hist, zero_words, lse, k_tail);  // also clears the selection histograms
    if (e == hipSuccess) e = launch_pool(p, raw, pooled, hist, w, st);
    bool gathered = false;  // the selection's last kernel gathers the kept rows itself unless it had to stream
    if (e == hipSuccess) e = launch_select(p, pooled, hist, w, idx, st, K, V, K_out, V_out, &gathered, nullptr, pos_in, pos_out);
    if (e == hipSuccess && !gathered) e = launch_compact(p, K, V, idx, K_out, V_out, st);
    return launch_status(e);
}

int jq_evict_inplace_workspace_bytes(const jq_shape* shape, size_t* bytes) {
    if (!bytes) return JQ_ERR_NULL;
    Plan p;
    const int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    *bytes = p.ws_bytes + align_up(2 * kv_out_bytes(p));
    return JQ_OK;
}

int jq_evict_inplace(const jq_shape* shape, const void* Q, void* K, void* V, const float* lse, int32_t* idx_out,
                     float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    Plan p;
    int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (!Q || !K || !V) return JQ_ERR_NULL;
    if (!ws) return JQ_ERR_NULL;
    const size_t stage_bytes = 2 * kv_out_bytes(p), need = p.ws_bytes + align_up(stage_bytes);
    if (misaligned(ws, 16) || ws_bytes < need) return JQ_ERR_WORKSPACE;
    if (misaligned(Q, 16) || misaligned(K, 16) || misaligned(V, 16) || (idx_out && misaligned(idx_out, 4)) ||
        (scores_out && misaligned(scores_out, 4)) || (lse && misaligned(lse, 4)))
        return JQ_ERR_UNSUPPORTED;
    const size_t nin = kv_bytes(p);
    const void* bufs[8] = {Q, K, V, lse, p.layer_budgets, idx_out, scores_out, ws};
    const size_t sizes[8] = {q_bytes(p), nin, nin, lse_bytes(p), lb_bytes(p), idx_bytes(p), score_bytes(p), need};
    for (int i = 0; i < 8; ++i)  // K and V are written: nothing may overlap them; outputs and workspace overlap nothing
        for (int j = i + 1; j < 8; ++j)
            if (bufs[i] && bufs[j] && (i == 1 || i == 2 || j == 1 || j == 2 || j >= 5) && overlaps(bufs[i], sizes[i], bufs[j], sizes[j]))
                return JQ_ERR_ALIAS;

    hipStream_t st = (hipStream_t)stream;
    char* w = (char*)ws;
    char* stage = w + p.ws_bytes;
    uint32_t* hist = (uint32_t*)(w + p.off_hist);
    float* raw = (float*)(w + p.off_scores);
    float* pooled = scores_out ? scores_out : (float*)(w + p.off_pooled);
    int32_t* idx = idx_out ? idx_out : (int32_t*)(w + p.off_idx);
    const size_t zero_words = (size_t)p.n_layers * p.n_seq * p.h_kv * kHistStride;
    hipError_t e = launch_score(p, Q, K, raw, w, st, hist, zero_words, lse, nullptr);
    if (e == hipSuccess) e = launch_pool(p, raw, pooled, hist, w, st);
    // The selection kernel saves the kept rows that are about to be overwritten; one more launch then writes every
    // kept row over the front of K and V.  (A streaming selection saves nothing: both launches of the stand-alone
    // in-place gather run.)
    bool staged = false;
    if (e == hipSuccess) e = launch_select(p, pooled, hist, w, idx, st, K, V, nullptr, nullptr, &staged, stage);
    if (e == hipSuccess) e = staged ? launch_compact_inplace_write(p, K, V, idx, stage, st) : launch_compact_inplace(p, K, V, idx, stage, st);
    return launch_status(e);
}

// workspace of the paged in-place eviction: the scratch of jq_evict, the staged rows, the destination-page bitmap
static size_t paged_inplace_bytes(const Plan& p, size_t* off_stage, size_t* off_bits) {
    *off_stage = p.ws_bytes;
    *off_bits = *off_stage + align_up(2 * (size_t)p.n_layers * p.TB * p.h_kv * p.d * 2);
    return *off_bits + align_up(((size_t)p.n_pages + 31) / 32 * 4);
}

int jq_evict_paged_inplace_workspace_bytes(const jq_shape* shape, const jq_pages* pages, size_t* bytes) {
    if (!bytes) return JQ_ERR_NULL;
    Plan p;
    int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if ((rc = apply_pages(pages, &p)) != JQ_OK) return rc;
    size_t o1, o2;
    *bytes = paged_inplace_bytes(p, &o1, &o2);
    return JQ_OK;
}

int jq_evict_paged_inplace(const jq_shape* shape, const jq_pages* pages, const jq_pages* out_pages, const void* Q, void* K_pool,
                           void* V_pool, const float* lse, int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes,
                           void* stream) {
    Plan p;
    int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if ((rc = apply_pages(pages, &p)) != JQ_OK) return rc;
    if ((rc = apply_out_pages(out_pages, &p)) != JQ_OK) return rc;
    // the kept rows go to other (or the same) pages of the very pools they are taken from
    if (out_pages->page_size != pages->page_size || out_pages->n_pages != pages->n_pages) return JQ_ERR_SHAPE;
    if (!Q || !K_pool || !V_pool || !ws) return JQ_ERR_NULL;
    size_t off_stage, off_bits;
    const size_t need = paged_inplace_bytes(p, &off_stage, &off_bits);
    if (misaligned(ws, 16) || ws_bytes < need) return JQ_ERR_WORKSPACE;
    if (misaligned(Q, 16) || misaligned(K_pool, 16) || misaligned(V_pool, 16) || (idx_out && misaligned(idx_out, 4)) ||
        (scores_out && misaligned(scores_out, 4)) || (lse && misaligned(lse, 4)))
        return JQ_ERR_UNSUPPORTED;
    const size_t nin = kv_bytes(p);
    const void* bufs[10] = {Q, K_pool, V_pool, lse, p.layer_budgets, p.block_table, p.out_map.block_table, idx_out, scores_out, ws};
    const size_t sizes[10] = {q_bytes(p), nin, nin, lse_bytes(p), lb_bytes(p), table_bytes(p), out_table_bytes(p), idx_bytes(p),
                              score_bytes(p), need};
    for (int i = 0; i < 10; ++i)  // the pools are written: nothing may overlap them; outputs and workspace overlap nothing
        for (int j = i + 1; j < 10; ++j)
            if (bufs[i] && bufs[j] && (i == 1 || i == 2 || j == 1 || j == 2 || j >= 7) && overlaps(bufs[i], sizes[i], bufs[j], sizes[j]))
                return JQ_ERR_ALIAS;

    hipStream_t st = (hipStream_t)stream;
    char* w = (char*)ws;
    char* stage = w + off_stage;
    uint32_t* dest_bits = (uint32_t*)(w + off_bits);
    uint32_t* hist = (uint32_t*)(w + p.off_hist);
    float* raw = (float*)(w + p.off_scores);
    float* pooled = scores_out ? scores_out : (float*)(w + p.off_pooled);
    int32_t* idx = idx_out ? idx_out : (int32_t*)(w + p.off_idx);
    const size_t zero_words = (size_t)p.n_layers * p.n_seq * p.h_kv * kHistStride;
    hipError_t e = launch_mark_dest_pages(p, dest_bits, st);  // which pages receive kept rows (read by the last two kernels)
    if (e == hipSuccess) e = launch_score(p, Q, K_pool, raw, w, st, hist, zero_words, lse, nullptr);
    if (e == hipSuccess) e = launch_pool(p, raw, pooled, hist, w, st);
    bool staged = false;
    if (e == hipSuccess) e = launch_select(p, pooled, hist, w, idx, st, K_pool, V_pool, nullptr, nullptr, &staged, stage, nullptr, nullptr, dest_bits);
    if (e == hipSuccess)
        e = staged ? launch_compact_inplace_write(p, K_pool, V_pool, idx, stage, st, dest_bits)
                   : launch_compact_inplace(p, K_pool, V_pool, idx, stage, st, dest_bits);
    return launch_status(e);
}

int jq_evict(const jq_shape* shape, const void* Q, const void* K, const void* V, void* K_out, void* V_out,
             int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    return evict_impl(shape, Q, K, V, nullptr, nullptr, K_out, V_out, idx_out, scores_out, ws, ws_bytes, stream, nullptr);
}

int jq_evict_stream(const jq_shape* shape, const void* Q, const void* K, const void* V, const int32_t* pos, const float* lse,
                    void* K_out, void* V_out, int32_t* pos_out, int32_t* idx_out, float* scores_out, void* ws,
                    size_t ws_bytes, void* stream) {
    if (!pos || !pos_out) return JQ_ERR_NULL;
    return evict_impl(shape, Q, K, V, lse, nullptr, K_out, V_out, idx_out, scores_out, ws, ws_bytes, stream, nullptr, nullptr,
                      false, nullptr, pos, pos_out);
}

int jq_evict_lse(const jq_shape* shape, const void* Q, const void* K, const void* V, const float* lse, void* K_out,
                 void* V_out, int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    if (!lse) return JQ_ERR_NULL;
    return evict_impl(shape, Q, K, V, lse, nullptr, K_out, V_out, idx_out, scores_out, ws, ws_bytes, stream, nullptr);
}

int jq_evict_tail(const jq_shape* shape, const void* Q, const void* K, const void* V, const void* K_tail, void* K_out,
                  void* V_out, int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream) {
    if (!K_tail) return JQ_ERR_NULL;
    return evict_impl(shape, Q, K, V, nullptr, K_tail, K_out, V_out, idx_out, scores_out, ws, ws_bytes, stream, nullptr);
}

// ---- jq_evict without a caller workspace ----------------------------------------------------------------
// The scratch memory of the eviction kernels (softmax partials, histograms, raw scores, candidate lists) in a
// file-scope device array instead of a caller buffer.  `scratch` names the array for the device compiler only; on
// the host it is a stand-in, so the array's device address is looked up once per device and only that address is
// ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[JQ_STATIC_WS_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_ptr[kMaxDevices];  // per device: the address of that device's copy of `scratch`

int static_scratch(void** out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return JQ_ERR_LAUNCH;
    void* p = scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {  // first call on this device (which is current): every thread that races here finds the same address
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return JQ_ERR_LAUNCH;
        scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return JQ_OK;
}
}  // namespace

int jq_evict_static(const jq_shape* shape, const void* Q, const void* K, const void* V, void* K_out, void* V_out,
                    int32_t* idx_out, float* scores_out, void* stream) {
    Plan p;
    const int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (p.ws_bytes > (size_t)JQ_STATIC_WS_BYTES) return JQ_ERR_WORKSPACE;  // the problem needs more scratch than the array holds
    if (!Q || !K || !V || !K_out || !V_out) return JQ_ERR_NULL;
    void* ws = nullptr;
    const int rs = static_scratch(&ws);
    if (rs != JQ_OK) return rs;
    // Nothing in the scratch area has to survive from, or be cleared before, a call: the first kernels write the
    // partial statistics and clear the histograms and list counters before anything reads them.
    return evict_impl(shape, Q, K, V, nullptr, nullptr, K_out, V_out, idx_out, scores_out, ws, JQ_STATIC_WS_BYTES, stream,
                      nullptr);
}

int jq_score_paged(const jq_shape* shape, const jq_pages* pages, const void* Q, const void* K_pool, const float* lse,
                   float* scores, void* ws, size_t ws_bytes, void* stream) {
    return score_impl(shape, Q, K_pool, lse, nullptr, false, scores, ws, ws_bytes, stream, pages, true);
}

int jq_evict_paged(const jq_shape* shape, const jq_pages* pages, const jq_pages* out_pages, const void* Q, const void* K_pool,
                   const void* V_pool, const float* lse, void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                   void* ws, size_t ws_bytes, void* stream) {
    return evict_impl(shape, Q, K_pool, V_pool, lse, nullptr, K_out, V_out, idx_out, scores_out, ws, ws_bytes, stream,
                      nullptr, pages, true, out_pages);
}

int jq_evict_traced(const jq_shape* shape, const void* Q, const void* K, const void* V, void* K_out, void* V_out,
                    int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes, void* stream,
                    void* const* marks, int n_marks) {
    if (!marks) return JQ_ERR_NULL;
    if (n_marks != JQ_TRACE_MARKS) return JQ_ERR_SHAPE;
    for (int i = 0; i < n_marks; ++i)
        if (!marks[i]) return JQ_ERR_NULL;
    return evict_impl(shape, Q, K, V, nullptr, nullptr, K_out, V_out, idx_out, scores_out, ws, ws_bytes, stream, marks);
}

int jq_hit_rate(const jq_shape* shape, const int32_t* idx_cur, const int32_t* idx_ref, const int32_t* ref_budgets,
                float* rate, void* stream) {
    Plan p;
    const int rc = make_plan(shape, true, &p);
    if (rc != JQ_OK) return rc;
    if (!idx_cur || !idx_ref || !rate) return JQ_ERR_NULL;
    int32_t cu_ref[JQ_MAX_SEQ + 1];
    int64_t tb_ref = 0;
    cu_ref[0] = 0;
    for (int s = 0; s < p.n_seq; ++s) {
        const int32_t L = shape->cu_seqlens[s + 1] - shape->cu_seqlens[s];
        const int32_t b = ref_budgets ? ref_budgets[s] : shape->budgets[s];
        if (b < 1 || b > L) return JQ_ERR_BUDGET;
        tb_ref += b;
        if (tb_ref > INT32_MAX) return JQ_ERR_UNSUPPORTED;
        cu_ref[s + 1] = (int32_t)tb_ref;
    }
    if (misaligned(idx_cur, 4) || misaligned(idx_ref, 4) || misaligned(rate, 4)) return JQ_ERR_UNSUPPORTED;
    const size_t rate_bytes = (size_t)p.n_layers * p.n_seq * p.h_kv * sizeof(float);
    const size_t ref_bytes = (size_t)p.n_layers * p.h_kv * (size_t)tb_ref * sizeof(int32_t);
    if (overlaps(rate, rate_bytes, idx_cur, idx_bytes(p)) || overlaps(rate, rate_bytes, idx_ref, ref_bytes)) return JQ_ERR_ALIAS;
    return launch_status(launch_hit_rate(p, cu_ref, tb_ref, idx_cur, idx_ref, rate, (hipStream_t)stream));
}

int jq_map_mse(const jq_shape* shape, const float* scores_a, float rows_a, const float* scores_b, float rows_b, float* mse,
               void* stream) {
    Plan p;
    const int rc = make_plan(shape, false, &p);
    if (rc != JQ_OK) return rc;
    if (!scores_a || !scores_b || !mse) return JQ_ERR_NULL;
    if (!(rows_a > 0.0f) || !(rows_b > 0.0f) || !std::isfinite(rows_a) || !std::isfinite(rows_b)) return JQ_ERR_SHAPE;
    if (misaligned(scores_a, 4) || misaligned(scores_b, 4) || misaligned(mse, 4)) return JQ_ERR_UNSUPPORTED;
    const size_t out_bytes = (size_t)p.n_layers * p.n_seq * p.h_kv * sizeof(float);
    if (overlaps(mse, out_bytes, scores_a, score_bytes(p)) || overlaps(mse, out_bytes, scores_b, score_bytes(p)))
        return JQ_ERR_ALIAS;
    return launch_status(launch_map_mse(p, scores_a, rows_a, scores_b, rows_b, mse, (hipStream_t)stream));
}

// Layout of the fused forward's workspace: the plan of either query set in full, then the partial sums.
static int mse_fused_plans(const jq_shape* shape, int32_t n_q_b, Plan* pa, Plan* pb, size_t* off_b, size_t* off_part, size_t* total) {
    int rc = make_plan(shape, false, pa);
    if (rc != JQ_OK) return rc;
    if (n_q_b < 1) return JQ_ERR_SHAPE;
    if (pa->window) return JQ_ERR_SHAPE;  // the maps of Eq. 3 / Eq. 4 have no window mode
    jq_shape sb = *shape;
    sb.n_q = n_q_b;
    if ((rc = make_plan(&sb, false, pb)) != JQ_OK) return rc;
    *off_b = pa->ws_bytes;
    *off_part = *off_b + pb->ws_bytes;
    *total = *off_part + align_up((size_t)pb->n_layers * pb->cu_cgrp2[pb->n_seq] * pb->h_kv * sizeof(double));
    return JQ_OK;
}

int jq_map_mse_fused_workspace_bytes(const jq_shape* shape, int32_t n_q_b, size_t* bytes) {
    if (!bytes) return JQ_ERR_NULL;
    Plan pa, pb;
    size_t off_b, off_part;
    return mse_fused_plans(shape, n_q_b, &pa, &pb, &off_b, &off_part, bytes);
}

int jq_map_mse_fused(const jq_shape* shape, const void* Q_a, const void* Q_b, int32_t n_q_b, const void* K, float* mse,
                     void* ws, size_t ws_bytes, void* stream) {
    Plan pa, pb;
    size_t off_b, off_part, total;
    const int rc = mse_fused_plans(shape, n_q_b, &pa, &pb, &off_b, &off_part, &total);
    if (rc != JQ_OK) return rc;
    if (!Q_a || !Q_b || !K || !mse) return JQ_ERR_NULL;
    if (!ws) return JQ_ERR_NULL;
    if (misaligned(ws, 16) || ws_bytes < total) return JQ_ERR_WORKSPACE;
    if (misaligned(Q_a, 16) || misaligned(Q_b, 16) || misaligned(K, 16) || misaligned(mse, 4)) return JQ_ERR_UNSUPPORTED;
    const size_t out_bytes = (size_t)pa.n_layers * pa.n_seq * pa.h_kv * sizeof(float);
    const void* ins[3] = {Q_a, Q_b, K};
    const size_t in_bytes[3] = {q_bytes(pa), q_bytes(pb), kv_bytes(pa)};
    for (int i = 0; i < 3; ++i)
        if (overlaps(ws, total, ins[i], in_bytes[i]) || overlaps(mse, out_bytes, ins[i], in_bytes[i])) return JQ_ERR_ALIAS;
    if (overlaps(mse, out_bytes, ws, total)) return JQ_ERR_ALIAS;
    hipStream_t st = (hipStream_t)stream;
    char* w = (char*)ws;
    float* map_a = (float*)(w + pa.off_scores);
    float* map_b = (float*)(w + off_b + pb.off_scores);  // holds the sums of the response's earlier row groups, if any
    hipError_t e = launch_score(pa, Q_a, K, map_a, w, st);
    MseFuse fuse;
    fuse.ref = map_a;
    fuse.inv_rows_ref = 1.0f / (float)pa.rows;
    fuse.inv_rows_own = 1.0f / (float)pb.rows;
    fuse.part = (double*)(w + off_part);
    if (e == hipSuccess) e = launch_score(pb, Q_b, K, map_b, w + off_b, st, nullptr, 0, nullptr, nullptr, &fuse);
    if (e == hipSuccess) e = launch_mse_reduce(pb, fuse.part, mse, st);
    return launch_status(e);
}

int jq_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst) return JQ_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return JQ_ERR_SHAPE;
    if (misaligned(src, 16) || misaligned(dst, 16)) return JQ_ERR_UNSUPPORTED;
    if (overlaps(src, bytes, dst, bytes)) return JQ_ERR_ALIAS;
    return launch_status(launch_copy_probe(src, dst, bytes, (hipStream_t)stream));
}

int jq_reload_knobs(void) {
    knobs_storage() = read_knobs();
    return JQ_OK;
}

const char* jq_status_string(int status) {
    switch (status) {
        case JQ_OK: return "ok";
        case JQ_ERR_NULL: return "a required pointer is NULL";
        case JQ_ERR_SHAPE: return "malformed shape (dimension, pool_k, scale or cu_seqlens)";
        case JQ_ERR_BUDGET: return "a budget is outside 1..L or below keep_first + keep_last";
        case JQ_ERR_UNSUPPORTED:
            return "valid but unsupported (d != 128, more than JQ_MAX_SEQ sequences, more than 65535 layers or 256 KV heads, "
                   "a sequence or a layer's page pool with 4 GiB or more of keys, more than 2^31 - 1 kept rows or "
                   "workgroups in one call, or a misaligned tensor)";
        case JQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case JQ_ERR_ALIAS: return "an output overlaps an input or another output";
        case JQ_ERR_LAUNCH: return "the HIP runtime refused a launch";
        default: return "unknown status";
    }
}

}  // extern "C"
