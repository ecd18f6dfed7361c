// Host side of the C ABI: argument validation, workspace layout, launch sequencing.
// No call here allocates device memory, synchronises, or reads device memory.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <unordered_map>

#include "ice_internal.h"

struct ice_index : ice::Host {};

namespace {

using namespace ice;

thread_local char g_err[512] = "";

ice_status_t fail(ice_status_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

ice_status_t check_cfg(const ice_config_t *c) {
    if (!c) return fail(ICE_ERR_INVALID_ARG, "config is null");
    if (c->batch < 1 || c->n_kv_heads < 1 || c->max_tokens < 1 || c->kmeans_iters < 1)
        return fail(ICE_ERR_INVALID_ARG, "batch, n_kv_heads, max_tokens and kmeans_iters must be >= 1");
    if (c->head_dim != kD) return fail(ICE_ERR_UNSUPPORTED, "head_dim %d: only 128 is supported", c->head_dim);
    if (c->group_size != 1 && c->group_size != 2 && c->group_size != 4 && c->group_size != 8)
        return fail(ICE_ERR_UNSUPPORTED, "group_size %d: only 1, 2, 4, 8 are supported", c->group_size);
    if ((long long)c->batch * c->n_kv_heads > 65535) return fail(ICE_ERR_UNSUPPORTED, "more than 65535 units");
    return ICE_OK;
}

ice_status_t check_shape(int page_size, int n_clusters) {
    if (page_size != 16 && page_size != 32 && page_size != 64)
        return fail(ICE_ERR_UNSUPPORTED, "page_size %d: only 16, 32, 64 are supported", page_size);
    if (n_clusters < 1) return fail(ICE_ERR_INVALID_ARG, "n_clusters must be >= 1");
    if (n_clusters > 8192) return fail(ICE_ERR_UNSUPPORTED, "n_clusters %d: at most 8192", n_clusters);
    return ICE_OK;
}

// Carves the workspace; with base == nullptr only measures.  Every region is 256-byte aligned.
size_t lay_out(const ice_config_t &cfg, int s, int C, char *base, Dev *out) {
    Dev d{};
    d.U = cfg.batch * cfg.n_kv_heads;
    d.G = cfg.group_size;
    d.s = s;
    d.C = C;
    d.Cpad = round_up(C, 32);
    d.max_tokens = cfg.max_tokens;
    d.max_pages = cfg.max_tokens / s + C;
    const size_t U = d.U, MP = d.max_pages, MT = d.max_tokens, CP = d.Cpad;
    size_t off = 0;
    auto take = [&](size_t bytes) -> char * {
        char *p = base ? base + off : nullptr;
        off += (bytes + 255) / 256 * 256;
        return p;
    };
    d.Kp = (bf16_t *)take(U * MP * s * kD * 2);
    d.Vp = (bf16_t *)take(U * MP * s * kD * 2);
    d.page_cluster = (int *)take(U * MP * 4);
    d.page_fill = (int *)take(U * MP * 4);
    d.page_pos = (int *)take(U * MP * s * 4);
    d.cluster_tail = (int *)take(U * C * 4);
    d.cluster_cnt = (int *)take(U * C * 4);
    d.tail_fill = (int *)take(U * C * 4);
    d.tail_sum = (float *)take(U * C * kD * 4);
    d.cluster_sum = (float *)take(U * C * kD * 4);
    d.centroid = (float *)take(U * C * kD * 4);
    d.page_sum = (float *)take(U * MP * kD * 4);
    d.rep = (bf16_t *)take(U * MP * kD * 2);
    d.n_pages = (int *)take(U * 4);
    d.n_tokens = (int *)take(U * 4);
    for (int b = 0; b < 2; ++b) {
        d.cent_bf16[b] = (bf16_t *)take(U * CP * kD * 2);
        d.cnorm[b] = (float *)take(U * CP * 4);
    }
    d.kaug = (bf16_t *)take(U * MT * 2);
    for (int b = 0; b < 2; ++b) d.caug[b] = (bf16_t *)take(U * CP * 2);
    d.cent_aug = (float *)take(U * C * 4);
    d.csum_aug = (float *)take(U * C * 4);
    d.c2 = (float *)take(U * 4);
    d.top_cent = (float *)take(U * kTopMax * kD * 4);
    d.top_bf16 = (bf16_t *)take(U * kTopMax * kD * 2);
    d.top_of = (int *)take(U * C * 4);
    d.top_cnt = (int *)take(U * kTopMax * 4);
    d.top_init = (int *)take(U * kTopMax * 4);
    d.init_idx = (int *)take(U * C * 4);
    d.assign = (int *)take(U * MT * 4);
    d.packed = (unsigned long long *)take(U * MT * 8);
    d.order = (int *)take(U * MT * 4);
    d.cluster_start = (int *)take(U * (CP + 1) * 4);
    d.page_base = (int *)take(U * (CP + 1) * 4);
    d.range_tot = (int *)take(std::max<size_t>(U, 256) * CP * 4);
    d.attn_part = (float *)take((size_t)256 * d.G * (kD + 2) * 4);
    d.attn_arrive = (int *)take(U * 4);
    d.scores = (uint32_t *)take(U * MP * 4);
    d.counter = (int *)take(U * 4);
    if (out) *out = d;
    return off;
}

ice_status_t ensure_layout(ice_index *ix, int s, int C) {
    if (ix->laid_out && ix->dev.s == s && ix->dev.C == C) return ICE_OK;
    const size_t need = lay_out(ix->cfg, s, C, nullptr, nullptr);
    if (need > ix->ws_bytes)
        return fail(ICE_ERR_CAPACITY, "workspace has %zu bytes, page_size %d / n_clusters %d need %zu", ix->ws_bytes, s,
                    C, need);
    lay_out(ix->cfg, s, C, ix->ws, &ix->dev);
    ix->dev.tk = ix->geometry;
    ix->laid_out = true;
    ix->built = false;
    return ICE_OK;
}

ice_status_t device_status(const char *what) {
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ICE_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return ICE_OK;
}

__global__ void fill_i32_kernel(int *p, int n, int v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// token counters, arrival counters and the empty marks of the score slots
void reset_decode_state(const Dev &d, int n_tokens, hipStream_t s) {
    hipLaunchKernelGGL(fill_i32_kernel, dim3((d.U + 255) / 256), dim3(256), 0, s, d.n_tokens, d.U, n_tokens);
    hipLaunchKernelGGL(fill_i32_kernel, dim3((d.U + 255) / 256), dim3(256), 0, s, d.counter, d.U, 0);
    hipLaunchKernelGGL(fill_i32_kernel, dim3((d.U + 255) / 256), dim3(256), 0, s, d.attn_arrive, d.U, 0);
    const int ns = d.U * d.max_pages;
    hipLaunchKernelGGL(fill_i32_kernel, dim3((ns + 255) / 256), dim3(256), 0, s, (int *)d.scores, ns, -1);
}

}  // namespace

namespace ice {

void allow_dynamic_lds(const void *kernel, size_t bytes) {
    static std::mutex mu;
    static std::unordered_map<uintptr_t, size_t> allowed;  // per (kernel, device): the largest size set so far
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::lock_guard<std::mutex> lock(mu);
    size_t &have = allowed[reinterpret_cast<uintptr_t>(kernel) * 64u + (uintptr_t)(dev & 63)];
    if (bytes <= have) return;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess) have = bytes;
}

}  // namespace ice

extern "C" {

const char *ice_last_error(void) { return g_err; }

size_t ice_workspace_bytes(const ice_config_t *cfg, int32_t page_size, int32_t n_clusters) {
    if (check_cfg(cfg) != ICE_OK || check_shape(page_size, n_clusters) != ICE_OK) return 0;
    return lay_out(*cfg, page_size, n_clusters, nullptr, nullptr);
}

ice_status_t ice_create(const ice_config_t *cfg, void *workspace, size_t workspace_bytes, ice_index_t **out) {
    if (!out) return fail(ICE_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (ice_status_t st = check_cfg(cfg)) return st;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return fail(ICE_ERR_INVALID_ARG, "workspace is null or not 256-byte aligned");
    if (workspace_bytes == 0) return fail(ICE_ERR_INVALID_ARG, "workspace_bytes is 0");
    ice_index *ix = new (std::nothrow) ice_index();
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "out of host memory");
    ix->cfg = *cfg;
    ix->ws = static_cast<char *>(workspace);
    ix->ws_bytes = workspace_bytes;
    ix->laid_out = false;
    ix->built = false;
    ix->n_tokens = 0;
    ix->build_n = 0;
    ix->n_top = 0;
    ix->cur = 0;
    ix->geometry = 0;
    *out = ix;
    return ICE_OK;
}

ice_status_t ice_destroy(ice_index_t *idx) {
    if (!idx) return fail(ICE_ERR_INVALID_ARG, "index is null");
    delete idx;
    return ICE_OK;
}

ice_status_t ice_build_index(ice_index_t *ix, const void *K, const void *V, int32_t n, int32_t page_size,
                             int32_t n_clusters, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!K || !V || !aligned16(K) || !aligned16(V)) return fail(ICE_ERR_INVALID_ARG, "K or V is null or misaligned");
    if (ix->cfg.init_idx && (reinterpret_cast<uintptr_t>(ix->cfg.init_idx) & 3u))
        return fail(ICE_ERR_INVALID_ARG, "init_idx is misaligned");
    if (ice_status_t st = check_shape(page_size, n_clusters)) return st;
    if (n < 1) return fail(ICE_ERR_INVALID_ARG, "n_tokens must be >= 1");
    if (n_clusters > n) return fail(ICE_ERR_SHAPE, "n_clusters %d exceeds n_tokens %d", n_clusters, n);
    if (n > ix->cfg.max_tokens) return fail(ICE_ERR_SHAPE, "n_tokens %d exceeds max_tokens %d", n, ix->cfg.max_tokens);
    if (ice_status_t st = ensure_layout(ix, page_size, n_clusters)) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    ix->dev.tk = ix->geometry;
    const Dev &d = ix->dev;
    const bf16_t *Kb = static_cast<const bf16_t *>(K), *Vb = static_cast<const bf16_t *>(V);
    ix->built = false;
    int cur = 0;
    if (d.tk) launch_key_aug(d, Kb, n, s);
    launch_init_centroids(d, Kb, n, ix->cfg.init_idx, ix->cfg.seed, cur, s);
    for (int t = 0; t < ix->cfg.kmeans_iters; ++t) {
        launch_assign(d, Kb, n, cur, s);
        launch_sort(d, n, nullptr, nullptr, s);
        launch_means(d, Kb, n, cur, s);
        cur ^= 1;
    }
    launch_paginate(d, Kb, Vb, n, s);
    reset_decode_state(d, n, s);
    if (ice_status_t st = device_status("ice_build_index")) return st;
    ix->cur = cur;
    ix->n_tokens = n;
    ix->build_n = n;
    ix->n_top = 0;
    ix->built = true;
    return ICE_OK;
}

ice_status_t ice_insert_batch(ice_index_t *ix, const void *k, const void *v, int32_t m, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_insert before ice_build_index");
    if (!k || !v || !aligned16(k) || !aligned16(v)) return fail(ICE_ERR_INVALID_ARG, "k or v is null or misaligned");
    if (m < 1) return fail(ICE_ERR_SHAPE, "number of tokens to insert must be >= 1");
    if ((long long)ix->n_tokens + m > ix->cfg.max_tokens)
        return fail(ICE_ERR_CAPACITY, "index holds %d tokens per unit, %d more exceed max_tokens = %d", ix->n_tokens, m,
                    ix->cfg.max_tokens);
    launch_insert(ix->dev, static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v), m, ix->cur,
                  static_cast<hipStream_t>(stream));
    if (ice_status_t st = device_status("ice_insert")) return st;
    ix->n_tokens += m;
    return ICE_OK;
}

ice_status_t ice_insert(ice_index_t *ix, const void *k, const void *v, void *stream) {
    return ice_insert_batch(ix, k, v, 1, stream);
}

static ice_status_t check_select(ice_index_t *ix, const void *q, int32_t budget, const int32_t *ids,
                                 const int32_t *n_sel, const char *who) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "%s before ice_build_index", who);
    if (!q || !aligned16(q)) return fail(ICE_ERR_INVALID_ARG, "q is null or misaligned");
    if (!ids || !n_sel) return fail(ICE_ERR_INVALID_ARG, "page_ids or n_selected is null");
    if (budget < ix->dev.s) return fail(ICE_ERR_SHAPE, "token_budget %d is below page_size %d", budget, ix->dev.s);
    if (ix->dev.max_pages > decode_step_max_pages(ix->dev.G))
        return fail(ICE_ERR_UNSUPPORTED, "%d pages per unit exceed the selection kernel's limit of %d", ix->dev.max_pages,
                    decode_step_max_pages(ix->dev.G));
    if (!decode_step_plan(ix->dev, budget / ix->dev.s, ix->n_tokens / ix->dev.s + ix->dev.C).fits)
        return fail(ICE_ERR_UNSUPPORTED, "token_budget %d (%d pages) and %d pages per unit need more LDS than a CU has for the "
                    "winner lists", budget, budget / ix->dev.s, ix->dev.max_pages);
    return ICE_OK;
}

ice_status_t ice_select(ice_index_t *ix, const void *q, int32_t budget, int32_t *ids, int32_t *n_sel, float *scores,
                        void *stream) {
    if (ice_status_t st = check_select(ix, q, budget, ids, n_sel, "ice_select")) return st;
    launch_decode_step(ix->dev, static_cast<const bf16_t *>(q), budget / ix->dev.s, ix->n_tokens / ix->dev.s + ix->dev.C,
                       ids, n_sel, scores, nullptr, nullptr, 0, nullptr, static_cast<hipStream_t>(stream));
    return device_status("ice_select");
}

static ice_status_t check_resident(const void *rk, const void *rv, int32_t n_res) {
    if (n_res < 0 || n_res > (1 << 20)) return fail(ICE_ERR_SHAPE, "n_resident %d is outside [0, 2^20]", n_res);
    if (n_res > 0 && (!rk || !rv || !aligned16(rk) || !aligned16(rv)))
        return fail(ICE_ERR_INVALID_ARG, "resident_k or resident_v is null or misaligned");
    return ICE_OK;
}

ice_status_t ice_attend_resident(ice_index_t *ix, const void *q, const int32_t *ids, const int32_t *n_sel, int32_t P,
                                 const void *rk, const void *rv, int32_t n_res, float *out, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_attend before ice_build_index");
    if (!q || !aligned16(q)) return fail(ICE_ERR_INVALID_ARG, "q is null or misaligned");
    if (!ids || !n_sel || !out) return fail(ICE_ERR_INVALID_ARG, "page_ids, n_selected or out is null");
    if (P < 1) return fail(ICE_ERR_SHAPE, "n_ids_per_unit must be >= 1");
    if (ice_status_t st = check_resident(rk, rv, n_res)) return st;
    const Resident res = {static_cast<const bf16_t *>(rk), static_cast<const bf16_t *>(rv), n_res, nullptr, nullptr, 0};
    launch_attend(ix->dev, static_cast<const bf16_t *>(q), ids, n_sel, P, res, out, static_cast<hipStream_t>(stream));
    return device_status("ice_attend");
}

ice_status_t ice_attend(ice_index_t *ix, const void *q, const int32_t *ids, const int32_t *n_sel, int32_t P, float *out,
                        void *stream) {
    return ice_attend_resident(ix, q, ids, n_sel, P, nullptr, nullptr, 0, out, stream);
}

ice_status_t ice_attend_noalloc(ice_index_t *ix, const void *q, const int32_t *ids, const int32_t *n_sel, int32_t P, float *out,
                                void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_attend_noalloc before ice_build_index");
    if (!q || !aligned16(q)) return fail(ICE_ERR_INVALID_ARG, "q is null or misaligned");
    if (!ids || !n_sel || !out) return fail(ICE_ERR_INVALID_ARG, "page_ids, n_selected or out is null");
    if (P < 1) return fail(ICE_ERR_SHAPE, "n_ids_per_unit must be >= 1");
    if (ix->dev.U > attend_static_max_units())
        return fail(ICE_ERR_UNSUPPORTED, "%d units: the static scratch array holds the partial results of at most %d",
                    ix->dev.U, attend_static_max_units());
    const hipError_t e = launch_attend_static(ix->dev, static_cast<const bf16_t *>(q), ids, n_sel, P, out,
                                              static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(ICE_ERR_DEVICE, "ice_attend_noalloc: %s", hipGetErrorString(e));
    return device_status("ice_attend_noalloc");
}

ice_status_t ice_select_attend_resident(ice_index_t *ix, const void *q, int32_t budget, const void *rk, const void *rv,
                                        int32_t n_res, int32_t *ids, int32_t *n_sel, float *out, void *stream) {
    if (ice_status_t st = check_select(ix, q, budget, ids, n_sel, "ice_select_attend")) return st;
    if (!out) return fail(ICE_ERR_INVALID_ARG, "out is null");
    if (ice_status_t st = check_resident(rk, rv, n_res)) return st;
    launch_decode_step(ix->dev, static_cast<const bf16_t *>(q), budget / ix->dev.s, ix->n_tokens / ix->dev.s + ix->dev.C, ids,
                       n_sel, nullptr, static_cast<const bf16_t *>(rk), static_cast<const bf16_t *>(rv), n_res, out,
                       static_cast<hipStream_t>(stream));
    return device_status("ice_select_attend");
}

ice_status_t ice_select_attend(ice_index_t *ix, const void *q, int32_t budget, int32_t *ids, int32_t *n_sel, float *out,
                               void *stream) {
    return ice_select_attend_resident(ix, q, budget, nullptr, nullptr, 0, ids, n_sel, out, stream);
}

ice_status_t ice_selected_tokens(ice_index_t *ix, const int32_t *ids, const int32_t *n_sel, int32_t P, int32_t *pos,
                                 int32_t *n_tok, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_selected_tokens before ice_build_index");
    if (!ids || !n_sel || !pos || !n_tok) return fail(ICE_ERR_INVALID_ARG, "a pointer is null");
    if (P < 1 || P > 1024) return fail(ICE_ERR_SHAPE, "n_ids_per_unit %d is outside [1, 1024]", P);
    launch_selected_tokens(ix->dev, ids, n_sel, P, pos, n_tok, static_cast<hipStream_t>(stream));
    return device_status("ice_selected_tokens");
}

ice_status_t ice_attend_tokens(ice_index_t *ix, const void *q, const void *K, const void *V, int32_t n_rows,
                               const int32_t *pos, const int32_t *n_tok, int32_t max_tok, float *out, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->laid_out) return fail(ICE_ERR_STATE, "ice_attend_tokens before ice_build_index or ice_import_index");
    if (!q || !aligned16(q) || !K || !V || !aligned16(K) || !aligned16(V))
        return fail(ICE_ERR_INVALID_ARG, "q, K or V is null or misaligned");
    if (!pos || !n_tok || !out) return fail(ICE_ERR_INVALID_ARG, "token_pos, n_tok or out is null");
    if (n_rows < 1 || max_tok < 1) return fail(ICE_ERR_SHAPE, "n_rows and max_tok must be >= 1");
    const Resident res = {static_cast<const bf16_t *>(K), static_cast<const bf16_t *>(V), max_tok, pos, n_tok, n_rows};
    launch_attend(ix->dev, static_cast<const bf16_t *>(q), nullptr, nullptr, 1, res, out, static_cast<hipStream_t>(stream));
    return device_status("ice_attend_tokens");
}

static ice_status_t select_hier_common(ice_index_t *ix, const void *q, int32_t budget, int32_t n_top, int32_t n_probe_top,
                                       int32_t n_probe, int32_t n_refine, int32_t *ids, int32_t *n_sel, float *scores,
                                       int32_t *clusters, int32_t *tops, float *out, void *stream, const char *who) {
    if (!q || !aligned16(q)) return fail(ICE_ERR_INVALID_ARG, "q is null or misaligned");
    if (!ids || !n_sel) return fail(ICE_ERR_INVALID_ARG, "page_ids or n_selected is null");
    if (budget < ix->dev.s) return fail(ICE_ERR_SHAPE, "token_budget %d is below page_size %d", budget, ix->dev.s);
    if (n_probe < 1) return fail(ICE_ERR_SHAPE, "n_probe must be >= 1");
    const int P = budget / ix->dev.s;
    if (n_refine != 0 && n_refine < P)
        return fail(ICE_ERR_SHAPE, "n_refine %d must be 0 (off) or at least the %d pages of the budget", n_refine, P);
    if (n_refine > ix->dev.max_pages) n_refine = ix->dev.max_pages;
    if (ix->dev.max_pages > decode_hier_max_pages(ix->dev.G))
        return fail(ICE_ERR_UNSUPPORTED, "%d pages per unit exceed the selection kernel's limit of %d", ix->dev.max_pages,
                    decode_hier_max_pages(ix->dev.G));
    if (decode_hier_lds_bytes(ix->dev, P, n_probe, n_refine) > 160u * 1024u - 6144u)
        return fail(ICE_ERR_UNSUPPORTED, "%d pages per unit, n_probe %d, n_refine %d and token_budget %d need more LDS than a CU has",
                    ix->dev.max_pages, n_probe, n_refine, budget);
    launch_decode_hier(ix->dev, static_cast<const bf16_t *>(q), ix->cur, P, n_top, n_probe_top, n_probe, n_refine,
                       ix->n_tokens / ix->dev.s + ix->dev.C, ids, n_sel, scores, clusters, tops, out, static_cast<hipStream_t>(stream));
    return device_status(who);
}

ice_status_t ice_select_hier(ice_index_t *ix, const void *q, int32_t budget, int32_t n_probe, int32_t n_refine, int32_t *ids,
                             int32_t *n_sel, float *scores, int32_t *clusters, float *out, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_select_hier before ice_build_index");
    return select_hier_common(ix, q, budget, 0, 0, n_probe, n_refine, ids, n_sel, scores, clusters, nullptr, out, stream,
                              "ice_select_hier");
}

ice_status_t ice_select_hier3(ice_index_t *ix, const void *q, int32_t budget, int32_t n_probe_top, int32_t n_probe,
                              int32_t n_refine, int32_t *ids, int32_t *n_sel, float *scores, int32_t *clusters, int32_t *tops,
                              float *out, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_select_hier3 before ice_build_index");
    if (ix->n_top == 0) return fail(ICE_ERR_STATE, "ice_select_hier3 before ice_build_top_level");
    if (n_probe_top < 1) return fail(ICE_ERR_SHAPE, "n_probe_top must be >= 1");
    return select_hier_common(ix, q, budget, ix->n_top, n_probe_top, n_probe, n_refine, ids, n_sel, scores, clusters, tops, out,
                              stream, "ice_select_hier3");
}

ice_status_t ice_build_top_level(ice_index_t *ix, int32_t n_top, int32_t iters, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_build_top_level before ice_build_index");
    if (n_top == 0) {  // (drops the level)
        ix->n_top = 0;
        return ICE_OK;
    }
    if (n_top < 1 || n_top > kTopMax || n_top > ix->dev.C)
        return fail(ICE_ERR_SHAPE, "n_top %d is outside [1, min(%d, n_clusters = %d)]", n_top, kTopMax, ix->dev.C);
    if (iters < 1) return fail(ICE_ERR_INVALID_ARG, "iters must be >= 1");
    launch_top_level(ix->dev, ix->cur, n_top, iters, static_cast<hipStream_t>(stream));
    if (ice_status_t st = device_status("ice_build_top_level")) return st;
    ix->n_top = n_top;
    return ICE_OK;
}

ice_status_t ice_export_top_level(ice_index_t *ix, ice_top_view_t *v) {
    if (!ix || !v) return fail(ICE_ERR_INVALID_ARG, "index or view is null");
    if (!ix->built || ix->n_top == 0) return fail(ICE_ERR_STATE, "ice_export_top_level before ice_build_top_level");
    memset(v, 0, sizeof(*v));
    v->n_top = ix->n_top;
    v->n_top_max = kTopMax;
    v->top_centroid = ix->dev.top_cent;
    v->top_centroid_bf16 = ix->dev.top_bf16;
    v->top_of = ix->dev.top_of;
    v->top_count = ix->dev.top_cnt;
    v->top_init = ix->dev.top_init;
    return ICE_OK;
}

ice_status_t ice_set_geometry(ice_index_t *ix, int32_t geometry) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (geometry != ICE_GEOMETRY_RAW && geometry != ICE_GEOMETRY_TRANSFORMED)
        return fail(ICE_ERR_INVALID_ARG, "geometry %d: ICE_GEOMETRY_RAW or ICE_GEOMETRY_TRANSFORMED", geometry);
    if (geometry != ix->geometry) ix->built = false;  // takes effect with the next build
    ix->geometry = geometry;
    return ICE_OK;
}

ice_status_t ice_export_geometry(ice_index_t *ix, ice_geometry_view_t *v) {
    if (!ix || !v) return fail(ICE_ERR_INVALID_ARG, "index or view is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_export_geometry before ice_build_index");
    const Dev &d = ix->dev;
    memset(v, 0, sizeof(*v));
    v->geometry = d.tk;
    if (d.tk) {
        v->key_extra = d.kaug;
        v->centroid_extra = d.cent_aug;
        v->cluster_sum_extra = d.csum_aug;
        v->radius_sq = d.c2;
        v->assign_centroid_extra_bf16 = d.caug[ix->cur ^ 1];
    }
    return ICE_OK;
}

ice_status_t ice_export_index(ice_index_t *ix, ice_index_view_t *v) {
    if (!ix || !v) return fail(ICE_ERR_INVALID_ARG, "index or view is null");
    if (!ix->built) return fail(ICE_ERR_STATE, "ice_export_index before ice_build_index");
    const Dev &d = ix->dev;
    memset(v, 0, sizeof(*v));
    v->n_units = d.U;
    v->group_size = d.G;
    v->head_dim = kD;
    v->page_size = d.s;
    v->n_clusters = d.C;
    v->cpad = d.Cpad;
    v->max_pages = d.max_pages;
    v->max_tokens = d.max_tokens;
    v->n_tokens = ix->n_tokens;
    v->Kp = d.Kp;
    v->Vp = d.Vp;
    v->page_cluster = d.page_cluster;
    v->page_fill = d.page_fill;
    v->page_pos = d.page_pos;
    v->cluster_tail = d.cluster_tail;
    v->cluster_cnt = d.cluster_cnt;
    v->cluster_sum = d.cluster_sum;
    v->centroid = d.centroid;
    v->page_sum = d.page_sum;
    v->rep = d.rep;
    v->n_pages = d.n_pages;
    v->assign = d.assign;
    v->assign_centroid_bf16 = d.cent_bf16[ix->cur ^ 1];
    v->init_idx = d.init_idx;
    return ICE_OK;
}

ice_status_t ice_import_index(ice_index_t *ix, const ice_index_view_t *v, void *stream) {
    if (!ix || !v) return fail(ICE_ERR_INVALID_ARG, "index or view is null");
    if (ice_status_t st = check_shape(v->page_size, v->n_clusters)) return st;
    if (v->n_units != ix->cfg.batch * ix->cfg.n_kv_heads || v->group_size != ix->cfg.group_size || v->head_dim != kD ||
        v->max_tokens != ix->cfg.max_tokens || v->max_pages != ix->cfg.max_tokens / v->page_size + v->n_clusters)
        return fail(ICE_ERR_SHAPE, "view dimensions do not match the index configuration");
    if (v->n_tokens < 0 || v->n_tokens > ix->cfg.max_tokens) return fail(ICE_ERR_SHAPE, "view n_tokens out of range");
    if (!v->Kp || !v->Vp || !v->page_cluster || !v->page_fill || !v->page_pos || !v->cluster_tail || !v->cluster_cnt ||
        !v->cluster_sum || !v->centroid || !v->page_sum || !v->rep || !v->n_pages)
        return fail(ICE_ERR_INVALID_ARG, "a view array is null");
    if (ice_status_t st = ensure_layout(ix, v->page_size, v->n_clusters)) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dev &d = ix->dev;
    const size_t U = d.U, MP = d.max_pages, C = d.C, ps = d.s;
    hipError_t e = hipSuccess;
    auto copy = [&](void *dst, const void *src, size_t bytes) {
        if (e == hipSuccess) e = hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToDevice, s);
    };
    copy(d.Kp, v->Kp, U * MP * ps * kD * 2);
    copy(d.Vp, v->Vp, U * MP * ps * kD * 2);
    copy(d.page_cluster, v->page_cluster, U * MP * 4);
    copy(d.page_fill, v->page_fill, U * MP * 4);
    copy(d.page_pos, v->page_pos, U * MP * ps * 4);
    copy(d.cluster_tail, v->cluster_tail, U * C * 4);
    copy(d.cluster_cnt, v->cluster_cnt, U * C * 4);
    copy(d.cluster_sum, v->cluster_sum, U * C * kD * 4);
    copy(d.centroid, v->centroid, U * C * kD * 4);
    copy(d.page_sum, v->page_sum, U * MP * kD * 4);
    copy(d.rep, v->rep, U * MP * kD * 2);
    copy(d.n_pages, v->n_pages, U * 4);
    if (e != hipSuccess) return fail(ICE_ERR_DEVICE, "ice_import_index: %s", hipGetErrorString(e));
    reset_decode_state(d, v->n_tokens, s);
    ix->cur = 0;
    ix->geometry = 0;  // (an imported index carries no extra coordinate)
    ix->dev.tk = 0;
    launch_refresh_centroids(d, 0, s);
    launch_refresh_centroids(d, 1, s);
    launch_refresh_tails(d, s);
    if (ice_status_t st = device_status("ice_import_index")) return st;
    ix->n_tokens = v->n_tokens;
    ix->build_n = 0;  // (not the product of a build here: no stage to re-run)
    ix->n_top = 0;
    ix->built = true;
    return ICE_OK;
}

ice_status_t ice_debug_assign(ice_index_t *ix, const void *K, int32_t n, const void *cent, int32_t n_clusters,
                              int32_t *assign_out, float *best_out, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!K || !cent || !aligned16(K) || !aligned16(cent))
        return fail(ICE_ERR_INVALID_ARG, "K or centroids is null or misaligned");
    if (n < 1) return fail(ICE_ERR_INVALID_ARG, "n must be >= 1");
    if (n > ix->cfg.max_tokens) return fail(ICE_ERR_SHAPE, "n %d exceeds max_tokens %d", n, ix->cfg.max_tokens);
    const int s_cur = ix->laid_out ? ix->dev.s : 16;
    if (ice_status_t st = check_shape(s_cur, n_clusters)) return st;
    if (ice_status_t st = ensure_layout(ix, s_cur, n_clusters)) return st;
    ix->dev.tk = 0;  // (the debug assignment is always on the raw keys)
    ix->built = false;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dev &d = ix->dev;
    launch_load_centroids(d, static_cast<const bf16_t *>(cent), 0, s);
    launch_assign(d, static_cast<const bf16_t *>(K), n, 0, s);
    if (assign_out) launch_sort(d, n, best_out, assign_out, s);  // (unpacks the winners; without it only the kernel is timed)
    return device_status("ice_debug_assign");
}

ice_status_t ice_debug_rerun_stage(ice_index_t *ix, const void *K, const void *V, int32_t stage, void *stream) {
    if (!ix) return fail(ICE_ERR_INVALID_ARG, "index is null");
    if (!ix->built || ix->build_n == 0 || ix->n_tokens != ix->build_n)
        return fail(ICE_ERR_STATE, "ice_debug_rerun_stage needs an index fresh from ice_build_index (no insertion since)");
    if (!K || !V || !aligned16(K) || !aligned16(V)) return fail(ICE_ERR_INVALID_ARG, "K or V is null or misaligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Dev &d = ix->dev;
    const bf16_t *Kb = static_cast<const bf16_t *>(K), *Vb = static_cast<const bf16_t *>(V);
    const int n = ix->build_n, prev = ix->cur ^ 1;  // the last round read buffer `prev` and wrote the live one
    switch (stage) {
        case ICE_STAGE_ASSIGN: launch_assign(d, Kb, n, prev, s); break;
        case ICE_STAGE_SORT: launch_sort(d, n, nullptr, nullptr, s); break;
        case ICE_STAGE_MEANS: launch_means(d, Kb, n, prev, s); break;
        case ICE_STAGE_PAGINATE: launch_paginate(d, Kb, Vb, n, s); break;
        default: return fail(ICE_ERR_INVALID_ARG, "stage %d: one of ICE_STAGE_ASSIGN .. ICE_STAGE_PAGINATE", stage);
    }
    return device_status("ice_debug_rerun_stage");
}

ice_status_t ice_debug_select_fault(ice_index_t *ix, const void *q, int32_t budget, int32_t *ids, int32_t *n_sel, float *out,
                                    int32_t muted_chunk, int32_t wait_log2, void *stream) {
    if (ice_status_t st = check_select(ix, q, budget, ids, n_sel, "ice_debug_select_fault")) return st;
    const int np_hint = ix->n_tokens / ix->dev.s + ix->dev.C;
    const int chunks = decode_step_chunks(ix->dev, np_hint);
    if (chunks < 2) return fail(ICE_ERR_UNSUPPORTED, "this index is served by one workgroup per unit: there is no score hand-off to disturb");
    if (muted_chunk < 0 || muted_chunk >= chunks) return fail(ICE_ERR_SHAPE, "muted_chunk %d is outside [0, %d)", muted_chunk, chunks);
    if (wait_log2 < 0 || wait_log2 > 20) return fail(ICE_ERR_SHAPE, "wait_log2 %d is outside [0, 20]", wait_log2);
    launch_decode_step(ix->dev, static_cast<const bf16_t *>(q), budget / ix->dev.s, np_hint, ids, n_sel, nullptr, nullptr, nullptr, 0,
                       out, static_cast<hipStream_t>(stream), wait_log2 | ((muted_chunk + 1) << 8));
    return device_status("ice_debug_select_fault");
}

}  // extern "C"
