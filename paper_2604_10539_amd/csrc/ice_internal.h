// Internal declarations shared by the host API and the kernel files (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "icecache.h"

// time stamps for performance work: empty in the product build
#ifdef ICE_PROF
#include "ice_prof.h"
#else
#define ICE_STAMP(i) do { } while (0)
#define ICE_USTAMP(i) do { } while (0)
#define ICE_BSTAMP(i) do { } while (0)
#define ICE_WSTAMP(t, i) do { } while (0)
#define ICE_HSTAMP(i) do { } while (0)
#define ICE_PROF_EXPORT(symbol)
#endif

namespace ice {

constexpr int kD = 128;          // head_dim
constexpr int kAssignTile = 256; // keys staged in LDS per step of the assign kernel
constexpr int kTopMax = 256;     // nodes of the optional level above the clusters, per unit

typedef uint16_t bf16_t;

// Everything a kernel needs, passed by value.  Pointers are into the caller's workspace.
struct Dev {
    int U, G, s, C, Cpad, max_pages, max_tokens;
    // index state
    bf16_t *Kp, *Vp;            // [U][max_pages][s][128]
    int *page_cluster, *page_fill; // [U][max_pages]
    int *page_pos;              // [U][max_pages][s]
    int *cluster_tail, *cluster_cnt; // [U][C]
    // what an insertion needs of a cluster's tail page, kept beside the cluster so that one round trip
    // fetches it (derived from the page tables by launch_refresh_tails; kept in step by the insertions)
    int *tail_fill;             // [U][C] tokens in the tail page; page_size when the cluster has no page
    float *tail_sum;            // [U][C][128] the tail page's fp32 key sum (page_sum of that page)
    float *cluster_sum, *centroid;   // [U][C][128]
    float *page_sum;            // [U][max_pages][128]
    bf16_t *rep;                // [U][max_pages][128]
    int *n_pages;               // [U]
    int *n_tokens;              // [U] device mirror of the token count (page_pos of inserts)
    bf16_t *cent_bf16[2];       // [U][Cpad][128] double buffer: [cur] is live, [cur^1] previous
    float *cnorm[2];            // [U][Cpad] squared norms of cent_bf16 (+inf in the padding)
    // optional extra coordinate of the clustering geometry (tk != 0): keys and centroids carry one
    // more dimension, see ice_set_geometry
    int tk;
    bf16_t *kaug;               // [U][max_tokens] extra coordinate of every token, by position
    bf16_t *caug[2];            // [U][Cpad] extra coordinate of the bf16 centroids (double buffer as cent_bf16)
    float *cent_aug, *csum_aug; // [U][C] its fp32 mean and running sum
    float *c2;                  // [U] squared radius c^2 of the key transformation
    // optional level above the clusters (ice_build_top_level): n_top nodes per unit, each the parent of
    // a group of clusters; fixed once built (insertions move centroids, not the level above them)
    float *top_cent;            // [U][kTopMax][128] position of a top node (mean of its clusters' bf16 centroids)
    bf16_t *top_bf16;           // [U][kTopMax][128] its bf16 rounding (rows >= n_top: zero)
    int *top_of;                // [U][C] top node of every cluster
    int *top_cnt;               // [U][kTopMax] clusters per top node
    int *top_init;              // [U][kTopMax] cluster each top node was promoted from
    // build scratch
    int *init_idx;              // [U][C]
    int *assign;                // [U][max_tokens]
    unsigned long long *packed; // [U][max_tokens] (ordered score << 32) | ~cluster
    int *order;                 // [U][max_tokens] tokens sorted by (cluster, position)
    int *cluster_start;         // [U][Cpad+1] exclusive scan of counts
    int *page_base;             // [U][Cpad+1] exclusive scan of pages per cluster
    float *attn_part;           // [256][G][130] partial results of the split attention (shares x units <= 256)
    int *attn_arrive;           // [U] arrival counters of its shares (zero between launches)
    int *range_tot;             // [U][R][Cpad] members per cluster in each of the sort's R token ranges (R = max(1, 256 / U) at most)
    // decode scratch
    uint32_t *scores;           // [U][max_pages] fp32 bits of the page scores; 0xFFFFFFFF = empty slot
    int *counter;               // [U] arrival counters of the decode-step kernel (zero between launches)
};

struct Host {
    ice_config_t cfg;
    char *ws;
    size_t ws_bytes;
    Dev dev;
    bool laid_out;   // dev pointers valid for (s, C)
    bool built;
    int n_tokens;    // per unit
    int build_n;     // tokens per unit of the last ice_build_index (0: none, or the index was imported)
    int n_top;       // nodes of the level above the clusters (0: not built)
    int cur;         // live centroid buffer
    int geometry;    // 0: distances on the raw keys; 1: on the transformed keys (one more coordinate)
};

__host__ __device__ inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Raises a kernel's dynamic-LDS limit when a launch needs more than any launch before it (the
// attribute is sticky: one runtime call per kernel instantiation and size class, not one per launch).
// Defined in ice_api.hip.
void allow_dynamic_lds(const void *kernel, size_t bytes);

// ---- launchers (host functions defined in the kernel files) ----
void launch_init_centroids(const Dev &d, const bf16_t *K, int n, const int *init_idx_or_null,
                           uint64_t seed, int cur, hipStream_t st);
void launch_load_centroids(const Dev &d, const bf16_t *cent, int cur, hipStream_t st);
void launch_key_aug(const Dev &d, const bf16_t *K, int n, hipStream_t st);
void launch_assign(const Dev &d, const bf16_t *K, int n, int cur, hipStream_t st);
void launch_sort(const Dev &d, int n, float *best_out_or_null, int *assign_out_or_null, hipStream_t st);
void launch_means(const Dev &d, const bf16_t *K, int n, int cur, hipStream_t st);
void launch_paginate(const Dev &d, const bf16_t *K, const bf16_t *V, int n, hipStream_t st);
void launch_refresh_centroids(const Dev &d, int cur, hipStream_t st);
void launch_refresh_tails(const Dev &d, hipStream_t st);  // tail_fill / tail_sum from the page tables (after a build or an import)
void launch_insert(const Dev &d, const bf16_t *k, const bf16_t *v, int m, int cur, hipStream_t st);
// scores + top-P selection (+ attention when out != nullptr) in one launch
// np_hint: host-side upper bound of the live pages per unit (tokens / page_size + clusters)
// res_k, res_v: n_res resident tokens per unit (bf16 [U][n_res][d]) attended on top of the pages; n_res may be 0
// wait_cfg: bits 0..7 = log2 of the bounded wait for a missing score, bits 8.. = 1 + the chunk whose
// score stores a test leaves out (0 in every product call)
constexpr int kDecodeWaitDefault = 16;
void launch_decode_step(const Dev &d, const bf16_t *q, int P, int np_hint, int *ids, int *n_sel, float *scores_out,
                        const bf16_t *res_k, const bf16_t *res_v, int n_res, float *out, hipStream_t st,
                        int wait_cfg = kDecodeWaitDefault);
int decode_step_chunks(const Dev &d, int np_hint);  // workgroups per unit of that launch
// two-stage selection (clusters, then their pages) (+ attention when out != nullptr) in one launch
// n_top > 0: three levels (the n_probe_top best top nodes first, only their clusters are scored)
void launch_decode_hier(const Dev &d, const bf16_t *q, int cur, int P, int n_top, int n_probe_top, int n_probe, int n_refine,
                        int np_hint, int *ids, int *n_sel, float *scores_out, int *clusters_out, int *tops_out, float *out,
                        hipStream_t st);
void launch_top_level(const Dev &d, int cur, int n_top, int iters, hipStream_t st);
int decode_hier_max_pages(int G);
size_t decode_hier_lds_bytes(const Dev &d, int P, int n_probe, int n_refine);
int decode_step_max_pages(int G);
struct DecodePlan {
    int chunks;      // workgroups per unit
    int np_hint;     // clamped upper bound of the live pages per unit
    int cand_cap;    // entries of the LDS candidate list
    int scores_off;  // byte offset of the LDS copy of the scores (one workgroup per unit only)
    size_t lds;      // dynamic LDS of the launch
    bool fits;       // ... within a CU's LDS
};
DecodePlan decode_step_plan(const Dev &d, int P, int np_hint);
// Resident tokens: tokens that are always attended on top of the listed pages, handled as further
// 16-token blocks dealt to the waves after the pages.  Two forms:
//   dense     a run of n tokens per unit, k, v bf16 [U][n][d] (the sink tokens and the recent
//             window of Alg. 1 / App. A), pos == nullptr;
//   gathered  rows pos[u][0 .. cnt[u]) of a whole cache k, v bf16 [U][rows][d] (token positions
//             chosen elsewhere, e.g. by another layer's selection, App. B); n is then the length of
//             a unit's position list.  Positions outside [0, rows) are clamped into the cache.
struct Resident {
    const bf16_t *k, *v;
    int n;
    const int *pos;
    const int *cnt;
    int rows;
};

void launch_attend(const Dev &d, const bf16_t *q, const int *ids_or_null, const int *n_sel, int P, const Resident &res,
                   float *out, hipStream_t st, int min_shares = 4);
// the same attention with the shares' partial results in the library's own static device array
// (no workspace region involved); at most attend_static_max_units() units
hipError_t launch_attend_static(const Dev &d, const bf16_t *q, const int *ids, const int *n_sel, int P, float *out,
                                hipStream_t st);
int attend_static_max_units();
bool launch_attend_would_split(const Dev &d, int P);  // few units, many pages: a selection call attends in a launch of its own
void launch_attend_split_after_select(const Dev &d, const bf16_t *q, const int *ids, const int *n_sel, int P, float *out,
                                      hipStream_t st);
void launch_selected_tokens(const Dev &d, const int *ids, const int *n_sel, int P, int *pos_out, int *n_tok_out,
                            hipStream_t st);

// ---- device helpers ----
__device__ inline float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ inline float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ inline float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round to nearest even; finite inputs
__device__ inline bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
// monotone map fp32 -> u32 (larger float <=> larger unsigned)
__device__ inline uint32_t f32_ordered(float f) {
    uint32_t u = __float_as_uint(f);
    return u ^ ((u & 0x80000000u) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ inline float ordered_f32(uint32_t k) {
    uint32_t u = k ^ ((k & 0x80000000u) ? 0x80000000u : 0xFFFFFFFFu);
    return __uint_as_float(u);
}

template <int CTRL>
__device__ inline float dpp_f32(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a DPP row; every lane of the row gets the same bits
__device__ inline float row16_sum(float x) {
    x += dpp_f32<0xB1>(x);  // quad_perm [1,0,3,2]
    x += dpp_f32<0x4E>(x);  // quad_perm [2,3,0,1]
    x += dpp_f32<0x141>(x); // row_half_mirror
    x += dpp_f32<0x140>(x); // row_mirror
    return x;
}
template <int CTRL>
__device__ inline uint32_t dpp_u32(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xF, 0xF, true);
}
// maximum / sum over the 16 lanes of a DPP row (every lane of the row gets the result)
__device__ inline uint32_t row16_max_u32(uint32_t x) {
    x = max(x, dpp_u32<0xB1>(x));
    x = max(x, dpp_u32<0x4E>(x));
    x = max(x, dpp_u32<0x141>(x));
    x = max(x, dpp_u32<0x140>(x));
    return x;
}
__device__ inline uint32_t row16_sum_u32(uint32_t x) {
    x += dpp_u32<0xB1>(x);
    x += dpp_u32<0x4E>(x);
    x += dpp_u32<0x141>(x);
    x += dpp_u32<0x140>(x);
    return x;
}
__device__ inline float wave_sum(float x) {
    x = row16_sum(x);
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}

// squared norm of a key held 8 dims per lane by a 16-lane row (fixed summation order), and the extra
// coordinate sqrt(c^2 - ||k||^2) of the transformed keys (Eq. 2), rounded to bf16
// Workgroup barrier that orders LDS traffic only: global loads that are still outstanding stay in
// flight across it (__syncthreads() waits for them as well).  For steps that exchange data through
// LDS alone.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// 16-byte load / store with the non-temporal hint, for data that a launch touches exactly once (the
// representative rows, key rows of a clustering pass, the page tiles being written)
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ inline uint4 load16_stream(const uint4 *p) {
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ inline void store16_stream(uint4 *p, const uint4 &w) {
    const u32x4 v = {w.x, w.y, w.z, w.w};
    __builtin_nontemporal_store(v, (u32x4 *)p);
}
template <bool STREAM>
__device__ inline uint4 load16(const uint4 *p) {
    if constexpr (STREAM) return load16_stream(p);
    else return *p;
}
template <bool STREAM>
__device__ inline void store16(uint4 *p, const uint4 &w) {
    if constexpr (STREAM) store16_stream(p, w);
    else *p = w;
}

// One direct global -> LDS load of 16 bytes per lane: lane l's bytes land at lds_base + 16 l
// (lds_base is the same for the whole wave).  Written as inline assembly so that the compiler's wait
// insertion does not know the load: told about it, it makes the wave wait for the load before the
// next LDS access that might alias its destination, which for a double-buffered tile is far too
// early.  The caller waits (wait_lds_dma) before the data is read, and before any barrier that
// hands the destination buffer over.
__device__ inline void lds_dma16(const uint4 *src, char *lds_base) {
    const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(__attribute__((address_space(3))) char *)lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory", "m0");
}
__device__ inline void wait_lds_dma() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }


// Kernel arguments beyond the preloaded dwords are fetched from memory where the compiler places the
// scalar load, which by default is next to each use: a load (and its wait) per use site, several of them
// on the critical path of a latency-bound kernel.  Pinning a value makes it opaque from here on, so it
// is fetched once, before this point, and then lives in a scalar register.
#define ICE_PIN(x) asm volatile("" : "+s"(x) : : "memory")
#define ICE_PIN_FIELD(dst, src, f) do { auto pinned_ = (src).f; ICE_PIN(pinned_); (dst).f = pinned_; } while (0)
// the fields of Dev that the insertion kernels use (the others stay unset)
__device__ inline void pin_insert_fields(Dev &d, const Dev &a, int cur, bf16_t *&caug_cur) {
    caug_cur = cur ? a.caug[1] : a.caug[0];
    ICE_PIN(caug_cur);
    ICE_PIN_FIELD(d, a, s); ICE_PIN_FIELD(d, a, C); ICE_PIN_FIELD(d, a, Cpad); ICE_PIN_FIELD(d, a, max_pages);
    ICE_PIN_FIELD(d, a, max_tokens); ICE_PIN_FIELD(d, a, tk);
    ICE_PIN_FIELD(d, a, Kp); ICE_PIN_FIELD(d, a, Vp); ICE_PIN_FIELD(d, a, page_cluster); ICE_PIN_FIELD(d, a, page_fill);
    ICE_PIN_FIELD(d, a, page_pos); ICE_PIN_FIELD(d, a, cluster_tail); ICE_PIN_FIELD(d, a, cluster_cnt);
    ICE_PIN_FIELD(d, a, tail_fill); ICE_PIN_FIELD(d, a, tail_sum); ICE_PIN_FIELD(d, a, cluster_sum);
    ICE_PIN_FIELD(d, a, centroid); ICE_PIN_FIELD(d, a, page_sum); ICE_PIN_FIELD(d, a, rep);
    ICE_PIN_FIELD(d, a, n_pages); ICE_PIN_FIELD(d, a, n_tokens);
    ICE_PIN_FIELD(d, a, kaug); ICE_PIN_FIELD(d, a, cent_aug); ICE_PIN_FIELD(d, a, csum_aug); ICE_PIN_FIELD(d, a, c2);
    // (caug is picked by the live buffer index at the call: an array indexed at run time would put the copy into scratch memory)
}

__device__ inline float key_sqnorm16(const uint4 &w) {  // this lane's 8 dims; summed over the 16-lane row
    float t = 0.f;
    t += bf16_lo(w.x) * bf16_lo(w.x); t += bf16_hi(w.x) * bf16_hi(w.x);
    t += bf16_lo(w.y) * bf16_lo(w.y); t += bf16_hi(w.y) * bf16_hi(w.y);
    t += bf16_lo(w.z) * bf16_lo(w.z); t += bf16_hi(w.z) * bf16_hi(w.z);
    t += bf16_lo(w.w) * bf16_lo(w.w); t += bf16_hi(w.w) * bf16_hi(w.w);
    return row16_sum(t);
}
__device__ inline bf16_t key_extra_coordinate(float c2, float n2) { return f32_to_bf16(sqrtf(fmaxf(c2 - n2, 0.f))); }


}  // namespace ice
