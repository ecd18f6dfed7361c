// Decode-step kernels: insertion of a new token, scoring of the page representatives, top-P page
// selection and sparse paged attention (Sec. 4.2-4.4, Alg. 1 and 3, Eq. 1 of the paper).
#include <algorithm>
#include <mutex>
#include <type_traits>
#include "ice_internal.h"

#include "ice_decode_common.h"

namespace ice {

constexpr uint32_t kScoreEmpty = 0xFFFFFFFFu;  // a NaN pattern no score can take (scores come out of fmaxf)
constexpr int kUnitFailed = -(1 << 30);        // arrival counter of a unit whose score hand-off gave up


// ------------------------------------------------------------------------------------------------
// Insertion of m tokens per unit, one after the other (Alg. 1 insertion loop; a node that outgrows
// its page gets a new one, Sec. 4.1; m > 1 is the page-at-a-time insertion of tokens that leave the
// recent window).  One workgroup per unit.  Per token: 15 waves scan the bf16 centroids (16 lanes x
// 16 bytes per row, four rows per wave and load, four loads in flight) for the nearest one, lowest
// id on ties; wave 0 then appends the key/value row to the cluster's tail page and updates, in
// ordered fp32 (one add per quantity): page sum -> representative, cluster sum -> centroid, its bf16
// rounding and squared norm.  The next token sees the moved centroid, exactly as m separate
// launches would; yet its scan does not wait for the update: only ONE centroid row changes, so
// while wave 0 appends token t the other waves scan for token t+1 over every row but that one, and
// wave 0 adds the moved row's distance (same 16-lane arithmetic, from the row it has just formed)
// before the barrier that ends the step.  k, v: bf16 [U, m, d].
constexpr int kInsertWaves = 16;
// (cent, cnorm: the live centroid buffer d.cent_bf16[cur] / d.cnorm[cur], which this kernel also
// writes, hence neither const nor restrict)
// RESIDENT (several tokens and the unit's centroids fit): the bf16 centroid rows, their norms and
// extra coordinates are copied to LDS once and scanned from there, the moved row patched in place:
// a token's scan then costs LDS time instead of another 256 C bytes through the CU.
template <bool RESIDENT>
__global__ __launch_bounds__(kInsertWaves * 64) void insert_kernel(const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                                                    bf16_t *cent, float *cnorm,
                                                                    int m, int cur, int C, int Cpad, Dev d) {  // (scalars first: preloaded)
    extern __shared__ __align__(16) char insert_lds[];  // RESIDENT: [C][128] bf16 rows, [C] fp32 norms, [C] fp32 extra coordinates
    __shared__ u64 best[3];  // token t's winner meets in best[t % 3]: (ordered distance, cluster id), minimum
    __shared__ __align__(16) uint32_t moved_row[64];  // the centroid row wave 0 has just moved (bf16 pairs)
    __shared__ float moved_norm, moved_aug;
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    // what the append needs and does not depend on the chosen cluster is requested before the scan
    int np = d.n_pages[u];
    int tok = d.n_tokens[u];
    const bf16_t *cb = cent + (size_t)u * Cpad * kD;
    const float *wn = cnorm + (size_t)u * Cpad;
    uint4 *lrow = (uint4 *)insert_lds;
    float *lnorm = (float *)(insert_lds + (size_t)C * kD * 2), *laug = lnorm + C;
    if constexpr (RESIDENT) {
        for (int x = tid; x < C * 16; x += kInsertWaves * 64) lrow[x] = ((const uint4 *)cb)[x];
        for (int r = tid; r < C; r += kInsertWaves * 64) {
            lnorm[r] = wn[r];
            laug[r] = d.tk ? bf16_to_f32(d.caug[cur][(size_t)u * Cpad + r]) : 0.f;
        }
    }
    const bf16_t *ku = k + (size_t)u * m * kD, *vu = v + (size_t)u * m * kD;
    const float c2 = d.tk ? d.c2[u] : 0.f;
    constexpr int RS = (kInsertWaves - 1) * 4;  // rows per pass of the scanning waves
    // transformed keys (Eq. 2): the new key's extra coordinate joins every comparison
    auto extra_of = [&](const uint4 &kq) -> bf16_t { return d.tk ? key_extra_coordinate(c2, key_sqnorm16(kq)) : (bf16_t)0; };
    // objective of one centroid row for a key: ||mu~||^2 - 2 k . mu~ (extra coordinate included)
    auto objective = [&](const uint4 &row, float w, float ce, const uint4 &kq, float kaf) {
        const float dot = row16_sum(dot8(row, kq)) + kaf * ce;
        return w - 2.0f * dot;
    };
    // waves 1..15: nearest row for token t among all rows but `skip`, into best[t % 3]
    auto scan = [&](int t, int skip) {
        const uint4 kq = ((const uint4 *)(ku + (size_t)t * kD))[ch];
        const float kaf = bf16_to_f32(extra_of(kq));
        float bv = INFINITY;
        int bi = 0x7FFFFFFF;
        for (int r0 = (wave - 1) * 4 + g; r0 < C; r0 += 4 * RS) {
            uint4 row[4];
            float w[4], ce[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int r = r0 + x * RS;
                if constexpr (RESIDENT) {
                    row[x] = r < C ? lrow[r * 16 + ch] : make_uint4(0, 0, 0, 0);
                    w[x] = r < C ? lnorm[r] : INFINITY;
                    ce[x] = r < C ? laug[r] : 0.f;
                } else {
                    row[x] = r < C ? ((const uint4 *)(cb + (size_t)r * kD))[ch] : make_uint4(0, 0, 0, 0);
                    w[x] = r < C ? wn[r] : INFINITY;
                    ce[x] = d.tk && r < C ? bf16_to_f32(d.caug[cur][(size_t)u * Cpad + r]) : 0.f;
                }
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {  // ascending r: a later row wins only when strictly smaller
                const float val = objective(row[x], w[x], ce[x], kq, kaf);
                if (val < bv && r0 + x * RS != skip) { bv = val; bi = r0 + x * RS; }
            }
        }
        if (ch == 0 && bi != 0x7FFFFFFF) atomicMin(&best[t % 3], ((u64)f32_ordered(bv) << 32) | (u64)(uint32_t)bi);
    };
    if (tid < 3) best[tid] = ~0ull;
    __syncthreads();
    if (wave > 0) scan(0, -1);
    __syncthreads();
    for (int t = 0; t < m; ++t) {
        // (no lane wins when every distance is NaN, i.e. a key with Inf / NaN coordinates: cluster 0 then,
        // the choice of an exhaustive search that never sees a smaller value)
        const u64 won = best[t % 3];
        const int c = won == ~0ull ? 0 : (int)(uint32_t)won;
        if (wave > 0) {
            if (t + 1 < m) scan(t + 1, c);
        } else {
            if (lane == 0) best[(t + 2) % 3] = ~0ull;  // (token t-1's slot, read for the last time before the previous barrier)
            const uint32_t kw = ((const uint32_t *)(ku + (size_t)t * kD))[lane];
            const uint32_t vw = ((const uint32_t *)(vu + (size_t)t * kD))[lane];
            const uint4 kq_now = ((const uint4 *)(ku + (size_t)t * kD))[ch];
            const int tn = min(t + 1, m - 1);
            const uint4 kq_next = ((const uint4 *)(ku + (size_t)tn * kD))[ch];
            const bf16_t ka = extra_of(kq_now);
            const float kaf = bf16_to_f32(ka);
            const size_t cl = (size_t)u * d.C + c;
            // two dependent round trips: what hangs on the cluster, then what hangs on its tail page
            // (fill and page sum together; the sum is dropped when a new page is opened)
            int tail = d.cluster_tail[cl];
            const int cnt = d.cluster_cnt[cl] + 1;
            float2 cs = ((const float2 *)(d.cluster_sum + cl * kD))[lane];
            const float es_old = d.tk ? d.csum_aug[cl] : 0.f;
            const size_t pg_old = (size_t)u * d.max_pages + max(tail, 0);
            int fill = d.page_fill[pg_old];
            float2 ps = ((const float2 *)(d.page_sum + pg_old * kD))[lane];
            if (tail < 0) fill = d.s;
            const bool fresh = fill == d.s;
            if (fresh) { tail = np; fill = 0; ps = make_float2(0.f, 0.f); }
            const size_t pg = (size_t)u * d.max_pages + tail;
            const int slot = fill;
            fill += 1;
            ((uint32_t *)(d.Kp + (pg * d.s + slot) * kD))[lane] = kw;
            ((uint32_t *)(d.Vp + (pg * d.s + slot) * kD))[lane] = vw;
            const float k0 = bf16_lo(kw), k1 = bf16_hi(kw);
            ps.x = ps.x + k0;
            ps.y = ps.y + k1;
            ((float2 *)(d.page_sum + pg * kD))[lane] = ps;
            const float ff = (float)fill;
            ((uint32_t *)(d.rep + pg * kD))[lane] = (uint32_t)f32_to_bf16(ps.x / ff) | ((uint32_t)f32_to_bf16(ps.y / ff) << 16);
            cs.x = cs.x + k0;
            cs.y = cs.y + k1;
            ((float2 *)(d.cluster_sum + cl * kD))[lane] = cs;
            const float fc = (float)cnt;
            const float2 mu = make_float2(cs.x / fc, cs.y / fc);
            ((float2 *)(d.centroid + cl * kD))[lane] = mu;
            const bf16_t b0 = f32_to_bf16(mu.x), b1 = f32_to_bf16(mu.y);
            const uint32_t packed = (uint32_t)b0 | ((uint32_t)b1 << 16);
            ((uint32_t *)(cent + ((size_t)u * Cpad + c) * kD))[lane] = packed;
            const float f0 = bf16_to_f32(b0), f1 = bf16_to_f32(b1);
            float nn = wave_sum(f0 * f0 + f1 * f1);
            float ef = 0.f;
            if (d.tk) {  // the cluster's extra coordinate follows its members' running mean as well
                const float es = es_old + kaf;
                const float e = es / fc;
                const bf16_t eb = f32_to_bf16(e);
                ef = bf16_to_f32(eb);
                nn += ef * ef;
                if (lane == 0) {
                    d.csum_aug[cl] = es;
                    d.cent_aug[cl] = e;
                    d.caug[cur][(size_t)u * d.Cpad + c] = eb;
                    d.kaug[(size_t)u * d.max_tokens + tok] = ka;
                }
            }
            if (lane == 0) {
                cnorm[(size_t)u * Cpad + c] = nn;
                d.cluster_cnt[cl] = cnt;
                d.cluster_tail[cl] = tail;
                d.page_fill[pg] = fill;
                d.page_pos[pg * d.s + slot] = tok;
                d.n_tokens[u] = tok + 1;
                if (fresh) {
                    d.page_cluster[pg] = c;
                    d.n_pages[u] = np + 1;
                }
            }
            if (fresh) np += 1;
            if (t + 1 < m) {
                // the moved row's distance to the next token, from the bits just stored (every 16-lane
                // row of the wave computes it, the way a scanning wave would)
                moved_row[lane] = packed;
                if (lane == 0) { moved_norm = nn; moved_aug = ef; }
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                const uint4 row = ((const uint4 *)moved_row)[ch];
                const float val = objective(row, moved_norm, moved_aug, kq_next, bf16_to_f32(extra_of(kq_next)));
                if (lane == 0 && !(val != val)) atomicMin(&best[(t + 1) % 3], ((u64)f32_ordered(val) << 32) | (u64)(uint32_t)c);
                if constexpr (RESIDENT) {  // (the scanning waves skip this row in this step: they may see it half written)
                    ((uint32_t *)(lrow + c * 16))[lane] = packed;
                    if (lane == 0) { lnorm[c] = nn; laug[c] = ef; }
                }
            }
        }
        tok += 1;
        // Token t+1's winner is complete.  Token t's updates must be visible to whoever reads them next:
        // with the centroids in LDS that is wave 0 alone (a wave's loads follow its own earlier stores
        // to the same address), so the stores may stay in flight; otherwise every wave re-reads the
        // moved row from memory and the barrier waits for the stores as well.
        if constexpr (RESIDENT) lds_barrier();
        else __syncthreads();
    }
}

void launch_insert(const Dev &d, const bf16_t *k, const bf16_t *v, int m, int cur, hipStream_t st) {
    const size_t lds = (size_t)d.C * (kD * 2 + 8);
    if (m >= 2 && lds <= 150u * 1024u) {
        allow_dynamic_lds((const void *)insert_kernel<true>, lds);
        hipLaunchKernelGGL(insert_kernel<true>, dim3(d.U), dim3(kInsertWaves * 64), lds, st, k, v, d.cent_bf16[cur], d.cnorm[cur], m, cur,
                           d.C, d.Cpad, d);
        return;
    }
    hipLaunchKernelGGL(insert_kernel<false>, dim3(d.U), dim3(kInsertWaves * 64), 0, st, k, v, d.cent_bf16[cur], d.cnorm[cur], m, cur, d.C, d.Cpad, d);
}

// ------------------------------------------------------------------------------------------------
template <int G, int NW, bool RES>
__global__ __launch_bounds__(NW * 64) void attend_kernel(const bf16_t *__restrict__ q, const int *__restrict__ ids,
                                                          const int *__restrict__ n_sel, int P, Dev d, Resident res,
                                                          float *__restrict__ out) {  // (scalars first: preloaded)
    extern __shared__ __align__(16) char smem[];
    const int u = blockIdx.x;
    bf16x8 qa[4];
    load_query_operand<G>(q, u, threadIdx.x & 63, qa, nullptr);
    const int *list = ids + (size_t)u * P;
    const int ns = ids ? max(0, min(n_sel[u], P)) : 0;  // (no page list: resident tokens only; negative count: none)
    attend_pages<G, NW, RES>(d, u, qa, [=](int x) { return list[x]; }, ns, res, out, (float *)smem, [] {});
}

// Few units and many pages per unit: one workgroup per unit would pull every tile through a single
// CU.  The page list of a unit is cut into S shares instead, one workgroup each (grid S x U); every
// workgroup leaves its partial result (attend_pages, PARTIAL) as device-scope words and bumps the
// unit's arrival counter once those stores have completed; the last one to arrive merges the shares:
// out = sum_s O_s e^(M_s - M) / sum_s L_s e^(M_s - M).  `arrive` is zero between launches (the last
// workgroup puts it back).
template <int G, int NW>
__global__ __launch_bounds__(NW * 64) void attend_split_kernel(const bf16_t *__restrict__ q, const int *__restrict__ ids,
                                                                const int *__restrict__ n_sel, int P, Dev d,
                                                                float *__restrict__ part, int *__restrict__ arrive,
                                                                float *__restrict__ out) {
    extern __shared__ __align__(16) char smem[];
    __shared__ int sh_last;
    const int s = blockIdx.x, S = gridDim.x, u = blockIdx.y, tid = threadIdx.x;
    if (s == 0) ICE_STAMP(16);
    bf16x8 qa[4];
    load_query_operand<G>(q, u, tid & 63, qa, nullptr);
    // shares are cut from the list's capacity P, not from the unit's count, so that every wave can ask
    // for its first page id together with the count (one round trip less); entries past the count
    // are dropped below
    const int per = (P + S - 1) / S, lo = min(P, s * per), wave = tid >> 6;
    const int *list = ids + (size_t)u * P + lo;
    const int first = lo + wave < P ? list[wave] : -1;
    const int ns = max(0, min(n_sel[u], P));
    const int cnt = max(0, min(ns - lo, per));
    attend_pages<G, NW, false, true>(d, u, qa, [=](int x) { return x == wave ? first : list[x]; }, cnt,
                                     Resident{nullptr, nullptr, 0, nullptr, nullptr, 0}, part + ((size_t)u * S + s) * G * (kD + 2),
                                     (float *)smem, [] {});
    if (s == 0) ICE_STAMP(17);
    __syncthreads();  // every wave's partial stores have completed
    if (s == 0) ICE_STAMP(18);
    if (tid == 0) {
        const int old = __hip_atomic_fetch_add(arrive + u, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = old == S - 1;
        if (last) __hip_atomic_store(arrive + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
        sh_last = last;
    }
    __syncthreads();
    if (!sh_last) return;
    ICE_STAMP(19);
    // The merge.  All partial results of the unit come to LDS in batches of independent loads (a
    // batch costs one round trip; the launch reserves room for S shares), then every output element is
    // combined from there.
    const float *pu = part + (size_t)u * S * G * (kD + 2);
    constexpr int NT = NW * 64, PW = G * (kD + 2);  // words of one share
    float *lp = (float *)smem;                       // (the attention's scratch is free again)
    const int words = S * PW;
    for (int x0 = tid; x0 < words; x0 += 8 * NT) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            v[i] = x0 + i * NT < words ? __hip_atomic_load(pu + x0 + i * NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (x0 + i * NT < words) lp[x0 + i * NT] = v[i];
    }
    __syncthreads();
    ICE_STAMP(20);
    for (int o = tid; o < G * kD; o += NT) {
        const int h = o / kD, j = o % kD;
        const float *ph = lp + h * (kD + 2);
        float M = -INFINITY;
        for (int sh = 0; sh < S; ++sh) M = fmaxf(M, ph[sh * PW + kD]);
        float num = 0.f, den = 0.f;
        for (int sh = 0; sh < S; ++sh) {
            const float ms = ph[sh * PW + kD];
            const float w = ms == -INFINITY ? 0.f : __expf(ms - M);  // (a share without tokens: no weight)
            num += ph[sh * PW + j] * w;
            den += ph[sh * PW + kD + 1] * w;
        }
        out[((size_t)u * G + h) * kD + j] = den > 0.f ? num / den : 0.f;
    }
    ICE_STAMP(21);
}
// LDS of a split launch: the attention's scratch, later the S shares' partial results side by side
static size_t attend_split_lds(int G, int NW, int S) {
    return sizeof(float) * std::max<size_t>(attend_scratch_floats(G, NW), (size_t)S * G * (kD + 2));
}
constexpr int kSplitMaxLdsBytes = 128 * 1024;
// shares per unit of the split attention: as many workgroups as the chip has CUs, at least one page
// per wave; below `min_shares` the exchange of the partial results costs more than the shares save
constexpr int kPagesPerShare = 4;
constexpr int kFusedSplitMinShares = 4;  // when the attention follows the selection of the same call (it then takes a launch of its own)
int attend_shares(const Dev &d, int P, int min_shares) {
    const int NW = d.G == 8 ? 8 : 16;
    // (a CU draws ~30 GB/s from cold HBM however many waves ask: what shortens the attention is the
    // number of CUs, so a share is kPagesPerShare pages even though a workgroup has a wave per page;
    // fewer than min_shares workgroups' worth of pages, counted NW to a workgroup, are not split)
    if ((P + NW - 1) / NW < min_shares) return 1;
    const int fit = kSplitMaxLdsBytes / (int)(sizeof(float) * d.G * (kD + 2));  // shares whose results fit the merging workgroup's LDS
    return std::max(1, std::min({256 / std::max(d.U, 1), (P + kPagesPerShare - 1) / kPagesPerShare, fit}));
}

// the token positions of the listed pages, in list and slot order, padded with -1
__global__ void selected_tokens_kernel(Dev d, const int *__restrict__ ids, const int *__restrict__ n_sel, int P,
                                       int *__restrict__ pos_out, int *__restrict__ n_tok_out) {
    const int u = blockIdx.x, s = d.s;
    __shared__ int base[1025];
    const int ns = max(0, min(n_sel[u], P));
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int x = 0; x < ns; ++x) {
            base[x] = acc;
            const int p = ids[(size_t)u * P + x];
            acc += (unsigned)p < (unsigned)d.max_pages ? d.page_fill[(size_t)u * d.max_pages + p] : 0;
        }
        base[ns] = acc;
        n_tok_out[u] = acc;
    }
    __syncthreads();
    const int tot = base[ns];
    for (int i = threadIdx.x; i < P * s; i += blockDim.x) pos_out[(size_t)u * P * s + i] = -1;
    __syncthreads();
    for (int i = threadIdx.x; i < ns * s; i += blockDim.x) {
        const int x = i / s, t = i % s, p = ids[(size_t)u * P + x];
        if ((unsigned)p >= (unsigned)d.max_pages) continue;
        const size_t pg = (size_t)u * d.max_pages + p;
        if (t < d.page_fill[pg]) pos_out[(size_t)u * P * s + base[x] + t] = d.page_pos[pg * s + t];
    }
    (void)tot;
}

void launch_selected_tokens(const Dev &d, const int *ids, const int *n_sel, int P, int *pos_out, int *n_tok_out,
                            hipStream_t st) {
    hipLaunchKernelGGL(selected_tokens_kernel, dim3(d.U), dim3(256), 0, st, d, ids, n_sel, P, pos_out, n_tok_out);
}

void launch_attend(const Dev &d, const bf16_t *q, const int *ids, const int *n_sel, int P, const Resident &res_in,
                   float *out, hipStream_t st, int min_shares) {
    const Resident res = res_in;
    const int n_res = res.n;
    const int S = ids && n_res == 0 && !res.pos ? attend_shares(d, P, min_shares) : 1;
    if (S > 1) {
#define ICE_ATTEND_SPLIT(g, nw)                                                                                            \
    do {                                                                                                                   \
        allow_dynamic_lds((const void *)attend_split_kernel<g, nw>, attend_split_lds(g, nw, S));                           \
        hipLaunchKernelGGL((attend_split_kernel<g, nw>), dim3(S, d.U), dim3(nw * 64), attend_split_lds(g, nw, S), st, q, ids, \
                           n_sel, P, d, d.attn_part, d.attn_arrive, out);                                                  \
    } while (0)
        switch (d.G) {
            case 1: ICE_ATTEND_SPLIT(1, 16); break;
            case 2: ICE_ATTEND_SPLIT(2, 16); break;
            case 4: ICE_ATTEND_SPLIT(4, 16); break;
            default: ICE_ATTEND_SPLIT(8, 8); break;
        }
#undef ICE_ATTEND_SPLIT
        return;
    }
#define ICE_ATTEND(g, nw)                                                                                                  \
    do {                                                                                                                   \
        if (n_res > 0)                                                                                                     \
            hipLaunchKernelGGL((attend_kernel<g, nw, true>), dim3(d.U), dim3(nw * 64),                                     \
                               sizeof(float) * attend_scratch_floats(g, nw), st, q, ids, n_sel, P, d, res, out);           \
        else                                                                                                               \
            hipLaunchKernelGGL((attend_kernel<g, nw, false>), dim3(d.U), dim3(nw * 64),                                    \
                               sizeof(float) * attend_scratch_floats(g, nw), st, q, ids, n_sel, P, d, res, out);           \
    } while (0)
    switch (d.G) {
        case 1: ICE_ATTEND(1, 16); break;
        case 2: ICE_ATTEND(2, 16); break;
        case 4: ICE_ATTEND(4, 16); break;
        default: ICE_ATTEND(8, 8); break;
    }
#undef ICE_ATTEND
}

// ------------------------------------------------------------------------------------------------
// Attention for callers that cannot allocate (code under HIP graph capture, serving loops and
// harnesses that forbid hipMalloc) and hold no workspace region to lend: the split attention above
// with its partial results in a device array of the library itself.  Every call on a GPU shares
// that GPU's array: calls that overlap on one GPU (two streams, two host threads) race on it.
// The partial results need no initial value (every share writes its whole block before the merge
// reads it); the arrival counters behind them start at zero (a static array does) and every launch
// puts them back to zero.
constexpr int kStaticPairs = 256;  // (unit, share) pairs the array holds, each 8 heads x 130 floats
constexpr int kStaticPartFloats = kStaticPairs * 8 * (kD + 2);
}  // namespace ice
static __device__ __align__(256) float scratch[ice::kStaticPartFloats + ice::kStaticPairs];  // partial results, then one counter per unit
namespace ice {

int attend_static_max_units() { return kStaticPairs; }

// The array's name is a host-side stand-in; its device address is looked up once per device, with
// that device current, and only that address is handed to kernels.
static float *scratch_on_current_device(hipError_t *err) {
    constexpr int kMaxDevices = 64;
    static float *ptr[kMaxDevices] = {};
    static std::mutex mu;
    int dev = -1;
    *err = hipGetDevice(&dev);
    if (*err != hipSuccess) return nullptr;
    if (dev < 0 || dev >= kMaxDevices) {
        *err = hipErrorInvalidDevice;
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (*err != hipSuccess) return nullptr;
        ptr[dev] = static_cast<float *>(p);
    }
    return ptr[dev];
}

// always the split form (shares, the last one to finish merges), also with one share per unit; d.U <= kStaticPairs
hipError_t launch_attend_static(const Dev &d, const bf16_t *q, const int *ids, const int *n_sel, int P, float *out,
                                hipStream_t st) {
    hipError_t err = hipSuccess;
    float *part = scratch_on_current_device(&err);
    if (!part) return err;
    const int NW = d.G == 8 ? 8 : 16;
    const int fit = kSplitMaxLdsBytes / (int)(sizeof(float) * d.G * (kD + 2));
    const int S = std::max(1, std::min({kStaticPairs / d.U, (P + kPagesPerShare - 1) / kPagesPerShare, fit}));
#define ICE_ATTEND_SPLIT(g, nw)                                                                                            \
    do {                                                                                                                   \
        allow_dynamic_lds((const void *)attend_split_kernel<g, nw>, attend_split_lds(g, nw, S));                           \
        hipLaunchKernelGGL((attend_split_kernel<g, nw>), dim3(S, d.U), dim3(nw * 64), attend_split_lds(g, nw, S), st, q, ids, \
                           n_sel, P, d, part, (int *)(part + kStaticPartFloats), out);                                     \
    } while (0)
    switch (d.G) {
        case 1: ICE_ATTEND_SPLIT(1, 16); break;
        case 2: ICE_ATTEND_SPLIT(2, 16); break;
        case 4: ICE_ATTEND_SPLIT(4, 16); break;
        default: ICE_ATTEND_SPLIT(8, 8); break;
    }
#undef ICE_ATTEND_SPLIT
    return hipSuccess;
}

// ------------------------------------------------------------------------------------------------
// One decode step for all units in ONE launch: score every page representative, pick the top-P
// pages, attend over them (Sec. 4.3-4.4, Alg. 3, Eq. 1).
//
// Phase A, every workgroup: a unit's representatives are one contiguous bf16 stream, split over
// `chunks` workgroups.  Scores come off the matrix cores, 16 pages per four
// v_mfma_f32_16x16x32_bf16 in the split-row operand form (SplitRow: every load instruction reads
// whole 128-byte lines, 8 rows x 128 bytes, with the non-temporal hint):
//   S[p] = max over the G query heads of (q_h . rep_p) / ||q_h||     (query normalisation of Eq. 3).
// The workgroup then bumps the unit's arrival counter; the LAST one to arrive carries on alone.
// Workgroup ids are mapped so that all chunks of a unit share (id mod 8), i.e. the same XCD and L2.
//
// Phase B, last workgroup of the unit: exact top-k over the composite key (score, lower id first),
// all keys distinct.  A threshold that at least k keys reach comes first.  Small budgets: the keys
// sit in registers, every 16-lane row (or, with one workgroup per unit, every (wave, unroll slot)
// group formed while scoring) takes the maximum of its keys, and the k-th largest of these maxima
// is such a threshold (k different groups hold a key at or above it); with 64 groups and k = 16 it
// lets through barely more than k keys.  Large budgets: the 16-bit prefix of the k-th largest key
// from two 8-bit LDS histograms; keys above the prefix are winners as they are.  What is left goes
// to an LDS candidate list, ranked exactly by counting (or by an LDS-histogram radix select when
// the list is long).  Winners are placed in ascending id order.
//
// Phase C, same workgroup: attention over the winners (attend_pages), ids never leave the chip.
// The leading scalar arguments are what the kernel needs before its first loads can be issued: the
// first 16 dwords of the kernel arguments are in scalar registers when a wave starts
// (kernel-argument preload; structures passed by value are not eligible), the rest arrives by
// scalar loads while the first loads are in flight.
template <int G, int NW, int EMAX, bool RES>
__global__ __launch_bounds__(NW * 64) void decode_step_kernel(int U, int max_pages, int P, int chunks, int np_hint, int lds_scores_off,
                                                               int wait_cfg, int cand_cap, const bf16_t *__restrict__ rep_all,
                                                               const bf16_t *__restrict__ q,
                                                               const int *__restrict__ n_pages, Dev d, int *__restrict__ ids_out,
                                                               int *__restrict__ n_sel_out, float *__restrict__ scores_out, Resident res,
                                                               float *__restrict__ out) {
    constexpr int NT = NW * 64;
    extern __shared__ __align__(16) char smem[];
    __shared__ int sh_last, sh_M, sh_M2, sh_W, sh_fail;
    __shared__ uint32_t sh_pre;
    __shared__ uint32_t sh_rowmax[4 * NW];
    __shared__ uint32_t sh_quadmax[16 * NW];
    __shared__ u64 sh_tau;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    const int xcd = blockIdx.x & 7, r = blockIdx.x >> 3;
    const int chunk = r % chunks, u_grid = xcd + 8 * (r / chunks);
    // (the grid is padded to a multiple of 8 units; a workgroup beyond the last unit leaves after the
    // first loads are issued: an early exit here would split the kernel-argument loads into
    // dependent round trips for every workgroup)
    const bool live = u_grid < U;
    const int u = live ? u_grid : U - 1;
    const int np = n_pages[u];  // first needed after the first loads are in flight
    const bf16_t *rep = rep_all + (size_t)u * max_pages * kD;
    uint32_t *S = d.scores + (size_t)u * d.max_pages;  // fp32 bits; kScoreEmpty = not written yet

    // one workgroup per unit: the scores never leave LDS and there is nobody to wait for
    const bool single = chunks == 1;
    // wait_cfg: bits 0..7 = log2 of the re-reads the last workgroup spends on a score slot that is
    // still empty; bits 8.. = 1 + the chunk whose score stores are left out (0: none).  The latter
    // exists for the test of the give-up path only: a hand-off that cannot complete, forced from the
    // host, with every wave still running to its end.
    const int spin_limit = 1 << (wait_cfg & 255);
    const bool muted = (wait_cfg >> 8) == chunk + 1;
    uint32_t *sc_lds = (uint32_t *)(smem + lds_scores_off);

    if (chunk == 0) ICE_STAMP(0);
    if (chunk == 0) ICE_USTAMP(0);
    if (tid == 0) {  // (visible to the workgroup after the barrier that ends phase A)
        sh_M = 0;
        sh_W = 0;
        sh_fail = 0;
        sh_pre = 0u;
        sh_tau = 0ull;
    }
    // ---- phase A: scores of this chunk, 16 pages per four v_mfma_f32_16x16x32_bf16 in the
    // split-row form (SplitRow: every load instruction reads whole 128-byte lines, 8 rows x 128
    // bytes; A operand = the G query rows twice).  Lane (.., c) of the owning row group ends up
    // with the score of page c of the 16.
    using SR = SplitRow<G>;
    bf16x8 qs[2];  // the query rows in split-row form (scoring); the attention takes them in plain form
    {
        const int per = round_up((np_hint + chunks - 1) / chunks, 16);  // (whole 16-page blocks)
        const int p0 = chunk * per, pend = min(np_hint, p0 + per);
        const int nblk = (pend - p0 + 15) >> 4;
        constexpr int UNR = 4;
        static_assert(NW * UNR == 4 * NW, "sh_rowmax holds one maximum per (wave, unroll slot)");
        uint4 bb[UNR][4];
        int word[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) word[j] = SR::word(lane, j >> 1, j & 1);
        const int row8 = ch & 7;
        auto request = [&](int b0, int lim) {
#pragma unroll
            for (int x = 0; x < UNR; ++x) {
                const int pb = p0 + 16 * (b0 + NW * x);
                const uint4 *src = (const uint4 *)(rep + (size_t)pb * kD);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    bb[x][j] = pb + 8 * (j >> 1) + row8 < lim ? load16_stream(src + word[j]) : make_uint4(0, 0, 0, 0);
            }
        };
        // The first round of representative rows is requested together with the query rows, before
        // anything waits for either (and before np is known: np <= np_hint <= max_pages): the
        // kernel starts with one memory round trip, not two.
        int b0 = wave;
        if (b0 < nblk) request(b0, pend);
        if (chunk == 0) ICE_STAMP(12);
        float invn;
        SR::load_query(q, u, lane, qs, &invn);
        if (!live) return;  // (nothing written, no barrier passed yet)
        float inv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) inv[v] = __shfl(invn, (4 * SR::head_group(lane) + v) & 15);
        const bool owner = SR::owner(lane);
        if (chunk == 0) ICE_STAMP(13);
        const int lim = min(np, pend);
        float gmax[UNR];  // running maximum of the scores this lane produced in unroll slot x
#pragma unroll
        for (int x = 0; x < UNR; ++x) gmax[x] = -INFINITY;
        while (b0 < nblk) {
#pragma unroll
            for (int x = 0; x < UNR; ++x) {
                if (b0 + NW * x >= nblk) break;  // (wave-uniform)
                f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qs[t], __builtin_bit_cast(bf16x8, bb[x][t]), acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qs[t], __builtin_bit_cast(bf16x8, bb[x][2 + t]), acc1, 0, 0, 0);
                }
                const float sc = SR::score(acc0, acc1, inv, lane);
                const int page = p0 + 16 * (b0 + NW * x) + ch;
                if (owner && page < lim) {
                    if (single) sc_lds[page] = __float_as_uint(sc);
                    else if (!muted) __hip_atomic_store(S + page, __float_as_uint(sc), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    gmax[x] = fmaxf(gmax[x], sc);
                }
            }
            b0 += NW * UNR;
            if (b0 < nblk) request(b0, lim);
        }
        // With one workgroup per unit the selection threshold needs the maxima of 4*NW disjoint
        // groups of scores: group (wave, x) is ready here, for free (the kernel is waiting for HBM).
        if (single) {
#pragma unroll
            for (int x = 0; x < UNR; ++x) {
                float r = gmax[x];
                r = fmaxf(r, dpp_f32<0xB1>(r));
                r = fmaxf(r, dpp_f32<0x4E>(r));
                r = fmaxf(r, dpp_f32<0x141>(r));
                r = fmaxf(r, dpp_f32<0x140>(r));
                r = fmaxf(r, __shfl_xor(r, 16));  // (the owners sit in two row groups)
                r = fmaxf(r, __shfl_xor(r, 32));
                if (lane == 0) sh_rowmax[wave * 4 + x] = f32_ordered(r);
            }
        }
    }
    // ---- arrival: count, and let the last workgroup of the unit go on.  No device-scope fence is
    // used (on this chip it writes back / invalidates a whole L2, per workgroup): scores travel as
    // device-scope atomic words, each slot doubles as its own ready flag (kScoreEmpty until written),
    // and the reader re-reads a slot until it is filled.  Writers never wait, so the reader only ever
    // waits for stores that were issued and completed (barrier below) before the counter moved.
    // (With one workgroup per unit only LDS is exchanged.)
    if (chunk == 0) ICE_STAMP(14);
    if (single) lds_barrier();
    else __syncthreads();
    if (chunk == 0) ICE_STAMP(15);
    // The score words a thread would rank are requested by EVERY workgroup right behind its counter
    // update, before it knows whether it is the last one: the last one then has them (or, for slots
    // whose writer's store had not landed yet, the empty mark, which finish_score re-reads) one round
    // trip earlier; the others drop them.  A slot is only ever re-armed by the last workgroup.
    uint32_t key[EMAX];
    const bool rank_some = P < np;  // (else every page is returned and nothing is ranked)
    if (!single) {
        int old = 0;
        if (tid == 0) old = __hip_atomic_fetch_add(d.counter + u, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (rank_some) {
#pragma unroll
            for (int e = 0; e < EMAX; ++e)
                key[e] = __hip_atomic_load(S + min(e * NT + tid, np - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (tid == 0) {
            // 1: the last to arrive carries on; 2: the unit was marked failed by an earlier launch (its
            // counter is negative until the index is rebuilt or imported again): chunk 0 says so again
            int role = old < 0 ? (chunk == 0 ? 2 : 0) : (old == chunks - 1 ? 1 : 0);
            if (role == 1) __hip_atomic_store(d.counter + u, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
            sh_last = role;
        }
        lds_barrier();  // (the score words stay in flight across it)
        if (!sh_last) return;
    }
    // A score hand-off that did not complete (a slot still empty after the bounded wait) is never
    // ranked: the unit reports n_selected = -1, ids -1 and a zero output, and stays marked (negative
    // arrival counter, slots left as they are) so that every later launch reports the same until
    // ice_build_index / ice_import_index re-arm the unit.
    auto report_failure = [&] {
        for (int x = tid; x < P; x += NT) {
            ids_out[(size_t)u * P + x] = -1;
            if (scores_out) scores_out[(size_t)u * P + x] = 0.f;
        }
        if (out)
            for (int o = tid; o < G * kD; o += NT) out[(size_t)u * G * kD + o] = 0.f;
        if (tid == 0) {
            n_sel_out[u] = -1;
            __hip_atomic_store(d.counter + u, kUnitFailed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };
    if (!single && sh_last == 2) {  // (workgroup-uniform)
        report_failure();
        return;
    }
    ICE_STAMP(1);
    ICE_USTAMP(1);
    // A thread's score words are all requested before any is looked at (clamped addresses, no
    // branches in between: one round trip, not E), and the slots are re-armed only after the last
    // one has been read: a store issued between two reads would make the second read wait for it.
    auto request_score = [&](int pid) -> uint32_t {
        return single ? sc_lds[pid] : __hip_atomic_load(S + pid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };
    auto finish_score = [&](int pid, uint32_t v) -> uint32_t {  // (several workgroups per unit only)
        if (v != kScoreEmpty) return v;
        for (int spin = 0; v == kScoreEmpty && spin < spin_limit; ++spin)
            v = __hip_atomic_load(S + pid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (v == kScoreEmpty) {  // never expected; a fence bounds the wait
            __threadfence();
            v = __hip_atomic_load(S + pid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (v == kScoreEmpty) sh_fail = 1;  // gave up: the workgroup reports the unit as failed
        return v;
    };
    auto rearm_score = [&](int pid) {
        __hip_atomic_store(S + pid, kScoreEmpty, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    };

    // ---- phase B: top-k pages
    const int k = min(P, np);
    int *ids = ids_out + (size_t)u * P;
    float *sco = scores_out ? scores_out + (size_t)u * P : nullptr;
    const int Pk = min(P, d.max_pages);
    u64 *sel_comp = (u64 *)(smem + round_up(Pk * 4, 16));         // [Pk] winners by rank
    char *region = smem + round_up(Pk * 4, 16) + (size_t)Pk * 8;  // candidates, later attention scratch
    u64 *cand = (u64 *)region;
    if (k == np) {
        // budget covers every page
        if (!single) {  // all slots filled?  (nothing is written or re-armed before that is known)
            for (int x = tid; x < k; x += NT) finish_score(x, request_score(x));
            lds_barrier();
            if (sh_fail) {
                report_failure();
                return;
            }
        }
        for (int x = tid; x < k; x += NT) {
            const uint32_t v = request_score(x);
            if (!single) rearm_score(x);
            ids[x] = x;
            if (sco) sco[x] = __uint_as_float(v);
        }
    } else {
        if (single) {
#pragma unroll
            for (int e = 0; e < EMAX; ++e) key[e] = sc_lds[min(e * NT + tid, np - 1)];
        } else {
#pragma unroll
            for (int e = 0; e < EMAX; ++e)
                if (e * NT + tid < np) key[e] = finish_score(e * NT + tid, key[e]);
            lds_barrier();
            if (sh_fail) {  // (workgroup-uniform)
                report_failure();
                return;
            }
#pragma unroll
            for (int e = 0; e < EMAX; ++e)
                if (e * NT + tid < np) rearm_score(e * NT + tid);
        }
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            const bool valid = e * NT + tid < np;
            key[e] = valid ? f32_ordered(__uint_as_float(key[e])) : 0u;
        }
        ICE_STAMP(2);
        constexpr int NR = 4 * NW;   // 16-lane rows in the workgroup
        constexpr int NO = 8 * NW;   // 8-lane groups
        constexpr int NQ = 16 * NW;  // 4-lane groups
        // The k-th largest of N disjoint groups' maxima is a threshold that k keys reach; it lets through
        // few more than k keys while k is at most N / 2: the NR rows up to k = NR / 2, then the NO
        // eight-lane groups, then the NQ four-lane groups; beyond k = NQ / 2 the prefix histograms.
        const bool by_groups = k > NR / 2 && k <= NQ / 2;
        const bool by_prefix = k > NQ / 2;
        if (by_groups) {
            // B1, medium budgets: group maxima of the key registers, made distinct by the group's number
            // in their low byte (the threshold need not be a key: any value that k keys reach will do),
            // so that ranking a maximum among the N is one comparison per pair; the lanes of a group
            // share its N comparisons.
            const bool quads = k > NO / 2;  // (workgroup-uniform)
            const int lg = quads ? 2 : 3, NGr = NT >> lg, gs = 1 << lg;
            uint32_t lmax = key[0];
#pragma unroll
            for (int e = 1; e < EMAX; ++e) lmax = max(lmax, key[e]);
            lmax = max(lmax, dpp_u32<0xB1>(lmax));  // quad_perm [1,0,3,2]
            lmax = max(lmax, dpp_u32<0x4E>(lmax));  // quad_perm [2,3,0,1]
            if (!quads) lmax = max(lmax, dpp_u32<0x141>(lmax));  // row_half_mirror: 8 lanes
            const int i = tid >> lg, part = tid & (gs - 1);
            if (part == 0) sh_quadmax[i] = (lmax & 0xFFFFFF00u) | (uint32_t)(255 - i);
            lds_barrier();
            const uint32_t v = sh_quadmax[i];
            const int len = NGr >> lg;  // comparisons per lane
            uint32_t c = 0;
#pragma unroll 8
            for (int jj = 0; jj < len; ++jj) c += sh_quadmax[part * len + jj] > v ? 1u : 0u;
            c += dpp_u32<0xB1>(c);
            c += dpp_u32<0x4E>(c);
            if (!quads) c += dpp_u32<0x141>(c);
            if (part == 0 && (int)c == k - 1) sh_pre = v & 0xFFFFFF00u;
        } else if (!by_prefix) {
            // B1, small budgets: the k-th largest of the 4*NW group maxima (groups without keys count as the
            // smallest key).  With several workgroups per unit the groups are the 16-lane rows of
            // the key registers; with one they were formed while scoring.
            if (!single) {
                uint32_t lmax = key[0];
#pragma unroll
                for (int e = 1; e < EMAX; ++e) lmax = max(lmax, key[e]);
                lmax = row16_max_u32(lmax);
                if (ch == 0) sh_rowmax[wave * 4 + g] = lmax;
                __syncthreads();
            }
            // rank of row maximum i among the NR (equal values: lower row first); 16 lanes share the work
            const int i = tid >> 4, part = tid & 15;
            const uint32_t v = sh_rowmax[i];
            uint32_t c = 0;
#pragma unroll
            for (int jj = 0; jj < NR / 16; ++jj) {
                const int j = part * (NR / 16) + jj;
                const uint32_t o = sh_rowmax[j];
                c += (o > v || (o == v && j < i)) ? 1u : 0u;
            }
            c = row16_sum_u32(c);
            if (part == 0 && (int)c == k - 1) sh_pre = v;
        } else {
            // B1, large budgets (the row maxima would let through a multiple of k): the 16-bit prefix
            // of the k-th largest key, from two 8-bit LDS histograms (top byte, then the second byte
            // inside the top byte's bucket), and how many keys of that prefix are still needed.
            int *h0 = (int *)region, *h1 = h0 + 272;  // (the candidate list starts here afterwards)
            if (tid < 256) { h0[tid] = 0; h1[tid] = 0; }
            lds_barrier();
            auto find_bucket = [&](int *h, int kk, int shift) {  // bins in descending order: thread t owns bin 255 - t
                int mine = 0, incl = 0;
                if (tid < 256) {
                    mine = h[255 - tid];
                    incl = mine;
                    for (int off = 1; off < 64; off <<= 1) {
                        const int t2 = __shfl_up(incl, off);
                        if (lane >= off) incl += t2;
                    }
                    if (lane == 63) h[256 + wave] = incl;
                }
                lds_barrier();
                if (tid < 256) {
                    for (int w2 = 0; w2 < wave; ++w2) incl += h[256 + w2];
                    const int excl = incl - mine;
                    if (incl >= kk && excl < kk) {  // exactly one bin
                        atomicOr(&sh_pre, (uint32_t)(255 - tid) << shift);
                        sh_M2 = kk - excl;
                    }
                }
                lds_barrier();
            };
            // (the top byte is sign and exponent: most keys of a wave share it, so the lanes that agree
            // with the first active lane are counted with one update)
#pragma unroll
            for (int e = 0; e < EMAX; ++e) {
                const int bin = e * NT + tid < np ? (int)(key[e] >> 24) : -1;
                const u64 act = __ballot(bin >= 0);
                if (act != 0ull) {  // (wave-uniform)
                    const int lead = (int)__builtin_ctzll(act);
                    const int first_bin = __shfl(bin, lead);
                    const u64 same = __ballot(bin == first_bin);
                    if (lane == lead) atomicAdd(&h0[first_bin], (int)__popcll(same));
                    if (bin >= 0 && bin != first_bin) atomicAdd(&h0[bin], 1);
                }
            }
            lds_barrier();
            find_bucket(h0, k, 24);
            const uint32_t top = sh_pre >> 24;
            const int k2 = sh_M2;
#pragma unroll
            for (int e = 0; e < EMAX; ++e)
                if (e * NT + tid < np && (key[e] >> 24) == top) atomicAdd(&h1[(int)((key[e] >> 16) & 255u)], 1);
            lds_barrier();
            find_bucket(h1, k2, 16);
        }
        lds_barrier();
        const uint32_t pre = sh_pre;
        ICE_STAMP(3);
        // B2: candidates = (score key, ~page id) composites at or above the threshold; all distinct.
        // One LDS counter bump per wave reserves the slots of all its candidates.  With the prefix
        // threshold only the keys that share the prefix are candidates: the keys above it are winners
        // as they are (k - need of them) and take the first places of the winner list, wave after
        // wave in a fixed order.
        const int need = by_prefix ? sh_M2 : k, first = k - need;
        auto list_candidates = [&](auto with_prefix) {
            constexpr bool PREFIX = decltype(with_prefix)::value;
            // (the lane masks are formed twice, once to count and once to place: keeping EMAX of them
            // would not fit the scalar registers of the instantiations with many keys per thread)
            auto listed = [&](int e) {
                const bool valid = e * NT + tid < np;
                if constexpr (PREFIX) return __ballot(valid && (key[e] >> 16) == (pre >> 16));
                else return __ballot(valid && key[e] >= pre);
            };
            auto is_above = [&](int e) { return __ballot(e * NT + tid < np && (key[e] >> 16) > (pre >> 16)); };
            int tot = 0, tot_a = 0;
#pragma unroll
            for (int e = 0; e < EMAX; ++e) {
                tot += (int)__popcll(listed(e));
                if constexpr (PREFIX) tot_a += (int)__popcll(is_above(e));
            }
            int base = 0;
            if (lane == 0 && tot) base = atomicAdd(&sh_M, tot);
            base = __shfl(base, 0);
            const u64 lower = (1ull << lane) - 1ull;
#pragma unroll
            for (int e = 0; e < EMAX; ++e) {
                const int pid = e * NT + tid;
                const u64 bal = listed(e);
                const int slot = base + (int)__popcll(bal & lower);
                if (((bal >> lane) & 1ull) && slot < cand_cap)  // (a list that overflows is not used: see B3)
                    cand[slot] = ((u64)key[e] << 32) | (u64)(0xFFFFFFFFu - (uint32_t)pid);
                base += (int)__popcll(bal);
            }
            if constexpr (PREFIX) {
                if (lane == 0) sh_rowmax[wave] = (uint32_t)tot_a;  // (the row maxima are not needed on this path)
                lds_barrier();
                int base_a = 0;
                for (int w2 = 0; w2 < wave; ++w2) base_a += (int)sh_rowmax[w2];
#pragma unroll
                for (int e = 0; e < EMAX; ++e) {
                    const int pid = e * NT + tid;
                    const u64 bal_a = is_above(e);
                    if ((bal_a >> lane) & 1ull)
                        sel_comp[base_a + (int)__popcll(bal_a & lower)] = ((u64)key[e] << 32) | (u64)(0xFFFFFFFFu - (uint32_t)pid);
                    base_a += (int)__popcll(bal_a);
                }
            }
        };
        if (by_prefix) list_candidates(std::true_type{});  // (workgroup-uniform)
        else list_candidates(std::false_type{});
        lds_barrier();
        const int M = sh_M;  // >= need
        ICE_STAMP(4);
        // B3: the `need` best of the M candidates, exactly, into sel_comp[first..k)
        if (M > cand_cap) {
            // More candidates than the list holds (many equal scores, or a threshold that cut little):
            // radix select straight from the key registers over ALL keys of the unit, 8 bits a pass over
            // the (32 + nb)-bit packed composite (score key, lower id first); it fills sel_comp[0..k) as
            // a whole, waves in a fixed order.
            int nb = 0;
            while ((1 << nb) < np) ++nb;
            const u64 idmask = (1ull << nb) - 1ull;
            auto packed = [&](int e) { return ((u64)key[e] << nb) | (idmask - (u64)(uint32_t)(e * NT + tid)); };
            int *hist = (int *)region;  // 256 bins + wave totals (the overflowed list is dead)
            u64 prefix = 0ull, known = 0ull;
            int kk = k;
            for (int sft = ((32 + nb - 1) / 8) * 8; sft >= 0; sft -= 8) {
                lds_barrier();
                if (tid < 256) hist[tid] = 0;
                lds_barrier();
#pragma unroll
                for (int e = 0; e < EMAX; ++e) {
                    // (keys that share the prefix mostly share the next byte as well: the lanes that agree
                    // with the first such lane are counted with one update)
                    const u64 pk = packed(e);
                    const int bin = e * NT + tid < np && (pk & known) == prefix ? (int)((pk >> sft) & 255ull) : -1;
                    const u64 act = __ballot(bin >= 0);
                    if (act != 0ull) {  // (wave-uniform)
                        const int lead = (int)__builtin_ctzll(act);
                        const int first_bin = __shfl(bin, lead);
                        const u64 same = __ballot(bin == first_bin);
                        if (lane == lead) atomicAdd(&hist[first_bin], (int)__popcll(same));
                        if (bin >= 0 && bin != first_bin) atomicAdd(&hist[bin], 1);
                    }
                }
                lds_barrier();
                int h = 0, incl = 0;
                if (tid < 256) {  // bins in descending order: thread t owns bin 255 - t
                    h = hist[255 - tid];
                    incl = h;
                    for (int off = 1; off < 64; off <<= 1) {
                        const int t2 = __shfl_up(incl, off);
                        if (lane >= off) incl += t2;
                    }
                    if (lane == 63) hist[256 + wave] = incl;
                }
                lds_barrier();
                if (tid < 256) {
                    for (int w2 = 0; w2 < wave; ++w2) incl += hist[256 + w2];
                    const int excl = incl - h;
                    if (incl >= kk && excl < kk) {
                        sh_tau = prefix | ((u64)(255 - tid) << sft);
                        sh_M2 = kk - excl;
                    }
                }
                lds_barrier();
                prefix = sh_tau;
                kk = sh_M2;
                known |= 255ull << sft;
            }
            // prefix = packed composite of the k-th largest key; everything at or above it wins
            const u64 lower = (1ull << lane) - 1ull;
            int tot = 0;
#pragma unroll
            for (int e = 0; e < EMAX; ++e) tot += (int)__popcll(__ballot(e * NT + tid < np && packed(e) >= prefix));
            lds_barrier();
            if (lane == 0) sh_rowmax[wave] = (uint32_t)tot;
            lds_barrier();
            int base = 0;
            for (int w2 = 0; w2 < wave; ++w2) base += (int)sh_rowmax[w2];
#pragma unroll
            for (int e = 0; e < EMAX; ++e) {
                const int pid = e * NT + tid;
                const u64 bal = __ballot(pid < np && packed(e) >= prefix);
                if ((bal >> lane) & 1ull) sel_comp[base + (int)__popcll(bal & lower)] = ((u64)key[e] << 32) | (u64)(0xFFFFFFFFu - (uint32_t)pid);
                base += (int)__popcll(bal);
            }
        } else if (M <= 512) {
            // every candidate counts the candidates that beat it; `parts` lanes share one candidate
            int lp = 0;
            while (lp < 6 && (M << (lp + 1)) <= NT) ++lp;
            const int parts = 1 << lp, i = tid >> lp, part = tid & (parts - 1), len = (M + parts - 1) >> lp;
            const u64 mine = i < M ? cand[i] : ~0ull;
            int rank = 0;
#pragma unroll 4
            for (int j = part * len; j < min(M, (part + 1) * len); ++j) rank += cand[j] > mine;
            // sum over the `parts` lanes of a candidate: DPP inside a 16-lane row, shuffles beyond
            if (parts >= 2) rank += (int)dpp_u32<0xB1>((uint32_t)rank);
            if (parts >= 4) rank += (int)dpp_u32<0x4E>((uint32_t)rank);
            if (parts >= 8) rank += (int)dpp_u32<0x141>((uint32_t)rank);
            if (parts >= 16) rank += (int)dpp_u32<0x140>((uint32_t)rank);
            if (parts >= 32) rank += __shfl_xor(rank, 16);
            if (parts >= 64) rank += __shfl_xor(rank, 32);
            if (part == 0 && i < M && rank < need) sel_comp[first + rank] = mine;
        } else {
            // radix select on LDS histograms, 8 bits a pass, over the (32 + nb)-bit packed composite
            int nb = 0;
            while ((1 << nb) < np) ++nb;
            const u64 idmask = (1ull << nb) - 1ull;
            int *hist = (int *)(cand + M);          // 256 bins + 4 wave totals, behind the candidates
            u64 prefix = 0ull, known = 0ull;
            int kk = need;
            for (int sft = ((32 + nb - 1) / 8) * 8; sft >= 0; sft -= 8) {
                if (tid < 256) hist[tid] = 0;
                lds_barrier();
                for (int t = tid; t < M; t += NT) {
                    const u64 cc = cand[t];
                    const u64 pk = ((cc >> 32) << nb) | (cc & idmask);
                    if ((pk & known) == prefix) atomicAdd(&hist[(int)((pk >> sft) & 255ull)], 1);
                }
                lds_barrier();
                int h = 0, incl = 0;
                if (tid < 256) {  // bins in descending order: thread t owns bin 255 - t
                    h = hist[255 - tid];
                    incl = h;
                    for (int off = 1; off < 64; off <<= 1) {
                        const int t2 = __shfl_up(incl, off);
                        if (lane >= off) incl += t2;
                    }
                    if (lane == 63) hist[256 + wave] = incl;
                }
                lds_barrier();
                if (tid < 256) {
                    for (int w2 = 0; w2 < wave; ++w2) incl += hist[256 + w2];
                    const int excl = incl - h;
                    if (incl >= kk && excl < kk) {
                        sh_tau = prefix | ((u64)(255 - tid) << sft);
                        sh_M2 = kk - excl;
                    }
                }
                lds_barrier();
                prefix = sh_tau;
                kk = sh_M2;
                known |= 255ull << sft;
                lds_barrier();
            }
            // prefix = packed composite of the k-th largest candidate; everything at or above it wins
            for (int t = tid; t < M; t += NT) {
                const u64 cc = cand[t];
                const u64 pk = ((cc >> 32) << nb) | (cc & idmask);
                if (pk >= prefix) sel_comp[first + atomicAdd(&sh_W, 1)] = cc;
            }
        }
    }
    lds_barrier();
    ICE_STAMP(5);
    ICE_USTAMP(2);
    // ---- phase C: attention over the winners, in rank order (the ids' ascending order is only an
    // output format and is produced afterwards, off the critical path)
    const bool all_pages = k == np;
    // B4: the winners' places in ascending id order; during the attention it runs where the first
    // waves would wait for the last ones
    auto order_ids = [&] {
        // (every global store of the selection is issued here, after the ranking: a store in flight
        // makes the next wait of its wave as long as a write to memory)
        for (int x = k + tid; x < P; x += NT) {
            ids[x] = -1;
            if (sco) sco[x] = 0.f;
        }
        if (tid == 0) n_sel_out[u] = k;
        if (all_pages) return;
        for (int t = tid; t < k; t += NT) {
            const u64 mine = sel_comp[t];
            const uint32_t myid = 0xFFFFFFFFu - (uint32_t)mine;
            int pos = 0;
            for (int j = 0; j < k; ++j) pos += (0xFFFFFFFFu - (uint32_t)sel_comp[j]) < myid;
            ids[pos] = (int)myid;
            if (sco) sco[pos] = ordered_f32((uint32_t)(mine >> 32));
        }
    };
    if (out) {
        ICE_STAMP(6);
        bf16x8 qa[4];
        SR::to_plain(qs, lane, qa);
        attend_pages<G, NW, RES>(d, u, qa, [=](int x) { return all_pages ? x : (int)(0xFFFFFFFFu - (uint32_t)sel_comp[x]); }, k,
                                 res, out, (float *)region, order_ids);
        ICE_STAMP(7);
    } else {
        order_ids();
    }
    ICE_USTAMP(3);
}

// Workgroups per unit: enough for every CU when units are few, but at least one 16-page block per
// wave each (smaller pieces were measured slower: 64 pages per workgroup 15.8 us per one-layer
// step, 128 pages 14.95, 256 pages 14.85: more arrivals per counter, no shorter scoring).
int decode_step_chunks(const Dev &d, int np_hint) {
    const int NW = d.G == 8 ? 8 : 16;
    np_hint = std::max(1, std::min(np_hint, d.max_pages));
    int chunks = 256 / d.U;
    const int max_chunks = (np_hint + 16 * NW - 1) / (16 * NW);
    if (chunks > max_chunks) chunks = max_chunks;
    return chunks < 1 ? 1 : chunks;
}

// the attention of a selection call as a launch of its own (few units, many pages per unit)
bool launch_attend_would_split(const Dev &d, int P) { return attend_shares(d, P, kFusedSplitMinShares) > 1; }
void launch_attend_split_after_select(const Dev &d, const bf16_t *q, const int *ids, const int *n_sel, int P, float *out, hipStream_t st) {
    launch_attend(d, q, ids, n_sel, P, Resident{nullptr, nullptr, 0, nullptr, nullptr, 0}, out, st, kFusedSplitMinShares);
}

// Launch shape and LDS of a decode step.  LDS: the winner lists ([Pk] ids, [Pk] composites), then
// one region used first for the candidate list (cand_cap entries + histograms) and later as the
// attention's scratch, then, with one workgroup per unit only, the unit's scores.  The candidate
// list is as long as the pages the index can hold, up to kCandCapMax entries (a longer list is
// never needed unless thousands of scores tie: then the selection runs from the key registers).
constexpr int kCandCapMax = 4096;
DecodePlan decode_step_plan(const Dev &d, int P, int np_hint) {
    const int NW = d.G == 8 ? 8 : 16;
    DecodePlan p;
    p.np_hint = std::max(1, std::min(np_hint, d.max_pages));
    p.chunks = decode_step_chunks(d, p.np_hint);
    const int Pk = P < d.max_pages ? P : d.max_pages;
    const size_t red_bytes = sizeof(float) * attend_scratch_floats(d.G, NW);
    const size_t fixed = round_up(Pk * 4, 16) + (size_t)Pk * 8 + (p.chunks == 1 ? (size_t)d.max_pages * 4 : 0);
    const size_t limit = 160u * 1024u - 2048u;  // (static LDS of the kernel: 1.7 KB)
    // no candidate list is needed when the budget covers every page the index can hold
    p.cand_cap = P >= d.max_pages ? 0 : std::min(d.max_pages, kCandCapMax);
    auto total = [&](int cap) {
        const size_t cand_bytes = cap ? (size_t)cap * 8 + 272 * 4 : 0;
        return fixed + round_up((int)std::max(cand_bytes, std::max(red_bytes, (size_t)272 * 4)), 16);
    };
    if (total(p.cand_cap) > limit && p.cand_cap > 1024) p.cand_cap = 1024;
    p.lds = total(p.cand_cap);
    p.scores_off = p.chunks == 1 ? (int)(p.lds - (size_t)d.max_pages * 4) : 0;
    p.fits = p.lds <= limit;
    return p;
}

void launch_decode_step(const Dev &d, const bf16_t *q, int P, int np_hint, int *ids, int *n_sel, float *scores_out,
                        const bf16_t *res_k, const bf16_t *res_v, int n_res, float *out, hipStream_t st, int wait_cfg) {
    const int NW = d.G == 8 ? 8 : 16;
    // a workgroup pass scores 16*NW pages per load round; few units -> split each unit over many
    // workgroups (one round each), many units -> one workgroup per unit and no cross-workgroup step
    const DecodePlan plan = decode_step_plan(d, P, np_hint);
    np_hint = plan.np_hint;
    const int chunks = plan.chunks;
    // few units and a large budget: select in this launch, attend with the unit's pages spread over
    // several workgroups (one more launch, see attend_split_kernel)
    const bool split_attend = out && chunks > 1 && n_res == 0 && launch_attend_would_split(d, P);
    float *out_fused = split_attend ? nullptr : out;
    const size_t lds = plan.lds;
    const int grid = round_up(d.U, 8) * chunks;
    const int E = (d.max_pages + NW * 64 - 1) / (NW * 64);
    const Resident res = {res_k, res_v, out_fused ? n_res : 0, nullptr, nullptr, 0};
#define ICE_STEP_R(g, nw, e, r)                                                                                     \
    do {                                                                                                            \
        allow_dynamic_lds((const void *)decode_step_kernel<g, nw, e, r>, lds);                                      \
        hipLaunchKernelGGL((decode_step_kernel<g, nw, e, r>), dim3(grid), dim3(nw * 64), lds, st, d.U, d.max_pages, P, chunks, np_hint, \
                           plan.scores_off, wait_cfg, plan.cand_cap, d.rep, q, d.n_pages, d, ids, n_sel, scores_out, res, out_fused); \
    } while (0)
#define ICE_STEP(g, nw, e)                                                                                          \
    do {                                                                                                            \
        if (res.n > 0) ICE_STEP_R(g, nw, e, true);                                                                  \
        else ICE_STEP_R(g, nw, e, false);                                                                           \
    } while (0)
    if (d.G == 8) { if (E <= 8) ICE_STEP(8, 8, 8); else if (E <= 32) ICE_STEP(8, 8, 32); else ICE_STEP(8, 8, 64); }
    else if (d.G == 4) { if (E <= 4) ICE_STEP(4, 16, 4); else if (E <= 16) ICE_STEP(4, 16, 16); else ICE_STEP(4, 16, 32); }
    else if (d.G == 2) { if (E <= 4) ICE_STEP(2, 16, 4); else if (E <= 16) ICE_STEP(2, 16, 16); else ICE_STEP(2, 16, 32); }
    else { if (E <= 4) ICE_STEP(1, 16, 4); else if (E <= 16) ICE_STEP(1, 16, 16); else ICE_STEP(1, 16, 32); }
#undef ICE_STEP
#undef ICE_STEP_R
    if (split_attend) launch_attend_split_after_select(d, q, ids, n_sel, P, out, st);
}

// largest page count launch_decode_step can serve (a unit's scores are ranked from one workgroup's registers)
int decode_step_max_pages(int G) { return (G == 8 ? 8 * 64 * 64 : 16 * 64 * 32); }

}  // namespace ice

ICE_PROF_EXPORT(ice_debug_prof_decode)
