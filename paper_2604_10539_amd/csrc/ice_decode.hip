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
// Insertion (Alg. 1 insertion loop; a node that outgrows its page gets a new one, Sec. 4.1).  One
// workgroup of 16 waves per unit.  A token goes to the nearest bf16 centroid, objective
// ||mu~||^2 - 2 k . mu~ (with the extra coordinate when the keys are transformed, Eq. 2), lowest id
// on ties; the dot products come off the matrix cores (v_mfma_f32_16x16x32_bf16: A = the tokens'
// keys, one per row; B = 16 centroid rows), and every one of them comes out of the same instruction
// sequence whichever row or column slot it sits in, so inserting m tokens in one launch and in m
// launches leaves the same bits.  The cluster then moves (ordered fp32: sum -> centroid -> bf16 row
// and squared norm) and the row is appended to the cluster's tail page (page sum -> representative).
constexpr int kInsertWaves = 16;
constexpr int kInsertTokens = 16;  // tokens per launch of the batched kernel at most (one per wave)

__device__ inline float insert_objective(float w, float dot, float kaf, float ce) {
    return __builtin_fmaf(-2.0f, __builtin_fmaf(kaf, ce, dot), w);
}
__device__ inline u64 insert_pack(float val, int c) { return ((u64)f32_ordered(val) << 32) | (u64)(uint32_t)c; }
__device__ inline int insert_winner(u64 b) { return b == ~0ull ? 0 : (int)(uint32_t)b; }  // (every objective NaN: cluster 0, as an exhaustive search that never sees a smaller value)
__device__ inline u64 readlane_u64(u64 x, int l) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, l);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), l);
    return ((u64)hi << 32) | lo;
}
// minimum over the 16 lanes of a DPP row / over the wave (vector unit only, no trip through LDS)
__device__ inline u64 row16_min_u64(u64 x) {
#define ICE_MIN_STEP(CTRL)                                                                         \
    do {                                                                                           \
        const u64 y = ((u64)dpp_u32<CTRL>((uint32_t)(x >> 32)) << 32) | dpp_u32<CTRL>((uint32_t)x); \
        x = y < x ? y : x;                                                                         \
    } while (0)
    ICE_MIN_STEP(0xB1);
    ICE_MIN_STEP(0x4E);
    ICE_MIN_STEP(0x141);
    ICE_MIN_STEP(0x140);
#undef ICE_MIN_STEP
    return x;
}
__device__ inline u64 wave_min_u64(u64 x) {
    x = row16_min_u64(x);
    const u64 a = readlane_u64(x, 0), b = readlane_u64(x, 16), c = readlane_u64(x, 32), e = readlane_u64(x, 48);
    const u64 ab = a < b ? a : b, ce = c < e ? c : e;
    return ab < ce ? ab : ce;
}
// the two smallest of the wave's values (each lane brings its own two smallest, a <= b)
__device__ inline void merge_min2(u64 &a, u64 &b, u64 pa, u64 pb) {
    const u64 hi = a < pa ? pa : a, lo2 = b < pb ? b : pb;
    a = a < pa ? a : pa;
    b = hi < lo2 ? hi : lo2;
}
__device__ inline void wave_min2_u64(u64 &a, u64 &b) {
#define ICE_MIN2_STEP(CTRL)                                                                          \
    do {                                                                                             \
        const u64 pa = ((u64)dpp_u32<CTRL>((uint32_t)(a >> 32)) << 32) | dpp_u32<CTRL>((uint32_t)a);  \
        const u64 pb = ((u64)dpp_u32<CTRL>((uint32_t)(b >> 32)) << 32) | dpp_u32<CTRL>((uint32_t)b);  \
        merge_min2(a, b, pa, pb);                                                                    \
    } while (0)
    ICE_MIN2_STEP(0xB1);
    ICE_MIN2_STEP(0x4E);
    ICE_MIN2_STEP(0x141);
    ICE_MIN2_STEP(0x140);
#undef ICE_MIN2_STEP
    u64 ra = readlane_u64(a, 0), rb = readlane_u64(b, 0);
    merge_min2(ra, rb, readlane_u64(a, 16), readlane_u64(b, 16));
    merge_min2(ra, rb, readlane_u64(a, 32), readlane_u64(b, 32));
    merge_min2(ra, rb, readlane_u64(a, 48), readlane_u64(b, 48));
    a = ra;
    b = rb;
}
// sum over the wave in a fixed order: the four row sums, then ((r0 + r1) + r2) + r3
__device__ inline float wave_sum_rows(float x) {
    x = row16_sum(x);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
    return ((r0 + r1) + r2) + r3;
}
// the four MFMAs of one 16-row tile: lane (g, n) ends with tokens 4g .. 4g+3 against column n
__device__ inline f32x4 insert_dots(const bf16x8 (&ka)[4], const uint4 (&b)[4]) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[ks], __builtin_bit_cast(bf16x8, b[ks]), acc, 0, 0, 0);
    return acc;
}
// what a token does to its cluster: ordered-fp32 running sums, the mean, its bf16 rounding and squared norm
struct ClusterMove {
    int cnt;
    float2 cs, mu;
    uint32_t packed;  // this lane's two bf16 coordinates of the moved row
    float nn, es, e, ef;
    bf16_t eb;
};
__device__ inline ClusterMove insert_move(int cnt_old, float2 cs, float es_old, uint32_t kw, float kaf, bool tk) {
    ClusterMove r;
    r.cnt = cnt_old + 1;
    cs.x = cs.x + bf16_lo(kw);
    cs.y = cs.y + bf16_hi(kw);
    r.cs = cs;
    const float fc = (float)r.cnt;
    r.mu = make_float2(cs.x / fc, cs.y / fc);
    const bf16_t b0 = f32_to_bf16(r.mu.x), b1 = f32_to_bf16(r.mu.y);
    r.packed = (uint32_t)b0 | ((uint32_t)b1 << 16);
    const float f0 = bf16_to_f32(b0), f1 = bf16_to_f32(b1);
    r.nn = wave_sum_rows(f0 * f0 + f1 * f1);
    r.es = 0.f; r.e = 0.f; r.ef = 0.f; r.eb = 0;
    if (tk) {  // the cluster's extra coordinate follows its members' running mean as well
        r.es = es_old + kaf;
        r.e = r.es / fc;
        r.eb = f32_to_bf16(r.e);
        r.ef = bf16_to_f32(r.eb);
        r.nn += r.ef * r.ef;
    }
    return r;
}
__device__ inline void insert_store_move(const Dev &d, bf16_t *cent, float *cnorm, bf16_t *caug_cur, int u, int c, int Cpad, int lane,
                                         const ClusterMove &mv, bool tk) {
    const size_t cl = (size_t)u * d.C + c;
    ((float2 *)(d.cluster_sum + cl * kD))[lane] = mv.cs;
    ((float2 *)(d.centroid + cl * kD))[lane] = mv.mu;
    ((uint32_t *)(cent + ((size_t)u * Cpad + c) * kD))[lane] = mv.packed;
    if (lane == 0) {
        cnorm[(size_t)u * Cpad + c] = mv.nn;
        d.cluster_cnt[cl] = mv.cnt;
        if (tk) {
            d.csum_aug[cl] = mv.es;
            d.cent_aug[cl] = mv.e;
            caug_cur[(size_t)u * Cpad + c] = mv.eb;
        }
    }
}

// A wave's own staging area for centroid tiles (16 rows x 256 bytes each): direct global -> LDS loads
// of four whole rows per instruction (a quad of lanes reads 64 contiguous bytes; loading the MFMA
// operand straight from memory would spread every quad over four rows), the 16-byte chunk c of row r
// in slot c ^ r so that the operand reads (lane (g, n): chunk 4 ks + g of row n) are conflict-free.
constexpr int kInsertTileBytes = 16 * kD * 2;
__device__ inline void insert_stage_tile(const bf16_t *cb, int tile, char *stg, int lane) {
    const int g = lane >> 4, i = lane & 15;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int rr = 4 * x + g;
        lds_dma16((const uint4 *)(cb + (size_t)(tile * 16 + rr) * kD) + (i ^ rr), stg + x * 1024);
    }
}
__device__ inline void insert_read_tile(const char *stg, int lane, uint4 (&b)[4]) {
    const int g = lane >> 4, n = lane & 15;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) b[ks] = *(const uint4 *)(stg + n * 256 + (((4 * ks + g) ^ n) << 4));
}

// One token per unit.  Every wave scans its share of the centroid tiles (both tiles of a round
// requested at once) and keeps its best row in registers; it then requests what hangs on THAT row
// (count and sum of the cluster, its tail page with fill and sum: all kept beside the cluster, one
// round trip) before the waves meet in one LDS word, so that for the wave whose row wins these loads
// have been in flight while it waited for the others.  That wave alone carries on, with nothing
// left to fetch: it moves the cluster and appends the row.
// (cent, cnorm: the live centroid buffer d.cent_bf16[cur] / d.cnorm[cur], which this kernel also
// writes, hence neither const nor restrict)
__global__ __launch_bounds__(kInsertWaves * 64) void insert_one_kernel(const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                                                        bf16_t *cent, float *cnorm, int m_total, int t0, int cur,
                                                                        int C, int Cpad, int tk_arg, Dev d_arg) {  // (scalars first: preloaded)
    extern __shared__ __align__(16) char insert_stage[];  // [16 waves][2 tiles]
    __shared__ u64 s_best;
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, i = lane & 15;
    char *stg = insert_stage + wave * 2 * kInsertTileBytes;
    const bf16_t *cb = cent + (size_t)u * Cpad * kD;
    const float *wn = cnorm + (size_t)u * Cpad;
    const bf16_t *ku = k + ((size_t)u * m_total + t0) * kD, *vu = v + ((size_t)u * m_total + t0) * kD;
    ICE_STAMP(40);
    if (tid == 0) s_best = ~0ull;
    const int tiles = (C + 15) / 16;
    if (wave < tiles) {  // (the first round's tiles go out before anything else is asked of memory)
        insert_stage_tile(cb, wave, stg, lane);
        if (wave + kInsertWaves < tiles) insert_stage_tile(cb, wave + kInsertWaves, stg + kInsertTileBytes, lane);
    }
    bf16x8 ka[4];  // A operand: the key in row 0
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {  // (a load under a condition, not a choice between two addresses: no zero constant in memory)
        uint4 w = make_uint4(0, 0, 0, 0);
        if (i == 0) w = ((const uint4 *)ku)[ks * 4 + g];
        ka[ks] = __builtin_bit_cast(bf16x8, w);
    }
    // The other arguments are fetched here, once, while tiles and key are on their way (waiting for them
    // only after the scan measured slower: their loads are then issued there as well).
    const bool tk = tk_arg != 0;
    Dev d;
    bf16_t *caug_cur;
    pin_insert_fields(d, d_arg, cur, caug_cur);
    bf16_t kab = 0;
    if (tk) kab = key_extra_coordinate(d.c2[u], key_sqnorm16(((const uint4 *)ku)[i]));
    const float kaf = bf16_to_f32(kab);
    u64 best = ~0ull;
    lds_barrier();  // (s_best is set before any wave's minimum can reach it)
    ICE_STAMP(41);
    for (int tile = wave; tile < tiles; tile += 2 * kInsertWaves) {
        const int tb = tile + kInsertWaves;
        const int ra = tile * 16 + i, rb = tb * 16 + i;
        if (tile != wave) {
            insert_stage_tile(cb, tile, stg, lane);
            if (tb < tiles) insert_stage_tile(cb, tb, stg + kInsertTileBytes, lane);
        }
        const float wa = ra < C ? wn[ra] : INFINITY, wb = tb < tiles && rb < C ? wn[rb] : INFINITY;
        const float ea = tk && ra < C ? bf16_to_f32(caug_cur[(size_t)u * Cpad + ra]) : 0.f;
        const float eb = tk && tb < tiles && rb < C ? bf16_to_f32(caug_cur[(size_t)u * Cpad + rb]) : 0.f;
        wait_lds_dma();
        ICE_STAMP(45);
        uint4 b0[4], b1[4];
        insert_read_tile(stg, lane, b0);
        insert_read_tile(stg + kInsertTileBytes, lane, b1);  // (no second tile: stale rows, results unused)
        const f32x4 a0 = insert_dots(ka, b0), a1 = insert_dots(ka, b1);
        ICE_STAMP(46);
        if (g == 0) {  // (row 0 of the output: the token against columns 0..15)
            const float va = insert_objective(wa, a0[0], kaf, ea), vb = insert_objective(wb, a1[0], kaf, eb);
            if (ra < C && !(va != va)) { const u64 key = insert_pack(va, ra); best = key < best ? key : best; }
            if (tb < tiles && rb < C && !(vb != vb)) { const u64 key = insert_pack(vb, rb); best = key < best ? key : best; }
        }
    }
    const u64 mine = readlane_u64(row16_min_u64(best), 0);  // (only row 0 of the wave holds candidates)
    ICE_STAMP(47);
    // what hangs on this wave's best row, requested before the waves meet
    const int c = insert_winner(mine);
    const size_t cl = (size_t)u * d.C + c;
    const int cnt = d.cluster_cnt[cl];
    const float2 cs = ((const float2 *)(d.cluster_sum + cl * kD))[lane];
    const float es_old = tk ? d.csum_aug[cl] : 0.f;
    int tail = d.cluster_tail[cl];
    int fill = d.tail_fill[cl];  // (page_size when the cluster has no page)
    float2 ps = ((const float2 *)(d.tail_sum + cl * kD))[lane];
    const int np = d.n_pages[u], tok = d.n_tokens[u];
    const uint32_t kw = ((const uint32_t *)ku)[lane], vw = ((const uint32_t *)vu)[lane];
    if (lane == 0 && mine != ~0ull) atomicMin(&s_best, mine);
    ICE_STAMP(42);
    lds_barrier();
    ICE_STAMP(43);
    const u64 won = s_best;
    if (won == ~0ull ? wave != 0 : mine != won) return;  // (every objective NaN: wave 0 carries on with cluster 0)
    ICE_STAMP(48);
    const ClusterMove mv = insert_move(cnt, cs, es_old, kw, kaf, tk);
    insert_store_move(d, cent, cnorm, caug_cur, u, c, Cpad, lane, mv, tk);
    if (tk && lane == 0) d.kaug[(size_t)u * d.max_tokens + tok] = kab;
    ICE_STAMP(49);
    // the row goes to the cluster's tail page, or to a new page when that one is full or the cluster
    // has none (the sum is dropped when a page is opened)
    const bool fresh = fill == d.s;
    if (fresh) { tail = np; fill = 0; ps = make_float2(0.f, 0.f); }
    const size_t pg = (size_t)u * d.max_pages + tail;
    ((uint32_t *)(d.Kp + (pg * d.s + fill) * kD))[lane] = kw;
    ((uint32_t *)(d.Vp + (pg * d.s + fill) * kD))[lane] = vw;
    ps.x = ps.x + bf16_lo(kw);
    ps.y = ps.y + bf16_hi(kw);
    ((float2 *)(d.page_sum + pg * kD))[lane] = ps;
    ((float2 *)(d.tail_sum + cl * kD))[lane] = ps;
    const float ff = (float)(fill + 1);
    ((uint32_t *)(d.rep + pg * kD))[lane] = (uint32_t)f32_to_bf16(ps.x / ff) | ((uint32_t)f32_to_bf16(ps.y / ff) << 16);
    if (lane == 0) {
        d.cluster_tail[cl] = tail;
        d.tail_fill[cl] = fill + 1;
        d.page_fill[pg] = fill + 1;
        d.page_pos[pg * d.s + fill] = tok;
        d.n_tokens[u] = tok + 1;
        if (fresh) {
            d.page_cluster[pg] = c;
            d.n_pages[u] = np + 1;
        }
    }
    ICE_STAMP(44);
}

// Up to 16 tokens per unit, with the result of inserting them one after the other (the
// page-at-a-time insertion of tokens that leave the recent window).  What makes the tokens depend on
// each other is small: token t moves ONE centroid row and touches one page.  Steps:
//   scan     all waves: D[t][c], the dot product of every token with every centroid row, into LDS.
//            The centroids cross the CU once for all tokens.
//   guess    wave t: token t's nearest centroid (and the runner-up) as if no token before it had
//            moved anything, the loads that hang on that cluster (count, sum, tail page with its
//            fill and sum: one round trip, all tokens' side by side), the cluster's move worked out
//            on that assumption, and the moved row's dot products with all tokens (one more MFMA
//            chain, the row in column 0).
//   check    wave t, the earlier tokens on its lanes: against which of the earlier guessed moves
//            token t's guess fails (same cluster guessed, or the moved row nearer than the guess).
//   settle   wave 0, everything in registers and LDS.  Tokens whose guess fails against no move that
//            stands are settled as guessed, whole runs at once; the others one by one: the nearest
//            centroid given the rows moved so far is the guess, or the runner-up when the guessed
//            row has moved, or one of the moved rows (their fresh objectives come from the dot
//            products the movers left); only when guess and runner-up have both moved a full pass
//            over D, which is then brought in step with the moves.  Such a token's move is worked out
//            from the cluster's current state (in LDS for every cluster some token guessed, read
//            from memory otherwise) and stored by wave 0, and the later guesses are checked
//            against it.  Meanwhile wave 1 works out the page table for the case that every token
//            goes where it guessed.
//   commit   wave t stores its own move if it stood.
//   append   wave t: token t's row into its cluster's tail page, or into a page opened by the
//            first token that finds the page full (page ids in the order single insertions hand
//            them out); the last token of a page adds the page's new keys to its sum in token
//            order and writes the representative; the tables follow.
// Worst case: all tokens of a launch crowd into a few clusters, and the settle step handles them one
// after the other (about 3 us each on one wave).
// k, v: bf16 [U, m_total, d], tokens t0 .. t0 + mt of them in this launch.
__host__ __device__ inline int insert_row_stride(int C) { return round_up(C, 16) + 4; }  // (+4: the four token groups of a store hit different banks)
// dynamic LDS: D [mt][stride], norms [Cr] (+ extras [Cr]), the tokens' keys and moved rows [16][64] words each,
// per slot the cluster sum before and after the guessed move and the tail page's sum [16][64] float2 each
__host__ __device__ inline size_t insert_fixed_lds(int C, bool tk) {
    return (size_t)round_up(C, 16) * 4 * (tk ? 2 : 1) + 2 * kInsertTokens * 64 * 4 + 3 * kInsertTokens * 64 * 8;
}

__global__ __launch_bounds__(kInsertWaves * 64) void insert_batch_kernel(const bf16_t *__restrict__ k, const bf16_t *__restrict__ v,
                                                                          bf16_t *cent, float *cnorm, int m_total, int t0, int mt,
                                                                          int cur, int C, int Cpad, int stage_tiles, int tk_arg,
                                                                          Dev d_arg) {  // (scalars first: preloaded)
    extern __shared__ __align__(16) char insert_lds[];
    __shared__ u64 s_best[kInsertTokens];        // the guess: (ordered objective, cluster), ~0 when every objective is NaN
    __shared__ int s_cluster[kInsertTokens];     // slot t caches the state of token t's guessed cluster
    __shared__ int s_cnt[kInsertTokens], s_tail[kInsertTokens], s_fill[kInsertTokens];
    __shared__ float s_es[kInsertTokens], s_es1[kInsertTokens], s_kaf[kInsertTokens];
    __shared__ float s_nn[kInsertTokens], s_ef[kInsertTokens];  // squared norm and extra coordinate of the row token t's move forms
    __shared__ float s_dm[kInsertTokens][kInsertTokens];        // [t'][t]: token t against the row token t' moved
    __shared__ bf16_t s_ka[kInsertTokens];
    __shared__ u64 s_best2[kInsertTokens];                      // the runner-up of the guess
    __shared__ int s_fail[kInsertTokens];                       // bit t': token t's guess fails if token t' < t moves as it guessed
    __shared__ int s_stood;                                     // bit t: token t's guessed move stands (wave t stores it); bit 16: every token went where it guessed
    __shared__ int t_cluster[2][kInsertTokens], t_page[2][kInsertTokens], t_slot[2][kInsertTokens], t_src[2][kInsertTokens], t_pages[2];  // page_table
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, i = lane & 15;
    const int Cr = round_up(C, 16), Cs = insert_row_stride(C);
    char *stg = insert_lds + wave * stage_tiles * kInsertTileBytes;  // this wave's staging area (first in LDS: placed by preloaded arguments alone)
    const bf16_t *cb = cent + (size_t)u * Cpad * kD;
    const float *wn = cnorm + (size_t)u * Cpad;
    const bf16_t *ku = k + ((size_t)u * m_total + t0) * kD, *vu = v + ((size_t)u * m_total + t0) * kD;

    // ---- scan (the tile loads go out first; the small tables are staged while they are in flight)
    ICE_STAMP(32);
    const int tiles = Cr / 16;
    if (wave < tiles) {
        insert_stage_tile(cb, wave, stg, lane);
        if (stage_tiles == 2 && wave + kInsertWaves < tiles) insert_stage_tile(cb, wave + kInsertWaves, stg + kInsertTileBytes, lane);
    }
    bf16x8 ka[4];  // A operand: row i = token i, lane (g, i) holds its dims [32 ks + 8 g, +8)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {  // (a load under a condition, not a choice between two addresses: no zero constant in memory)
        uint4 w = make_uint4(0, 0, 0, 0);
        if (i < mt) w = ((const uint4 *)(ku + (size_t)i * kD))[ks * 4 + g];
        ka[ks] = __builtin_bit_cast(bf16x8, w);
    }
    // The other arguments are fetched here, once, while tiles and keys are on their way.
    const bool tk = tk_arg != 0;
    Dev d;
    bf16_t *caug_cur;
    pin_insert_fields(d, d_arg, cur, caug_cur);
    float *Dl = (float *)(insert_lds + kInsertWaves * stage_tiles * kInsertTileBytes);
    float *lw = Dl + (size_t)mt * Cs;
    float *lce = lw + Cr;
    uint32_t *lkey = (uint32_t *)(lce + (tk ? Cr : 0));
    uint32_t *lrow = lkey + kInsertTokens * 64;  // [t][64]: the bf16 row token t's move forms (a B operand is read back from it)
    float2 *s_cs = (float2 *)(lrow + kInsertTokens * 64);  // slot t: the guessed cluster's sum as it stands
    float2 *s_cs1 = s_cs + kInsertTokens * 64;             // ... and after token t's guessed move
    float2 *s_ps = s_cs1 + kInsertTokens * 64;             // ... and its tail page's sum before this launch
    uint32_t vw = 0;
    if (wave < mt) {
        lkey[wave * 64 + lane] = ((const uint32_t *)(ku + (size_t)wave * kD))[lane];
        vw = ((const uint32_t *)(vu + (size_t)wave * kD))[lane];
    }
    for (int r = tid; r < Cr; r += kInsertWaves * 64) {
        lw[r] = r < C ? wn[r] : INFINITY;
        if (tk) lce[r] = r < C ? bf16_to_f32(caug_cur[(size_t)u * Cpad + r]) : 0.f;
    }
    auto store_dots = [&](const f32x4 &acc, int tile) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * g + j < mt) Dl[(size_t)(4 * g + j) * Cs + tile * 16 + i] = acc[j];
    };
    for (int tile = wave; tile < tiles; tile += stage_tiles * kInsertWaves) {
        const int tb = tile + kInsertWaves;
        const bool two = stage_tiles == 2 && tb < tiles;
        if (tile != wave) {
            insert_stage_tile(cb, tile, stg, lane);
            if (two) insert_stage_tile(cb, tb, stg + kInsertTileBytes, lane);
        }
        wait_lds_dma();
        uint4 b0[4];
        insert_read_tile(stg, lane, b0);
        store_dots(insert_dots(ka, b0), tile);
        if (two) {
            uint4 b1[4];
            insert_read_tile(stg + kInsertTileBytes, lane, b1);
            store_dots(insert_dots(ka, b1), tb);
        }
    }
    const int np0 = d.n_pages[u], tok0 = d.n_tokens[u];
    ICE_STAMP(33);
    __syncthreads();
    ICE_STAMP(34);

    // nearest row for token t over all rows, from LDS
    auto nearest = [&](int t, float kaf) {
        u64 b = ~0ull;
        for (int c = lane; c < C; c += 64) {
            const float val = insert_objective(lw[c], Dl[(size_t)t * Cs + c], kaf, tk ? lce[c] : 0.f);
            if (!(val != val)) {
                const u64 key = insert_pack(val, c);
                b = key < b ? key : b;
            }
        }
        return wave_min_u64(b);
    };
    // the row a move forms against every token: lanes (g, 0) end with tokens 4g .. 4g+3
    auto row_dots = [&](const uint32_t *row) {
        uint4 bm[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bm[ks] = make_uint4(0, 0, 0, 0);
            if (i == 0) bm[ks] = ((const uint4 *)row)[ks * 4 + g];
        }
        return insert_dots(ka, bm);
    };

    // ---- guess
    ClusterMove mine = {};
    if (wave < mt) {
        const int t = wave;
        bf16_t kab = 0;
        if (tk) kab = key_extra_coordinate(d.c2[u], key_sqnorm16(((const uint4 *)(ku + (size_t)t * kD))[i]));
        const float kaf = bf16_to_f32(kab);
        u64 b = ~0ull, b2 = ~0ull;  // the nearest row and the runner-up
        for (int c = lane; c < C; c += 64) {
            const float val = insert_objective(lw[c], Dl[(size_t)t * Cs + c], kaf, tk ? lce[c] : 0.f);
            if (!(val != val)) merge_min2(b, b2, insert_pack(val, c), ~0ull);
        }
        wave_min2_u64(b, b2);
        const int p = insert_winner(b);
        const size_t cl = (size_t)u * d.C + p;
        const int cnt = d.cluster_cnt[cl];
        const float2 cs = ((const float2 *)(d.cluster_sum + cl * kD))[lane];
        const float es = tk ? d.csum_aug[cl] : 0.f;
        const int tail = d.cluster_tail[cl];
        const int fill = d.tail_fill[cl];
        const float2 ps = ((const float2 *)(d.tail_sum + cl * kD))[lane];
        mine = insert_move(cnt, cs, es, lkey[t * 64 + lane], kaf, tk);
        lrow[t * 64 + lane] = mine.packed;
        if (lane == 0) {
            s_best[t] = b;
            s_best2[t] = b2;
            s_cluster[t] = p;
            s_cnt[t] = cnt;
            s_es[t] = es;
            s_es1[t] = mine.es;
            s_tail[t] = tail;
            s_fill[t] = fill;
            s_kaf[t] = kaf;
            s_ka[t] = kab;
            s_nn[t] = mine.nn;
            s_ef[t] = mine.ef;
        }
        s_cs[t * 64 + lane] = cs;
        s_cs1[t * 64 + lane] = mine.cs;
        s_ps[t * 64 + lane] = ps;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        const f32x4 acc = row_dots(lrow + t * 64);
        if (i == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) s_dm[t][4 * g + j] = acc[j];
        }
    }
    ICE_STAMP(35);
    __syncthreads();
    ICE_STAMP(36);

    // ---- check, all pairs at once (wave t, the earlier tokens on its lanes): token t's guess fails against an
    // earlier token t' that moves as IT guessed if both guessed the same cluster or the row t' moves comes
    // out nearer to t than t's guess.  A token whose guess fails against no earlier move goes where it
    // guessed, with the move its wave worked out.
    if (wave < mt) {
        const int t = wave, lt = lane < mt ? lane : 0;
        const int p_l = s_cluster[lt];
        const float val = insert_objective(s_nn[lt], s_dm[lt][t], s_kaf[t], s_ef[lt]);
        const bool bad = lane < t && (p_l == s_cluster[t] || (!(val != val) && insert_pack(val, p_l) < s_best[t]));
        const u64 bads = __ballot(bad);
        if (lane == 0) s_fail[t] = (int)bads;
    }
    lds_barrier();

    // Where every token goes, token j on lane j: cj = its cluster, gj / tail_s / fill_s = what slot j
    // caches (the guessed cluster, its tail page and that page's fill before this launch).  Written to
    // table `buf` in LDS; one wave works it out.
    auto page_table = [&](int buf, int cj, int gj, int tail_s, int fill_s) {
        const int s = d.s;
        int src = -1;  // lowest slot that caches this token's cluster (-1: nobody guessed it)
        u64 equal = 0; // tokens of the same cluster
        for (int jj = 0; jj < mt; ++jj) {
            const int gjj = __builtin_amdgcn_readlane(gj, jj), cjj = __builtin_amdgcn_readlane(cj, jj);
            if (src < 0 && gjj == cj) src = jj;
            const u64 eq = __ballot(cjj == cj);
            if (lane == jj) equal = eq;
        }
        int tail0 = __shfl(tail_s, max(src, 0)), fill0 = __shfl(fill_s, max(src, 0));
        if (lane < mt && src < 0) {
            tail0 = d.cluster_tail[(size_t)u * d.C + cj];
            fill0 = d.tail_fill[(size_t)u * d.C + cj];
        }
        const int r = __popcll(equal & ((1ull << lane) - 1ull));  // tokens of the same cluster before this one
        const int q = fill0 + r;
        const bool onold = q < s;
        const int slot = onold ? q : (q - s) % s;
        const u64 openers = __ballot(lane < mt && !onold && slot == 0);
        u64 mm = equal;  // the token that opened this token's page: the (r - slot)-th of its cluster
        for (int x = 0; x < r - slot; ++x) mm &= mm - 1;
        const int opener = mm ? __ffsll((long long)mm) - 1 : lane;
        const int page = onold ? tail0 : np0 + __popcll(openers & ((1ull << opener) - 1ull));
        if (lane < mt) {
            t_cluster[buf][lane] = cj;
            t_page[buf][lane] = page;
            t_slot[buf][lane] = slot | (onold ? 1 << 30 : 0);
            t_src[buf][lane] = src;
        }
        if (lane == 0) t_pages[buf] = __popcll(openers);
    };

    if (wave == 1) {
        // while wave 0 settles: the table as it is if every token goes where it guessed
        const int lt = lane < mt ? lane : 0;
        const int gj = lane < mt ? s_cluster[lt] : -1 - lane;
        page_table(0, gj, gj, s_tail[lt], s_fill[lt]);
    }
    // ---- settle (wave 0; token j's entry lives on lane j)
    if (wave == 0) {
        const int lt = lane < mt ? lane : 0;
        const int r_guess = lane < mt ? s_cluster[lt] : -1 - lane;  // the cluster slot `lane` caches
        const int r_tail = s_tail[lt], r_fill = s_fill[lt];
        const u64 r_best = s_best[lt];
        const float r_kaf = s_kaf[lt];
        float r_nn = s_nn[lt], r_ef = s_ef[lt];  // of the row token `lane` moves (the guessed move until settled otherwise)
        int r_row = -1 - lane;                   // cluster token `lane` went to (set when it is settled)
        u64 live = 0;     // the latest move of its row
        u64 stood = 0;    // the guessed move stands (and no later token moved the cluster again): wave t stores it
        u64 post = 0;     // slot t's cluster is in the state AFTER token t's guessed move (s_cnt + 1, s_cs1, s_es1)
        u64 patched = 0;  // D and the norms hold this move
        bool all_guessed = true;
        const u64 r_best2 = s_best2[lt];
        const int r_fail = lane < mt ? s_fail[lt] : 0;  // against the guessed moves of earlier tokens
        u64 dfail = 0;                                  // tokens whose guess fails against a move settled here
        const u64 all = mt >= 64 ? ~0ull : (1ull << mt) - 1ull;
        int t = -1;
        for (;;) {
            // the next token whose guess does not stand, taking every token up to it as standing
            const u64 done = t < 0 ? 0ull : (2ull << t) - 1ull;  // tokens 0 .. t
            const u64 assumed = stood | (all & ~done);
            const bool bad = lane > t && lane < mt &&
                             ((((u64)(uint32_t)r_fail & assumed & ((1ull << lane) - 1ull)) != 0ull) || ((dfail >> lane) & 1ull));
            const u64 bads = __ballot(bad);
            const int next = bads ? __ffsll((long long)bads) - 1 : mt;
            const u64 run = ((1ull << next) - 1ull) & ~done;  // tokens t+1 .. next-1: settled as guessed
            stood |= run;
            post |= run;
            live |= run;
            if ((run >> lane) & 1ull) r_row = r_guess;
            if (next >= mt) break;
            t = next;
            const float kaf = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r_kaf), t));
            const u64 b1 = readlane_u64(r_best, t), b2 = readlane_u64(r_best2, t);
            const int p = insert_winner(b1);
            const bool is_live = (live >> lane) & 1ull;
            // fresh objectives of the rows moved so far
            u64 cand = ~0ull;
            if (is_live) {
                const float val = insert_objective(r_nn, s_dm[lt][t], kaf, r_ef);
                if (!(val != val)) cand = insert_pack(val, r_row);
            }
            cand = readlane_u64(row16_min_u64(cand), 0);
            const bool p_moved = __ballot(is_live && r_row == p) != 0ull;
            const bool p2_moved = b2 != ~0ull && __ballot(is_live && r_row == insert_winner(b2)) != 0ull;
            u64 b;
            if (!p_moved) {
                b = cand < b1 ? cand : b1;  // the guess still stands among the rows that have not moved
            } else if (!p2_moved) {
                b = cand < b2 ? cand : b2;  // ... or the runner-up does
            } else {
                // a full pass: D and the norms first catch up with the moves that are live
                for (u64 need = live & ~patched; need; need &= need - 1) {
                    const int j = __ffsll((long long)need) - 1;
                    const int row = __builtin_amdgcn_readlane(r_row, j);
                    if (lane >= t && lane < mt) Dl[(size_t)lane * Cs + row] = s_dm[j][lane];
                    if (lane == 0) {
                        lw[row] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r_nn), j));
                        if (tk) lce[row] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r_ef), j));
                    }
                }
                patched |= live;
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                b = nearest(t, kaf);
            }
            const int c = insert_winner(b);
            all_guessed = all_guessed && c == p;
            const u64 same_slot = __ballot(r_guess == c);  // slots that cache this cluster
            if (c == p && !p_moved) {
                // the guessed move stands after all: wave t stores it; slot t now stands for the state after it
                stood |= 1ull << t;
                post |= 1ull << t;
            } else {
                // (a move of this cluster that stood is superseded: everything it would store is stored here)
                stood &= ~__ballot(lane < t && r_row == c);
                const size_t cl = (size_t)u * d.C + c;
                int cnt;
                float2 cs;
                float es_old;
                if (same_slot & post) {
                    const int j = __ffsll((long long)(same_slot & post)) - 1;
                    cnt = s_cnt[j] + 1;
                    cs = s_cs1[j * 64 + lane];
                    es_old = s_es1[j];
                } else if (same_slot) {
                    const int j = __ffsll((long long)same_slot) - 1;
                    cnt = s_cnt[j];
                    cs = s_cs[j * 64 + lane];
                    es_old = s_es[j];
                } else {
                    cnt = d.cluster_cnt[cl];
                    cs = ((const float2 *)(d.cluster_sum + cl * kD))[lane];
                    es_old = tk ? d.csum_aug[cl] : 0.f;
                }
                const ClusterMove mv = insert_move(cnt, cs, es_old, lkey[t * 64 + lane], kaf, tk);
                insert_store_move(d, cent, cnorm, caug_cur, u, c, Cpad, lane, mv, tk);
                if (same_slot) {  // the lowest slot that caches this cluster holds its state from now on
                    const int j = __ffsll((long long)same_slot) - 1;
                    s_cs[j * 64 + lane] = mv.cs;
                    if (lane == 0) { s_cnt[j] = mv.cnt; s_es[j] = mv.es; }
                }
                post &= ~same_slot;
                if (lane == t) { r_nn = mv.nn; r_ef = mv.ef; }
                if (t + 1 < mt) {
                    lrow[t * 64 + lane] = mv.packed;
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    const f32x4 acc = row_dots(lrow + t * 64);
                    if (i == 0) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) s_dm[t][4 * g + j] = acc[j];
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                    // the later tokens against this move: same cluster guessed, or the moved row nearer than their guess
                    const float val = insert_objective(mv.nn, s_dm[t][lt], r_kaf, mv.ef);
                    dfail |= __ballot(lane > t && lane < mt && (r_guess == c || (!(val != val) && insert_pack(val, c) < r_best)));
                }
            }
            live &= ~__ballot(is_live && r_row == c);
            live |= 1ull << t;
            if (lane == t) r_row = c;
        }
        if (lane == 0) s_stood = (int)stood | (all_guessed ? 1 << 16 : 0);
        if (!all_guessed) page_table(1, r_row, r_guess, r_tail, r_fill);
    }
    ICE_STAMP(37);
    __syncthreads();
    ICE_STAMP(38);

    // ---- commit
    const int stood_all = s_stood;
    if (wave < mt && ((stood_all >> wave) & 1)) insert_store_move(d, cent, cnorm, caug_cur, u, s_cluster[wave], Cpad, lane, mine, tk);

    // ---- append
    ICE_STAMP(53);
    if (wave < mt) {
        const int s = d.s, t = wave, buf = (stood_all >> 16) & 1 ? 0 : 1;
        const int lt = lane < mt ? lane : 0;
        const int cj = lane < mt ? t_cluster[buf][lt] : -1 - lane, page = lane < mt ? t_page[buf][lt] : -1 - lane;
        const int c = t_cluster[buf][t], pg_t = t_page[buf][t], slot_t = t_slot[buf][t] & ~(1 << 30), src_t = t_src[buf][t];
        const bool onold_t = (t_slot[buf][t] >> 30) & 1;
        const size_t cl = (size_t)u * d.C + c;
        const size_t pg = (size_t)u * d.max_pages + pg_t;
        ((uint32_t *)(d.Kp + (pg * s + slot_t) * kD))[lane] = lkey[t * 64 + lane];
        ((uint32_t *)(d.Vp + (pg * s + slot_t) * kD))[lane] = vw;
        if (lane == 0) {
            d.page_pos[pg * s + slot_t] = tok0 + t;
            if (tk) d.kaug[(size_t)u * d.max_tokens + tok0 + t] = s_ka[t];
        }
        const u64 members = __ballot(page == pg_t);
        if ((members >> t) == 1ull) {  // the page's last token of this launch: its sum and representative
            float2 ps = make_float2(0.f, 0.f);
            // (the page's own sum when nobody cached it: the cluster's copy may already belong to a later page)
            if (onold_t) ps = src_t >= 0 ? s_ps[src_t * 64 + lane] : ((const float2 *)(d.page_sum + pg * kD))[lane];
            for (u64 hm = members; hm; hm &= hm - 1) {  // ascending token order, one add per key
                const uint32_t kwj = lkey[(__ffsll((long long)hm) - 1) * 64 + lane];
                ps.x = ps.x + bf16_lo(kwj);
                ps.y = ps.y + bf16_hi(kwj);
            }
            ((float2 *)(d.page_sum + pg * kD))[lane] = ps;
            const float ff = (float)(slot_t + 1);
            ((uint32_t *)(d.rep + pg * kD))[lane] = (uint32_t)f32_to_bf16(ps.x / ff) | ((uint32_t)f32_to_bf16(ps.y / ff) << 16);
            if (lane == 0) {
                d.page_fill[pg] = slot_t + 1;
                if (!onold_t) d.page_cluster[pg] = c;
            }
            const u64 same_cluster = __ballot(cj == c);
            if ((same_cluster >> t) == 1ull) {  // ... and the cluster's last: this page is its tail from now on
                ((float2 *)(d.tail_sum + cl * kD))[lane] = ps;
                if (lane == 0) {
                    d.cluster_tail[cl] = pg_t;
                    d.tail_fill[cl] = slot_t + 1;
                }
            }
        }
        if (t == 0 && lane == 0) {
            d.n_pages[u] = np0 + t_pages[buf];
            d.n_tokens[u] = tok0 + mt;
        }
    }
    ICE_STAMP(55);
}

void launch_insert(const Dev &d, const bf16_t *k, const bf16_t *v, int m, int cur, hipStream_t st) {
    // LDS of the batched kernel: the fixed tables, one staging tile per wave at least, a row of D per token
    const size_t budget = 156u * 1024u, stage1 = (size_t)kInsertWaves * kInsertTileBytes;
    const size_t fixed = insert_fixed_lds(d.C, d.tk != 0), row = (size_t)insert_row_stride(d.C) * 4;
    const int cap = (int)std::min<size_t>(kInsertTokens, (budget - fixed - stage1) / row);  // >= 1 up to 8192 clusters
    const size_t one_lds = 2 * stage1;
    for (int t0 = 0; t0 < m; t0 += std::max(cap, 1)) {
        const int mt = std::min(std::max(cap, 1), m - t0);
        if (mt == 1) {
            allow_dynamic_lds((const void *)insert_one_kernel, one_lds);
            hipLaunchKernelGGL(insert_one_kernel, dim3(d.U), dim3(kInsertWaves * 64), one_lds, st, k, v, d.cent_bf16[cur], d.cnorm[cur], m,
                               t0, cur, d.C, d.Cpad, d.tk, d);
            continue;
        }
        const int stage_tiles = fixed + mt * row + 2 * stage1 <= budget ? 2 : 1;
        const size_t lds = fixed + mt * row + stage_tiles * stage1;
        allow_dynamic_lds((const void *)insert_batch_kernel, lds);
        hipLaunchKernelGGL(insert_batch_kernel, dim3(d.U), dim3(kInsertWaves * 64), lds, st, k, v, d.cent_bf16[cur], d.cnorm[cur], m, t0,
                           mt, cur, d.C, d.Cpad, stage_tiles, d.tk, d);
    }
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
