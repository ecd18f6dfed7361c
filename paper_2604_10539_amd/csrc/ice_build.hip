// Index build at prefill: promotion of the initial centroids, nearest-centroid assignment on the
// matrix cores, deterministic per-cluster means, and the node -> page layout (Sec. 4.1-4.2,
// Alg. 2 of the paper restricted to two levels and iterated as Lloyd rounds).
#include <algorithm>

#include "ice_internal.h"

namespace ice {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned long long u64;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
// a.lo*b.lo + a.hi*b.hi + c on packed bf16 pairs, fp32 accumulate (v_dot2_f32_bf16)
__device__ inline float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

__device__ inline uint64_t splitmix64(uint64_t x) {
    x += 0x9E3779B97F4A7C15ull;
    x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
    x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
    return x ^ (x >> 31);
}

// ------------------------------------------------------------------------------------------------
// Transformed keys (Sec. 4.2, Eq. 2): T_K(k) = [k / c, sqrt(1 - ||k||^2 / c^2)] with c >= the largest
// key norm.  Distances are only compared, so everything is kept times c: the key itself plus ONE
// more coordinate a(k) = sqrt(c^2 - ||k||^2), stored as bf16 beside the keys; c^2 is the largest
// squared norm of the unit's prefill keys (a later key with a larger norm gets a(k) = 0).
// Pass 1: squared norms (16 lanes per key, fixed summation order) and their maximum per unit;
// pass 2: the extra coordinate.
__global__ __launch_bounds__(256) void key_norms_kernel(Dev d, const bf16_t *__restrict__ K, int n, float *n2_out) {
    // 256 keys per workgroup (16 at a time, 16 lanes each); one atomic maximum per wave
    const int u = blockIdx.y, row = threadIdx.x >> 4, ch = threadIdx.x & 15;
    float mx = 0.f;
    uint4 w[16];  // the workgroup's 64 KB of key rows are requested at once (read once: streaming loads)
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int i = blockIdx.x * 256 + it * 16 + row;
        w[it] = i < n ? load16_stream((const uint4 *)(K + ((size_t)u * n + i) * kD) + ch) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int it = 0; it < 16; ++it) {
        const int i = blockIdx.x * 256 + it * 16 + row;
        const float n2 = key_sqnorm16(w[it]);  // (uniform over the 16 lanes of a key: no divergent reduction)
        if (i < n) {
            if (ch == 0) n2_out[(size_t)u * d.max_tokens + i] = n2;
            mx = fmaxf(mx, n2);
        }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if ((threadIdx.x & 63) == 0) atomicMax((unsigned int *)d.c2 + u, __float_as_uint(mx));  // (non-negative floats order like their bits)
}
__global__ __launch_bounds__(256) void key_aug_kernel(Dev d, int n, const float *n2_in) {
    const int u = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) d.kaug[(size_t)u * d.max_tokens + i] = key_extra_coordinate(d.c2[u], n2_in[(size_t)u * d.max_tokens + i]);
}
__global__ void fill_f32_kernel(float *p, int n, float v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

void launch_key_aug(const Dev &d, const bf16_t *K, int n, hipStream_t st) {
    float *n2 = (float *)d.order;  // (free until the first sort)
    hipLaunchKernelGGL(fill_f32_kernel, dim3((d.U + 255) / 256), dim3(256), 0, st, d.c2, d.U, 0.f);
    hipLaunchKernelGGL(key_norms_kernel, dim3((n + 255) / 256, d.U), dim3(256), 0, st, d, K, n, n2);
    hipLaunchKernelGGL(key_aug_kernel, dim3((n + 255) / 256, d.U), dim3(256), 0, st, d, n, n2);
}

// ------------------------------------------------------------------------------------------------
// Initial centroids = the promoted keys (Alg. 2, "random promotion" with an exact count): cluster c
// of unit u starts at key init_idx[u][c], or, without a list, at a hashed position inside the c-th
// of C equal strata of the sequence (distinct by construction).  One wave per centroid row; rows
// >= C are padding (zero vector, infinite norm) in both centroid buffers.
__global__ __launch_bounds__(64) void init_centroids_kernel(Dev d, const bf16_t *K, int n,
                                                            const int *init_idx, uint64_t seed, int cur) {
    const int c = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
    uint32_t *cb0 = (uint32_t *)(d.cent_bf16[cur] + ((size_t)u * d.Cpad + c) * kD);
    uint32_t *cb1 = (uint32_t *)(d.cent_bf16[cur ^ 1] + ((size_t)u * d.Cpad + c) * kD);
    if (c >= d.C) {
        cb0[lane] = 0u;
        cb1[lane] = 0u;
        if (lane == 0) {
            d.cnorm[cur][(size_t)u * d.Cpad + c] = INFINITY;
            d.cnorm[cur ^ 1][(size_t)u * d.Cpad + c] = INFINITY;
            if (d.tk) d.caug[cur][(size_t)u * d.Cpad + c] = d.caug[cur ^ 1][(size_t)u * d.Cpad + c] = 0;
        }
        return;
    }
    int idx;
    if (init_idx) {
        idx = init_idx[(size_t)u * d.C + c];
        idx = idx < 0 ? 0 : (idx >= n ? n - 1 : idx);
    } else {
        long long lo = (long long)c * n / d.C, hi = (long long)(c + 1) * n / d.C;
        idx = (int)(lo + (long long)(splitmix64(seed ^ ((uint64_t)u << 32) ^ (uint64_t)c) % (uint64_t)(hi - lo)));
    }
    const uint32_t w = ((const uint32_t *)(K + ((size_t)u * n + idx) * kD))[lane];
    const float lo = bf16_lo(w), hi = bf16_hi(w);
    cb0[lane] = w;
    ((float2 *)(d.centroid + ((size_t)u * d.C + c) * kD))[lane] = make_float2(lo, hi);
    float nn = wave_sum(lo * lo + hi * hi);
    if (lane == 0) {
        if (d.tk) {  // the promoted key's extra coordinate
            const bf16_t a = d.kaug[(size_t)u * d.max_tokens + idx];
            const float af = bf16_to_f32(a);
            d.caug[cur][(size_t)u * d.Cpad + c] = a;
            d.cent_aug[(size_t)u * d.C + c] = af;
            nn += af * af;
        }
        d.cnorm[cur][(size_t)u * d.Cpad + c] = nn;
        d.init_idx[(size_t)u * d.C + c] = idx;
    }
}

void launch_init_centroids(const Dev &d, const bf16_t *K, int n, const int *init_idx, uint64_t seed, int cur,
                           hipStream_t st) {
    hipLaunchKernelGGL(init_centroids_kernel, dim3(d.Cpad, d.U), dim3(64), 0, st, d, K, n, init_idx, seed, cur);
}

// Caller-supplied bf16 centroids [U][C][128] -> live centroid buffer (padding + squared norms).
__global__ __launch_bounds__(64) void load_centroids_kernel(Dev d, const bf16_t *cent, int cur) {
    const int c = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
    uint32_t *cb = (uint32_t *)(d.cent_bf16[cur] + ((size_t)u * d.Cpad + c) * kD);
    if (c >= d.C) {
        cb[lane] = 0u;
        if (lane == 0) d.cnorm[cur][(size_t)u * d.Cpad + c] = INFINITY;
        return;
    }
    const uint32_t w = ((const uint32_t *)(cent + ((size_t)u * d.C + c) * kD))[lane];
    cb[lane] = w;
    const float lo = bf16_lo(w), hi = bf16_hi(w);
    const float nn = wave_sum(lo * lo + hi * hi);
    if (lane == 0) d.cnorm[cur][(size_t)u * d.Cpad + c] = nn;
}

void launch_load_centroids(const Dev &d, const bf16_t *cent, int cur, hipStream_t st) {
    hipLaunchKernelGGL(load_centroids_kernel, dim3(d.Cpad, d.U), dim3(64), 0, st, d, cent, cur);
}

// Recompute the bf16 rounding and squared norm of every centroid from the fp32 centroids.
__global__ __launch_bounds__(64) void refresh_centroids_kernel(Dev d, int cur) {
    const int c = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
    uint32_t *cb = (uint32_t *)(d.cent_bf16[cur] + ((size_t)u * d.Cpad + c) * kD);
    if (c >= d.C) {
        cb[lane] = 0u;
        if (lane == 0) d.cnorm[cur][(size_t)u * d.Cpad + c] = INFINITY;
        return;
    }
    const float2 m = ((const float2 *)(d.centroid + ((size_t)u * d.C + c) * kD))[lane];
    const bf16_t b0 = f32_to_bf16(m.x), b1 = f32_to_bf16(m.y);
    cb[lane] = (uint32_t)b0 | ((uint32_t)b1 << 16);
    const float lo = bf16_to_f32(b0), hi = bf16_to_f32(b1);
    const float nn = wave_sum(lo * lo + hi * hi);
    if (lane == 0) d.cnorm[cur][(size_t)u * d.Cpad + c] = nn;
}

void launch_refresh_centroids(const Dev &d, int cur, hipStream_t st) {
    hipLaunchKernelGGL(refresh_centroids_kernel, dim3(d.Cpad, d.U), dim3(64), 0, st, d, cur);
}

// The copy of every cluster's tail-page state that the insertions work on (fill and key sum).
__global__ __launch_bounds__(256) void refresh_tails_kernel(Dev d) {
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), u = blockIdx.y, lane = threadIdx.x & 63;
    if (c >= d.C) return;
    const size_t cl = (size_t)u * d.C + c;
    const int tail = d.cluster_tail[cl];
    float2 ps = make_float2(0.f, 0.f);
    int fill = d.s;
    if (tail >= 0) {
        const size_t pg = (size_t)u * d.max_pages + tail;
        fill = d.page_fill[pg];
        ps = ((const float2 *)(d.page_sum + pg * kD))[lane];
    }
    ((float2 *)(d.tail_sum + cl * kD))[lane] = ps;
    if (lane == 0) d.tail_fill[cl] = fill;
}
void launch_refresh_tails(const Dev &d, hipStream_t st) {
    hipLaunchKernelGGL(refresh_tails_kernel, dim3((d.C + 3) / 4, d.U), dim3(256), 0, st, d);
}

__global__ void fill_u64_kernel(u64 *p, size_t n, u64 v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

// ------------------------------------------------------------------------------------------------
// Nearest centroid on the matrix cores.
//   score(i, c) = k_i . mu~_c - ||mu~_c||^2 / 2      (argmax score == argmin ||k_i - mu~_c||^2)
// A dense (keys x 128) by (128 x centroids) contraction: v_mfma_f32_32x32x16_bf16 with the
// centroids as the A operand (rows) and the keys as the B operand (columns), so one lane ends up
// with 16 centroid scores of ONE key per 32x32 tile and the argmax over centroids stays in-lane.
// The accumulator is seeded with -||mu~||^2/2, so the epilogue is compare/select only.
//
// A workgroup of 8 waves covers CW * CT * 32 centroids (wave w keeps CT tiles of 32 centroids in
// registers for its whole life) and streams its share of the unit's keys through LDS in tiles of
// 256 keys (direct global -> LDS loads into unpadded rows whose 16-byte chunks are swizzled by row,
// so the 32-row operand reads are bank-conflict free).  When CW < 8 the remaining waves split the
// key tile instead.  Per key
// the waves' candidates meet in an LDS 64-bit max of (ordered score, ~centroid id): the exact fp32
// maximum with the lowest centroid id on ties.  More than CW*CT*32 centroids are covered by
// blockIdx.y slices that meet the same way in global memory.
//
// In-lane argmax over the 16 scores of one accumulator tile: a tournament with three entries per
// node.  The value of a node is one v_max3; its index follows by equality with that value, the
// first of the three entries winning ties (lowest element index), i.e. two v_cmp and two v_cndmask:
// 5 vector operations for every two entries removed, 38 per tile (a binary tournament of (value,
// index) pairs needs 45, and measured 2 % slower; carrying the index bits as lane masks on the
// scalar unit needs 30 vector + ~40 scalar operations and measured 5 % slower: what limits the
// kernel is the number of instructions a wave has to issue per MFMA).  The index comes out as the
// local centroid id 8 (v / 4) + v % 4 of element v.  Written level by level (all maxima, then all
// comparisons, then all selects) so that a comparison and the select that consumes its lane mask
// need not be adjacent.
__device__ inline float max3f(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }
__device__ inline void argmax16(const f32x16 &x, float &m, uint32_t &idx) {
    auto id = [](int v) { return (uint32_t)(8 * (v >> 2) + (v & 3)); };
    float t1[6], t2[2];
    uint32_t i1[6], i2[2];
    bool ea[5], eb[5];
#pragma unroll
    for (int p = 0; p < 5; ++p) t1[p] = max3f(x[3 * p], x[3 * p + 1], x[3 * p + 2]);
    t1[5] = x[15];
    t2[0] = max3f(t1[0], t1[1], t1[2]);
    t2[1] = max3f(t1[3], t1[4], t1[5]);
#pragma unroll
    for (int p = 0; p < 5; ++p) {
        ea[p] = x[3 * p] == t1[p];
        eb[p] = x[3 * p + 1] == t1[p];
    }
    const bool fa0 = t1[0] == t2[0], fb0 = t1[1] == t2[0], fa1 = t1[3] == t2[1], fb1 = t1[4] == t2[1];
    const bool g = t2[1] > t2[0];
#pragma unroll
    for (int p = 0; p < 5; ++p) {
        const uint32_t t = eb[p] ? id(3 * p + 1) : id(3 * p + 2);
        i1[p] = ea[p] ? id(3 * p) : t;
    }
    i1[5] = id(15);
    const uint32_t u0 = fb0 ? i1[1] : i1[2], u1 = fb1 ? i1[4] : i1[5];
    i2[0] = fa0 ? i1[0] : u0;
    i2[1] = fa1 ? i1[3] : u1;
    m = g ? t2[1] : t2[0];
    idx = g ? i2[1] : i2[0];
}
// LDS layout of a 256-row tile (keys, or the centroid block while it is staged): rows of 256 bytes
// without padding, the 16-byte chunk c of row r stored in slot c ^ (r & 15).  A fragment read (lane
// = row r, chunk 2 ks + half) then hits 16 different 16-byte bank groups per 16 lanes (measured: the
// full 160 B/clk/CU), and a wave can write four whole rows with ONE direct global -> LDS load (lane
// l lands at 16 l; it fetches chunk (l & 15) ^ (row & 15) of its row), so a key tile never passes
// through registers.  With the extra coordinate (transformed keys) each row has a 32-byte
// companion (the coordinate, then zeros: the two chunks of a ninth contraction step) in a
// separate array.
__host__ __device__ constexpr int assign_lds_bytes(bool aug) {
    return 2 * 256 * 256 + (aug ? 2 * 256 * 32 : 0) + 2 * 256 * 8;
}

template <int CT, int CW, bool AUG>
__global__ __launch_bounds__(512) void assign_kernel(const bf16_t *__restrict__ K, const bf16_t *__restrict__ cent,
                                                      const float *__restrict__ cnorm, int n, int keys_per_wg, int zsplit,
                                                      int Cpad, int cur, Dev d) {  // (scalars first: preloaded at wave start)
    constexpr int KW = 8 / CW;
    constexpr int KS = AUG ? 9 : 8;  // 16-wide steps of the contraction
    extern __shared__ __align__(16) char smem[];
    char *keys = smem;                                                // [2][256][256 B], chunks swizzled
    uint4 *kext = (uint4 *)(smem + 2 * kAssignTile * 256);            // (AUG) [2][256][2] companion chunks
    u64 *best = (u64 *)(smem + 2 * kAssignTile * 256 + (AUG ? 2 * kAssignTile * 32 : 0));  // [2][256]
    // byte offset of chunk c of row r inside a buffer
    auto slot = [](int r, int c) { return r * 256 + ((c ^ (r & 15)) << 4); };

    const int u = blockIdx.z, tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, col = lane & 31, half = lane >> 5;
    const int cw = wave % CW, kw = wave / CW;
    const int cbase = (blockIdx.y * CW + cw) * CT * 32;
    const int k0 = blockIdx.x * keys_per_wg;
    const int kend = min(n, k0 + keys_per_wg);
    const int ntiles = (kend - k0 + kAssignTile - 1) / kAssignTile;
    const bf16_t *Ku = K + (size_t)u * n * kD;

    ICE_BSTAMP(0);
    // Prologue.  The workgroup's block of centroid rows goes to LDS with fully coalesced 16-byte
    // loads (the staging area is the key buffers, not yet in use) and every wave then picks its
    // MFMA fragments from there: reading the fragments straight from global memory touches 32
    // separate rows per load instruction.  The first key tile is in flight meanwhile.
    constexpr int R = CW * CT * 32;  // centroid rows of this workgroup
    const int crow0 = blockIdx.y * R;
    uint4 cst[R / 32];
    {
        const bf16_t *csrc = cent + ((size_t)u * Cpad + crow0) * kD;
#pragma unroll
        for (int i = 0; i < R / 32; ++i) {
            const int id = tid + 512 * i, row = id >> 4, ch = id & 15;
            cst[i] = crow0 + row < Cpad ? ((const uint4 *)(csrc + (size_t)row * kD))[ch] : make_uint4(0, 0, 0, 0);
        }
    }
    // accumulator seeds -||mu~||^2 / 2 (rows past Cpad: -inf), resident for the whole kernel: element v
    // of a lane of half h belongs to local centroid 8 (v / 4) + 4 h + v % 4 of its tile
    f32x16 seed[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int row0 = cbase + ct * 32;
        if (row0 < Cpad) {
            const float *wn = cnorm + (size_t)u * Cpad + row0;
#pragma unroll
            for (int v = 0; v < 16; ++v) seed[ct][v] = -0.5f * wn[8 * (v >> 2) + 4 * half + (v & 3)];
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) seed[ct][v] = -INFINITY;
        }
    }

    // The first key tile travels through registers (it is requested before the centroid block is
    // staged in the very buffers it goes to); every later tile goes straight to LDS.
    uint32_t stage_aug = 0;  // (AUG) extra coordinate of key `tid` of the next tile, threads 0..255
    auto load_aug = [&](int t) {
        if constexpr (AUG) {
            const int key = k0 + t * kAssignTile + tid;
            stage_aug = tid < kAssignTile && key < kend ? d.kaug[(size_t)u * d.max_tokens + key] : 0u;
        }
    };
    auto store_aug = [&](int buf) {
        if constexpr (AUG) {
            if (tid < kAssignTile) {
                kext[(buf * kAssignTile + tid) * 2] = make_uint4(stage_aug, 0, 0, 0);
                kext[(buf * kAssignTile + tid) * 2 + 1] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    // rows past the end of the range are never written back: they may hold any valid key
    auto request_tile = [&](int t, int buf) {
        const int base = k0 + t * kAssignTile;
        const int ch = tid & 15, r16 = (tid >> 4) & 15;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = (tid >> 4) + 32 * i;
            const int key = min(base + row, kend - 1);
            const uint4 *src = (const uint4 *)(Ku + (size_t)key * kD) + (ch ^ r16);
            char *dst = keys + buf * (kAssignTile * 256) + (4 * wave + 32 * i) * 256;  // this wave's four rows
            lds_dma16(src, dst);
        }
    };
    u32x4 first[8];  // (the grid leaves no workgroup without keys: ntiles >= 1)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int id = tid + 512 * i, row = id >> 4, ch = id & 15;
        const int key = min(k0 + row, kend - 1);
        first[i] = ((const u32x4 *)(Ku + (size_t)key * kD))[ch];
    }
    load_aug(0);
#pragma unroll
    for (int i = 0; i < R / 32; ++i) {
        const int id = tid + 512 * i, row = id >> 4, ch = id & 15;
        *(uint4 *)(keys + slot(row, ch)) = cst[i];
    }
    if constexpr (AUG) {
        if (tid < R) {  // the centroids' extra coordinate, then 15 zeros
            const uint32_t a = crow0 + tid < Cpad ? d.caug[cur][(size_t)u * Cpad + crow0 + tid] : 0u;
            kext[tid * 2] = make_uint4(a, 0, 0, 0);
            kext[tid * 2 + 1] = make_uint4(0, 0, 0, 0);
        }
    }
    if (tid < 2 * kAssignTile) best[tid] = 0ull;
    __syncthreads();
    // centroid operand, resident for the whole kernel
    bf16x8 A[CT][KS];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        const int r = (cw * CT + ct) * 32 + col;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) A[ct][ks] = __builtin_bit_cast(bf16x8, *(const uint4 *)(keys + slot(r, 2 * ks + half)));
        if constexpr (AUG) A[ct][8] = __builtin_bit_cast(bf16x8, kext[r * 2 + half]);
    }
    __syncthreads();  // every wave holds its fragments before the first key tile overwrites them
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int id = tid + 512 * i, row = id >> 4, ch = id & 15;
        *(u32x4 *)(keys + slot(row, ch)) = first[i];
    }
    store_aug(0);
    __syncthreads();
    // byte address of this lane's fragment chunk ks in row `col` of buffer 0; sub-tiles and the
    // other buffer are constant offsets from it
    uint32_t frag[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) frag[ks] = (uint32_t)slot(col, 2 * ks + half);
    ICE_BSTAMP(1);

    constexpr int NSUB = 8 / KW;  // 32-key sub-tiles of this wave per tile
    const uint32_t inv_cid0 = 0xFFFFFFFFu - (uint32_t)(cbase + 4 * half);  // low word for local centroid id 0
    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        u64 *bestt = best + buf * kAssignTile;
        ICE_WSTAMP(t, 0);
        if (t + 1 < ntiles) {
            request_tile(t + 1, buf ^ 1);
            load_aug(t + 1);
        }
        // Software pipeline over "slots" j = (sub-tile i, centroid tile ct): while the matrix cores
        // run the 8-MFMA chain of slot j+1 into one accumulator set, the vector unit
        // reduces slot j's 16 scores per lane from the other set (argmax16).  The key operand of a
        // sub-tile is read from LDS one sub-tile ahead.
        constexpr int NSLOT = NSUB * CT;
        bf16x8 B[2][KS];
        auto load_b = [&](int i, bf16x8 (&dst)[KS]) {
            const char *sub = keys + buf * (kAssignTile * 256) + (kw + i * KW) * 32 * 256;  // (32 rows: r & 15 is col & 15)
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) dst[ks] = __builtin_bit_cast(bf16x8, *(const uint4 *)(sub + frag[ks]));
            if constexpr (AUG) dst[8] = __builtin_bit_cast(bf16x8, kext[(buf * kAssignTile + (kw + i * KW) * 32 + col) * 2 + half]);
        };
        f32x16 acc[2];
        auto chain = [&](int j, f32x16 &dst) {
            const int i = j / CT, ct = j % CT;
            dst = seed[ct];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                dst = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[ct][ks], B[i & 1][ks], dst, 0, 0, 0);
        };
        load_b(0, B[0]);
        if (CT == 1 && NSUB > 1) load_b(1, B[1]);
        chain(0, acc[0]);
        float sv = 0.f;
        uint32_t sidx = 0;
#pragma unroll
        for (int j = 0; j < NSLOT; ++j) {
            const int i = j / CT, ct = j % CT;
            // LDS reads for the sub-tile whose first chain is issued in the NEXT iteration
            if ((j + 2) % CT == 0 && (j + 2) / CT < NSUB && (j + 2) / CT >= 1 && !(CT == 1 && j + 2 == 1))
                load_b((j + 2) / CT, B[((j + 2) / CT) & 1]);
            if (j + 1 < NSLOT) chain(j + 1, acc[(j + 1) & 1]);
            // element v of this lane has local centroid id ct*32 + 8*(v/4) + v%4 (+ 4*half), ascending in v
            float m;
            uint32_t li;
            argmax16(acc[j & 1], m, li);
            if (ct == 0) {
                sv = m;
                sidx = li;
            } else {
                const bool gt = m > sv;
                sv = gt ? m : sv;
                sidx = gt ? li + 32u * ct : sidx;
            }
            if (ct == CT - 1) {
                const u64 pk = ((u64)f32_ordered(sv + 0.0f) << 32) | (u64)(inv_cid0 - sidx);
                atomicMax(&bestt[(kw + i * KW) * 32 + col], pk);
            }
        }
        ICE_BSTAMP(2 + 2 * (t & 3));
        ICE_WSTAMP(t, 1);
        if (t + 1 < ntiles) {
            store_aug(buf ^ 1);
            wait_lds_dma();  // this wave's share of the next tile is in LDS
        }
        ICE_WSTAMP(t, 2);
        __syncthreads();
        ICE_WSTAMP(t, 3);
        ICE_BSTAMP(3 + 2 * (t & 3));
        // the per-key winners of this tile leave through the first 256 threads; the other buffer
        // collects the next tile meanwhile, and this one is not touched again before the barrier
        // of the next tile
        if (tid < kAssignTile) {
            const int key = k0 + t * kAssignTile + tid;
            if (key < kend) {
                u64 *dst = d.packed + (size_t)u * d.max_tokens + key;
                if (zsplit == 1) *dst = bestt[tid];
                else atomicMax(dst, bestt[tid]);
            }
            bestt[tid] = 0ull;
        }
    }
}

void launch_assign(const Dev &d, const bf16_t *K, int n, int cur, hipStream_t st) {
    const int tiles = d.Cpad / 32;
    int CT = tiles == 1 ? 1 : 2, CW = 1;
    while (CW < 8 && CW * CT < tiles) CW *= 2;
    const int cblock = CT * CW * 32;
    const int zsplit = (d.Cpad + cblock - 1) / cblock;
    // One workgroup per CU when the work allows it (a workgroup fills a CU: 132-148 KB of LDS, 8 waves
    // of 226-256 registers), each amortising its prologue over as many key tiles as possible.
    int keys_per_wg = kAssignTile;
    const int wg_target = 256;
    while ((long long)((n + keys_per_wg - 1) / keys_per_wg) * zsplit * d.U > wg_target && keys_per_wg < n) keys_per_wg *= 2;
    dim3 grid((n + keys_per_wg - 1) / keys_per_wg, zsplit, d.U);
    const size_t lds = assign_lds_bytes(d.tk != 0);
    if (zsplit > 1) {
        const size_t tot = (size_t)d.U * d.max_tokens;
        hipLaunchKernelGGL(fill_u64_kernel, dim3(1024), dim3(256), 0, st, d.packed, tot, 0ull);
    }
#define ICE_ASSIGN_A(ct, cw, aug)                                                                   \
    do {                                                                                            \
        allow_dynamic_lds((const void *)assign_kernel<ct, cw, aug>, lds);                           \
        hipLaunchKernelGGL((assign_kernel<ct, cw, aug>), grid, dim3(512), lds, st, K, d.cent_bf16[cur], d.cnorm[cur], n, keys_per_wg, \
                           zsplit, d.Cpad, cur, d);                                                 \
    } while (0)
#define ICE_ASSIGN(ct, cw)                                                                          \
    do {                                                                                            \
        if (d.tk) ICE_ASSIGN_A(ct, cw, true);                                                       \
        else ICE_ASSIGN_A(ct, cw, false);                                                           \
    } while (0)
    if (CT == 1) ICE_ASSIGN(1, 1);
    else if (CW == 1) ICE_ASSIGN(2, 1);
    else if (CW == 2) ICE_ASSIGN(2, 2);
    else if (CW == 4) ICE_ASSIGN(2, 4);
    else ICE_ASSIGN(2, 8);
#undef ICE_ASSIGN
#undef ICE_ASSIGN_A
}

// ------------------------------------------------------------------------------------------------
// Stable counting sort of the tokens by cluster (ascending position inside a cluster): the order
// both the deterministic means and the page layout need.  A unit's tokens are cut into R ranges,
// one workgroup of 16 waves each (R = 1 once there are 256 units; with fewer units more workgroups
// per unit keep the chip busy), all counters in LDS.  With R > 1 a first kernel leaves every
// range's member count per cluster in global memory (sort_totals_kernel).  The sorting kernel
// cuts its range into W segments of `seg` tokens (a multiple of 64), wave w owns segment w:
//   count  the wave unpacks its tokens' winners (and writes the assignment) and bumps
//          cnt[w][cluster]; with REG (a segment has at most 32 groups of 64 tokens) the cluster
//          ids stay in registers for the last phase;
//   scan   per cluster an exclusive scan over the earlier ranges (their totals) and over the
//          segments, then over the clusters (member counts and page counts of the whole unit),
//          which turns cnt[w][c] into the first output slot of segment w's members of cluster c
//          and yields the cluster and page offsets (written by the workgroup of range 0);
//   rank   the wave walks its segment in token order, 64 tokens at a time: lanes with the same
//          cluster find each other through a lane mask per cluster, the first of them moves the
//          cluster's cursor past all of them.
// A segment and cluster take 12 bytes of LDS (counter + lane mask): W = min(16, 12288 / Cpad)
// segments fit in 144 KB.
__global__ __launch_bounds__(1024) void sort_totals_kernel(Dev d, int n, int range_len) {
    extern __shared__ int tot[];  // [Cpad]
    const int r = blockIdx.x, u = blockIdx.y, tid = threadIdx.x;
    const int Cpad = d.Cpad;
    const uint32_t *pk = (const uint32_t *)(d.packed + (size_t)u * d.max_tokens);
    const int rb = r * range_len, re = min(n, rb + range_len);
    uint32_t v[4];  // (the first 4096 tokens are in flight while the counters are cleared)
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = rb + j * 1024 + tid < re ? pk[2 * (rb + j * 1024 + tid)] : 0u;
    for (int c = tid; c < Cpad; c += 1024) tot[c] = 0;
    __syncthreads();
    for (int i0 = rb; i0 < re; i0 += 4096) {
        if (i0 > rb) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = i0 + j * 1024 + tid < re ? pk[2 * (i0 + j * 1024 + tid)] : 0u;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i0 + j * 1024 + tid < re) atomicAdd(&tot[(int)min(0xFFFFFFFFu - v[j], (uint32_t)Cpad - 1u)], 1);
    }
    __syncthreads();
    int *out = d.range_tot + ((size_t)u * gridDim.x + r) * Cpad;
    for (int c = tid; c < Cpad; c += 1024) out[c] = tot[c];
}

constexpr int kSortRegGroups = 32;

template <bool REG>
__global__ __launch_bounds__(1024) void sort_unit_kernel(Dev d, int n, int range_len, int W, int seg, float *best_out,
                                                         int *assign_out) {
    extern __shared__ __align__(8) int cnt[];  // [W][Cpad] counters, then [W][Cpad] 64-bit lane masks
    __shared__ int wsum[2][16];
    __shared__ int carry[2];
    const int r = blockIdx.x, R = gridDim.x, u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Cpad = d.Cpad;
    const int rb = r * range_len, re = min(n, rb + range_len);  // this workgroup's tokens
    // low word of a packed winner = ~cluster id (the high word, the score, is read only for best_out)
    const uint32_t *pk = (const uint32_t *)(d.packed + (size_t)u * d.max_tokens);
    const int beg = min(re, rb + wave * seg), end = wave < W ? min(re, beg + seg) : beg;  // this wave's tokens
    // the winners of the first groups are in flight while the counters are cleared
    constexpr int NB = REG ? kSortRegGroups : 16;  // groups per batch of loads
    uint32_t v[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int i = beg + j * 64 + lane;
        v[j] = i < end ? pk[2 * i] : 0u;
    }
    u64 *mask_all = (u64 *)(cnt + W * Cpad);  // [W][Cpad] lane masks of the rank phase
    for (int x = tid; x < W * Cpad; x += 1024) { cnt[x] = 0; mask_all[x] = 0ull; }
    if (tid < 2) carry[tid] = 0;
    __syncthreads();
    int *pos = cnt + (wave < W ? wave : 0) * Cpad;
    u64 *mask = mask_all + (size_t)(wave < W ? wave : 0) * Cpad;
    // cluster id of a packed winner (always < Cpad for finite keys; clamped so that no input can
    // send a counter update or an output slot out of range)
    auto cluster_of = [&](uint32_t w) { return (int)min(0xFFFFFFFFu - w, (uint32_t)Cpad - 1u); };
    auto count_one = [&](int i, uint32_t w) {
        const int a = cluster_of(w);
        d.assign[(size_t)u * d.max_tokens + i] = a;
        if (assign_out) assign_out[(size_t)u * n + i] = a;
        if (best_out) best_out[(size_t)u * n + i] = -2.0f * ordered_f32(pk[2 * i + 1]);
        atomicAdd(&pos[a], 1);
        return a;
    };
    int areg[REG ? kSortRegGroups : 1];
    // ---- count
    if constexpr (REG) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const int i = beg + j * 64 + lane;
            areg[j] = i < end ? count_one(i, v[j]) : 0;
        }
    } else {
        for (int g0 = beg; g0 < end; g0 += NB * 64) {
            if (g0 > beg) {
#pragma unroll
                for (int j = 0; j < NB; ++j) {
                    const int i = g0 + j * 64 + lane;
                    v[j] = i < end ? pk[2 * i] : 0u;
                }
            }
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int i = g0 + j * 64 + lane;
                if (i < end) count_one(i, v[j]);
            }
        }
    }
    __syncthreads();
    // ---- scan
    const int *rtot = d.range_tot + (size_t)u * R * Cpad;
    for (int c0 = 0; c0 < Cpad; c0 += 1024) {
        const int c = c0 + tid;
        int own = 0, before = 0, tot = 0;
        if (c < Cpad) {
            for (int w = 0; w < W; ++w) {
                const int t = cnt[w * Cpad + c];
                cnt[w * Cpad + c] = own;
                own += t;
            }
            tot = own;
            if (R > 1) {
                tot = 0;
                for (int q0 = 0; q0 < R; q0 += 32) {  // 32 counts in flight per round trip
                    int t[32];
#pragma unroll
                    for (int j = 0; j < 32; ++j) t[j] = q0 + j < R ? rtot[(size_t)(q0 + j) * Cpad + c] : 0;
#pragma unroll
                    for (int j = 0; j < 32; ++j) {
                        if (q0 + j < r) before += t[j];
                        tot += t[j];
                    }
                }
            }
        }
        const int pages = (tot + d.s - 1) / d.s;
        int a = tot, b = pages;  // inclusive wave scans of (tot, pages)
        for (int off = 1; off < 64; off <<= 1) {
            const int ta = __shfl_up(a, off), tb = __shfl_up(b, off);
            if (lane >= off) { a += ta; b += tb; }
        }
        if (lane == 63) { wsum[0][wave] = a; wsum[1][wave] = b; }
        __syncthreads();
        int pa = carry[0], pb = carry[1];
        for (int w = 0; w < wave; ++w) { pa += wsum[0][w]; pb += wsum[1][w]; }
        const int ex_a = pa + a - tot, ex_b = pb + b - pages;
        if (c < Cpad) {
            for (int w = 0; w < W; ++w) cnt[w * Cpad + c] += ex_a + before;
            if (r == 0) {
                d.cluster_start[(size_t)u * (Cpad + 1) + c] = ex_a;
                d.page_base[(size_t)u * (Cpad + 1) + c] = ex_b;
                if (c < d.C) {
                    d.cluster_cnt[(size_t)u * d.C + c] = tot;
                    d.cluster_tail[(size_t)u * d.C + c] = tot > 0 ? ex_b + pages - 1 : -1;
                }
            }
        }
        __syncthreads();
        if (tid == 1023) { carry[0] = pa + a; carry[1] = pb + b; }
        __syncthreads();
    }
    if (tid == 0 && r == 0) {
        d.cluster_start[(size_t)u * (Cpad + 1) + Cpad] = carry[0];
        d.page_base[(size_t)u * (Cpad + 1) + Cpad] = carry[1];
        d.n_pages[u] = carry[1];
    }
    // ---- rank (row `wave` of the counters is touched by this wave only from here on)
    int *order = d.order + (size_t)u * d.max_tokens;
    const u64 lt = (1ull << lane) - 1ull;
    // Lanes of one group with the same cluster find each other through a 64-bit lane mask per
    // cluster in LDS (a table of this wave's own): every lane ORs its bit into its cluster's entry,
    // reads the entry back and clears it.  The LDS unit executes one wave's instructions in order,
    // so the three steps need no wait between them, only their program order.
    auto rank_group = [&](int i, int a) {
        const bool valid = i < end;
        u64 peers = 0ull;
        int base = 0;
        if (valid) atomicOr(&mask[a], 1ull << lane);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (valid) { peers = mask[a]; base = pos[a]; }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        if (valid) {
            mask[a] = 0ull;
            if ((peers & lt) == 0ull) pos[a] = base + (int)__popcll(peers);  // the first of them moves the cursor
            order[base + (int)__popcll(peers & lt)] = i;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    };
    if constexpr (REG) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if (beg + j * 64 >= end) break;  // (wave-uniform)
            rank_group(beg + j * 64 + lane, areg[j]);
        }
    } else {
        for (int g0 = beg; g0 < end; g0 += NB * 64) {
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const int i = g0 + j * 64 + lane;
                v[j] = i < end ? pk[2 * i] : 0u;  // (read again; nothing written above is read back)
            }
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                if (g0 + j * 64 >= end) break;  // (wave-uniform)
                rank_group(g0 + j * 64 + lane, cluster_of(v[j]));
            }
        }
    }
}

// ranges per unit of the sort: enough workgroups for the chip, at least 1024 tokens each
int sort_ranges(int U, int n, int *range_len) {
    int R = std::max(1, std::min(256 / std::max(U, 1), (n + 1023) / 1024));
    *range_len = round_up((n + R - 1) / R, 64);
    return (n + *range_len - 1) / *range_len;
}

void launch_sort(const Dev &d, int n, float *best_out, int *assign_out, hipStream_t st) {
    int range_len;
    const int R = sort_ranges(d.U, n, &range_len);
    const int W = d.Cpad <= 768 ? 16 : 12288 / d.Cpad;  // (12 bytes per segment and cluster in 144 KB; Cpad <= 8192: W >= 1)
    const int seg = round_up((range_len + W - 1) / W, 64);
    const size_t lds = (size_t)W * d.Cpad * 12;
    if (R > 1)
        hipLaunchKernelGGL(sort_totals_kernel, dim3(R, d.U), dim3(1024), (size_t)d.Cpad * sizeof(int), st, d, n, range_len);
    if (seg <= kSortRegGroups * 64) {
        allow_dynamic_lds((const void *)sort_unit_kernel<true>, lds);
        hipLaunchKernelGGL(sort_unit_kernel<true>, dim3(R, d.U), dim3(1024), lds, st, d, n, range_len, W, seg, best_out, assign_out);
    } else {
        allow_dynamic_lds((const void *)sort_unit_kernel<false>, lds);
        hipLaunchKernelGGL(sort_unit_kernel<false>, dim3(R, d.U), dim3(1024), lds, st, d, n, range_len, W, seg, best_out, assign_out);
    }
}
// The key rows of one clustering pass are read by assign, then by means (and once more by paginate).
// While they fit the chip's last-level cache (256 MB) the second reader finds them there; beyond
// that every pass streams from HBM, and the non-temporal hint is what gets the most out of it.
static bool keys_exceed_cache(const Dev &d, int n) { return (size_t)d.U * (size_t)n * kD * sizeof(bf16_t) >= ((size_t)256 << 20); }

// ------------------------------------------------------------------------------------------------
// Centroid update: one workgroup of four waves per cluster.  Wave w gathers the w-th quarter of the
// cluster's members in sorted order (key rows of 256 contiguous bytes, 16 lanes x 16 bytes, four
// rows per load) and sums them in fp32 in a fixed order; the four partial sums meet in LDS and are
// added in wave order, so the result is the same on every run (no floating-point atomics) and a
// large cluster costs a quarter of the dependent round trips.  Writes sum, count, mean, and the
// bf16 rounding + squared norm of the mean into the OTHER centroid buffer; an empty cluster keeps
// its centroid.
template <bool STREAM>
__global__ __launch_bounds__(256) void means_kernel(Dev d, const bf16_t *__restrict__ K, int n, int cur) {
    __shared__ float4 part_sum[3][16][2];
    const int u = blockIdx.y, c = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane >> 4, ch = lane & 15;
    const int start = d.cluster_start[(size_t)u * (d.Cpad + 1) + c];
    const int cnt = d.cluster_start[(size_t)u * (d.Cpad + 1) + c + 1] - start;
    const int *ord = d.order + (size_t)u * d.max_tokens + start;
    const bf16_t *Ku = K + (size_t)u * n * kD;
    const int quarter = (cnt + 3) / 4;
    const int lo = min(cnt, wave * quarter), hi = min(cnt, lo + quarter);
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
    // Group g of a wave sums rows g, g+4, g+8, ... of the wave's range in that order.  The member
    // list is read 64 entries at a time (one per lane) and the rows are fetched eight per group at
    // once, so a wave keeps 8 KB of key rows in flight instead of one dependent load pair per step.
    for (int base = lo; base < hi; base += 64) {
        const int mine = base + lane < hi ? ord[base + lane] : -1;
        const int rows = min(64, hi - base);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            if (h * 32 >= rows) break;
            uint4 w[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int tok = __shfl(mine, 4 * (h * 8 + k) + g);
                w[k] = tok >= 0 ? load16<STREAM>((const uint4 *)(Ku + (size_t)tok * kD) + ch) : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {  // rows past the end add +0
                acc[0] += bf16_lo(w[k].x); acc[1] += bf16_hi(w[k].x);
                acc[2] += bf16_lo(w[k].y); acc[3] += bf16_hi(w[k].y);
                acc[4] += bf16_lo(w[k].z); acc[5] += bf16_hi(w[k].z);
                acc[6] += bf16_lo(w[k].w); acc[7] += bf16_hi(w[k].w);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        acc[j] += __shfl_xor(acc[j], 16);
        acc[j] += __shfl_xor(acc[j], 32);
    }
    // (transformed keys) sum of the members' extra coordinates: lane-strided partial sums in member
    // order by the first wave, requested before the waves meet
    float aug_part = 0.f;
    if (d.tk && wave == 0)
        for (int r = lane; r < cnt; r += 64) aug_part += bf16_to_f32(d.kaug[(size_t)u * d.max_tokens + ord[r]]);
    if (wave > 0 && g == 0) {
        part_sum[wave - 1][ch][0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        part_sum[wave - 1][ch][1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w) {
        const float4 p0 = part_sum[w][ch][0], p1 = part_sum[w][ch][1];
        acc[0] += p0.x; acc[1] += p0.y; acc[2] += p0.z; acc[3] += p0.w;
        acc[4] += p1.x; acc[5] += p1.y; acc[6] += p1.z; acc[7] += p1.w;
    }
    float mu[8];
    float *cen = d.centroid + ((size_t)u * d.C + c) * kD + ch * 8;
    if (cnt > 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) mu[j] = acc[j] / (float)cnt;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) mu[j] = cen[j];
    }
    uint32_t pk[4];
    float nn = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const bf16_t b0 = f32_to_bf16(mu[2 * j]), b1 = f32_to_bf16(mu[2 * j + 1]);
        pk[j] = (uint32_t)b0 | ((uint32_t)b1 << 16);
        const float f0 = bf16_to_f32(b0), f1 = bf16_to_f32(b1);
        nn += f0 * f0 + f1 * f1;
    }
    nn = row16_sum(nn);
    if (d.tk) {
        // the centroid's extra coordinate: mean of the members' extra coordinates (the fixed wave
        // reduction of the partial sums above)
        const float asum = wave_sum(aug_part);
        const float e = cnt > 0 ? asum / (float)cnt : d.cent_aug[(size_t)u * d.C + c];
        const bf16_t eb = f32_to_bf16(e);
        const float ef = bf16_to_f32(eb);
        if (lane == 0) {
            d.csum_aug[(size_t)u * d.C + c] = asum;
            d.cent_aug[(size_t)u * d.C + c] = e;
            d.caug[cur ^ 1][(size_t)u * d.Cpad + c] = eb;
        }
        nn += ef * ef;
    }
    if (g == 0) {
        float *sum = d.cluster_sum + ((size_t)u * d.C + c) * kD + ch * 8;
        ((float4 *)sum)[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        ((float4 *)sum)[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        ((float4 *)cen)[0] = make_float4(mu[0], mu[1], mu[2], mu[3]);
        ((float4 *)cen)[1] = make_float4(mu[4], mu[5], mu[6], mu[7]);
        ((uint4 *)(d.cent_bf16[cur ^ 1] + ((size_t)u * d.Cpad + c) * kD))[ch] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        if (ch == 0) d.cnorm[cur ^ 1][(size_t)u * d.Cpad + c] = nn;
    }
}

void launch_means(const Dev &d, const bf16_t *K, int n, int cur, hipStream_t st) {
    if (keys_exceed_cache(d, n)) hipLaunchKernelGGL(means_kernel<true>, dim3(d.C, d.U), dim3(256), 0, st, d, K, n, cur);
    else hipLaunchKernelGGL(means_kernel<false>, dim3(d.C, d.U), dim3(256), 0, st, d, K, n, cur);
}

// ------------------------------------------------------------------------------------------------
// Node -> pages (Sec. 4.1): clusters in id order, members in ascending position, cut every s
// tokens; consecutive page ids.  One wave per page copies the s key rows and s value rows into
// the page's contiguous tiles, records their positions, and forms the representative: the fp32
// sum of the page's keys in slot order (one add per slot), divided by the fill, rounded to bf16.
template <bool STREAM>
__global__ __launch_bounds__(256) void paginate_kernel(Dev d, const bf16_t *__restrict__ K,
                                                        const bf16_t *__restrict__ V, int n) {
    extern __shared__ __align__(16) char smem[];  // [4][s][128] bf16
    const int u = blockIdx.y, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + wave;
    if (p >= d.max_pages) return;
    const int s = d.s;
    const size_t pg = (size_t)u * d.max_pages + p;
    const int np = d.n_pages[u];
    if (p >= np) {  // unused page: clear its table entries
        if (lane == 0) { d.page_cluster[pg] = -1; d.page_fill[pg] = 0; }
        for (int t = lane; t < s; t += 64) d.page_pos[pg * s + t] = -1;
        return;
    }
    const int *pb = d.page_base + (size_t)u * (d.Cpad + 1);
    int lo = 0, hi = d.Cpad;  // largest c with pb[c] <= p (clusters without pages are skipped)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (pb[mid] <= p) lo = mid; else hi = mid;
    }
    const int c = lo;
    const int start = d.cluster_start[(size_t)u * (d.Cpad + 1) + c];
    const int cnt = d.cluster_start[(size_t)u * (d.Cpad + 1) + c + 1] - start;
    const int r0 = (p - pb[c]) * s;
    const int fill = min(s, cnt - r0);
    const int *ord = d.order + (size_t)u * d.max_tokens + start + r0;
    const int g = lane >> 4, ch = lane & 15;
    bf16_t *tile = (bf16_t *)smem + (size_t)wave * s * kD;
    for (int t4 = 0; t4 < s; t4 += 4) {
        const int slot = t4 + g;
        const bool valid = slot < fill;
        const int tok = valid ? ord[slot] : -1;
        uint4 kw = make_uint4(0, 0, 0, 0), vw = kw;
        if (valid) {
            kw = load16<STREAM>((const uint4 *)(K + ((size_t)u * n + tok) * kD) + ch);
            vw = load16<STREAM>((const uint4 *)(V + ((size_t)u * n + tok) * kD) + ch);
        }
        store16<STREAM>((uint4 *)(d.Kp + (pg * s + slot) * kD) + ch, kw);
        store16<STREAM>((uint4 *)(d.Vp + (pg * s + slot) * kD) + ch, vw);
        ((uint4 *)(tile + (size_t)slot * kD))[ch] = kw;
        if (ch == 0) d.page_pos[pg * s + slot] = tok;
    }
    if (lane == 0) { d.page_cluster[pg] = c; d.page_fill[pg] = fill; }
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the tile writes above are visible to the wave
    float a0 = 0.f, a1 = 0.f;
    for (int t = 0; t < fill; ++t) {
        const uint32_t w = ((const uint32_t *)(tile + (size_t)t * kD))[lane];
        a0 = a0 + bf16_lo(w);
        a1 = a1 + bf16_hi(w);
    }
    ((float2 *)(d.page_sum + pg * kD))[lane] = make_float2(a0, a1);
    const float f = (float)fill;
    ((uint32_t *)(d.rep + pg * kD))[lane] = (uint32_t)f32_to_bf16(a0 / f) | ((uint32_t)f32_to_bf16(a1 / f) << 16);
}

void launch_paginate(const Dev &d, const bf16_t *K, const bf16_t *V, int n, hipStream_t st) {
    const size_t lds = (size_t)4 * d.s * kD * 2;
    if (keys_exceed_cache(d, n)) hipLaunchKernelGGL(paginate_kernel<true>, dim3((d.max_pages + 3) / 4, d.U), dim3(256), lds, st, d, K, V, n);
    else hipLaunchKernelGGL(paginate_kernel<false>, dim3((d.max_pages + 3) / 4, d.U), dim3(256), lds, st, d, K, V, n);
    launch_refresh_tails(d, st);
}

// ------------------------------------------------------------------------------------------------
// The level above the clusters (Sec. 3.3: every point's parent is a point one level up).  A small
// Lloyd iteration over the unit's C bf16 centroids as points, one workgroup per unit:
//   promote  top node t starts at the centroid in the middle of the t-th of n_top equal strata of the
//            cluster ids;
//   assign   every cluster to the nearest top node: ||t~||^2 - 2 c . t~, fp32 accumulate on the matrix cores
//            (16 clusters x 16 nodes per v_mfma_f32_16x16x32_bf16 chain) against the nodes' bf16 rounding held
//            in LDS, lowest id on ties;
//   means    the clusters of a node are listed in ascending id (one wave per node walks the
//            assignment with lane masks) and summed in that order in fp32, four dimensions per thread;
//            an empty node keeps its position.
// The state left is the last assignment and the means of that assignment, as for the clusters.
// LDS: [n_top][128] bf16 rows, [n_top] norms, [n_top + 1] list starts, [C] assignment, [C] member list.
__global__ __launch_bounds__(1024) void top_level_kernel(Dev d, const bf16_t *__restrict__ cent, int n_top, int iters) {
    extern __shared__ __align__(16) char smem[];
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int C = d.C;
    uint4 *rows = (uint4 *)smem;                                   // [n_top][16]
    float *norm = (float *)(smem + (size_t)n_top * 256);           // [n_top]
    int *start = (int *)(norm + n_top);                            // [n_top + 1]
    int *asg = start + n_top + 1;                                  // [C]
    int *members = asg + C;                                        // [C]
    const bf16_t *pts = cent + (size_t)u * d.Cpad * kD;            // the clusters' bf16 centroids: the points
    float *tc = d.top_cent + (size_t)u * kTopMax * kD;
    // promote
    for (int x = tid; x < n_top * 16; x += 1024) {
        const int t = x >> 4, ch = x & 15;
        const int c = (int)(((long long)(2 * t + 1) * C) / (2 * n_top));
        const uint4 w = ((const uint4 *)(pts + (size_t)c * kD))[ch];
        rows[x] = w;
        float *dst = tc + (size_t)t * kD + ch * 8;
        dst[0] = bf16_lo(w.x); dst[1] = bf16_hi(w.x); dst[2] = bf16_lo(w.y); dst[3] = bf16_hi(w.y);
        dst[4] = bf16_lo(w.z); dst[5] = bf16_hi(w.z); dst[6] = bf16_lo(w.w); dst[7] = bf16_hi(w.w);
        if (ch == 0) d.top_init[(size_t)u * kTopMax + t] = c;
    }
    __syncthreads();
    for (int it = 0; it < iters; ++it) {
        for (int t = tid; t < n_top; t += 1024) {
            float nn = 0.f;
            for (int ch = 0; ch < 16; ++ch) {
                const uint4 w = rows[t * 16 + ch];
                nn += bf16_lo(w.x) * bf16_lo(w.x) + bf16_hi(w.x) * bf16_hi(w.x) + bf16_lo(w.y) * bf16_lo(w.y) + bf16_hi(w.y) * bf16_hi(w.y) +
                      bf16_lo(w.z) * bf16_lo(w.z) + bf16_hi(w.z) * bf16_hi(w.z) + bf16_lo(w.w) * bf16_lo(w.w) + bf16_hi(w.w) * bf16_hi(w.w);
            }
            norm[t] = nn;
        }
        __syncthreads();
        // assign on the matrix cores: a wave takes 16 clusters at a time as the columns of the B operand (lane
        // (g, n): dims [32 ks + 8 g, +8) of cluster n) and walks the nodes 16 at a time as the rows of A, read from
        // LDS; lane (g, n) ends with nodes 4g .. 4g+3 of the tile against cluster n and keeps the best, lowest node
        // id on ties; the four row groups meet by lane exchange
        {
            const int g = lane >> 4, i16 = lane & 15;
            const int ptiles = (C + 15) >> 4, ntiles = (n_top + 15) >> 4;
            auto cluster_rows = [&](int pt, uint4 (&b)[4]) {
                const int c = pt * 16 + i16;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    b[ks] = make_uint4(0, 0, 0, 0);
                    if (c < C) b[ks] = ((const uint4 *)(pts + (size_t)c * kD))[ks * 4 + g];
                }
            };
            uint4 b[4], bn[4];
            if (wave < ptiles) cluster_rows(wave, b);
            for (int pt = wave; pt < ptiles; pt += 16) {
                const int c = pt * 16 + i16;
                if (pt + 16 < ptiles) cluster_rows(pt + 16, bn);  // (the next tile's rows are on their way during this one)
                u64 best = ~0ull;
                for (int nt = 0; nt < ntiles; ++nt) {
                    const int node_a = nt * 16 + i16;
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < 4; ++ks) {
                        uint4 a = make_uint4(0, 0, 0, 0);
                        if (node_a < n_top) a = rows[node_a * 16 + ks * 4 + g];
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b[ks]), acc, 0, 0, 0);
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int node = nt * 16 + 4 * g + j;
                        const float val = __builtin_fmaf(-2.0f, acc[j], node < n_top ? norm[node] : INFINITY);
                        if (node < n_top && !(val != val)) {
                            const u64 key = ((u64)f32_ordered(val) << 32) | (u64)(uint32_t)node;
                            best = key < best ? key : best;
                        }
                    }
                }
                u64 o = __shfl_xor(best, 16);
                best = o < best ? o : best;
                o = __shfl_xor(best, 32);
                best = o < best ? o : best;
                if (g == 0 && c < C) {
                    const int bi = best == ~0ull ? 0 : (int)(uint32_t)best;
                    asg[c] = bi;
                    d.top_of[(size_t)u * C + c] = bi;
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) b[ks] = bn[ks];
            }
        }
        __syncthreads();
        // list the clusters of every node in ascending id: counts, starts, then placement
        for (int t = wave; t < n_top; t += 16) {
            int cnt = 0;
            for (int c0 = 0; c0 < C; c0 += 64) cnt += (int)__popcll(__ballot(c0 + lane < C && asg[c0 + lane] == t));
            if (lane == 0) start[t + 1] = cnt;
        }
        __syncthreads();
        if (tid == 0) {
            start[0] = 0;
            for (int t = 0; t < n_top; ++t) start[t + 1] += start[t];
        }
        __syncthreads();
        for (int t = wave; t < n_top; t += 16) {
            int base = start[t];
            for (int c0 = 0; c0 < C; c0 += 64) {
                const bool is = c0 + lane < C && asg[c0 + lane] == t;
                const u64 bal = __ballot(is);
                if (is) members[base + (int)__popcll(bal & ((1ull << lane) - 1ull))] = c0 + lane;
                base += (int)__popcll(bal);
            }
        }
        __syncthreads();
        // means: (node, four dimensions) per thread, members in list order
        for (int x = tid; x < n_top * 32; x += 1024) {
            const int t = x >> 5, qd = x & 31;
            const int lo = start[t], cnt = start[t + 1] - lo;
            float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
            constexpr int MB = 32;  // rows requested at once (the sum itself stays in list order)
            for (int i0 = 0; i0 < cnt; i0 += MB) {
                uint2 w[MB];
#pragma unroll
                for (int x = 0; x < MB; ++x) {
                    w[x] = make_uint2(0u, 0u);
                    if (i0 + x < cnt) w[x] = ((const uint2 *)(pts + (size_t)members[lo + i0 + x] * kD))[qd];
                }
#pragma unroll
                for (int x = 0; x < MB; ++x)
                    if (i0 + x < cnt) { a0 += bf16_lo(w[x].x); a1 += bf16_hi(w[x].x); a2 += bf16_lo(w[x].y); a3 += bf16_hi(w[x].y); }
            }
            float *dst = tc + (size_t)t * kD + qd * 4;
            if (cnt > 0) {
                const float f = (float)cnt;
                a0 /= f; a1 /= f; a2 /= f; a3 /= f;
                dst[0] = a0; dst[1] = a1; dst[2] = a2; dst[3] = a3;
            } else {
                a0 = dst[0]; a1 = dst[1]; a2 = dst[2]; a3 = dst[3];
            }
            ((uint2 *)rows)[t * 32 + qd] = make_uint2((uint32_t)f32_to_bf16(a0) | ((uint32_t)f32_to_bf16(a1) << 16),
                                                      (uint32_t)f32_to_bf16(a2) | ((uint32_t)f32_to_bf16(a3) << 16));
            if (qd == 0) d.top_cnt[(size_t)u * kTopMax + t] = cnt;
        }
        __syncthreads();
    }
    // the nodes' bf16 rows for the search (rows from n_top on: zero)
    uint4 *dst = (uint4 *)(d.top_bf16 + (size_t)u * kTopMax * kD);
    for (int x = tid; x < kTopMax * 16; x += 1024) dst[x] = x < n_top * 16 ? rows[x] : make_uint4(0, 0, 0, 0);
}

void launch_top_level(const Dev &d, int cur, int n_top, int iters, hipStream_t st) {
    const size_t lds = (size_t)n_top * 256 + (size_t)(2 * n_top + 1) * 4 + (size_t)d.C * 8;
    allow_dynamic_lds((const void *)top_level_kernel, lds);
    hipLaunchKernelGGL(top_level_kernel, dim3(d.U), dim3(1024), lds, st, d, d.cent_bf16[cur], n_top, iters);
}

}  // namespace ice

ICE_PROF_EXPORT(ice_debug_prof_build)
