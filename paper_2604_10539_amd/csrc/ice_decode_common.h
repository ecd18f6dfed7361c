// Device code shared by the decode-step kernels (flat and hierarchical page selection): vector
// types, packed-bf16 dot products, the query operand of the scoring / logit MFMAs, and sparse
// paged attention over a list of pages.
#pragma once
#include "ice_internal.h"

namespace ice {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short bf16x4s __attribute__((ext_vector_type(4)));  // operand type of the 16x16x16 bf16 MFMA builtin
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef unsigned long long u64;

// a.lo*b.lo + a.hi*b.hi + c on packed bf16 pairs, fp32 accumulate (v_dot2_f32_bf16)
__device__ inline float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ inline float dot8(const uint4 &a, const uint4 &b) {
    return dot2(a.w, b.w, dot2(a.z, b.z, dot2(a.y, b.y, dot2(a.x, b.x, 0.f))));
}

// Sparse paged attention over a list of pages (Eq. 1 with the mask set on the tokens of the listed
// pages), for one unit, by the NW waves of the calling workgroup.  Wave w streams pages w, w+NW, ...;
// a page's key tile and value tile are each s x 256 contiguous bytes.  Per 16-token block:
//   logits   one v_mfma_f32_16x16x32_bf16 chain, A = the G query rows, B = the 16 key rows (lane
//            (g, r) reads bytes [64*ks + 16*g, +16) of key row r): lane r of row group 0 gets the
//            logits of token r for heads 0..3 (group 1: heads 4..7);
//   softmax  running maximum and denominator per head, shared by the whole wave (DPP row maxima),
//            fp32; the 16 x G weights cross to the matrix-operand layout via LDS;
//   values   also on the matrix cores: out[head][dim] += sum_token p[head][token] v[token][dim] as
//            v_mfma_f32_16x16x16_bf16 with A = the weights, split into two bf16 terms (p = hi + lo,
//            relative error 2^-16, so the fp32 softmax survives), and B = the value rows.  Lane
//            (g, c) loads value rows 4t+g, 16 bytes each (1 KiB per load instruction): it holds
//            tokens {g, 4+g, 8+g, 12+g} x dims 8c..8c+7, which is exactly the B operand of eight
//            column tiles if tile j is made of dims {8c + j} and contraction slot 4g+i stands for
//            token 4i+g (a permutation of the sum); two byte-permutes per tile pack it.
// The NW waves are merged by the (max, sum, output) rule.  page_of(x) names the x-th listed page;
// `red` is LDS scratch of attend_scratch_floats() floats; aside() is work of the caller that needs
// no barrier and runs where a wave would otherwise wait for the slowest wave's pages.
__host__ __device__ constexpr int attend_scratch_floats(int G, int NW) { return NW * (G * (kD + 2) + 16 * 8); }

template <int G>
__device__ inline void load_query_operand(const bf16_t *q, int u, int lane, bf16x8 (&qa)[4], float *sumsq) {
    const int g = lane >> 4, ch = lane & 15;
    float nn = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const uint4 w = ch < G ? ((const uint4 *)(q + ((size_t)u * G + ch) * kD))[ks * 4 + g] : make_uint4(0, 0, 0, 0);
        qa[ks] = __builtin_bit_cast(bf16x8, w);
        nn += dot8(w, w);
    }
    if (sumsq) *sumsq = nn;
}

// Split-row form of the scoring contraction.  In the plain form lane (g, c) of a B operand reads
// 16 bytes of row c at 64*ks + 16*g, so one load instruction touches half a 128-byte line of each of
// 16 rows.  Here a load instruction covers whole lines: lanes c and c+8 read the two 64-byte halves
// of a line of row c%8, i.e. column c < 8 of the B operand carries dims [64t, 64t+32) of the row and
// column c+8 dims [64t+32, 64t+64) (t = 0, 1: two MFMAs per 8 rows, as many as before per byte).
// The A operand holds every query row twice: row h with the dims of the lower halves, row G+h with
// those of the upper halves (load_query).  Output (row h, column c < 8) and (row G+h, column c+8) are then the
// two halves of q_h . row_c; the other outputs are discarded.  A pair of 8-row blocks shares one
// exchange: lanes c < 8 keep the first block, lanes c >= 8 the second, each sends the partner
// (lane xor kXor) the half it does not keep, and lane (.., c) ends with the scores of row c of the
// 16 for its heads.
template <int G>
struct SplitRow {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8, "2G query rows must fit the 16 operand rows");
    static constexpr int kDG = G >= 4 ? G / 4 : 0;  // 16-lane row groups between row h and row G+h
    static constexpr int kDV = G >= 4 ? 0 : G;      // accumulator slots between them
    static constexpr int kXor = 8 + 16 * kDG;
    static constexpr int kHV = G < 4 ? G : 4;       // heads per lane

    // The A operand straight from memory: lane (g, c) holds q_c dims [64t + 8g, +8) for c < G and
    // q_{c-G} dims [64t + 32 + 8g, +8) for G <= c < 2G (t = 0, 1), zeros from row 2G on.  *inv_norm =
    // 1 / max(||q_h||, 1e-20) on the lanes with c = h and c = G + h.
    __device__ static void load_query(const bf16_t *q, int u, int lane, bf16x8 (&qs)[2], float *inv_norm) {
        const int g = lane >> 4, c = lane & 15;
        const int upper = c >= G ? 1 : 0, h = c - G * upper;
        const uint4 *row = (const uint4 *)(q + ((size_t)u * G + h) * kD);
        float nn = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint4 w = c < 2 * G ? row[8 * t + 4 * upper + g] : make_uint4(0, 0, 0, 0);
            qs[t] = __builtin_bit_cast(bf16x8, w);
            nn += dot8(w, w);
        }
        nn += __shfl_xor(nn, 16);
        nn += __shfl_xor(nn, 32);
        nn += __shfl_xor(nn, G);  // the other half of the row
        *inv_norm = 1.0f / fmaxf(sqrtf(nn), 1e-20f);
    }
    // The plain operand of the logit MFMAs (lane (g, h): dims [32ks + 8g, +8) of q_h, zero rows from
    // G on) out of the split one, by lane exchange: no second trip to memory for the query rows.
    __device__ static void to_plain(const bf16x8 (&qs)[2], int lane, bf16x8 (&qa)[4]) {
        const bool low = (lane & 15) < G;
        const uint4 zero = make_uint4(0, 0, 0, 0);
        const int src = (lane + G) & 63;  // row G + h holds the upper halves of q_h
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint4 w = __builtin_bit_cast(uint4, qs[t]);
            uint4 up;
            up.x = __shfl(w.x, src);
            up.y = __shfl(w.y, src);
            up.z = __shfl(w.z, src);
            up.w = __shfl(w.w, src);
            qa[2 * t] = __builtin_bit_cast(bf16x8, low ? w : zero);
            qa[2 * t + 1] = __builtin_bit_cast(bf16x8, low ? up : zero);
        }
    }
    // uint4 index inside a 16-row block (rows of 16 uint4) of the load that feeds MFMA t of 8-row
    // block blk
    __device__ static int word(int lane, int blk, int t) {
        const int g = lane >> 4, c = lane & 15;
        return (8 * blk + (c & 7)) * 16 + 8 * t + 4 * (c >> 3) + g;
    }
    // lanes whose result is a row's score: row c of the 16, heads 4 * head_group(lane) + v
    __device__ static bool owner(int lane) { return (lane >> 4) == ((lane & 8) ? kDG : 0); }
    __device__ static int head_group(int lane) { return (lane >> 4) - ((lane & 8) ? kDG : 0); }
    // max over the group's heads of (q_h . row) * inv[v]; acc0 / acc1 = accumulators of the two blocks
    __device__ static float score(const f32x4 &acc0, const f32x4 &acc1, const float (&inv)[4], int lane) {
        const bool hi = (lane & 8) != 0;
        float sc = -INFINITY;
#pragma unroll
        for (int v = 0; v < kHV; ++v) {
            const float a0 = (kDV && hi) ? acc0[(v + kDV) & 3] : acc0[v];
            const float a1 = (kDV && hi) ? acc1[(v + kDV) & 3] : acc1[v];
            const float tot = (hi ? a1 : a0) + __shfl_xor(hi ? a0 : a1, kXor);
            sc = fmaxf(sc, tot * inv[v]);
        }
        if (G > 4) sc = fmaxf(sc, __shfl_xor(sc, 16));
        return sc;
    }
};

// With PARTIAL the workgroup attends to a share of a unit's pages and leaves, instead of the output,
// what a later merge needs: per head h the unnormalised sum at out[h * (kD + 2) + j], the running
// maximum at [.. + kD] and the denominator at [.. + kD + 1] (`out` then points at the workgroup's own
// block and `u` only addresses the pages).
template <int G, int NW, bool RES, bool PARTIAL = false, typename PageOf, typename Aside>
__device__ inline void attend_pages(const Dev &d, int u, const bf16x8 (&qa)[4], PageOf page_of, int ns, Resident res,
                                    float *__restrict__ out, float *red, Aside aside) {
    constexpr int GR = (G + 3) / 4;  // row groups that hold logits and outputs
    float(*wacc)[G][kD] = (float(*)[G][kD])red;                   // [NW][G][128]
    float(*wm)[G] = (float(*)[G])(red + NW * G * kD);             // [NW][G]
    float(*wl)[G] = (float(*)[G])(red + NW * G * (kD + 1));       // [NW][G]
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    float *px = red + NW * G * (kD + 2) + wave * (16 * 8);        // [16 tokens][8 heads] weights of this wave
    const float scale = 0.08838834764831845f;  // 1/sqrt(128)
    const int s = d.s;
    // lane (g, r): m, l of heads 4g..4g+3 (wave-wide maxima, own-token denominators);
    // acc[j][v] = output of head 4g+v, dim 8r+j
    float m[4], l[4];
    f32x4 acc[8];
#pragma unroll
    for (int v = 0; v < 4; ++v) { m[v] = -INFINITY; l[v] = 0.f; }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    bool first = true;
    // one 16-token block whose key pieces (kb) and value rows (vt) are in registers; tokens from
    // nvalid on are masked
    auto block = [&](int b0, int fill, uint4 (&kb)[4], uint4 (&vt)[4]) {
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks], __builtin_bit_cast(bf16x8, kb[ks]), z, 0, 0, 0);
#ifdef ICE_PROF_ATTEND
        if (threadIdx.x == 0 && u == 0 && z[0] != 12345.f) ice::prof::stamps[9] = wall_clock64();
#endif
        const bool tok_ok = b0 + ch < fill;  // this lane's logits belong to token b0 + ch
        float pw[4], alpha[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float zz = tok_ok ? z[v] * scale : -INFINITY;
            float mx = zz;
            mx = fmaxf(mx, dpp_f32<0xB1>(mx));
            mx = fmaxf(mx, dpp_f32<0x4E>(mx));
            mx = fmaxf(mx, dpp_f32<0x141>(mx));
            mx = fmaxf(mx, dpp_f32<0x140>(mx));   // block maximum of head 4g+v on all 16 lanes of the row
            const float mn = fmaxf(m[v], mx);     // finite: every live page has at least one token
            alpha[v] = __expf(m[v] - mn);
            pw[v] = __expf(zz - mn);
            l[v] = l[v] * alpha[v] + pw[v];
            m[v] = mn;
        }
        if (g < GR) *(float4 *)(px + ch * 8 + 4 * g) = make_float4(pw[0], pw[1], pw[2], pw[3]);
        __builtin_amdgcn_wave_barrier();
        // A operand: lane (g, h) holds p[head h][token 4i+g], i = 0..3, as hi + lo bf16 terms
        float pa[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float t = px[(4 * i + g) * 8 + (ch & 7)];  // (unconditional read, then select: no branch)
            pa[i] = ch < G ? t : 0.f;
        }
        uint32_t hi[4], lo[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            hi[i] = __float_as_uint(pa[i]) & 0xFFFF0000u;
            lo[i] = __float_as_uint(pa[i] - __uint_as_float(hi[i]));
        }
        const v2u ahi = {__builtin_amdgcn_perm(hi[1], hi[0], 0x07060302u), __builtin_amdgcn_perm(hi[3], hi[2], 0x07060302u)};
        const v2u alo = {__builtin_amdgcn_perm(lo[1], lo[0], 0x07060302u), __builtin_amdgcn_perm(lo[3], lo[2], 0x07060302u)};
        if (!first) {  // rescale what earlier blocks left (same lanes hold the factors)
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[j][v] *= alpha[v];
        }
        first = false;
        if (fill - b0 < 16) {  // a partly filled block: rows past the end must not reach the matrix core
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (b0 + 4 * t + g >= fill) vt[t] = make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // column tile j: dims {8c + j}; contraction slot 4g+i = token 4i+g
            const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
            const uint32_t w0 = j < 2 ? vt[0].x : j < 4 ? vt[0].y : j < 6 ? vt[0].z : vt[0].w;
            const uint32_t w1 = j < 2 ? vt[1].x : j < 4 ? vt[1].y : j < 6 ? vt[1].z : vt[1].w;
            const uint32_t w2 = j < 2 ? vt[2].x : j < 4 ? vt[2].y : j < 6 ? vt[2].z : vt[2].w;
            const uint32_t w3 = j < 2 ? vt[3].x : j < 4 ? vt[3].y : j < 6 ? vt[3].z : vt[3].w;
            const v2u bv = {__builtin_amdgcn_perm(w1, w0, sel), __builtin_amdgcn_perm(w3, w2, sel)};
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4s, ahi), __builtin_bit_cast(bf16x4s, bv), acc[j], 0, 0, 0);
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(bf16x4s, alo), __builtin_bit_cast(bf16x4s, bv), acc[j], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();  // the next block overwrites px
    };
    // the first 16-token block of a page is fetched before its fill count is known (one fewer
    // dependent round trip); slots >= fill may hold stale bytes and are masked after the load
    for (int x = wave; x < ns; x += NW) {
        const int p = page_of(x);
        if ((unsigned)p >= (unsigned)d.max_pages) continue;  // not a page id: ignored
        const size_t pg = (size_t)u * d.max_pages + p;
        uint4 kb[4], vt[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            kb[t] = ((const uint4 *)(d.Kp + (pg * s + ch) * kD))[t * 4 + g];
            vt[t] = ((const uint4 *)(d.Vp + (pg * s + 4 * t + g) * kD))[ch];
        }
        const int fill = d.page_fill[pg];
        ICE_STAMP(8);
        for (int b0 = 0; b0 < fill; b0 += 16) {
            if (b0 > 0) {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    kb[t] = ((const uint4 *)(d.Kp + (pg * s + b0 + ch) * kD))[t * 4 + g];
                    vt[t] = ((const uint4 *)(d.Vp + (pg * s + b0 + 4 * t + g) * kD))[ch];
                }
            }
            block(b0, fill, kb, vt);
        }
    }
    if constexpr (RES) {
        // resident tokens, 16 per block, dealt to the waves where the pages left off; rows past the
        // end of the run are not there to be read
        const int nres = res.pos ? min(res.cnt[u], res.n) : res.n;
        const int nrb = (nres + 15) >> 4;
        for (int j = ((wave - ns) % NW + NW) % NW; j < nrb; j += NW) {
            const int r0 = 16 * j, fill = min(16, nres - r0);
            uint4 kb[4], vt[4];
            if (!res.pos) {
                const bf16_t *ktile = res.k + ((size_t)u * res.n + r0) * kD;
                const bf16_t *vtile = res.v + ((size_t)u * res.n + r0) * kD;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    kb[t] = ch < fill ? ((const uint4 *)(ktile + (size_t)ch * kD))[t * 4 + g] : make_uint4(0, 0, 0, 0);
                    vt[t] = 4 * t + g < fill ? ((const uint4 *)(vtile + (size_t)(4 * t + g) * kD))[ch] : make_uint4(0, 0, 0, 0);
                }
            } else {
                const int *pl = res.pos + (size_t)u * res.n + r0;
                const int krow = ch < fill ? min(max(pl[ch], 0), res.rows - 1) : 0;
                int vrow[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) vrow[t] = 4 * t + g < fill ? min(max(pl[4 * t + g], 0), res.rows - 1) : 0;
                const bf16_t *kbase = res.k + (size_t)u * res.rows * kD, *vbase = res.v + (size_t)u * res.rows * kD;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    kb[t] = ch < fill ? ((const uint4 *)(kbase + (size_t)krow * kD))[t * 4 + g] : make_uint4(0, 0, 0, 0);
                    vt[t] = 4 * t + g < fill ? ((const uint4 *)(vbase + (size_t)vrow[t] * kD))[ch] : make_uint4(0, 0, 0, 0);
                }
            }
            block(0, fill, kb, vt);
        }
    }
    ICE_STAMP(10);
    if (g < GR) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (4 * g + v < G) {
                float *dst = &wacc[wave][4 * g + v][ch * 8];
                *(float4 *)dst = make_float4(acc[0][v], acc[1][v], acc[2][v], acc[3][v]);
                *(float4 *)(dst + 4) = make_float4(acc[4][v], acc[5][v], acc[6][v], acc[7][v]);
            }
        }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) l[v] = row16_sum(l[v]);
    if (g < GR && ch == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (4 * g + v < G) { wm[wave][4 * g + v] = m[v]; wl[wave][4 * g + v] = l[v]; }
    }
    aside();
    __syncthreads();
    ICE_STAMP(11);
    // per head: the waves' merge weights exp(m_w - M) / L, one 16-lane row per head, one lane per wave
    static_assert(NW <= 16, "one DPP row holds the waves of a head");
    if (tid < 16 * G) {
        const int h = tid >> 4, w = tid & 15;
        const float mw = w < NW ? wm[w][h] : -INFINITY, lw = w < NW ? wl[w][h] : 0.f;
        float M = mw;
        M = fmaxf(M, dpp_f32<0xB1>(M));
        M = fmaxf(M, dpp_f32<0x4E>(M));
        M = fmaxf(M, dpp_f32<0x141>(M));
        M = fmaxf(M, dpp_f32<0x140>(M));
        const float e = M == -INFINITY ? 0.f : __expf(mw - M);
        const float L = row16_sum(lw * e);
        if constexpr (PARTIAL) {  // (device-scope words: another workgroup merges them)
            if (w < NW) wm[w][h] = e;
            if (w == 0) {
                __hip_atomic_store(out + h * (kD + 2) + kD, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(out + h * (kD + 2) + kD + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        } else {
            if (w < NW) wm[w][h] = L > 0.f ? e / L : 0.f;
        }
    }
    __syncthreads();
    for (int o = tid; o < G * kD; o += NW * 64) {
        const int h = o / kD, j = o % kD;
        float O = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) O += wacc[w][h][j] * wm[w][h];
        if constexpr (PARTIAL) __hip_atomic_store(out + h * (kD + 2) + j, O, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else out[((size_t)u * G + h) * kD + j] = O;
    }
}

}  // namespace ice
