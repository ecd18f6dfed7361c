// Decode-step kernels: insertion of a new token, scoring of the page representatives, top-P page
// selection and sparse paged attention (Sec. 4.2-4.4, Alg. 1 and 3, Eq. 1 of the paper).
#include "ice_internal.h"

namespace ice {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef unsigned long long u64;

// a.lo*b.lo + a.hi*b.hi + c on packed bf16 pairs, fp32 accumulate (v_dot2_f32_bf16)
__device__ inline float dot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}
__device__ inline float dot8(const uint4 &a, const uint4 &b) {
    return dot2(a.w, b.w, dot2(a.z, b.z, dot2(a.y, b.y, dot2(a.x, b.x, 0.f))));
}

// ------------------------------------------------------------------------------------------------
// Insertion of one token per unit (Alg. 1 insertion loop; a node that outgrows its page gets a new
// one, Sec. 4.1).  One workgroup per unit: the four waves scan the bf16 centroids
// (16 lanes x 16 bytes per row) for the nearest one, lowest id on ties; wave 0 then appends the
// key/value row to the cluster's tail page and updates, in ordered fp32 (one add per quantity):
// page sum -> representative, cluster sum -> centroid, its bf16 rounding and squared norm.
__global__ __launch_bounds__(256) void insert_kernel(Dev d, const bf16_t *__restrict__ k,
                                                      const bf16_t *__restrict__ v, int cur) {
    __shared__ u64 best;
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    if (tid == 0) best = ~0ull;
    __syncthreads();
    const uint4 kq = ((const uint4 *)(k + (size_t)u * kD))[ch];
    const bf16_t *cb = d.cent_bf16[cur] + (size_t)u * d.Cpad * kD;
    const float *wn = d.cnorm[cur] + (size_t)u * d.Cpad;
    float bv = INFINITY;
    int bi = 0x7FFFFFFF;
    for (int r = wave * 4 + g; r < d.C; r += 16) {
        const uint4 row = ((const uint4 *)(cb + (size_t)r * kD))[ch];
        const float dot = row16_sum(dot8(row, kq));
        const float val = wn[r] - 2.0f * dot;
        if (val < bv) { bv = val; bi = r; }
    }
    if (ch == 0 && bi != 0x7FFFFFFF) atomicMin(&best, ((u64)f32_ordered(bv) << 32) | (u64)(uint32_t)bi);
    __syncthreads();
    if (wave != 0) return;
    const int c = (int)(uint32_t)best;
    const size_t cl = (size_t)u * d.C + c;
    int tail = d.cluster_tail[cl];
    int fill = tail >= 0 ? d.page_fill[(size_t)u * d.max_pages + tail] : d.s;
    const int np = d.n_pages[u];
    const int tok = d.n_tokens[u];
    const int cnt = d.cluster_cnt[cl] + 1;
    const bool fresh = fill == d.s;
    if (fresh) { tail = np; fill = 0; }
    const size_t pg = (size_t)u * d.max_pages + tail;
    const int slot = fill;
    fill += 1;
    const uint32_t kw = ((const uint32_t *)(k + (size_t)u * kD))[lane];
    const uint32_t vw = ((const uint32_t *)(v + (size_t)u * kD))[lane];
    ((uint32_t *)(d.Kp + (pg * d.s + slot) * kD))[lane] = kw;
    ((uint32_t *)(d.Vp + (pg * d.s + slot) * kD))[lane] = vw;
    const float k0 = bf16_lo(kw), k1 = bf16_hi(kw);
    float2 ps = fresh ? make_float2(0.f, 0.f) : ((const float2 *)(d.page_sum + pg * kD))[lane];
    ps.x = ps.x + k0;
    ps.y = ps.y + k1;
    ((float2 *)(d.page_sum + pg * kD))[lane] = ps;
    const float ff = (float)fill;
    ((uint32_t *)(d.rep + pg * kD))[lane] = (uint32_t)f32_to_bf16(ps.x / ff) | ((uint32_t)f32_to_bf16(ps.y / ff) << 16);
    float2 cs = ((const float2 *)(d.cluster_sum + cl * kD))[lane];
    cs.x = cs.x + k0;
    cs.y = cs.y + k1;
    ((float2 *)(d.cluster_sum + cl * kD))[lane] = cs;
    const float fc = (float)cnt;
    const float2 mu = make_float2(cs.x / fc, cs.y / fc);
    ((float2 *)(d.centroid + cl * kD))[lane] = mu;
    const bf16_t b0 = f32_to_bf16(mu.x), b1 = f32_to_bf16(mu.y);
    ((uint32_t *)(d.cent_bf16[cur] + ((size_t)u * d.Cpad + c) * kD))[lane] = (uint32_t)b0 | ((uint32_t)b1 << 16);
    const float f0 = bf16_to_f32(b0), f1 = bf16_to_f32(b1);
    const float nn = wave_sum(f0 * f0 + f1 * f1);
    if (lane == 0) {
        d.cnorm[cur][(size_t)u * d.Cpad + c] = nn;
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
}

void launch_insert(const Dev &d, const bf16_t *k, const bf16_t *v, int cur, hipStream_t st) {
    hipLaunchKernelGGL(insert_kernel, dim3(d.U), dim3(256), 0, st, d, k, v, cur);
}

// ------------------------------------------------------------------------------------------------
// Representative scoring (Sec. 4.3-4.4; query normalisation of Eq. 3): for every live page p
//   S[p] = max over the G query heads of the group of  (q_h . rep_p) / ||q_h||.
// The representatives of a unit are one contiguous bf16 stream; a wave reads 1 KiB (four rows)
// per load instruction, 16 lanes x 16 bytes per row, and reduces each row's partial dot products
// inside its 16-lane DPP row.  The unit's pages are split over gridDim.x workgroups.
template <int G>
__global__ __launch_bounds__(256) void score_kernel(Dev d, const bf16_t *__restrict__ q) {
    const int u = blockIdx.y, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    const int np = d.n_pages[u];
    const int per = round_up((np + gridDim.x - 1) / gridDim.x, 16);
    const int p0 = blockIdx.x * per, p1 = min(np, p0 + per);
    if (p0 >= p1) return;
    uint4 qr[G];
    float inv[G];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        qr[h] = ((const uint4 *)(q + ((size_t)u * G + h) * kD))[ch];
        const float nn = row16_sum(dot8(qr[h], qr[h]));
        inv[h] = 1.0f / fmaxf(sqrtf(nn), 1e-20f);
    }
    const bf16_t *rep = d.rep + (size_t)u * d.max_pages * kD;
    float *S = d.scores + (size_t)u * d.max_pages;
    constexpr int UNR = 4;
    for (int base = p0; base < p1; base += 64 * UNR / 4) {  // 64 pages per workgroup iteration
        uint4 r[UNR];
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            const int pp = base + 16 * x + wave * 4 + g;
            r[x] = pp < p1 ? ((const uint4 *)(rep + (size_t)pp * kD))[ch] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int x = 0; x < UNR; ++x) {
            float sc = -INFINITY;
#pragma unroll
            for (int h = 0; h < G; ++h) sc = fmaxf(sc, row16_sum(dot8(r[x], qr[h])) * inv[h]);
            const int pp = base + 16 * x + wave * 4 + g;
            if (ch == 0 && pp < p1) S[pp] = sc;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Top-P page selection (Alg. 3 with pages ranked directly): exact radix select on the
// order-preserving integer image of the fp32 scores finds the P-th largest score; pages above it,
// plus the lowest-id pages equal to it, are written in ascending id order (ordered compaction).
// One workgroup per unit; the scores are re-read from L2 in each of the four 8-bit passes.
__global__ __launch_bounds__(1024) void select_kernel(Dev d, int P, int *__restrict__ ids_out,
                                                       int *__restrict__ n_sel_out, float *__restrict__ scores_out) {
    __shared__ int hist[256];
    __shared__ int wtot[16];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_kk, sh_base_eq, sh_base_out;
    const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int np = d.n_pages[u];
    const int k = min(P, np);
    const float *S = d.scores + (size_t)u * d.max_pages;
    int *ids = ids_out + (size_t)u * P;
    float *sco = scores_out ? scores_out + (size_t)u * P : nullptr;
    for (int x = k + tid; x < P; x += 1024) {
        ids[x] = -1;
        if (sco) sco[x] = 0.f;
    }
    if (tid == 0) n_sel_out[u] = k;
    if (k == 0) return;

    uint32_t prefix = 0, mask = 0;
    int kk = k;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < np; i += 1024) {
            const uint32_t key = f32_ordered(S[i]);
            if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1);
        }
        __syncthreads();
        // bins in descending order: thread t < 256 owns bin 255 - t
        int h = 0, incl = 0;
        if (tid < 256) {
            h = hist[255 - tid];
            incl = h;
            for (int off = 1; off < 64; off <<= 1) {
                const int t = __shfl_up(incl, off);
                if (lane >= off) incl += t;
            }
            if (lane == 63) wtot[wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            for (int w = 0; w < wave; ++w) incl += wtot[w];
            const int excl = incl - h;
            if (incl >= kk && excl < kk) {
                sh_prefix = prefix | ((uint32_t)(255 - tid) << shift);
                sh_kk = kk - excl;
            }
        }
        __syncthreads();
        prefix = sh_prefix;
        kk = sh_kk;
        mask |= 255u << shift;
        __syncthreads();
    }
    // prefix = key of the k-th largest score; kk = how many pages equal to it are still wanted
    if (tid == 0) { sh_base_eq = 0; sh_base_out = 0; }
    __syncthreads();
    for (int i0 = 0; i0 < np; i0 += 1024) {
        const int i = i0 + tid;
        uint32_t key = 0;
        float sc = 0.f;
        if (i < np) { sc = S[i]; key = f32_ordered(sc); }
        const bool gt = i < np && key > prefix, eq = i < np && key == prefix;
        // exclusive rank among the "equal" pages, in id order
        const u64 beq = __ballot(eq);
        if (lane == 0) wtot[wave] = (int)__popcll(beq);
        __syncthreads();
        int eqr = sh_base_eq + (int)__popcll(beq & ((1ull << lane) - 1ull));
        int tot_eq = 0;
        for (int w = 0; w < 16; ++w) { if (w < wave) eqr += wtot[w]; tot_eq += wtot[w]; }
        const bool take = gt || (eq && eqr < kk);
        __syncthreads();
        const u64 bt = __ballot(take);
        if (lane == 0) wtot[wave] = (int)__popcll(bt);
        __syncthreads();
        int pos = sh_base_out + (int)__popcll(bt & ((1ull << lane) - 1ull));
        int tot_out = 0;
        for (int w = 0; w < 16; ++w) { if (w < wave) pos += wtot[w]; tot_out += wtot[w]; }
        if (take) {
            ids[pos] = i;
            if (sco) sco[pos] = sc;
        }
        __syncthreads();
        if (tid == 0) { sh_base_eq += tot_eq; sh_base_out += tot_out; }
        __syncthreads();
    }
}

void launch_select(const Dev &d, const bf16_t *q, int P, int *ids, int *n_sel, float *scores_out, hipStream_t st) {
    // split each unit's representatives over enough workgroups to occupy the 256 CUs
    int chunks = (512 + d.U - 1) / d.U;
    const int max_chunks = (d.max_pages + 63) / 64;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    dim3 grid(chunks, d.U);
    switch (d.G) {
        case 1: hipLaunchKernelGGL(score_kernel<1>, grid, dim3(256), 0, st, d, q); break;
        case 2: hipLaunchKernelGGL(score_kernel<2>, grid, dim3(256), 0, st, d, q); break;
        case 4: hipLaunchKernelGGL(score_kernel<4>, grid, dim3(256), 0, st, d, q); break;
        default: hipLaunchKernelGGL(score_kernel<8>, grid, dim3(256), 0, st, d, q); break;
    }
    hipLaunchKernelGGL(select_kernel, dim3(d.U), dim3(1024), 0, st, d, P, ids, n_sel, scores_out);
}

// ------------------------------------------------------------------------------------------------
// Sparse paged attention (Eq. 1 with the mask set on the tokens of the selected pages).  One
// workgroup of 16 waves per unit; wave w streams selected pages w, w+16, ...: a page's key tile
// and value tile are each s x 256 contiguous bytes, read 1 KiB (four token rows) per load.  For
// every 16-token block the G heads' logits are reduced inside 16-lane DPP rows, so each row group
// of lanes runs its own online softmax (running max, denominator, 8 output dims per lane) over the
// tokens it sees; the four row groups, then the 16 waves, are merged with the usual
// (max, sum, weighted output) rule.  fp32 throughout, bf16 only as the storage format.
template <int G, int NW>
__global__ __launch_bounds__(NW * 64) void attend_kernel(Dev d, const bf16_t *__restrict__ q,
                                                          const int *__restrict__ ids, const int *__restrict__ n_sel,
                                                          int P, float *__restrict__ out) {
    extern __shared__ __align__(16) char smem[];
    float(*wacc)[G][kD] = (float(*)[G][kD])smem;                                  // [NW][G][128]
    float(*wm)[G] = (float(*)[G])(smem + sizeof(float) * NW * G * kD);            // [NW][G]
    float(*wl)[G] = (float(*)[G])(smem + sizeof(float) * NW * G * (kD + 1));      // [NW][G]
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    const int ns = min(n_sel[u], P);
    const float scale = 0.08838834764831845f;  // 1/sqrt(128)
    uint4 qr[G];
    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        qr[h] = ((const uint4 *)(q + ((size_t)u * G + h) * kD))[ch];
        m[h] = -INFINITY;
        l[h] = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[h][j] = 0.f;
    }
    const int s = d.s;
    for (int x = wave; x < ns; x += NW) {
        const int p = ids[(size_t)u * P + x];
        if ((unsigned)p >= (unsigned)d.max_pages) continue;  // not a page id: ignored
        const size_t pg = (size_t)u * d.max_pages + p;
        const int fill = d.page_fill[pg];
        for (int b0 = 0; b0 < fill; b0 += 16) {  // 16-token blocks of the page
            uint4 kt[4], vt[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int slot = b0 + 4 * t + g;  // < s; slots >= fill may hold stale bytes: not read
                const bool valid = slot < fill;
                kt[t] = valid ? ((const uint4 *)(d.Kp + (pg * s + slot) * kD))[ch] : make_uint4(0, 0, 0, 0);
                vt[t] = valid ? ((const uint4 *)(d.Vp + (pg * s + slot) * kD))[ch] : make_uint4(0, 0, 0, 0);
            }
            float z[G][4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const bool valid = b0 + 4 * t + g < fill;
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float dot = row16_sum(dot8(kt[t], qr[h]));
                    z[h][t] = valid ? dot * scale : -INFINITY;
                }
            }
            float pw[G][4];
#pragma unroll
            for (int h = 0; h < G; ++h) {
                const float mn = fmaxf(fmaxf(fmaxf(z[h][0], z[h][1]), fmaxf(z[h][2], z[h][3])), m[h]);
                const float mm = mn == -INFINITY ? 0.f : mn;
                const float alpha = __expf(m[h] - mm);
                float ps = 0.f;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    pw[h][t] = __expf(z[h][t] - mm);
                    ps += pw[h][t];
                }
                l[h] = l[h] * alpha + ps;
                m[h] = mn;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[h][j] *= alpha;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float v0 = bf16_lo(vt[t].x), v1 = bf16_hi(vt[t].x), v2 = bf16_lo(vt[t].y), v3 = bf16_hi(vt[t].y);
                const float v4 = bf16_lo(vt[t].z), v5 = bf16_hi(vt[t].z), v6 = bf16_lo(vt[t].w), v7 = bf16_hi(vt[t].w);
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float pp = pw[h][t];
                    acc[h][0] = fmaf(pp, v0, acc[h][0]); acc[h][1] = fmaf(pp, v1, acc[h][1]);
                    acc[h][2] = fmaf(pp, v2, acc[h][2]); acc[h][3] = fmaf(pp, v3, acc[h][3]);
                    acc[h][4] = fmaf(pp, v4, acc[h][4]); acc[h][5] = fmaf(pp, v5, acc[h][5]);
                    acc[h][6] = fmaf(pp, v6, acc[h][6]); acc[h][7] = fmaf(pp, v7, acc[h][7]);
                }
            }
        }
    }
    // merge the four row groups of the wave
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float mo = __shfl_xor(m[h], off), lo = __shfl_xor(l[h], off);
            const float mn = fmaxf(m[h], mo);
            const float mm = mn == -INFINITY ? 0.f : mn;
            const float a = __expf(m[h] - mm), b = __expf(mo - mm);
            l[h] = l[h] * a + lo * b;
            m[h] = mn;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[h][j] = acc[h][j] * a + __shfl_xor(acc[h][j], off) * b;
        }
    }
    if (g == 0) {
#pragma unroll
        for (int h = 0; h < G; ++h) {
            if (ch == 0) { wm[wave][h] = m[h]; wl[wave][h] = l[h]; }
#pragma unroll
            for (int j = 0; j < 8; ++j) wacc[wave][h][ch * 8 + j] = acc[h][j];
        }
    }
    __syncthreads();
    for (int o = tid; o < G * kD; o += NW * 64) {
        const int h = o / kD, j = o % kD;
        float M = -INFINITY;
        for (int w = 0; w < NW; ++w) M = fmaxf(M, wm[w][h]);
        float L = 0.f, O = 0.f;
        if (M != -INFINITY) {
            for (int w = 0; w < NW; ++w) {
                const float e = __expf(wm[w][h] - M);
                L += wl[w][h] * e;
                O += wacc[w][h][j] * e;
            }
        }
        out[((size_t)u * G + h) * kD + j] = L > 0.f ? O / L : 0.f;
    }
}

void launch_attend(const Dev &d, const bf16_t *q, const int *ids, const int *n_sel, int P, float *out,
                   hipStream_t st) {
#define ICE_ATTEND(g, nw)                                                                              \
    hipLaunchKernelGGL((attend_kernel<g, nw>), dim3(d.U), dim3(nw * 64), sizeof(float) * nw * g * (kD + 2), st, d, q, \
                       ids, n_sel, P, out)
    switch (d.G) {
        case 1: ICE_ATTEND(1, 16); break;
        case 2: ICE_ATTEND(2, 16); break;
        case 4: ICE_ATTEND(4, 16); break;
        default: ICE_ATTEND(8, 8); break;
    }
#undef ICE_ATTEND
}

}  // namespace ice
