// Hierarchical page selection: the two-level form of the paper's top-down search (Sec. 4.3,
// Alg. 3: descend from the parents that score best to their children).  One launch, one workgroup
// per unit:
//   stage 1  score the C cluster centroids (their bf16 rounding, the same rows the assignment
//            uses) against the group's queries, keep the n_probe best by (score, lower id first);
//   stage 2  find the live pages of the kept clusters (a scan of the 4-byte page -> cluster table
//            against a bitmask of kept clusters; pages opened by insertions sit anywhere in the
//            page range), score only their representatives, keep the top-P;
//   attend   over the winners (attend_pages), ids never leave the chip.
// Against the flat scan this reads C + n_probe/C * n_p representative rows instead of n_p.
// Scores are the flat scan's: max over the G heads of (q_h . row) / ||q_h||, fp32 MFMA accumulate.
#include "ice_decode_common.h"

namespace ice {

namespace {

constexpr int kListCap = 512;  // entries of the short list that is ranked by all-pairs counting

struct SelShared {
    int M, W, M2;
    uint32_t pre;
    u64 tau;
    uint32_t rowmax[64];
};

// Exact top-k of n distinct 64-bit composites (ordered score << 32 | ~id) held in LDS, into
// sel[0..k) (in no particular order when the radix path runs, by rank otherwise); requires
// 1 <= k < n.  A threshold that at least k composites reach comes from the k-th largest of the
// 4*NW sixteen-lane row maxima of the per-thread maxima; what passes it goes to a short list that
// is ranked by counting.  If the list overflows (or k exceeds the row count) an 8-bit-per-pass
// radix select over LDS histograms runs on the whole array instead.  `nb` = bits of the id field
// that can be set.  Every thread of the workgroup must call it; it ends with a barrier.
template <int NW>
__device__ void select_topk_lds(const u64 *comp, int n, int k, int nb, u64 *sel, u64 *list, int *hist, SelShared &sh) {
    constexpr int NT = NW * 64, NR = 4 * NW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, ch = lane & 15;
    if (tid == 0) { sh.M = 0; sh.W = 0; sh.pre = 0u; sh.tau = 0ull; }
    bool listed = false;
    if (k <= NR) {
        uint32_t lmax = 0u;
        for (int j = tid; j < n; j += NT) lmax = max(lmax, (uint32_t)(comp[j] >> 32));
        lmax = row16_max_u32(lmax);
        if (ch == 0) sh.rowmax[wave * 4 + g] = lmax;
        __syncthreads();
        const int i = tid >> 4, part = tid & 15;
        const uint32_t v = sh.rowmax[i];
        uint32_t c = 0;
#pragma unroll
        for (int jj = 0; jj < NR / 16; ++jj) {
            const int j = part * (NR / 16) + jj;
            const uint32_t o = sh.rowmax[j];
            c += (o > v || (o == v && j < i)) ? 1u : 0u;
        }
        c = row16_sum_u32(c);
        if (part == 0 && (int)c == k - 1) sh.pre = v;
        __syncthreads();
        const uint32_t pre = sh.pre;
        // short list of everything at or above the threshold (>= k entries)
        for (int j0 = 0; j0 < n; j0 += NT) {
            const int j = j0 + tid;
            const u64 cc = j < n ? comp[j] : 0ull;
            const bool is = j < n && (uint32_t)(cc >> 32) >= pre;
            const u64 bal = __ballot(is);
            int base = 0;
            if (lane == 0 && bal) base = atomicAdd(&sh.M, (int)__popcll(bal));
            base = __shfl(base, 0);
            const int slot = base + (int)__popcll(bal & ((1ull << lane) - 1ull));
            if (is && slot < kListCap) list[slot] = cc;
        }
        __syncthreads();
        const int M = sh.M;
        if (M <= kListCap) {
            listed = true;
            // every listed composite counts the listed composites that beat it
            int lp = 0;
            while (lp < 6 && (M << (lp + 1)) <= NT) ++lp;
            const int parts = 1 << lp, len = (M + parts - 1) >> lp;
            for (int i0 = 0; i0 < M; i0 += NT >> lp) {
                const int ii = i0 + (tid >> lp), part2 = tid & (parts - 1);
                const u64 mine = ii < M ? list[ii] : ~0ull;
                int rank = 0;
                for (int j = part2 * len; j < min(M, (part2 + 1) * len); ++j) rank += list[j] > mine;
                if (parts >= 2) rank += (int)dpp_u32<0xB1>((uint32_t)rank);
                if (parts >= 4) rank += (int)dpp_u32<0x4E>((uint32_t)rank);
                if (parts >= 8) rank += (int)dpp_u32<0x141>((uint32_t)rank);
                if (parts >= 16) rank += (int)dpp_u32<0x140>((uint32_t)rank);
                if (parts >= 32) rank += __shfl_xor(rank, 16);
                if (parts >= 64) rank += __shfl_xor(rank, 32);
                if (part2 == 0 && ii < M && rank < k) sel[rank] = mine;
            }
        }
    } else {
        __syncthreads();  // (sh initialised)
    }
    if (!listed) {  // (workgroup-uniform)
        const u64 idmask = (1ull << nb) - 1ull;
        u64 prefix = 0ull, known = 0ull;
        int kk = k;
        for (int sft = ((32 + nb - 1) / 8) * 8; sft >= 0; sft -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int t = tid; t < n; t += NT) {
                const u64 cc = comp[t];
                const u64 pk = ((cc >> 32) << nb) | (cc & idmask);
                if ((pk & known) == prefix) atomicAdd(&hist[(int)((pk >> sft) & 255ull)], 1);
            }
            __syncthreads();
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
            __syncthreads();
            if (tid < 256) {
                for (int w2 = 0; w2 < wave; ++w2) incl += hist[256 + w2];
                const int excl = incl - h;
                if (incl >= kk && excl < kk) {
                    sh.tau = prefix | ((u64)(255 - tid) << sft);
                    sh.M2 = kk - excl;
                }
            }
            __syncthreads();
            prefix = sh.tau;
            kk = sh.M2;
            known |= 255ull << sft;
            __syncthreads();
        }
        // prefix = packed composite of the k-th largest; everything at or above it wins
        for (int t = tid; t < n; t += NT) {
            const u64 cc = comp[t];
            const u64 pk = ((cc >> 32) << nb) | (cc & idmask);
            if (pk >= prefix) sel[atomicAdd(&sh.W, 1)] = cc;
        }
    }
    __syncthreads();
}

__host__ __device__ inline size_t align16(size_t x) { return (x + 15) & ~(size_t)15; }

}  // namespace

// LDS carve-up (bytes), shared by host and device
struct HierLds {
    size_t comp1, member, comp2, list, hist, sel1, sel2, red, total;
};
__host__ __device__ inline HierLds hier_lds(int Cpad, int max_pages, int n_probe, int P, int G, int NW) {
    HierLds L;
    size_t off = 0;
    L.comp1 = off;  off += align16((size_t)Cpad * 8);
    L.member = off; off += align16((size_t)(Cpad / 32 + 1) * 4);
    L.comp2 = off;  off += align16((size_t)max_pages * 8);
    L.list = off;   off += (size_t)kListCap * 8;
    L.hist = off;   off += (256 + 16) * 4;
    L.sel1 = off;   off += align16((size_t)n_probe * 8);
    L.sel2 = off;   off += align16((size_t)P * 8);
    L.red = off;    off += align16(sizeof(float) * (size_t)attend_scratch_floats(G, NW));
    L.total = off;
    return L;
}

template <int G, int NW>
__global__ __launch_bounds__(NW * 64) void decode_hier_kernel(Dev d, const bf16_t *__restrict__ q, int cur, int P, int n_probe,
                                                               int *__restrict__ ids_out, int *__restrict__ n_sel_out,
                                                               float *__restrict__ scores_out, int *__restrict__ clusters_out,
                                                               float *__restrict__ out) {
    constexpr int NT = NW * 64;
    extern __shared__ __align__(16) char smem[];
    __shared__ SelShared sh;
    __shared__ int sh_ncand;
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    const HierLds L = hier_lds(d.Cpad, d.max_pages, n_probe, P, G, NW);
    u64 *comp1 = (u64 *)(smem + L.comp1);
    uint32_t *member = (uint32_t *)(smem + L.member);
    u64 *comp2 = (u64 *)(smem + L.comp2);
    u64 *list = (u64 *)(smem + L.list);
    int *hist = (int *)(smem + L.hist);
    u64 *sel1 = (u64 *)(smem + L.sel1);
    u64 *sel2 = (u64 *)(smem + L.sel2);
    float *red = (float *)(smem + L.red);

    const int np = d.n_pages[u];
    const int C = d.C;
    // the query operand of every scoring MFMA, and 1/||q_h|| where the scores land
    bf16x8 qa[4];
    float inv[4];
    {
        float nn;
        load_query_operand<G>(q, u, lane, qa, &nn);
        nn += __shfl_xor(nn, 16);
        nn += __shfl_xor(nn, 32);  // ||q_h||^2 on every lane with lane%16 == h
        const float invn = 1.0f / fmaxf(sqrtf(nn), 1e-20f);
#pragma unroll
        for (int v = 0; v < 4; ++v) inv[v] = __shfl(invn, (4 * g + v) & 15);
    }
    // group score of the 16 rows a wave just multiplied: valid on the lanes of row group 0
    auto group_score = [&](const f32x4 &acc) {
        float sc = -INFINITY;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (4 * g + v < G) sc = fmaxf(sc, acc[v] * inv[v]);
        if (G > 4) sc = fmaxf(sc, __shfl_xor(sc, 16));
        return sc;
    };
    for (int i = tid; i < d.Cpad / 32 + 1; i += NT) member[i] = 0u;
    if (tid == 0) sh_ncand = 0;

    // ---- stage 1: centroid scores, 16 centroids per MFMA chain (rows of C..Cpad are padding)
    {
        const bf16_t *cb = d.cent_bf16[cur] + (size_t)u * d.Cpad * kD;
        const int nblk = d.Cpad >> 4;
        for (int b = wave; b < nblk; b += NW) {
            const int c = 16 * b + ch;
            const uint4 *src = (const uint4 *)(cb + (size_t)c * kD);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks], __builtin_bit_cast(bf16x8, src[ks * 4 + g]), acc, 0, 0, 0);
            const float sc = group_score(acc);
            if (g == 0 && c < C) comp1[c] = ((u64)f32_ordered(sc) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)c);
        }
    }
    __syncthreads();
    const int n_keep = min(n_probe, C);
    if (n_keep == C) {
        for (int c = tid; c < C; c += NT) sel1[c] = comp1[c];
        __syncthreads();
    } else {
        int nb = 0;
        while ((1 << nb) < C) ++nb;
        select_topk_lds<NW>(comp1, C, n_keep, nb, sel1, list, hist, sh);
    }
    // kept clusters: bitmask for stage 2, and the optional ascending id list
    for (int t = tid; t < n_keep; t += NT) {
        const uint32_t c = 0xFFFFFFFFu - (uint32_t)sel1[t];
        atomicOr(&member[c >> 5], 1u << (c & 31));
    }
    if (clusters_out) {
        int *co = clusters_out + (size_t)u * n_probe;
        for (int t = tid; t < n_probe; t += NT) {
            if (t < n_keep) {
                const uint32_t myc = 0xFFFFFFFFu - (uint32_t)sel1[t];
                int pos = 0;
                for (int j = 0; j < n_keep; ++j) pos += (0xFFFFFFFFu - (uint32_t)sel1[j]) < myc;
                co[pos] = (int)myc;
            } else {
                co[t] = -1;
            }
        }
    }
    __syncthreads();

    // ---- stage 2a: the live pages of the kept clusters, in any order, ids in the low words of comp2
    {
        const int *pc = d.page_cluster + (size_t)u * d.max_pages;
        for (int p0 = 0; p0 < np; p0 += NT) {
            const int p = p0 + tid;
            const int c = p < np ? pc[p] : -1;
            const bool is = c >= 0 && c < C && ((member[c >> 5] >> (c & 31)) & 1u);
            const u64 bal = __ballot(is);
            int base = 0;
            if (lane == 0 && bal) base = atomicAdd(&sh_ncand, (int)__popcll(bal));
            base = __shfl(base, 0);
            if (is) comp2[base + (int)__popcll(bal & ((1ull << lane) - 1ull))] = (u64)(uint32_t)p;
        }
    }
    __syncthreads();
    const int ncand = sh_ncand;
    // ---- stage 2b: their representatives' scores, 16 candidates per MFMA chain (gathered rows)
    {
        const bf16_t *rep = d.rep + (size_t)u * d.max_pages * kD;
        const int nblk = (ncand + 15) >> 4;
        for (int b = wave; b < nblk; b += NW) {
            const int j = 16 * b + ch;
            const uint32_t p = j < ncand ? (uint32_t)comp2[j] : 0u;  // (page 0 stands in past the end; its score is dropped)
            const uint4 *src = (const uint4 *)(rep + (size_t)p * kD);
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[ks], __builtin_bit_cast(bf16x8, src[ks * 4 + g]), acc, 0, 0, 0);
            const float sc = group_score(acc);
            __builtin_amdgcn_wave_barrier();  // every lane has read its page id before the entries change
            if (g == 0 && j < ncand) comp2[j] = ((u64)f32_ordered(sc) << 32) | (u64)(0xFFFFFFFFu - p);
        }
    }
    __syncthreads();
    const int k = min(P, ncand);
    int *ids = ids_out + (size_t)u * P;
    float *sco = scores_out ? scores_out + (size_t)u * P : nullptr;
    for (int x = k + tid; x < P; x += NT) {
        ids[x] = -1;
        if (sco) sco[x] = 0.f;
    }
    if (tid == 0) n_sel_out[u] = k;
    if (k == ncand) {
        for (int x = tid; x < k; x += NT) sel2[x] = comp2[x];
        __syncthreads();
    } else {
        int nb = 0;
        while ((1 << nb) < d.max_pages) ++nb;
        select_topk_lds<NW>(comp2, ncand, k, nb, sel2, list, hist, sh);
    }
    // the winners' places in ascending id order; during the attention it runs where the first
    // waves would wait for the last ones
    auto order_ids = [&] {
        for (int t = tid; t < k; t += NT) {
            const u64 mine = sel2[t];
            const uint32_t myid = 0xFFFFFFFFu - (uint32_t)mine;
            int pos = 0;
            for (int j = 0; j < k; ++j) pos += (0xFFFFFFFFu - (uint32_t)sel2[j]) < myid;
            ids[pos] = (int)myid;
            if (sco) sco[pos] = ordered_f32((uint32_t)(mine >> 32));
        }
    };
    if (out) attend_pages<G, NW>(d, u, qa, [=](int x) { return (int)(0xFFFFFFFFu - (uint32_t)sel2[x]); }, k, out, red, order_ids);
    else order_ids();
}

size_t decode_hier_lds_bytes(const Dev &d, int P, int n_probe) {
    const int NW = d.G == 8 ? 8 : 16;
    return hier_lds(d.Cpad, d.max_pages, n_probe, P, d.G, NW).total;
}

void launch_decode_hier(const Dev &d, const bf16_t *q, int cur, int P, int n_probe, int *ids, int *n_sel, float *scores_out,
                        int *clusters_out, float *out, hipStream_t st) {
    const size_t lds = decode_hier_lds_bytes(d, P, n_probe);
#define ICE_HIER(g, nw)                                                                                              \
    do {                                                                                                             \
        (void)hipFuncSetAttribute((const void *)decode_hier_kernel<g, nw>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        hipLaunchKernelGGL((decode_hier_kernel<g, nw>), dim3(d.U), dim3(nw * 64), lds, st, d, q, cur, P, n_probe, ids, n_sel, \
                           scores_out, clusters_out, out);                                                           \
    } while (0)
    switch (d.G) {
        case 1: ICE_HIER(1, 16); break;
        case 2: ICE_HIER(2, 16); break;
        case 4: ICE_HIER(4, 16); break;
        default: ICE_HIER(8, 8); break;
    }
#undef ICE_HIER
}

}  // namespace ice
