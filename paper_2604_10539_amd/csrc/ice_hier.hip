// Hierarchical page selection: the two-level form of the paper's top-down search (Sec. 3.3,
// Alg. 4: descend level by level from the parents that score best to their children; Alg. 3,
// page selection, calls it).  One launch, one workgroup
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
    int M, W, M2, A;
    uint32_t pre;
    u64 tau;
    uint32_t rowmax[64];
};

// Exact top-k of n distinct 64-bit composites (ordered score << 32 | ~id) held in LDS, into
// sel[0..k) (in no particular order); requires
// 1 <= k < n.  First a 32-bit threshold that at least k keys reach, and few more:
//   k <= 2*NW  the k-th largest of the 4*NW sixteen-lane row maxima, element j belonging to row
//              j mod 4*NW (so short arrays still spread over every row);
//   else       the 16-bit key prefix of the k-th largest key, from two 8-bit LDS histograms.
// What passes goes to a short list that is ranked by counting; with the prefix threshold only the
// keys that share the prefix are listed (those above it are winners as they are, and the
// histograms say how many of the listed ones are still needed), so the list stays a handful of
// entries however large k is.  If the list overflows, an 8-bit-per-pass radix select over LDS
// histograms runs on the whole array instead.  `nb` = bits of
// the id field that can be set.  hist: 2 x 272 ints.  Every thread of the workgroup must call it;
// it ends with a barrier.
template <int NW>
__device__ void select_topk_lds(const u64 *comp, int n, int k, int nb, u64 *sel, u64 *list, int *hist, SelShared &sh) {
    constexpr int NT = NW * 64, NR = 4 * NW;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) { sh.M = 0; sh.W = 0; sh.A = 0; sh.pre = 0u; sh.tau = 0ull; }
    const bool by_prefix = k > NR / 2;
    if (!by_prefix) {
        const int row = tid >> 4, l16 = tid & 15;
        uint32_t lmax = 0u;
        for (int j = row + NR * l16; j < n; j += NR * 16) lmax = max(lmax, (uint32_t)(comp[j] >> 32));
        lmax = row16_max_u32(lmax);
        if (l16 == 0) sh.rowmax[row] = lmax;
        __syncthreads();
        const uint32_t v = sh.rowmax[row];
        uint32_t c = 0;
#pragma unroll
        for (int jj = 0; jj < NR / 16; ++jj) {
            const int j = l16 * (NR / 16) + jj;
            const uint32_t o = sh.rowmax[j];
            c += (o > v || (o == v && j < row)) ? 1u : 0u;
        }
        c = row16_sum_u32(c);
        if (l16 == 0 && (int)c == k - 1) sh.pre = v;
    } else {
        // bucket of the k-th largest key by its top byte, then by its second byte inside that bucket
        int *h0 = hist, *h1 = hist + 272;
        if (tid < 256) { h0[tid] = 0; h1[tid] = 0; }
        __syncthreads();
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
            __syncthreads();
            if (tid < 256) {
                for (int w2 = 0; w2 < wave; ++w2) incl += h[256 + w2];
                const int excl = incl - mine;
                if (incl >= kk && excl < kk) {  // exactly one bin
                    sh.pre |= (uint32_t)(255 - tid) << shift;
                    sh.M2 = kk - excl;
                }
            }
            __syncthreads();
        };
        // (the top byte is sign and exponent: most keys of a wave share it, so the lanes that agree
        // with the first active lane are counted with one update)
        for (int j0 = 0; j0 < n; j0 += NT) {
            const int j = j0 + tid;
            const int bin = j < n ? (int)(comp[j] >> 56) : -1;
            const u64 act = __ballot(bin >= 0);
            if (act == 0ull) continue;  // (wave-uniform)
            const int first_bin = __shfl(bin, (int)__builtin_ctzll(act));
            const u64 same = __ballot(bin == first_bin);
            if (lane == (int)__builtin_ctzll(act)) atomicAdd(&h0[first_bin], (int)__popcll(same));
            if (bin >= 0 && bin != first_bin) atomicAdd(&h0[bin], 1);
        }
        __syncthreads();
        find_bucket(h0, k, 24);
        const uint32_t top = sh.pre >> 24;
        const int k2 = sh.M2;
        for (int j = tid; j < n; j += NT) {
            const uint32_t key = (uint32_t)(comp[j] >> 32);
            if ((key >> 24) == top) atomicAdd(&h1[(int)((key >> 16) & 255u)], 1);
        }
        __syncthreads();
        find_bucket(h1, k2, 16);
    }
    __syncthreads();
    const uint32_t pre = sh.pre;
    // With the prefix threshold: keys above the prefix are winners (k - need of them, need = what
    // the histograms left for the prefix's own bucket) and go straight to sel; the bucket is listed.
    // With the row-maxima threshold: everything at or above it is listed (>= k entries).
    const int need = by_prefix ? sh.M2 : k, first = k - need;
    for (int j0 = 0; j0 < n; j0 += NT) {
        const int j = j0 + tid;
        const u64 cc = j < n ? comp[j] : 0ull;
        const uint32_t key = (uint32_t)(cc >> 32);
        const bool above = j < n && by_prefix && (key >> 16) > (pre >> 16);
        const bool is = j < n && key >= pre && !above;
        const u64 bal = __ballot(is), bal_a = __ballot(above);
        int base = 0, base_a = 0;
        if (lane == 0 && bal) base = atomicAdd(&sh.M, (int)__popcll(bal));
        if (lane == 0 && bal_a) base_a = atomicAdd(&sh.A, (int)__popcll(bal_a));
        base = __shfl(base, 0);
        base_a = __shfl(base_a, 0);
        const u64 lower = (1ull << lane) - 1ull;
        const int slot = base + (int)__popcll(bal & lower);
        if (is && slot < kListCap) list[slot] = cc;
        if (above) sel[base_a + (int)__popcll(bal_a & lower)] = cc;  // (exactly `first` of them)
    }
    __syncthreads();
    const int M = sh.M;
    const bool listed = M <= kListCap;
    if (listed) {
        // every listed composite counts the listed composites that beat it
        int lp = 0;
        while (lp < 6 && (M << (lp + 1)) <= NT) ++lp;
        const int parts = 1 << lp, len = (M + parts - 1) >> lp;
        for (int i0 = 0; i0 < M; i0 += NT >> lp) {
            const int ii = i0 + (tid >> lp), part2 = tid & (parts - 1);
            const u64 mine = ii < M ? list[ii] : ~0ull;
            int rank = 0;
#pragma unroll 8
            for (int j = part2 * len; j < min(M, (part2 + 1) * len); ++j) rank += list[j] > mine;
            if (parts >= 2) rank += (int)dpp_u32<0xB1>((uint32_t)rank);
            if (parts >= 4) rank += (int)dpp_u32<0x4E>((uint32_t)rank);
            if (parts >= 8) rank += (int)dpp_u32<0x141>((uint32_t)rank);
            if (parts >= 16) rank += (int)dpp_u32<0x140>((uint32_t)rank);
            if (parts >= 32) rank += __shfl_xor(rank, 16);
            if (parts >= 64) rank += __shfl_xor(rank, 32);
            if (part2 == 0 && ii < M && rank < need) sel[first + rank] = mine;
        }
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
    size_t comp1, member, comp2, list, hist, sel1, sel2, comp3, sel3, red, total;
};
__host__ __device__ inline HierLds hier_lds(int Cpad, int max_pages, int n_probe, int n_refine, int P, int G, int NW) {
    HierLds L;
    size_t off = 0;
    L.comp1 = off;  off += align16((size_t)Cpad * 8);
    L.member = off; off += align16((size_t)(Cpad / 32 + 1) * 4);
    L.comp2 = off;  off += align16((size_t)max_pages * 8);
    L.list = off;   off += (size_t)kListCap * 8;
    L.hist = off;   off += 2 * 272 * 4;
    // (lists are as long as what can be kept: at most every cluster, at most every page)
    const int n_keep = n_probe < Cpad ? n_probe : Cpad, Pk = P < max_pages ? P : max_pages;
    const int n_ref = n_refine < max_pages ? n_refine : max_pages;
    L.sel1 = off;   off += align16((size_t)n_keep * 8);
    L.sel2 = off;   off += align16((size_t)(n_ref > Pk ? n_ref : Pk) * 8);
    L.comp3 = off;  off += align16((size_t)n_ref * 8);
    L.sel3 = off;   off += align16((size_t)Pk * 8);
    L.red = off;    off += align16(sizeof(float) * (size_t)attend_scratch_floats(G, NW));
    L.total = off;
    return L;
}

// (The leading scalar arguments are those needed before the first loads: they are preloaded into
// scalar registers at wave start; cent_all = the centroid rows in use.)
// TOP: three levels (a stage in front that ranks the top nodes; compiled apart so that the two-level
// instantiations keep their register budget).
template <int G, int NW, int EMAX, bool TOP>
__global__ __launch_bounds__(NW * 64) void decode_hier_kernel(int Cpad, int max_pages, int np_hint, int P, int n_probe, int n_refine,
                                                               const bf16_t *__restrict__ cent_all, const bf16_t *__restrict__ q,
                                                               const int *__restrict__ page_cluster, const int *__restrict__ n_pages, Dev d,
                                                               int *__restrict__ ids_out, int *__restrict__ n_sel_out,
                                                               float *__restrict__ scores_out, int *__restrict__ clusters_out,
                                                               float *__restrict__ out, int n_top, int n_probe_top,
                                                               int *__restrict__ tops_out) {
    constexpr int NT = NW * 64;
    extern __shared__ __align__(16) char smem[];
    __shared__ SelShared sh;
    __shared__ int sh_ncand;
    __shared__ u64 comp0[TOP ? kTopMax : 1], sel0[TOP ? kTopMax : 1];  // three levels: the top nodes' composites, the kept ones
    __shared__ uint32_t member0[kTopMax / 32];
    const int u = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int g = lane >> 4, ch = lane & 15;
    const HierLds L = hier_lds(Cpad, max_pages, n_probe, n_refine, P, G, NW);
    u64 *comp1 = (u64 *)(smem + L.comp1);
    uint32_t *member = (uint32_t *)(smem + L.member);
    u64 *comp2 = (u64 *)(smem + L.comp2);
    u64 *list = (u64 *)(smem + L.list);
    int *hist = (int *)(smem + L.hist);
    u64 *sel1 = (u64 *)(smem + L.sel1);
    u64 *sel2 = (u64 *)(smem + L.sel2);
    u64 *comp3 = (u64 *)(smem + L.comp3);
    u64 *sel3 = (u64 *)(smem + L.sel3);
    float *red = (float *)(smem + L.red);

    ICE_HSTAMP(0);
    const int np = n_pages[u];  // first needed in stage 2
    const int C = d.C;
    // the page -> cluster table is requested now and used in stage 2; np_hint is the host's upper
    // bound of the live pages (entries past the live pages are read and ignored)
    int pcl[EMAX];
    {
        const int *pc = page_cluster + (size_t)u * max_pages;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) pcl[e] = e * NT + tid < np_hint ? pc[e * NT + tid] : -1;
    }
    // ---- stage 1 loads: 16 centroids per four MFMAs in the split-row form (SplitRow: whole
    // 128-byte lines per load instruction), four such blocks in flight per wave (rows of C..Cpad
    // are padding).  The first round is requested together with the query rows, before anything
    // waits for either.
    using SR = SplitRow<G>;
    const bf16_t *cb = cent_all + (size_t)u * Cpad * kD;
    const int nblk1 = Cpad >> 4;
    constexpr int UNR1 = 4;
    uint4 bb1[UNR1][4];
    int word[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) word[j] = SR::word(lane, j >> 1, j & 1);
    auto request1 = [&](int b0) {
#pragma unroll
        for (int x = 0; x < UNR1; ++x) {
            const int c0 = 16 * (b0 + NW * x);  // (Cpad is a multiple of 16: a block is there or not)
            const uint4 *src = (const uint4 *)(cb + (size_t)c0 * kD);
#pragma unroll
            for (int j = 0; j < 4; ++j) bb1[x][j] = c0 < Cpad ? load16_stream(src + word[j]) : make_uint4(0, 0, 0, 0);
        }
    };
    if constexpr (!TOP) request1(wave);
    // the query operand of every scoring MFMA, and 1/||q_h|| where the scores land
    bf16x8 qs[2];
    float inv[4];
    {
        float invn;
        SR::load_query(q, u, lane, qs, &invn);
#pragma unroll
        for (int v = 0; v < 4; ++v) inv[v] = __shfl(invn, (4 * SR::head_group(lane) + v) & 15);
    }
    const bool owner = SR::owner(lane);
    // group scores of 16 rows whose loads are bw[0..3] (SplitRow::word order): valid on the owner
    // lanes, lane (.., c) for row c
    auto group_score = [&](const uint4 (&bw)[4]) {
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qs[t], __builtin_bit_cast(bf16x8, bw[t]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qs[t], __builtin_bit_cast(bf16x8, bw[2 + t]), acc1, 0, 0, 0);
        }
        return SR::score(acc0, acc1, inv, lane);
    };
    for (int i = tid; i < Cpad / 32 + 1; i += NT) member[i] = 0u;
    if (tid < kTopMax / 32) member0[tid] = 0u;
    if (tid == 0) sh_ncand = 0;
    // Scores of `cnt` rows gathered through a list (16 per block: lanes c and c+8 read the two halves
    // of a line of row 8*blk + c%8; two blocks in flight per wave).  lst[j] holds row id j in its low
    // word and is overwritten by the row's composite (ordered score, lower id first).
    auto score_listed = [&](const bf16_t *rows, u64 *lst, int cnt) {
        const int nblk = (cnt + 15) >> 4;
        constexpr int UNR = 2;
        const int piece = 4 * ((ch >> 3) & 1) + g;  // uint4 inside the 128-byte line
        for (int b0 = wave; b0 < nblk; b0 += NW * UNR) {
            uint4 bb[UNR][4];
            uint32_t rid[UNR];
#pragma unroll
            for (int x = 0; x < UNR; ++x) {
                const int j0 = 16 * (b0 + NW * x), j = j0 + ch;
                rid[x] = j < cnt ? (uint32_t)lst[j] : 0u;  // (row 0 stands in past the end; its score is dropped)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    const int jr = j0 + 8 * blk + (ch & 7);
                    const uint32_t rr = jr < cnt ? (uint32_t)lst[jr] : 0u;
                    const uint4 *src = (const uint4 *)(rows + (size_t)rr * kD);
                    bb[x][2 * blk] = load16_stream(src + piece);
                    bb[x][2 * blk + 1] = load16_stream(src + 8 + piece);
                }
            }
            __builtin_amdgcn_wave_barrier();  // every lane has read its row ids before the entries change
#pragma unroll
            for (int x = 0; x < UNR; ++x) {
                const int j = 16 * (b0 + NW * x) + ch;
                const float sc = group_score(bb[x]);
                if (owner && j < cnt) lst[j] = ((u64)f32_ordered(sc) << 32) | (u64)(0xFFFFFFFFu - rid[x]);
            }
        }
    };

    int n_keep, n_keep0 = 0;
    if constexpr (!TOP) {
        // ---- stage 1: centroid scores
        for (int b0 = wave; b0 < nblk1;) {
#pragma unroll
            for (int x = 0; x < UNR1; ++x) {
                if (b0 + NW * x >= nblk1) break;  // (wave-uniform)
                const int c = 16 * (b0 + NW * x) + ch;
                const float sc = group_score(bb1[x]);
                if (owner && c < C) comp1[c] = ((u64)f32_ordered(sc) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)c);
            }
            b0 += NW * UNR1;
            if (b0 < nblk1) request1(b0);
        }
        __syncthreads();
        ICE_HSTAMP(1);
        n_keep = min(n_probe, C);
        if (n_keep == C) {
            for (int c = tid; c < C; c += NT) sel1[c] = comp1[c];
            __syncthreads();
        } else {
            int nb = 0;
            while ((1 << nb) < C) ++nb;
            select_topk_lds<NW>(comp1, C, n_keep, nb, sel1, list, hist, sh);
        }
    } else {
        // ---- stage 0 (three levels): scores of the top nodes, 16 rows per block as in stage 1
        const bf16_t *tb = d.top_bf16 + (size_t)u * kTopMax * kD;
        for (int b0 = wave; 16 * b0 < n_top; b0 += NW) {
            uint4 bw[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) bw[j] = load16_stream((const uint4 *)(tb + (size_t)16 * b0 * kD) + word[j]);
            const int t = 16 * b0 + ch;
            const float sc = group_score(bw);
            if (owner && t < n_top) comp0[t] = ((u64)f32_ordered(sc) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)t);
        }
        __syncthreads();
        n_keep0 = min(n_probe_top, n_top);
        if (n_keep0 == n_top) {
            for (int t = tid; t < n_top; t += NT) sel0[t] = comp0[t];
            __syncthreads();
        } else {
            int nb0 = 0;
            while ((1 << nb0) < n_top) ++nb0;
            select_topk_lds<NW>(comp0, n_top, n_keep0, nb0, sel0, list, hist, sh);
        }
        for (int t = tid; t < n_keep0; t += NT) {
            const uint32_t tn = 0xFFFFFFFFu - (uint32_t)sel0[t];
            atomicOr(&member0[tn >> 5], 1u << (tn & 31));
        }
        __syncthreads();
        // the clusters hanging under the kept nodes, in any order, ids in the low words of comp1
        const int *tof = d.top_of + (size_t)u * C;
        for (int c0 = 0; c0 < C; c0 += NT) {
            const int c = c0 + tid;
            const int tn = c < C ? tof[c] : -1;
            const bool is = tn >= 0 && tn < n_top && ((member0[tn >> 5] >> (tn & 31)) & 1u);
            const u64 bal = __ballot(is);
            int base = 0;
            if (lane == 0 && bal) base = atomicAdd(&sh_ncand, (int)__popcll(bal));
            base = __shfl(base, 0);
            if (is) comp1[base + (int)__popcll(bal & ((1ull << lane) - 1ull))] = (u64)(uint32_t)c;
        }
        __syncthreads();
        const int ncl = sh_ncand;
        __syncthreads();
        if (tid == 0) sh_ncand = 0;  // (counts the candidate pages next)
        // ---- stage 1: scores of those clusters' centroids
        score_listed(cb, comp1, ncl);
        __syncthreads();
        ICE_HSTAMP(1);
        n_keep = min(n_probe, ncl);
        if (n_keep == ncl) {
            for (int c = tid; c < ncl; c += NT) sel1[c] = comp1[c];
            __syncthreads();
        } else {
            int nb = 0;
            while ((1 << nb) < C) ++nb;
            select_topk_lds<NW>(comp1, ncl, n_keep, nb, sel1, list, hist, sh);
        }
    }
    ICE_HSTAMP(2);
    // kept clusters: bitmask for stage 2 (their ascending id list is written later, off the critical path)
    for (int t = tid; t < n_keep; t += NT) {
        const uint32_t c = 0xFFFFFFFFu - (uint32_t)sel1[t];
        atomicOr(&member[c >> 5], 1u << (c & 31));
    }
    __syncthreads();

    ICE_HSTAMP(3);
    // ---- stage 2a: the live pages of the kept clusters, in any order, ids in the low words of comp2
    {
        u64 bal[EMAX];
        int tot = 0;
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            const int p = e * NT + tid, c = pcl[e];
            bal[e] = __ballot(p < np && c >= 0 && c < C && ((member[c >> 5] >> (c & 31)) & 1u));
            tot += (int)__popcll(bal[e]);
        }
        int base = 0;
        if (lane == 0 && tot) base = atomicAdd(&sh_ncand, tot);
        base = __shfl(base, 0);
#pragma unroll
        for (int e = 0; e < EMAX; ++e) {
            if ((bal[e] >> lane) & 1ull) comp2[base + (int)__popcll(bal[e] & ((1ull << lane) - 1ull))] = (u64)(uint32_t)(e * NT + tid);
            base += (int)__popcll(bal[e]);
        }
    }
    __syncthreads();
    const int ncand = sh_ncand;
    ICE_HSTAMP(4);
    // ---- stage 2b: their representatives' scores
    score_listed(d.rep + (size_t)u * d.max_pages * kD, comp2, ncand);
    __syncthreads();
    ICE_HSTAMP(5);
    // how many pages stage 2 keeps: P, or n_refine of which stage 3 then keeps P
    const int k2 = min(n_refine > 0 ? n_refine : P, ncand);
    int k = min(P, k2);
    int *ids = ids_out + (size_t)u * P;
    float *sco = scores_out ? scores_out + (size_t)u * P : nullptr;
    for (int x = k + tid; x < P; x += NT) {
        ids[x] = -1;
        if (sco) sco[x] = 0.f;
    }
    if (tid == 0) n_sel_out[u] = k;
    int nb = 0;
    while ((1 << nb) < d.max_pages) ++nb;
    if (k2 == ncand) {
        for (int x = tid; x < k2; x += NT) sel2[x] = comp2[x];
        __syncthreads();
    } else {
        select_topk_lds<NW>(comp2, ncand, k2, nb, sel2, list, hist, sh);
    }
    const u64 *win = sel2;  // the winners, as composites
    if (n_refine > 0) {
        // ---- stage 3: the kept pages re-scored by their best key (the paper ranks keys and loads the
        // pages that hold them, Alg. 3): one wave per page, logits of 16 tokens per MFMA chain as in the
        // attention, normalised like the page scores, maximum over heads and live tokens
        const int s = d.s;
        constexpr int UNR3 = 4;  // pages whose first blocks are in flight per wave
        for (int x0 = wave; x0 < k2; x0 += NW * UNR3) {
            uint4 kb[UNR3][4];
            uint32_t pp[UNR3];
            int fl[UNR3];
#pragma unroll
            for (int y = 0; y < UNR3; ++y) {
                const int x = x0 + NW * y;
                pp[y] = x < k2 ? 0xFFFFFFFFu - (uint32_t)sel2[x] : 0u;  // (page 0 stands in past the end)
                const size_t pg = (size_t)u * d.max_pages + pp[y];
#pragma unroll
                for (int t = 0; t < 4; ++t) kb[y][t] = ((const uint4 *)(d.Kp + pg * s * kD))[word[t]];
                fl[y] = d.page_fill[pg];
            }
#pragma unroll
            for (int y = 0; y < UNR3; ++y) {
                const int x = x0 + NW * y;
                const size_t pg = (size_t)u * d.max_pages + pp[y];
                float best = -INFINITY;
                for (int b0 = 0; b0 < fl[y]; b0 += 16) {
                    if (b0 > 0) {
#pragma unroll
                        for (int t = 0; t < 4; ++t) kb[y][t] = ((const uint4 *)(d.Kp + (pg * s + b0) * kD))[word[t]];
                    }
                    const float sc = group_score(kb[y]);   // token b0 + ch, on the owner lanes
                    if (owner && b0 + ch < fl[y]) best = fmaxf(best, sc);
                }
                best = fmaxf(best, dpp_f32<0xB1>(best));
                best = fmaxf(best, dpp_f32<0x4E>(best));
                best = fmaxf(best, dpp_f32<0x141>(best));
                best = fmaxf(best, dpp_f32<0x140>(best));
                best = fmaxf(best, __shfl_xor(best, 16));  // (the owners sit in two row groups)
                best = fmaxf(best, __shfl_xor(best, 32));
                if (lane == 0 && x < k2) comp3[x] = ((u64)f32_ordered(best) << 32) | (u64)(0xFFFFFFFFu - pp[y]);
            }
        }
        __syncthreads();
        if (k == k2) {
            for (int x = tid; x < k; x += NT) sel3[x] = comp3[x];
            __syncthreads();
        } else {
            select_topk_lds<NW>(comp3, k2, k, nb, sel3, list, hist, sh);
        }
        win = sel3;
    }
    ICE_HSTAMP(6);
    // the winners' places in ascending id order; during the attention it runs where the first
    // waves would wait for the last ones
    auto order_ids = [&] {
        if (TOP && tops_out) {  // the kept top nodes, ascending
            int *to = tops_out + (size_t)u * n_probe_top;
            for (int t = tid; t < n_probe_top; t += NT) {
                if (t < n_keep0) {
                    const uint32_t mine = 0xFFFFFFFFu - (uint32_t)sel0[t];
                    int pos = 0;
                    for (int j = 0; j < n_keep0; ++j) pos += (0xFFFFFFFFu - (uint32_t)sel0[j]) < mine;
                    to[pos] = (int)mine;
                } else {
                    to[t] = -1;
                }
            }
        }
        if (clusters_out) {  // the kept clusters, ascending
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
        for (int t = tid; t < k; t += NT) {
            const u64 mine = win[t];
            const uint32_t myid = 0xFFFFFFFFu - (uint32_t)mine;
            int pos = 0;
            for (int j = 0; j < k; ++j) pos += (0xFFFFFFFFu - (uint32_t)win[j]) < myid;
            ids[pos] = (int)myid;
            if (sco) sco[pos] = ordered_f32((uint32_t)(mine >> 32));
        }
    };
    bf16x8 qa[4];
    if (out) SR::to_plain(qs, lane, qa);
    if (out) attend_pages<G, NW, false>(d, u, qa, [=](int x) { return (int)(0xFFFFFFFFu - (uint32_t)win[x]); }, k, Resident{nullptr, nullptr, 0, nullptr, nullptr, 0}, out, red, order_ids);
    else order_ids();
    ICE_HSTAMP(7);
}

size_t decode_hier_lds_bytes(const Dev &d, int P, int n_probe, int n_refine) {
    const int NW = d.G == 8 ? 8 : 16;
    return hier_lds(d.Cpad, d.max_pages, n_probe, n_refine, P, d.G, NW).total;
}

void launch_decode_hier(const Dev &d, const bf16_t *q, int cur, int P, int n_top, int n_probe_top, int n_probe, int n_refine,
                        int np_hint, int *ids, int *n_sel, float *scores_out, int *clusters_out, int *tops_out, float *out,
                        hipStream_t st) {
    const size_t lds = decode_hier_lds_bytes(d, P, n_probe, n_refine);
    const int NW = d.G == 8 ? 8 : 16;
    // few units and many pages: the attention moves to a launch of its own that spreads a unit's pages
    // over several workgroups (see attend_split_kernel)
    float *out_split = nullptr;
    if (out && launch_attend_would_split(d, P)) {
        out_split = out;
        out = nullptr;
    }
    if (np_hint > d.max_pages) np_hint = d.max_pages;
    const int E = (d.max_pages + NW * 64 - 1) / (NW * 64);
#define ICE_HIER_T(g, nw, e, top)                                                                                    \
    do {                                                                                                             \
        allow_dynamic_lds((const void *)decode_hier_kernel<g, nw, e, top>, lds);                                     \
        hipLaunchKernelGGL((decode_hier_kernel<g, nw, e, top>), dim3(d.U), dim3(nw * 64), lds, st, d.Cpad, d.max_pages, np_hint, P, \
                           n_probe, n_refine, d.cent_bf16[cur], q, d.page_cluster, d.n_pages, d, ids, n_sel, scores_out,   \
                           clusters_out, out, n_top, n_probe_top, tops_out);                                         \
    } while (0)
#define ICE_HIER(g, nw, e)                                                                                           \
    do {                                                                                                             \
        if (n_top > 0) ICE_HIER_T(g, nw, e, true);                                                                   \
        else ICE_HIER_T(g, nw, e, false);                                                                            \
    } while (0)
    if (d.G == 8) { if (E <= 8) ICE_HIER(8, 8, 8); else ICE_HIER(8, 8, 32); }
    else if (d.G == 4) { if (E <= 4) ICE_HIER(4, 16, 4); else ICE_HIER(4, 16, 16); }
    else if (d.G == 2) { if (E <= 4) ICE_HIER(2, 16, 4); else ICE_HIER(2, 16, 16); }
    else { if (E <= 4) ICE_HIER(1, 16, 4); else ICE_HIER(1, 16, 16); }
#undef ICE_HIER
#undef ICE_HIER_T
    if (out_split) launch_attend_split_after_select(d, q, ids, n_sel, P, out_split, st);
}

// largest page count per unit the kernel serves (page -> cluster entries held in registers)
int decode_hier_max_pages(int G) { return G == 8 ? 8 * 64 * 32 : 16 * 64 * 16; }

}  // namespace ice

ICE_PROF_EXPORT(ice_debug_prof_hier)
