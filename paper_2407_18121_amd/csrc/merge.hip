// ec_merge_compact / ec_remerge_compact: bucket division (Sec. 3.3, Eq. 2), cache merging
// (Eq. 3) and compaction (Alg. 1's gather) in one pass over K and V.
//
// HBM-bound: every prompt K/V row is read once, every cache row written once.
// Buckets are contiguous position ranges, so the rows of bucket j are one
// contiguous slab of memory.  A group of LPR = row_bytes/16 lanes owns bucket j:
// it derives the bucket's bounds from the three neighbouring anchors, streams the
// slab with 16-byte loads in ascending position, accumulates in fp32, divides by
// the count once and stores the row.  Neighbouring groups own neighbouring
// buckets, so a wave reads one contiguous stretch of the prompt.  Importance scores
// put most anchors next to each other and leave a few buckets of hundreds of rows:
// those are summed by all lane groups of the workgroup together.
#include "ec_common.h"

namespace ec {

constexpr int kMergeThreads = 256;
constexpr int kMergeUnroll = 8;  // rows of K and of V in flight per bucket (16 loads per lane)
constexpr int kMergeLong = 128;  // buckets with more rows are summed by the whole workgroup

// Inclusive bounds of bucket j for ascending anchors a[0..n).  Clamped so that a
// malformed anchor list can never index outside [0,T).
__device__ __forceinline__ void bucket_bounds(const int32_t* __restrict__ a, int j, int n, int T,
                                              int& lo, int& hi)
{
    const int t = a[j];
    lo = (j == 0) ? 0 : ((a[j - 1] + t) >> 1) + 1;
    hi = (j == n - 1) ? T - 1 : ((t + a[j + 1]) >> 1);
    lo = max(lo, 0);
    hi = min(hi, T - 1);
}

// WEIGHTED: every source row t carries an integer weight w_t (the number of original tokens it already
// stands for, when rows of an earlier merge are merged again); the cache row is sum w_t x_t / sum w_t
// and counts receives sum w_t.  Without it every row weighs 1 (Eq. 3).  src_rows is the distance in rows
// between the heads of k/v (>= T); src_pos, if given, maps a source row to its original position.
template <int DT, int D, bool WEIGHTED>
__global__ __launch_bounds__(kMergeThreads) void merge_compact_kernel(
    const uint4* __restrict__ k, const uint4* __restrict__ v, const int32_t* __restrict__ anchor_idx,
    const int32_t* __restrict__ weights, const int32_t* __restrict__ src_pos,
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache, int32_t* __restrict__ counts,
    int32_t* __restrict__ assign, int32_t* __restrict__ pos, int H, int G, int T_max, int src_rows, int n_max,
    int cap, int evict_only, const int32_t* __restrict__ seq_len, const int32_t* __restrict__ n_anchor_b)
{
    constexpr int LPR = D * Elem<DT>::kBytes / 16;
    constexpr int EPL = Elem<DT>::kPerChunk;
    constexpr int GROUPS = kMergeThreads / LPR;
    __shared__ int sh_nlong;
    __shared__ int sh_long[GROUPS];
    __shared__ int sh_wsum[GROUPS];
    __shared__ float sh_part[GROUPS][LPR * EPL * 2];

    const int bh = blockIdx.y;
    const int b = bh / H, h = bh % H;
    const int tid = threadIdx.x;
    const int sub = tid % LPR, grp = tid / LPR;
    // Long and short buckets sit at the same chunk numbers in every head, and workgroups go to the 8
    // XCDs round-robin by linear id: rotating the chunk number by the head index keeps the heavy chunks
    // from piling onto the same XCDs.
    const int chunk = (blockIdx.x + blockIdx.y) % gridDim.x;
    const int j = chunk * GROUPS + grp;
    // ragged batches: batch element b has T positions and n_anchor anchors; array rows stay T_max / n_max apart
    const int T = ragged_rows(seq_len, b, T_max);
    const int n_anchor = n_anchor_b ? min(max(n_anchor_b[b], 0), min(T, n_max)) : n_max;
    if (chunk * GROUPS >= n_anchor) return;  // whole workgroup
    const bool valid = j < n_anchor;

    const size_t bg = (size_t)b * G + (G == 1 ? 0 : h);
    const int32_t* a = anchor_idx + bg * n_max;
    const int32_t* wrow = WEIGHTED ? weights + bg * T_max : nullptr;
    const bool owner = (G == H || h == 0);  // writes the bookkeeping of its score group
    // K and V of a bucket are streamed side by side: two independent load streams per lane
    const uint4* src_k = k + (size_t)bh * src_rows * LPR + sub;
    const uint4* src_v = v + (size_t)bh * src_rows * LPR + sub;

    float acc_k[EPL], acc_v[EPL];
    int wsum;
    // rows first, first + step, ... <= hi of one bucket; `whole` = this group sums the bucket alone
    auto stream = [&](int first, int hi, int step, bool whole) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc_k[e] = acc_v[e] = 0.f;
        wsum = 0;
        // a bucket of one row is copied (weight 1 whatever it carries), so it stays bit-exact
        const bool use_w = WEIGHTED && !(whole && first == hi);
        for (int t = first; t <= hi; t += kMergeUnroll * step) {
            uint4 ck[kMergeUnroll], cv[kMergeUnroll];
            int wt[kMergeUnroll];
#pragma unroll
            for (int u = 0; u < kMergeUnroll; ++u) {
                ck[u] = make_uint4(0, 0, 0, 0);
                cv[u] = make_uint4(0, 0, 0, 0);
                wt[u] = 1;
                const int r = t + u * step;
                if (r <= hi) {
                    if (WEIGHTED) wt[u] = max(wrow[r], 1);
                    ck[u] = load_stream(src_k + (size_t)r * LPR);
                    cv[u] = load_stream(src_v + (size_t)r * LPR);
                }
            }
#pragma unroll
            for (int u = 0; u < kMergeUnroll; ++u) {
                if (t + u * step <= hi) {
                    float xk[EPL], xv[EPL];
                    unpack<DT>(ck[u], xk);
                    unpack<DT>(cv[u], xv);
                    const bool start = (u == 0 && t == first);  // the sum starts from the first row, so a bucket
                    if (WEIGHTED) {                             // of one is a bit-exact copy (-0 stays -0)
                        wsum += wt[u];
                        const float w = use_w ? (float)wt[u] : 1.f;
#pragma unroll
                        for (int e = 0; e < EPL; ++e) {
                            acc_k[e] = start ? w * xk[e] : fmaf(w, xk[e], acc_k[e]);
                            acc_v[e] = start ? w * xv[e] : fmaf(w, xv[e], acc_v[e]);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < EPL; ++e) {
                            acc_k[e] = start ? xk[e] : acc_k[e] + xk[e];
                            acc_v[e] = start ? xv[e] : acc_v[e] + xv[e];
                        }
                    }
                }
            }
        }
    };
    // The share of one lane group in a bucket that the whole workgroup sums: rows first, first + step, ...
    // A slot is loaded again as soon as its row has been added, so the loads in flight do not drain
    // between rounds.  The additions are made in the order of stream().
    auto stream_ring = [&](int first, int hi, int step) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc_k[e] = acc_v[e] = 0.f;
        wsum = 0;
        uint4 ck[kMergeUnroll], cv[kMergeUnroll];
        int wt[kMergeUnroll];
#pragma unroll
        for (int u = 0; u < kMergeUnroll; ++u) {
            const int r = first + u * step;
            ck[u] = make_uint4(0, 0, 0, 0);
            cv[u] = make_uint4(0, 0, 0, 0);
            wt[u] = 1;
            if (r <= hi) {
                if (WEIGHTED) wt[u] = max(wrow[r], 1);
                ck[u] = load_stream(src_k + (size_t)r * LPR);
                cv[u] = load_stream(src_v + (size_t)r * LPR);
            }
        }
        for (int t = first; t <= hi; t += kMergeUnroll * step) {
#pragma unroll
            for (int u = 0; u < kMergeUnroll; ++u) {
                const int r = t + u * step;
                if (r <= hi) {
                    float xk[EPL], xv[EPL];
                    unpack<DT>(ck[u], xk);
                    unpack<DT>(cv[u], xv);
                    if (WEIGHTED) {
                        wsum += wt[u];
                        const float w = (float)wt[u];
#pragma unroll
                        for (int e = 0; e < EPL; ++e) {
                            acc_k[e] = fmaf(w, xk[e], acc_k[e]);
                            acc_v[e] = fmaf(w, xv[e], acc_v[e]);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < EPL; ++e) {
                            acc_k[e] += xk[e];
                            acc_v[e] += xv[e];
                        }
                    }
                    const int rn = r + kMergeUnroll * step;
                    if (rn <= hi) {
                        if (WEIGHTED) wt[u] = max(wrow[rn], 1);
                        ck[u] = load_stream(src_k + (size_t)rn * LPR);
                        cv[u] = load_stream(src_v + (size_t)rn * LPR);
                    }
                }
            }
        }
    };
    // divide by the count, round once, store cache row jj and its bookkeeping
    auto finish = [&](int jj, int n_rows, int w_total) {
        const int count = WEIGHTED ? w_total : n_rows;
        if (n_rows > 1) {
            const float cf = (float)count;
#pragma unroll
            for (int e = 0; e < EPL; ++e) {
                acc_k[e] = acc_k[e] / cf;
                acc_v[e] = acc_v[e] / cf;
            }
        }
        k_cache[((size_t)bh * cap + jj) * LPR + sub] = pack<DT>(acc_k);
        v_cache[((size_t)bh * cap + jj) * LPR + sub] = pack<DT>(acc_v);
        if (owner && sub == 0) {
            if (counts) counts[bg * n_max + jj] = count;
            if (pos) {
                const int t = min(max(a[jj], 0), T - 1);
                pos[bg * cap + jj] = src_pos ? src_pos[bg * T_max + t] : a[jj];
            }
        }
    };

    int lo = 0, hi = -1, blo = 0, bhi = -1;
    if (valid) {
        bucket_bounds(a, j, n_anchor, T, lo, hi);
        blo = lo;
        bhi = hi;  // the bucket, for the bookkeeping
        if (evict_only) lo = hi = min(max(a[j], 0), T - 1);  // eviction-only ablation: the anchor's own row
    }
    // Buckets of more than kMergeLong rows are left to the whole workgroup (below): one lane group would
    // stream them as a long chain of dependent loads while its neighbours sit idle.
    const bool is_long = valid && (hi - lo + 1) > kMergeLong;
    if (tid == 0) sh_nlong = 0;
    __syncthreads();
    if (is_long && sub == 0) sh_long[atomicAdd(&sh_nlong, 1)] = grp;
    __syncthreads();

    if (valid && !is_long) {
        stream(lo, hi, 1, true);
        finish(j, hi - lo + 1, wsum);
        if (owner && assign)
            for (int t = blo + sub; t <= bhi; t += LPR) assign[bg * T_max + t] = (!evict_only || t == lo) ? j : -1;
    }

    // Long buckets, one after the other: group g sums rows lo+g, lo+g+GROUPS, ...; the partial sums are
    // added in ascending group order, so the result does not depend on which bucket is taken first.
    const int n_long = sh_nlong;
    for (int i = 0; i < n_long; ++i) {
        const int jj = chunk * GROUPS + sh_long[i];
        int llo, lhi;
        bucket_bounds(a, jj, n_anchor, T, llo, lhi);
        stream_ring(llo + grp, lhi, GROUPS);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            sh_part[grp][(sub * EPL + e) * 2] = acc_k[e];
            sh_part[grp][(sub * EPL + e) * 2 + 1] = acc_v[e];
        }
        if (sub == 0) sh_wsum[grp] = wsum;
        __syncthreads();
        if (grp == 0) {
            int w_total = 0;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc_k[e] = acc_v[e] = 0.f;
            for (int g = 0; g < GROUPS; ++g) {
                w_total += sh_wsum[g];
#pragma unroll
                for (int e = 0; e < EPL; ++e) {
                    acc_k[e] += sh_part[g][(sub * EPL + e) * 2];
                    acc_v[e] += sh_part[g][(sub * EPL + e) * 2 + 1];
                }
            }
            finish(jj, lhi - llo + 1, w_total);
        }
        if (owner && assign)
            for (int t = llo + tid; t <= lhi; t += kMergeThreads) assign[bg * T_max + t] = jj;
        __syncthreads();  // the partial sums are free again
    }
}

template <int DT, int D>
static int launch_merge(const void* k, const void* v, const int32_t* anchor_idx, const int32_t* weights,
                        const int32_t* src_pos, int B, int H, int G, int T, int src_rows, int n_anchor, void* k_cache,
                        void* v_cache, int cap, int32_t* counts, int32_t* assign, int32_t* pos, int evict_only,
                        const int32_t* seq_len, const int32_t* n_anchor_b, hipStream_t stream)
{
    constexpr int LPR = D * Elem<DT>::kBytes / 16;
    constexpr int GROUPS = kMergeThreads / LPR;
    dim3 grid((n_anchor + GROUPS - 1) / GROUPS, B * H);
    if (weights != nullptr && !evict_only)
        hipLaunchKernelGGL((merge_compact_kernel<DT, D, true>), grid, dim3(kMergeThreads), 0, stream,
                           (const uint4*)k, (const uint4*)v, anchor_idx, weights, src_pos, (uint4*)k_cache,
                           (uint4*)v_cache, counts, assign, pos, H, G, T, src_rows, n_anchor, cap, evict_only, seq_len,
                           n_anchor_b);
    else
        hipLaunchKernelGGL((merge_compact_kernel<DT, D, false>), grid, dim3(kMergeThreads), 0, stream,
                           (const uint4*)k, (const uint4*)v, anchor_idx, weights, src_pos, (uint4*)k_cache,
                           (uint4*)v_cache, counts, assign, pos, H, G, T, src_rows, n_anchor, cap, evict_only, seq_len,
                           n_anchor_b);
    return status_from_hip(hipGetLastError());
}

int merge_dispatch(const void* k, const void* v, const int32_t* anchor_idx, const int32_t* weights,
                   const int32_t* src_pos, int B, int H, int G, int T, int src_rows, int D, int n_anchor, int dt,
                   int evict_only, void* k_cache, void* v_cache, int cap, int32_t* counts, int32_t* assign,
                   int32_t* pos, const int32_t* seq_len, const int32_t* n_anchor_b, hipStream_t stream)
{
#define EC_MERGE_CASE(DT_, D_)                                                                               \
    if (dt == DT_ && D == D_)                                                                                \
        return launch_merge<DT_, D_>(k, v, anchor_idx, weights, src_pos, B, H, G, T, src_rows, n_anchor, k_cache, \
                                     v_cache, cap, counts, assign, pos, evict_only, seq_len, n_anchor_b, stream);
    EC_MERGE_CASE(EC_BF16, 128)
    EC_MERGE_CASE(EC_BF16, 64)
    EC_MERGE_CASE(EC_F32, 128)
    EC_MERGE_CASE(EC_F32, 64)
#undef EC_MERGE_CASE
    return EC_EUNSUPPORTED;
}

}  // namespace ec
