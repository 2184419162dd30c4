// ec_decode_step: single-query attention over the compressed cache, with the
// append of the new key/value row and the fixed-point elimination folded into
// the same launch (Sec. 3.1 Output Generation; Sec. 3.3; Alg. 1's last branch).
//
// HBM-bound: every K and V row of the cache is read exactly once with 16-byte
// loads.  The rows of one (batch, head) are cut into `n_splits` contiguous
// ranges, one workgroup each (flash-decoding style), so that small batches still
// fill 256 CUs.  A group of LPR = row_bytes/16 lanes owns one row per load; each
// group keeps its own running (max, sum, weighted V) and never talks to other
// groups inside the streaming loop.  Workgroup partials go to the workspace; the
// last workgroup of a (batch, head) to arrive -- decided by an atomic ticket --
// merges them, writes `out`, and only then shifts the tail rows over the evicted
// row and stores the new row, so no row is overwritten before every reader of
// that (batch, head) is done.
#include "ec_common.h"

namespace ec {

constexpr int kDecodeThreads = 256;
constexpr int kDecodeWaves = kDecodeThreads / kWave;
constexpr int kDecodeUnroll = 4;
constexpr int kDecodeMaxSplits = 64;

template <int DT, int D> struct DecodeShape {
    static constexpr int kRowBytes = D * Elem<DT>::kBytes;
    static constexpr int kLPR = kRowBytes / 16;           // lanes per row
    static constexpr int kRPW = kWave / kLPR;             // rows per wave load
    static constexpr int kEPL = Elem<DT>::kPerChunk;      // elements per lane
    static constexpr int kGroups = kDecodeWaves * kRPW;   // row groups per workgroup
    static constexpr int kTile = kDecodeWaves * kDecodeUnroll * kRPW;  // rows per WG iteration
};

// Workspace layout: [BH][kDecodeMaxSplits][D + 2] floats (unnormalised out, max, sum),
// then [BH] uint32 tickets.
__host__ __device__ inline size_t decode_partial_floats(int BH, int D)
{
    return (size_t)BH * kDecodeMaxSplits * (size_t)(D + 2);
}

template <int DT, int D>
__global__ __launch_bounds__(kDecodeThreads) void decode_step_kernel(
    const uint4* __restrict__ q, const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
    uint4* k_cache, uint4* v_cache, int32_t* pos, uint4* __restrict__ out, float* ws_partial,
    unsigned int* ws_ticket, int H, int G, int cap, int cache_len, int evict_idx, int32_t new_pos,
    float scale_log2e, int rows_per_split, int n_splits)
{
    using S = DecodeShape<DT, D>;
    constexpr int LPR = S::kLPR, RPW = S::kRPW, EPL = S::kEPL;
    const int split = blockIdx.x;
    const int bh = blockIdx.y;
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = tid % kWave;
    const int sub = lane % LPR;   // which 16-byte chunk of the row
    const int rgrp = lane / LPR;  // which row of the wave's load

    const int n_rows = cache_len + 1;  // row cache_len is the new one, still in k_new/v_new
    const int row_begin = split * rows_per_split;
    const int row_end = min(n_rows, row_begin + rows_per_split);

    const uint4* kc = k_cache + (size_t)bh * cap * LPR;
    const uint4* vc = v_cache + (size_t)bh * cap * LPR;
    const uint4* kn = k_new + (size_t)bh * LPR;
    const uint4* vn = v_new + (size_t)bh * LPR;

    float qf[EPL];
    {
        uint4 qc = q[(size_t)bh * LPR + sub];
        unpack<DT>(qc, qf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[e] *= scale_log2e;
    }

    float m_run = -INFINITY, l_run = 0.f;
    float acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

    for (int base = row_begin; base < row_end; base += S::kTile) {
        uint4 kf[kDecodeUnroll], vf[kDecodeUnroll];
        bool valid[kDecodeUnroll];
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            const int r = base + (u * kDecodeWaves + wave) * RPW + rgrp;
            valid[u] = r < row_end;
            const bool is_new = (r == cache_len);
            const uint4* kp = is_new ? kn + sub : kc + (size_t)r * LPR + sub;
            const uint4* vp = is_new ? vn + sub : vc + (size_t)r * LPR + sub;
            if (valid[u]) {
                kf[u] = *kp;
                vf[u] = *vp;
            } else {
                kf[u] = make_uint4(0, 0, 0, 0);
                vf[u] = make_uint4(0, 0, 0, 0);
            }
        }
        float s[kDecodeUnroll];
        float m_tile = -INFINITY;
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            float kx[EPL];
            unpack<DT>(kf[u], kx);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kx[e], d);
            d = group_sum<LPR>(d);
            s[u] = valid[u] ? d : -INFINITY;
            m_tile = fmaxf(m_tile, s[u]);
        }
        const float m_new = fmaxf(m_run, m_tile);
        if (m_new > -INFINITY) {  // uniform inside a row group
            const float corr = exp2f(m_run - m_new);
            l_run *= corr;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] *= corr;
#pragma unroll
            for (int u = 0; u < kDecodeUnroll; ++u) {
                const float p = exp2f(s[u] - m_new);
                l_run += p;
                float vx[EPL];
                unpack<DT>(vf[u], vx);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vx[e], acc[e]);
            }
            m_run = m_new;
        }
    }

    // ---- merge the row groups of this workgroup through LDS ----
    __shared__ float sh_acc[S::kGroups][D];
    __shared__ float sh_m[S::kGroups];
    __shared__ float sh_l[S::kGroups];
    __shared__ int sh_last;
    const int grp = wave * RPW + rgrp;
#pragma unroll
    for (int e = 0; e < EPL; ++e) sh_acc[grp][sub * EPL + e] = acc[e];
    if (sub == 0) {
        sh_m[grp] = m_run;
        sh_l[grp] = l_run;
    }
    __syncthreads();

    float* part = ws_partial + ((size_t)bh * kDecodeMaxSplits + split) * (D + 2);
    float o_d = 0.f, M = -INFINITY, L = 0.f;
    if (tid < D) {
#pragma unroll
        for (int g = 0; g < S::kGroups; ++g) M = fmaxf(M, sh_m[g]);
#pragma unroll
        for (int g = 0; g < S::kGroups; ++g) {
            const float w = (sh_m[g] > -INFINITY) ? exp2f(sh_m[g] - M) : 0.f;
            L = fmaf(sh_l[g], w, L);
            o_d = fmaf(sh_acc[g][tid], w, o_d);
        }
    }

    if (n_splits > 1) {
        if (tid < D) {
            part[tid] = o_d;
            if (tid == 0) {
                part[D] = M;
                part[D + 1] = L;
            }
        }
        __threadfence();  // partials visible device-wide before the ticket is taken
        __syncthreads();
        if (tid == 0) {
            const unsigned int old = atomicInc(&ws_ticket[bh], (unsigned int)(n_splits - 1));
            sh_last = (old == (unsigned int)(n_splits - 1));  // ticket wraps back to 0 for the next call
        }
        __syncthreads();
        if (!sh_last) return;
        __threadfence();
        if (tid < D) {
            const float* pb = ws_partial + (size_t)bh * kDecodeMaxSplits * (D + 2);
            M = -INFINITY;
            for (int sp = 0; sp < n_splits; ++sp)
                M = fmaxf(M, __hip_atomic_load(pb + sp * (D + 2) + D, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT));
            L = 0.f;
            o_d = 0.f;
            for (int sp = 0; sp < n_splits; ++sp) {
                const float ms = __hip_atomic_load(pb + sp * (D + 2) + D, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                const float ls = __hip_atomic_load(pb + sp * (D + 2) + D + 1, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                const float os = __hip_atomic_load(pb + sp * (D + 2) + tid, __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
                const float w = (ms > -INFINITY) ? exp2f(ms - M) : 0.f;
                L = fmaf(ls, w, L);
                o_d = fmaf(os, w, o_d);
            }
        }
    }

    // ---- write out[bh, :] ----
    if (tid < D) {
        const float r = o_d / L;
        typename Elem<DT>::type* o = reinterpret_cast<typename Elem<DT>::type*>(out) + (size_t)bh * D;
        if constexpr (DT == EC_F32)
            o[tid] = r;
        else
            o[tid] = f32_to_bf16(r);
    }

    // ---- every reader of this (b,h) is done: evict (shift the tail up) and append ----
    // Rows evict_idx+1 .. cache_len-1 of the cache move to evict_idx .. cache_len-2; the new row
    // lands at cache_len-1 (eviction) or cache_len (none); it is dropped if it is the victim.
    uint4* kcw = k_cache + (size_t)bh * cap * LPR;
    uint4* vcw = v_cache + (size_t)bh * cap * LPR;
    if (evict_idx >= 0) {
        const int n_move = cache_len - 1 - evict_idx;  // rows taken from the cache itself
        const int total = n_move * LPR;                // 16-byte chunks per tensor
        for (int c0 = 0; c0 < total; c0 += kDecodeThreads) {
            const int c = c0 + tid;
            uint4 kk, vv;
            if (c < total) {
                kk = kcw[(size_t)(evict_idx + 1) * LPR + c];
                vv = vcw[(size_t)(evict_idx + 1) * LPR + c];
            }
            __syncthreads();  // all reads of this slab before any write into it
            if (c < total) {
                kcw[(size_t)evict_idx * LPR + c] = kk;
                vcw[(size_t)evict_idx * LPR + c] = vv;
            }
        }
    }
    const int new_row = (evict_idx < 0) ? cache_len : ((evict_idx == cache_len) ? -1 : cache_len - 1);
    if (new_row >= 0 && tid < 2 * LPR) {
        if (tid < LPR)
            kcw[(size_t)new_row * LPR + tid] = kn[tid];
        else
            vcw[(size_t)new_row * LPR + (tid - LPR)] = vn[tid - LPR];
    }

    // ---- positions: one copy per score group ----
    if (pos != nullptr) {
        const int b = bh / H, h = bh % H;
        if (G == H || h == 0) {
            int32_t* pp = pos + ((size_t)b * G + (G == 1 ? 0 : h)) * cap;
            if (evict_idx >= 0) {
                const int n_move = cache_len - 1 - evict_idx;
                for (int c0 = 0; c0 < n_move; c0 += kDecodeThreads) {
                    const int c = c0 + tid;
                    int32_t pv = 0;
                    if (c < n_move) pv = pp[evict_idx + 1 + c];
                    __syncthreads();
                    if (c < n_move) pp[evict_idx + c] = pv;
                }
            }
            if (new_row >= 0 && tid == 0) pp[new_row] = new_pos;
        }
    }
}

template <int DT, int D>
static int launch_decode(const void* q, const void* k_new, const void* v_new, void* k_cache,
                         void* v_cache, int32_t* pos, int B, int H, int G, int cap, int cache_len,
                         int evict_idx, int32_t new_pos, float scale, void* out, void* ws,
                         int forced_splits, hipStream_t stream)
{
    using S = DecodeShape<DT, D>;
    const int BH = B * H;
    const int n_rows = cache_len + 1;
    const int max_by_rows = (n_rows + S::kTile - 1) / S::kTile;
    int splits = forced_splits > 0 ? forced_splits : (1024 + BH - 1) / BH;
    splits = max(1, min(min(splits, kDecodeMaxSplits), max_by_rows));
    int rows_per_split = (n_rows + splits - 1) / splits;
    rows_per_split = ((rows_per_split + S::kTile - 1) / S::kTile) * S::kTile;
    splits = (n_rows + rows_per_split - 1) / rows_per_split;

    float* ws_partial = reinterpret_cast<float*>(ws);
    unsigned int* ws_ticket = reinterpret_cast<unsigned int*>(ws_partial + decode_partial_floats(BH, D));
    dim3 grid(splits, BH);
    hipLaunchKernelGGL((decode_step_kernel<DT, D>), grid, dim3(kDecodeThreads), 0, stream,
                       (const uint4*)q, (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache,
                       (uint4*)v_cache, pos, (uint4*)out, ws_partial, ws_ticket, H, G, cap, cache_len,
                       evict_idx, new_pos, scale * kLog2e, rows_per_split, splits);
    return status_from_hip(hipGetLastError());
}

size_t decode_workspace_bytes(int B, int H, int D)
{
    const int BH = B * H;
    return decode_partial_floats(BH, D) * sizeof(float) + (size_t)BH * sizeof(unsigned int);
}

int decode_dispatch(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                    int32_t* pos, int B, int H, int G, int D, int cap, int cache_len, int evict_idx,
                    int32_t new_pos, float scale, int dt, void* out, void* ws, int forced_splits,
                    hipStream_t stream)
{
#define EC_DECODE_CASE(DT_, D_)                                                                     \
    if (dt == DT_ && D == D_)                                                                       \
        return launch_decode<DT_, D_>(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, cap, cache_len, \
                                      evict_idx, new_pos, scale, out, ws, forced_splits, stream);
    EC_DECODE_CASE(EC_BF16, 128)
    EC_DECODE_CASE(EC_BF16, 64)
    EC_DECODE_CASE(EC_F32, 128)
    EC_DECODE_CASE(EC_F32, 64)
#undef EC_DECODE_CASE
    return EC_EUNSUPPORTED;
}

}  // namespace ec
