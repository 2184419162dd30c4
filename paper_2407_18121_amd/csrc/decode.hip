// ec_decode_step: single-query attention over the compressed cache, with the
// append of the new key/value row and the fixed-point elimination folded into
// the same launch (Sec. 3.1 Output Generation; Sec. 3.3; Alg. 1's last branch).
//
// HBM-bound: every K and V row of the cache is read exactly once with 16-byte
// loads.  Two launch shapes:
//   fused : one workgroup of up to 16 waves owns a whole (batch, head); nothing is exchanged
//           between workgroups and the elimination is a register-held shift (below).
//   split : when there are too few (batch, head) pairs to fill the chip, or too few bytes in flight
//           per compute unit, the rows of one (batch, head) are divided over `splits` workgroups
//           that each write an un-normalised partial (max, sum, weighted V) to the caller's
//           workspace; a second, small launch merges the partials, writes the output and performs
//           the append and the elimination through memory.  The two launches are ordered by the
//           stream: no ticket, no device-scope fence inside a kernel.
// A group of LPR = row_bytes/16
// lanes owns one row per load, so a wave load covers 1 KB of contiguous cache;
// each group keeps its own running (max, sum, weighted V) and never talks to
// other groups inside the streaming loop.  Loads of the next tile are issued
// before the current tile is consumed.  Tiles are aligned to the END of the
// cache, so when the loop finishes the registers still hold the newest rows:
// after the workgroup barrier that ends all reads, the rows behind the evicted
// one are stored one slot up straight from those registers, and so is the new
// row -- the elimination costs no extra read.
#include <algorithm>

#include "ec_common.h"

namespace ec {

template <int DT, int D, int WAVES, int UNROLL> struct DecodeShape {
    static constexpr int kThreads = WAVES * kWave;
    static constexpr int kRowBytes = D * Elem<DT>::kBytes;
    static constexpr int kLPR = kRowBytes / 16;                 // lanes per row
    static constexpr int kRPW = kWave / kLPR;                   // rows per wave load
    static constexpr int kEPL = Elem<DT>::kPerChunk;            // elements per lane
    static constexpr int kTile = WAVES * UNROLL * kRPW;       // rows per workgroup iteration
};

// EMIT (frequency discard policy): the kernel also stores every row's scaled score (base-2 units) into
// raw [B,H,cap] and the head's softmax maximum and denominator into stats [B,H,2], from which
// freq_accumulate_kernel forms this step's probabilities.
template <int DT, int D, int WAVES, int UNROLL, bool EMIT>
__global__ __launch_bounds__(WAVES * kWave) void decode_step_kernel(
    const uint4* __restrict__ q, const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
    uint4* k_cache, uint4* v_cache, int32_t* pos, uint4* __restrict__ out, int H, int G, int cap,
    int cache_len, int evict_idx, int32_t new_pos, float scale_log2e, float* __restrict__ raw,
    float* __restrict__ stats, const int32_t* __restrict__ len_b, const int32_t* __restrict__ evict_b,
    const int32_t* __restrict__ new_pos_b)
{
    using S = DecodeShape<DT, D, WAVES, UNROLL>;
    if (len_b) {  // ragged batch: every batch element has its own cache length, victim and position
        const int b = blockIdx.x / H;
        cache_len = min(max(len_b[b], 0), cap - 1);
        evict_idx = evict_b ? min(max(evict_b[b], -1), cache_len) : -1;
        if (new_pos_b) new_pos = new_pos_b[b];
    }
    constexpr int kDecodeUnroll = UNROLL;
    constexpr int LPR = S::kLPR, RPW = S::kRPW, EPL = S::kEPL, THREADS = S::kThreads, TILE = S::kTile;
    const int bh = blockIdx.x;
    const int tid = threadIdx.x;
    const int wave = tid / kWave;
    const int lane = tid % kWave;
    const int sub = lane % LPR;   // which 16-byte chunk of the row
    const int rgrp = lane / LPR;  // which row of the wave's load

    const int n_rows = cache_len + 1;  // row cache_len is the new one, still in k_new/v_new
    const int n_tiles = (n_rows + TILE - 1) / TILE;
    const int first_row = n_rows - n_tiles * TILE;  // <= 0: tile 0 is the ragged one

    uint4* kc = k_cache + (size_t)bh * cap * LPR;
    uint4* vc = v_cache + (size_t)bh * cap * LPR;
    const uint4* kn = k_new + (size_t)bh * LPR;
    const uint4* vn = v_new + (size_t)bh * LPR;

    // positions of the rows behind the victim, fetched early (stored after the barrier)
    const bool owns_pos = pos != nullptr && (G == H || (bh % H) == 0);
    int32_t* pp = owns_pos ? pos + ((size_t)(bh / H) * G + (G == 1 ? 0 : bh % H)) * cap : nullptr;
    const int n_move = (evict_idx >= 0) ? max(cache_len - 1 - evict_idx, 0) : 0;
    int32_t pos_pref = 0;
    if (owns_pos && tid < n_move) pos_pref = pp[evict_idx + 1 + tid];

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

    uint4 kf[kDecodeUnroll], vf[kDecodeUnroll], kf2[kDecodeUnroll], vf2[kDecodeUnroll];
    const int lane_row = wave * RPW + rgrp;  // row offset of this lane group inside one unroll slab

    auto load_tile = [&](int t, uint4* kd, uint4* vd) {
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            const int r = first_row + t * TILE + u * (WAVES * RPW) + lane_row;
            if (r >= 0) {
                const bool is_new = (r == cache_len);
                kd[u] = load_stream(is_new ? kn + sub : kc + (size_t)r * LPR + sub);
                vd[u] = load_stream(is_new ? vn + sub : vc + (size_t)r * LPR + sub);
            } else {
                kd[u] = make_uint4(0, 0, 0, 0);
                vd[u] = make_uint4(0, 0, 0, 0);
            }
        }
    };

    load_tile(0, kf, vf);
    for (int t = 0;; ++t) {
        const bool more = t + 1 < n_tiles;
        if (more) load_tile(t + 1, kf2, vf2);

        float s[kDecodeUnroll];
        float m_tile = -INFINITY;
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            const int r = first_row + t * TILE + u * (WAVES * RPW) + lane_row;
            float kx[EPL];
            unpack<DT>(kf[u], kx);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kx[e], d);
            d = group_sum<LPR>(d);
            s[u] = (r >= 0) ? d : -INFINITY;
            if (EMIT && r >= 0 && sub == 0) raw[(size_t)bh * cap + r] = d;
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
        if (!more) break;  // kf/vf keep the last tile: the newest rows
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            kf[u] = kf2[u];
            vf[u] = vf2[u];
        }
    }

    // ---- merge the RPW row groups of each wave with shuffles (lanes that hold the same chunk) ----
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
        const float m_o = __shfl_xor(m_run, off, kWave);
        const float l_o = __shfl_xor(l_run, off, kWave);
        const float m_n = fmaxf(m_run, m_o);
        const float w_s = (m_run > -INFINITY) ? exp2f(m_run - m_n) : 0.f;
        const float w_o = (m_o > -INFINITY) ? exp2f(m_o - m_n) : 0.f;
        l_run = l_run * w_s + l_o * w_o;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float a_o = __shfl_xor(acc[e], off, kWave);
            acc[e] = acc[e] * w_s + a_o * w_o;
        }
        m_run = m_n;
    }

    // ---- merge the waves through LDS ----
    __shared__ float sh_acc[WAVES][D];
    __shared__ float sh_m[WAVES];
    __shared__ float sh_l[WAVES];
    if (rgrp == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sh_acc[wave][sub * EPL + e] = acc[e];
        if (sub == 0) {
            sh_m[wave] = m_run;
            sh_l[wave] = l_run;
        }
    }
    __syncthreads();  // also: every wave of this workgroup has finished reading the cache

    if (tid < D) {
        float M = -INFINITY, L = 0.f, o_d = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) M = fmaxf(M, sh_m[w]);
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float wt = (sh_m[w] > -INFINITY) ? exp2f(sh_m[w] - M) : 0.f;
            L = fmaf(sh_l[w], wt, L);
            o_d = fmaf(sh_acc[w][tid], wt, o_d);
        }
        if (EMIT && tid == 0) {
            stats[(size_t)bh * 2] = M;
            stats[(size_t)bh * 2 + 1] = L;
        }
        const float r = o_d / L;
        typename Elem<DT>::type* o = reinterpret_cast<typename Elem<DT>::type*>(out) + (size_t)bh * D;
        if constexpr (DT == EC_F32)
            o[tid] = r;
        else
            o[tid] = f32_to_bf16(r);
    }

    // ---- fixed-point elimination + append ----
    // With a victim, rows evict_idx+1 .. cache_len (the last being the new row) move up by one; the
    // new row is dropped if it is the victim itself.  Without one, the new row lands at cache_len.
    const int last_tile_row0 = first_row + (n_tiles - 1) * TILE;  // first row still held in registers
    if (evict_idx >= 0) {
        // rows behind the victim that left the registers long ago (only when more than a tile moves)
        const int slow_end = min(last_tile_row0, cache_len);  // rows [evict_idx+1, slow_end) via memory
        const int total = max(slow_end - (evict_idx + 1), 0) * LPR;
        for (int c0 = 0; c0 < total; c0 += THREADS) {
            const int c = c0 + tid;
            uint4 kk, vv;
            if (c < total) {
                kk = kc[(size_t)(evict_idx + 1) * LPR + c];
                vv = vc[(size_t)(evict_idx + 1) * LPR + c];
            }
            __syncthreads();  // all reads of this slab before any write into it
            if (c < total) {
                kc[(size_t)evict_idx * LPR + c] = kk;
                vc[(size_t)evict_idx * LPR + c] = vv;
            }
        }
        if (total > 0) __syncthreads();
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            const int r = last_tile_row0 + u * (WAVES * RPW) + lane_row;
            if (r > evict_idx && r >= 0) {
                kc[(size_t)(r - 1) * LPR + sub] = kf[u];
                vc[(size_t)(r - 1) * LPR + sub] = vf[u];
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < kDecodeUnroll; ++u) {
            const int r = last_tile_row0 + u * (WAVES * RPW) + lane_row;
            if (r == cache_len) {
                kc[(size_t)r * LPR + sub] = kf[u];
                vc[(size_t)r * LPR + sub] = vf[u];
            }
        }
    }

    // ---- positions: one copy per score group ----
    if (owns_pos) {
        if (tid < n_move) pp[evict_idx + tid] = pos_pref;  // fetched before the barrier above
        for (int c0 = THREADS; c0 < n_move; c0 += THREADS) {  // beyond one workgroup's worth
            const int c = c0 + tid;
            int32_t pv = 0;
            if (c < n_move) pv = pp[evict_idx + 1 + c];
            __syncthreads();
            if (c < n_move) pp[evict_idx + c] = pv;
        }
        const int new_row = (evict_idx < 0) ? cache_len : ((evict_idx == cache_len) ? -1 : cache_len - 1);
        if (new_row >= 0 && tid == 0) pp[new_row] = new_pos;
    }
}

// ------------------------------------------------------------------ split launch shape
// Workgroup (bh, s) attends rows [s * chunk, (s + 1) * chunk) of its (batch, head), chunk =
// ceil(n_rows / splits), and stores its partial to part[(bh * splits + s) * (D + 2)]: D weighted-V sums
// relative to its own maximum, then that maximum (base-2 units; -inf for an empty range) and the sum of
// its weights.  Nothing in the cache is written here.
template <int DT, int D, int WAVES, int UNROLL>
__global__ __launch_bounds__(WAVES * kWave) void decode_split_kernel(
    const uint4* __restrict__ q, const uint4* __restrict__ k_new, const uint4* __restrict__ v_new,
    const uint4* __restrict__ k_cache, const uint4* __restrict__ v_cache, float* __restrict__ part, int cap,
    int cache_len, int splits, float scale_log2e)
{
    using S = DecodeShape<DT, D, WAVES, UNROLL>;
    constexpr int LPR = S::kLPR, RPW = S::kRPW, EPL = S::kEPL, TILE = S::kTile;
    const int bh = blockIdx.x / splits, sp = blockIdx.x % splits;
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int sub = lane % LPR, rgrp = lane / LPR;

    const int n_rows = cache_len + 1;  // row cache_len is the new one, still in k_new/v_new
    const int chunk = (n_rows + splits - 1) / splits;
    const int r0 = sp * chunk, r1 = min(r0 + chunk, n_rows);
    const int n_tiles = (max(r1 - r0, 0) + TILE - 1) / TILE;

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

    uint4 kf[UNROLL], vf[UNROLL], kf2[UNROLL], vf2[UNROLL];
    const int lane_row = wave * RPW + rgrp;
    auto load_tile = [&](int t, uint4* kd, uint4* vd) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = r0 + t * TILE + u * (WAVES * RPW) + lane_row;
            if (r < r1) {
                const bool is_new = (r == cache_len);
                kd[u] = load_stream(is_new ? kn + sub : kc + (size_t)r * LPR + sub);
                vd[u] = load_stream(is_new ? vn + sub : vc + (size_t)r * LPR + sub);
            } else {
                kd[u] = make_uint4(0, 0, 0, 0);
                vd[u] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    if (n_tiles > 0) load_tile(0, kf, vf);
    for (int t = 0; t < n_tiles; ++t) {
        const bool more = t + 1 < n_tiles;
        if (more) load_tile(t + 1, kf2, vf2);
        float s[UNROLL];
        float m_tile = -INFINITY;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int r = r0 + t * TILE + u * (WAVES * RPW) + lane_row;
            float kx[EPL];
            unpack<DT>(kf[u], kx);
            float d = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d = fmaf(qf[e], kx[e], d);
            d = group_sum<LPR>(d);
            s[u] = (r < r1) ? d : -INFINITY;
            m_tile = fmaxf(m_tile, s[u]);
        }
        const float m_new = fmaxf(m_run, m_tile);
        if (m_new > -INFINITY) {
            const float corr = exp2f(m_run - m_new);
            l_run *= corr;
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[e] *= corr;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const float p = exp2f(s[u] - m_new);
                l_run += p;
                float vx[EPL];
                unpack<DT>(vf[u], vx);
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vx[e], acc[e]);
            }
            m_run = m_new;
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            kf[u] = kf2[u];
            vf[u] = vf2[u];
        }
    }
    // row groups of a wave, then the waves: same order of operations as the fused kernel
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
        const float m_o = __shfl_xor(m_run, off, kWave);
        const float l_o = __shfl_xor(l_run, off, kWave);
        const float m_n = fmaxf(m_run, m_o);
        const float w_s = (m_run > -INFINITY) ? exp2f(m_run - m_n) : 0.f;
        const float w_o = (m_o > -INFINITY) ? exp2f(m_o - m_n) : 0.f;
        l_run = l_run * w_s + l_o * w_o;
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            const float a_o = __shfl_xor(acc[e], off, kWave);
            acc[e] = acc[e] * w_s + a_o * w_o;
        }
        m_run = m_n;
    }
    __shared__ float sh_acc[WAVES][D];
    __shared__ float sh_m[WAVES];
    __shared__ float sh_l[WAVES];
    if (rgrp == 0) {
#pragma unroll
        for (int e = 0; e < EPL; ++e) sh_acc[wave][sub * EPL + e] = acc[e];
        if (sub == 0) {
            sh_m[wave] = m_run;
            sh_l[wave] = l_run;
        }
    }
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY, L = 0.f, o_d = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) M = fmaxf(M, sh_m[w]);
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float wt = (sh_m[w] > -INFINITY) ? exp2f(sh_m[w] - M) : 0.f;
            L = fmaf(sh_l[w], wt, L);
            o_d = fmaf(sh_acc[w][tid], wt, o_d);
        }
        float* dst = part + (size_t)blockIdx.x * (D + 2);
        dst[tid] = o_d;
        if (tid == 0) {
            dst[D] = M;
            dst[D + 1] = L;
        }
    }
}

// Second launch of the split shape, one workgroup per (batch, head): merges the partials in ascending split
// order, writes the output, then appends the new row and removes the victim through memory (the rows behind
// it move up by one, slab by slab: a slab is read completely before any of it is overwritten).
constexpr int kCombineThreads = 256;
template <int DT, int D>
__global__ __launch_bounds__(kCombineThreads) void decode_combine_kernel(
    const float* __restrict__ part, const uint4* __restrict__ k_new, const uint4* __restrict__ v_new, uint4* k_cache,
    uint4* v_cache, int32_t* pos, void* __restrict__ out, int H, int G, int cap, int cache_len, int evict_idx,
    int32_t new_pos, int splits)
{
    constexpr int LPR = D * Elem<DT>::kBytes / 16;
    const int bh = blockIdx.x, tid = threadIdx.x;
    if (tid < D) {
        const float* p = part + (size_t)bh * splits * (D + 2);
        float M = -INFINITY;
        for (int s = 0; s < splits; ++s) M = fmaxf(M, p[s * (D + 2) + D]);
        float L = 0.f, o_d = 0.f;
        for (int s = 0; s < splits; ++s) {
            const float ms = p[s * (D + 2) + D];
            const float wt = (ms > -INFINITY) ? exp2f(ms - M) : 0.f;
            L = fmaf(p[s * (D + 2) + D + 1], wt, L);
            o_d = fmaf(p[s * (D + 2) + tid], wt, o_d);
        }
        const float r = o_d / L;
        typename Elem<DT>::type* o = reinterpret_cast<typename Elem<DT>::type*>(out) + (size_t)bh * D;
        if constexpr (DT == EC_F32)
            o[tid] = r;
        else
            o[tid] = f32_to_bf16(r);
    }

    uint4* kc = k_cache + (size_t)bh * cap * LPR;
    uint4* vc = v_cache + (size_t)bh * cap * LPR;
    // rows evict_idx+1 .. cache_len-1 move up by one, then the new row lands behind them
    const int n_move = (evict_idx >= 0) ? max(cache_len - 1 - evict_idx, 0) : 0;
    const int total = n_move * LPR;
    for (int c0 = 0; c0 < total; c0 += kCombineThreads) {
        const int c = c0 + tid;
        uint4 kk, vv;
        if (c < total) {
            kk = kc[(size_t)(evict_idx + 1) * LPR + c];
            vv = vc[(size_t)(evict_idx + 1) * LPR + c];
        }
        __syncthreads();
        if (c < total) {
            kc[(size_t)evict_idx * LPR + c] = kk;
            vc[(size_t)evict_idx * LPR + c] = vv;
        }
        __syncthreads();
    }
    const int new_row = (evict_idx < 0) ? cache_len : ((evict_idx == cache_len) ? -1 : cache_len - 1);
    if (new_row >= 0 && tid < LPR) {
        kc[(size_t)new_row * LPR + tid] = k_new[(size_t)bh * LPR + tid];
        vc[(size_t)new_row * LPR + tid] = v_new[(size_t)bh * LPR + tid];
    }
    if (pos != nullptr && (G == H || (bh % H) == 0)) {
        int32_t* pp = pos + ((size_t)(bh / H) * G + (G == 1 ? 0 : bh % H)) * cap;
        for (int c0 = 0; c0 < n_move; c0 += kCombineThreads) {
            const int c = c0 + tid;
            int32_t pv = 0;
            if (c < n_move) pv = pp[evict_idx + 1 + c];
            __syncthreads();
            if (c < n_move) pp[evict_idx + c] = pv;
            __syncthreads();
        }
        if (new_row >= 0 && tid == 0) pp[new_row] = new_pos;
    }
}

template <int DT, int D, int WAVES, int UNROLL>
static int launch_decode_split(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                               int32_t* pos, int B, int H, int G, int cap, int cache_len, int evict_idx,
                               int32_t new_pos, float scale, void* out, float* part, int splits, hipStream_t stream)
{
    using S = DecodeShape<DT, D, WAVES, UNROLL>;
    hipLaunchKernelGGL((decode_split_kernel<DT, D, WAVES, UNROLL>), dim3(B * H * splits), dim3(S::kThreads), 0, stream,
                       (const uint4*)q, (const uint4*)k_new, (const uint4*)v_new, (const uint4*)k_cache,
                       (const uint4*)v_cache, part, cap, cache_len, splits, scale * kLog2e);
    int rc = status_from_hip(hipGetLastError());
    if (rc != EC_OK) return rc;
    hipLaunchKernelGGL((decode_combine_kernel<DT, D>), dim3(B * H), dim3(kCombineThreads), 0, stream, part,
                       (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache, (uint4*)v_cache, pos, out, H, G, cap,
                       cache_len, evict_idx, new_pos, splits);
    return status_from_hip(hipGetLastError());
}

template <int DT, int D, int WAVES, int UNROLL>
static int launch_decode_w(const void* q, const void* k_new, const void* v_new, void* k_cache,
                           void* v_cache, int32_t* pos, int B, int H, int G, int cap, int cache_len,
                           int evict_idx, int32_t new_pos, float scale, void* out, const int32_t* len_b,
                           const int32_t* evict_b, const int32_t* new_pos_b, hipStream_t stream)
{
    using S = DecodeShape<DT, D, WAVES, UNROLL>;
    hipLaunchKernelGGL((decode_step_kernel<DT, D, WAVES, UNROLL, false>), dim3(B * H), dim3(S::kThreads), 0, stream,
                       (const uint4*)q, (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache,
                       (uint4*)v_cache, pos, (uint4*)out, H, G, cap, cache_len, evict_idx, new_pos,
                       scale * kLog2e, (float*)nullptr, (float*)nullptr, len_b, evict_b, new_pos_b);
    return status_from_hip(hipGetLastError());
}

// Number of workgroups one (batch, head) is divided over when the caller leaves the choice to the library.
// Measured on MI355X (graph replay, 32 layers): the merging launch costs about as much as an empty dispatch
// (3-5 us), which is more than the split saves at every workload shape tried -- B*H = 32, 640 rows: 9.9 us
// fused, 10.3 us best split; B*H = 160: 13.1 vs 16.8 us; B*H = 256: 16.0 vs 20.2 us -- because one launch is
// ~3 us of dispatch plus bytes at 5.3-5.9 TB/s already.  The library therefore always picks the fused shape;
// the split shape stays reachable through ec_decode_step_shaped.
int decode_auto_splits(int BH, int n_rows)
{
    (void)BH;
    (void)n_rows;
    return 1;
}

// Workspace floats the split shape needs at most (any cache length up to `cap` rows).
size_t decode_part_floats(int B, int H, int cap, int D)
{
    const int s = decode_auto_splits(B * H, cap);
    return s < 2 ? 0 : (size_t)B * H * s * (D + 2);
}

// Workgroup width and loads in flight grow with the number of rows to stream.  splits: 0 = choose, 1 = fused
// kernel, n > 1 = n workgroups per (batch, head) + combine launch (needs `part`, part_floats >= B*H*n*(D+2)).
template <int DT, int D>
static int launch_decode(const void* q, const void* k_new, const void* v_new, void* k_cache,
                         void* v_cache, int32_t* pos, int B, int H, int G, int cap, int cache_len,
                         int evict_idx, int32_t new_pos, float scale, void* out, int forced_waves,
                         int forced_unroll, int splits, bool strict, float* part, size_t part_floats,
                         const int32_t* len_b, const int32_t* evict_b, const int32_t* new_pos_b, hipStream_t stream)
{
    const int n_rows = cache_len + 1;  // ragged batches pass the longest length the buffers allow
    if (splits <= 0 || len_b != nullptr) splits = decode_auto_splits(B * H, n_rows);  // ragged batches: fused only
    if (splits > 1 && (part == nullptr || part_floats < (size_t)B * H * splits * (D + 2))) {
        if (strict) return EC_EWORKSPACE;  // an explicit request that cannot be met
        splits = 1;                        // no workspace: the fused shape needs none
    }
    int waves = forced_waves, unroll = forced_unroll;
    if (splits > 1) {
        if (waves <= 0) waves = ((n_rows + splits - 1) / splits >= 192) ? 8 : 4;
        if (unroll <= 0) unroll = 4;
#define EC_DECODE_S(W_, U_)                                                                                    \
    if (waves == W_ && unroll == U_)                                                                           \
        return launch_decode_split<DT, D, W_, U_>(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, cap, cache_len, \
                                                  evict_idx, new_pos, scale, out, part, splits, stream);
        EC_DECODE_S(4, 4)
        EC_DECODE_S(8, 4)
        EC_DECODE_S(4, 8)
        EC_DECODE_S(2, 4)
        EC_DECODE_S(2, 8)
#undef EC_DECODE_S
        return EC_EINVAL;
    }
    // Width of a workgroup.  Measured (us per launch, 4 loads of K and of V in flight per lane; 2 / 4 / 8 / 16 waves):
    //   B*H =   32,  640 rows: 20.6 / 12.4 /  9.8 / 10.8      B*H =  160,  640 rows: 22.4 / 14.6 / 12.4 / 13.1
    //   B*H =  256,  576 rows: 23.8 / 16.1 / 15.5 / 16.1      B*H =  320,  256 rows: 13.1 / 11.7 / 12.8 / 15.4
    //   B*H =  512,  870 rows: 40.6 / 39.7 / 42.0 / 45.5      B*H = 1536,  150 rows: 24.9 / 26.6 / 28.4 / 37.0
    // With one workgroup per compute unit or less the wide workgroup streams fastest; once several workgroups
    // share a compute unit, narrower ones (more of them resident, shorter tails) do.
    if (waves <= 0) {
        const long long bh = (long long)B * H;
        waves = bh >= 1024 ? 2 : bh > 256 ? 4 : (n_rows >= 96 ? 8 : 4);
    }
    if (unroll <= 0) unroll = 4;
#define EC_DECODE_W(W_, U_)                                                                              \
    if (waves == W_ && unroll == U_)                                                                     \
        return launch_decode_w<DT, D, W_, U_>(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, cap, cache_len, \
                                              evict_idx, new_pos, scale, out, len_b, evict_b, new_pos_b, stream);
    EC_DECODE_W(2, 4)
    EC_DECODE_W(2, 8)
    EC_DECODE_W(4, 4)
    EC_DECODE_W(4, 6)
    EC_DECODE_W(4, 8)
    EC_DECODE_W(8, 4)
    EC_DECODE_W(16, 4)
    EC_DECODE_W(16, 6)
    EC_DECODE_W(8, 8)
    EC_DECODE_W(8, 12)
    EC_DECODE_W(4, 12)
#undef EC_DECODE_W
    return EC_EINVAL;
}

// strict: the launch shape is an explicit request; a split without enough workspace is then an error instead
// of falling back to the fused kernel.
int decode_dispatch(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                    int32_t* pos, int B, int H, int G, int D, int cap, int cache_len, int evict_idx,
                    int32_t new_pos, float scale, int dt, void* out, int forced_waves, int forced_unroll,
                    int splits, bool strict, float* part, size_t part_floats, const int32_t* len_b,
                    const int32_t* evict_b, const int32_t* new_pos_b, hipStream_t stream)
{
#define EC_DECODE_CASE(DT_, D_)                                                                       \
    if (dt == DT_ && D == D_)                                                                         \
        return launch_decode<DT_, D_>(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, cap, cache_len,    \
                                      evict_idx, new_pos, scale, out, forced_waves, forced_unroll, splits, \
                                      strict, part, part_floats, len_b, evict_b, new_pos_b, stream);
    EC_DECODE_CASE(EC_BF16, 128)
    EC_DECODE_CASE(EC_BF16, 64)
    EC_DECODE_CASE(EC_F32, 128)
    EC_DECODE_CASE(EC_F32, 64)
#undef EC_DECODE_CASE
    return EC_EUNSUPPORTED;
}

// ------------------------------------------------------------------ frequency discard policy
// freq[b,g,j] += this step's attention mass of row j (head mean when G == 1); the row just appended
// (j = n - 1) starts at its own mass.  A workgroup covers 64 rows; its 4 thread groups each add up a quarter
// of the heads (ascending), and the quarters are added in ascending order: the result does not depend on
// scheduling.
constexpr int kFreqRows = 64;
constexpr int kFreqParts = 4;
__global__ __launch_bounds__(kFreqRows * kFreqParts) void freq_accumulate_kernel(const float* __restrict__ raw,
                                                                                const float* __restrict__ stats,
                                                                                float* __restrict__ freq, int H, int G,
                                                                                int n, int cap)
{
    __shared__ float part[kFreqParts][kFreqRows];
    const int bg = blockIdx.y;
    const int r = threadIdx.x % kFreqRows, grp = threadIdx.x / kFreqRows;
    const int j = blockIdx.x * kFreqRows + r;
    const int b = bg / G, g = bg % G;
    const int h_first = (G == H) ? g : 0, h_count = (G == H) ? 1 : H;
    const int per = (h_count + kFreqParts - 1) / kFreqParts;
    const int h0 = h_first + grp * per, h1 = min(h0 + per, h_first + h_count);
    float acc = 0.f;
    if (j < n)
        for (int h = h0; h < h1; ++h) {
            const size_t bh = (size_t)b * H + h;
            acc += exp2f(raw[bh * cap + j] - stats[bh * 2]) / stats[bh * 2 + 1];
        }
    part[grp][r] = acc;
    __syncthreads();
    if (grp == 0 && j < n) {
        float mass = part[0][r];
#pragma unroll
        for (int p = 1; p < kFreqParts; ++p) mass += part[p][r];
        mass /= (float)h_count;
        float* f = freq + (size_t)bg * cap + j;
        *f = (j == n - 1) ? mass : *f + mass;
    }
}

template <int DT, int D, int WAVES>
static int launch_decode_score(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                               int32_t* pos, float* freq, int B, int H, int G, int cap, int cache_len,
                               int32_t new_pos, float scale, void* out, float* raw, float* stats,
                               hipStream_t stream)
{
    using S = DecodeShape<DT, D, WAVES, 4>;
    hipLaunchKernelGGL((decode_step_kernel<DT, D, WAVES, 4, true>), dim3(B * H), dim3(S::kThreads), 0, stream,
                       (const uint4*)q, (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache,
                       (uint4*)v_cache, pos, (uint4*)out, H, G, cap, cache_len, -1, new_pos, scale * kLog2e, raw,
                       stats, (const int32_t*)nullptr, (const int32_t*)nullptr, (const int32_t*)nullptr);
    int rc = status_from_hip(hipGetLastError());
    if (rc != EC_OK) return rc;
    const int n = cache_len + 1;
    hipLaunchKernelGGL(freq_accumulate_kernel, dim3((n + kFreqRows - 1) / kFreqRows, B * G),
                       dim3(kFreqRows * kFreqParts), 0, stream, raw, stats, freq, H, G, n, cap);
    return status_from_hip(hipGetLastError());
}

int decode_score_dispatch(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                          int32_t* pos, float* freq, int B, int H, int G, int D, int cap, int cache_len,
                          int32_t new_pos, float scale, int dt, void* out, float* raw, float* stats,
                          hipStream_t stream)
{
    const bool wide = cache_len + 1 >= 96;
#define EC_DSCORE_CASE(DT_, D_)                                                                                \
    if (dt == DT_ && D == D_)                                                                                  \
        return wide ? launch_decode_score<DT_, D_, 8>(q, k_new, v_new, k_cache, v_cache, pos, freq, B, H, G, cap,  \
                                                      cache_len, new_pos, scale, out, raw, stats, stream)     \
                    : launch_decode_score<DT_, D_, 4>(q, k_new, v_new, k_cache, v_cache, pos, freq, B, H, G, cap,  \
                                                      cache_len, new_pos, scale, out, raw, stats, stream);
    EC_DSCORE_CASE(EC_BF16, 128)
    EC_DSCORE_CASE(EC_BF16, 64)
    EC_DSCORE_CASE(EC_F32, 128)
    EC_DSCORE_CASE(EC_F32, 64)
#undef EC_DSCORE_CASE
    return EC_EUNSUPPORTED;
}

// Least-mass row of one score group: lowest index among equal fp32 values, rows [lo, hi] only.
__device__ __forceinline__ int argmin_row(const float* __restrict__ f, int lo, int hi, int tid, int threads,
                                          float* sh_v, int* sh_i)
{
    float bv = INFINITY;
    int bi = 0x7fffffff;
    for (int j = lo + tid; j <= hi; j += threads) {  // ascending per thread: strict < keeps the first
        const float v = f[j];
        if (v < bv || bi == 0x7fffffff) {
            bv = v;
            bi = j;
        }
    }
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const float ov = __shfl_xor(bv, off, kWave);
        const int oi = __shfl_xor(bi, off, kWave);
        if (oi != 0x7fffffff && (bi == 0x7fffffff || ov < bv || (ov == bv && oi < bi))) {
            bv = ov;
            bi = oi;
        }
    }
    const int wave = tid / kWave, lane = tid % kWave;
    if (lane == 0) {
        sh_v[wave] = bv;
        sh_i[wave] = bi;
    }
    __syncthreads();
    bv = sh_v[0];
    bi = sh_i[0];
    for (int w = 1; w < threads / kWave; ++w) {
        const float ov = sh_v[w];
        const int oi = sh_i[w];
        if (oi != 0x7fffffff && (bi == 0x7fffffff || ov < bv || (ov == bv && oi < bi))) {
            bv = ov;
            bi = oi;
        }
    }
    return bi;
}

constexpr int kEvictThreads = 256;
constexpr int kEvictUnroll = 4;

// Every (b,h) workgroup finds its group's victim itself (freq is only read here) and moves its own K and V
// rows up by one; the group's first head also publishes the index.
__global__ __launch_bounds__(kEvictThreads) void evict_min_rows_kernel(uint4* k_cache, uint4* v_cache,
                                                                       const float* __restrict__ freq,
                                                                       int32_t* __restrict__ victim, int H, int G,
                                                                       int cap, int len, int lo, int hi, int lpr)
{
    __shared__ float sh_v[kEvictThreads / kWave];
    __shared__ int sh_i[kEvictThreads / kWave];
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int b = bh / H, h = bh % H;
    const size_t bg = (size_t)b * G + (G == 1 ? 0 : h);
    const int vic = argmin_row(freq + bg * cap, lo, hi, tid, kEvictThreads, sh_v, sh_i);
    if (tid == 0 && (G == H || h == 0)) victim[bg] = vic;

    uint4* kc = k_cache + (size_t)bh * cap * lpr;
    uint4* vc = v_cache + (size_t)bh * cap * lpr;
    const int total = (len - 1 - vic) * lpr;  // 16-byte chunks that move, in ascending address order
    for (int c0 = 0; c0 < total; c0 += kEvictThreads * kEvictUnroll) {
        uint4 kk[kEvictUnroll], vv[kEvictUnroll];
#pragma unroll
        for (int u = 0; u < kEvictUnroll; ++u) {
            const int c = c0 + u * kEvictThreads + tid;
            if (c < total) {
                kk[u] = kc[(size_t)(vic + 1) * lpr + c];
                vv[u] = vc[(size_t)(vic + 1) * lpr + c];
            }
        }
        __syncthreads();  // the slab is read completely before any of it is overwritten
#pragma unroll
        for (int u = 0; u < kEvictUnroll; ++u) {
            const int c = c0 + u * kEvictThreads + tid;
            if (c < total) {
                kc[(size_t)vic * lpr + c] = kk[u];
                vc[(size_t)vic * lpr + c] = vv[u];
            }
        }
        __syncthreads();  // and written before the next slab, which overlaps it by one row, is read
    }
}

// The group's positions and masses follow their rows.
__global__ __launch_bounds__(kEvictThreads) void evict_min_meta_kernel(float* freq, int32_t* pos,
                                                                       const int32_t* __restrict__ victim, int cap,
                                                                       int len)
{
    const int bg = blockIdx.x, tid = threadIdx.x;
    const int vic = victim[bg];
    float* f = freq + (size_t)bg * cap;
    int32_t* p = pos ? pos + (size_t)bg * cap : nullptr;
    const int total = len - 1 - vic;
    for (int c0 = 0; c0 < total; c0 += kEvictThreads) {
        const int c = c0 + tid;
        float fv = 0.f;
        int32_t pv = 0;
        if (c < total) {
            fv = f[vic + 1 + c];
            if (p) pv = p[vic + 1 + c];
        }
        __syncthreads();
        if (c < total) {
            f[vic + c] = fv;
            if (p) p[vic + c] = pv;
        }
        __syncthreads();
    }
}

int evict_min_dispatch(void* k_cache, void* v_cache, int32_t* pos, float* freq, int B, int H, int G, int D, int cap,
                       int len, int protect_first, int protect_recent, int dt, int32_t* victim, hipStream_t stream)
{
    const int lpr = D * (dt == EC_F32 ? 4 : 2) / 16;
    hipLaunchKernelGGL(evict_min_rows_kernel, dim3(B * H), dim3(kEvictThreads), 0, stream, (uint4*)k_cache,
                       (uint4*)v_cache, freq, victim, H, G, cap, len, protect_first, len - 1 - protect_recent, lpr);
    int rc = status_from_hip(hipGetLastError());
    if (rc != EC_OK) return rc;
    hipLaunchKernelGGL(evict_min_meta_kernel, dim3(B * G), dim3(kEvictThreads), 0, stream, freq, pos, victim, cap, len);
    return status_from_hip(hipGetLastError());
}

}  // namespace ec
