// ec_select_anchors: per (batch, score group) choice of the N_I highest-scoring
// positions (Sec. 3.3), protected first/last positions always kept (Sec. 4.1),
// equal scores resolved toward the lower position, output ascending.
//
// One workgroup of 1024 threads per problem.  Scores are mapped to 32-bit keys
// whose unsigned order equals the fp32 order (-0 folded onto +0).  An MSB-first
// radix select (four 8-bit digits, LDS histograms) finds the key of the last
// selected element and how many elements equal to it are needed; one ordered
// sweep over the positions then emits the selected indices in ascending order,
// taking equal keys lowest-position-first.  Pure integer work: the result is
// bit-exact by construction.
#include "ec_common.h"

namespace ec {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSelLdsKeys = 8192;  // keys are cached in LDS up to this T

__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if (u == 0x80000000u) u = 0u;  // -0 compares equal to +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Ragged batches: seq_len[b] positions and n_anchor_b[b] anchors for batch element b (both clamped), rows
// of score and anchor_idx stay T_max and n_max apart.
__global__ __launch_bounds__(kSelThreads) void select_anchors_kernel(
    const float* __restrict__ score, int T_max, int n_max, int protect_first, int protect_last,
    int32_t* __restrict__ anchor_idx, int keys_in_lds, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ n_anchor_b, int G)
{
    extern __shared__ uint32_t lds_keys[];
    __shared__ int hist[256];
    __shared__ int wave_tot[2][kSelWaves];  // two sets, used in turn: one barrier per sweep step
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_need;

    const int tid = threadIdx.x;
    const int lane = tid % kWave, wave = tid / kWave;
    const int b = blockIdx.x / G;
    const int T = ragged_rows(seq_len, b, T_max);
    const int n_anchor = n_anchor_b ? min(max(n_anchor_b[b], 0), min(T, n_max)) : n_max;
    if (T == 0 || n_anchor == 0) return;  // whole workgroup
    protect_first = min(protect_first, n_anchor);
    protect_last = min(protect_last, n_anchor - protect_first);
    const float* s = score + (size_t)blockIdx.x * T_max;
    int32_t* dst = anchor_idx + (size_t)blockIdx.x * n_max;
    const int free_lo = protect_first, free_hi = T - protect_last;  // unprotected: [free_lo, free_hi)
    const int n_free = n_anchor - protect_first - protect_last;

    if (keys_in_lds)
        for (int t = tid; t < T; t += kSelThreads) lds_keys[t] = score_key(s[t]);
    if (tid < 256) hist[tid] = 0;
    if (tid == 0) {
        sh_prefix = 0u;
        sh_need = n_free;
    }
    __syncthreads();

    // ---- radix select of the n_free-th largest unprotected key ----
    if (n_free > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            const uint32_t hi_mask = (pass == 0) ? 0u : (0xffffffffu << (shift + 8));
            const uint32_t prefix = sh_prefix;
            const int need = sh_need;
            for (int t = free_lo + tid; t < free_hi; t += kSelThreads) {
                const uint32_t key = keys_in_lds ? lds_keys[t] : score_key(s[t]);
                if ((key & hi_mask) == prefix) atomicAdd(&hist[(key >> shift) & 0xffu], 1);
            }
            __syncthreads();
            // One wave finds the digit: lane l owns digits 4l..4l+3; a shuffle scan from the top gives the
            // number of candidates in the lanes above, and the four digits of a lane are walked in registers.
            if (wave == 0) {
                int c[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) c[i] = hist[4 * lane + i];
#pragma unroll
                for (int i = 0; i < 4; ++i) hist[4 * lane + i] = 0;  // ready for the next pass
                const int mine = c[0] + c[1] + c[2] + c[3];
                int incl = mine;  // candidates in lanes >= this one
#pragma unroll
                for (int off = 1; off < kWave; off <<= 1) {
                    const int x = __shfl_down(incl, off, kWave);
                    if (lane + off < kWave) incl += x;
                }
                int above = incl - mine;  // candidates with a digit above this lane's four
#pragma unroll
                for (int i = 3; i >= 0; --i) {
                    if (above < need && need <= above + c[i]) {  // exactly one digit satisfies this
                        sh_prefix = prefix | ((uint32_t)(4 * lane + i) << shift);
                        sh_need = need - above;
                    }
                    above += c[i];
                }
            }
            __syncthreads();
        }
    }
    const uint32_t kth = sh_prefix;  // key of the last selected unprotected element
    const int need_eq = sh_need;     // how many elements equal to kth are selected (lowest positions)

    // ---- ordered emission ----
    // One workgroup scan per 1024 positions carries two counts, packed into one word: elements that are
    // kept outright (protected or above the threshold key) and elements equal to it.  Of the equal ones the
    // first need_eq are kept, so an element's output slot is (kept outright before it) + min(equal before
    // it, need_eq).
    int base_keep = 0, base_eq = 0, set = 0;
    for (int t0 = 0; t0 < T; t0 += kSelThreads, set ^= 1) {
        const int t = t0 + tid;
        bool keep = false, eq = false;
        if (t < T) {
            keep = (t < free_lo) || (t >= free_hi);
            if (!keep && n_free > 0) {
                const uint32_t key = keys_in_lds ? lds_keys[t] : score_key(s[t]);
                keep = key > kth;
                eq = key == kth;
            }
        }
        const unsigned long long ball_keep = __ballot(keep), ball_eq = __ballot(eq);
        const unsigned long long below = (1ull << lane) - 1ull;
        if (lane == 0) wave_tot[set][wave] = __popcll(ball_keep) | (__popcll(ball_eq) << 16);
        __syncthreads();
        int before = 0, tot = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) {
            const int c = wave_tot[set][w];
            before += (w < wave) ? c : 0;
            tot += c;
        }
        const int keep_before = base_keep + (before & 0xffff) + __popcll(ball_keep & below);
        const int eq_before = base_eq + (before >> 16) + __popcll(ball_eq & below);
        const int o = keep_before + min(eq_before, need_eq);
        if ((keep || (eq && eq_before < need_eq)) && o < n_anchor) dst[o] = t;
        base_keep += tot & 0xffff;
        base_eq += tot >> 16;
    }
}

int select_dispatch(const float* score, int B, int G, int T, int n_anchor, int protect_first,
                    int protect_last, int32_t* anchor_idx, const int32_t* seq_len, const int32_t* n_anchor_b,
                    hipStream_t stream)
{
    const int keys_in_lds = T <= kSelLdsKeys;
    const size_t dyn = keys_in_lds ? (size_t)T * sizeof(uint32_t) : 0;
    hipLaunchKernelGGL(select_anchors_kernel, dim3(B * G), dim3(kSelThreads), dyn, stream, score, T,
                       n_anchor, protect_first, protect_last, anchor_idx, keys_in_lds, seq_len, n_anchor_b, G);
    return status_from_hip(hipGetLastError());
}

// ------------------------------------------------------------------ retention test on the device
// Per-sequence bookkeeping of a ragged generation loop (Alg. 1's del_num and fix_idx in integer arithmetic,
// the same rules as the host function ec_evict_index), one thread per batch element.
__global__ __launch_bounds__(256) void retention_step_kernel(int32_t* __restrict__ n_seen_b,
                                                             int32_t* __restrict__ cache_len_b,
                                                             int32_t* __restrict__ evict_idx_b,
                                                             int32_t* __restrict__ new_pos_b,
                                                             int32_t* __restrict__ pending_b, int B, int gamma_num,
                                                             int gamma_den, int budget_mode, int fixed_len,
                                                             int trunc_mode, int recent, int n_tl, int protect_first,
                                                             int flush_only)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int len = cache_len_b[b];
    if (pending_b[b]) {  // the step prepared by the previous call has run: a row was appended, maybe one removed
        len += (evict_idx_b[b] < 0) ? 1 : 0;
        pending_b[b] = 0;
    }
    if (!flush_only) {
        const long long seen = (long long)n_seen_b[b] + 1;
        const long long after = (long long)len + 1;
        long long keep;
        if (budget_mode == EC_BUDGET_RATIO) {
            const long long prod = (long long)gamma_num * seen;
            keep = prod / gamma_den + ((prod % gamma_den) ? 1 : 0);
        } else {
            keep = fixed_len;
        }
        long long victim = -1;
        if (after > keep) {
            victim = (trunc_mode == EC_TRUNC_RECENT) ? after - 1 - recent : (long long)n_tl;
            if (victim < protect_first) victim = protect_first;
            if (victim >= after - 1) victim = -1;
        }
        n_seen_b[b] = (int32_t)seen;
        evict_idx_b[b] = (int32_t)victim;
        new_pos_b[b] = (int32_t)(seen - 1);
        pending_b[b] = 1;
    }
    cache_len_b[b] = len;
}

int retention_step_launch(int32_t* n_seen_b, int32_t* cache_len_b, int32_t* evict_idx_b, int32_t* new_pos_b,
                          int32_t* pending_b, int B, int gamma_num, int gamma_den, int budget_mode, int fixed_len,
                          int trunc_mode, int recent, int n_tl, int protect_first, int flush_only, hipStream_t stream)
{
    hipLaunchKernelGGL(retention_step_kernel, dim3((B + 255) / 256), dim3(256), 0, stream, n_seen_b, cache_len_b,
                       evict_idx_b, new_pos_b, pending_b, B, gamma_num, gamma_den, budget_mode, fixed_len, trunc_mode,
                       recent, n_tl, protect_first, flush_only);
    return status_from_hip(hipGetLastError());
}

}  // namespace ec
