// ec_prefill_score / ec_chunk_score, matrix-core path for bf16 inputs (Sec. 3.3, Eq. 1 and I_n = sum_m A_mn).
// Geometry (ScoreGeom): Tq queries over L = P + Tq key rows, query m sees rows n <= P + m; the first-turn
// prompt pass is P = 0.
//
// Three kernels, none of which stores the T x T matrix:
//   vt_transpose : V [T,D] -> V^T [D,Tp] per head (zero-padded to a multiple of 64 keys), so that
//                  the contraction index of P.V is contiguous in memory for the MFMA operands.
//   attn_fwd     : one workgroup = 128 or 256 queries (4 or 8 waves x 32), key tiles of 64 double-
//                  buffered in LDS.  The score tile is computed TRANSPOSED, S^T = K.Q^T, with
//                  v_mfma_f32_32x32x16_bf16: in the accumulator layout a lane then owns one query
//                  (column) and 16 keys (rows), so the row max / row sum of the online softmax are
//                  in-lane reductions plus one exchange between the two half-waves, the rescale
//                  factor is a per-lane scalar, and the fp32 accumulators -- rounded to bf16 -- are
//                  directly the B operand of O^T += V^T.P^T (the contraction index is permuted the
//                  same way on both operands).  Emits out (optional) and the row log-sum-exp.
//   colsum       : one workgroup = 128 keys (4 waves x 32) whose K fragments stay in registers;
//                  query tiles of 64 at or below the diagonal are streamed through LDS, S = Q.K^T
//                  is recomputed un-transposed so that a lane owns one key (column): p =
//                  exp(s - lse_row) is summed down the column in-lane.  One workgroup owns a column,
//                  so there are no atomics and the result is deterministic.
//
// MFMA operand layout used throughout (wave64, lane l, half h = l / 32):
//   A (32 x 16): lane holds A[l % 32][8h .. 8h+7]      B (16 x 32): lane holds B[8h .. 8h+7][l % 32]
//   C (32 x 32): lane holds C[8g + 4h + t][l % 32] in register 4g + t, g,t in 0..3
#include "ec_common.h"

namespace ec {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;  // 16-byte staging register (native vector: stays in VGPRs)

constexpr int kMfmaThreads = 256;
constexpr int kFwdBN = 64;   // keys per LDS tile
constexpr int kColBN = 128;  // keys per workgroup in colsum (32 per wave)
constexpr int kColBM = 64;   // queries per LDS tile in colsum (128 measured slower: it halves the occupancy)
constexpr int kVtPitch = kFwdBN + 8;  // bf16 elements per V^T row in LDS (144 B: conflict-free b128 reads)

__host__ __device__ inline int padded_T(int T) { return (T + 63) / 64 * 64; }

// Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.  Work
// items are therefore renumbered so that one XCD gets a CONTIGUOUS range of items: all tiles of a
// head (which share its K and V) then sit behind the same L2 instead of being fetched eight times.
constexpr int kXcds = 8;
inline int xcd_grid(int total) { return (total + kXcds - 1) / kXcds * kXcds; }
__device__ __forceinline__ int xcd_contiguous_item(int linear_id, int total)
{
    const int per_xcd = (total + kXcds - 1) / kXcds;
    if (linear_id / kXcds >= per_xcd) return total;
    return (linear_id % kXcds) * per_xcd + linear_id / kXcds;  // may be >= total: caller exits
}

// ------------------------------------------------------------------ V^T
__global__ __launch_bounds__(256) void vt_transpose_kernel(const uint16_t* __restrict__ v,
                                                           uint16_t* __restrict__ vt, int T_max, int Tp, int D,
                                                           int kv_rows, const int32_t* __restrict__ seq_len, int H)
{
    __shared__ uint16_t tile[64][64 + 2];
    const int bh = blockIdx.z;
    const int T = ragged_rows(seq_len, bh / H, T_max);  // rows beyond it are written as zeros
    const int n0 = blockIdx.x * 64, d0 = blockIdx.y * 64;
    const uint16_t* src = v + (size_t)bh * kv_rows * D;
    uint16_t* dst = vt + (size_t)bh * D * Tp;
    for (int i = threadIdx.x; i < 64 * 32; i += 256) {  // pairs of elements along d
        const int r = i / 32, c = (i % 32) * 2;
        uint32_t x = 0;
        if (n0 + r < T) x = *reinterpret_cast<const uint32_t*>(src + (size_t)(n0 + r) * D + d0 + c);
        tile[r][c] = (uint16_t)(x & 0xffffu);
        tile[r][c + 1] = (uint16_t)(x >> 16);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < 64 * 32; i += 256) {  // pairs of elements along n
        const int d = i / 32, c = (i % 32) * 2;
        const uint32_t x = (uint32_t)tile[c][d] | ((uint32_t)tile[c + 1][d] << 16);
        *reinterpret_cast<uint32_t*>(dst + (size_t)(d0 + d) * Tp + n0 + c) = x;
    }
}

// ------------------------------------------------------------------ forward
// Double-buffered: the global loads of key tile i+1 are issued before tile i is consumed and land
// in the other LDS buffer after it, so there is one barrier per tile and the HBM/L2 latency is
// hidden behind the MFMA + softmax work of the current tile.
template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * kWave, 2) void attn_fwd_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ vt,
    uint16_t* __restrict__ out, float* __restrict__ lse, ScoreGeom geo, int Tp, float scale_log2e, int n_qtiles,
    int n_heads, const int32_t* __restrict__ seq_len, int H)
{
    constexpr int THREADS = WAVES * kWave;
    constexpr int BM = WAVES * 32;   // queries per workgroup
    constexpr int KB = D / 16;       // contraction blocks of Q.K
    constexpr int DB = D / 32;       // 32-row blocks of O^T
    constexpr int KP = D + 8;        // K tile pitch in elements (272 B for D=128: conflict-free b128)
    constexpr int KCH = kFwdBN * (D / 8) / THREADS;  // 16-byte chunks of the K tile per thread
    constexpr int VCH = D * (kFwdBN / 8) / THREADS;  // 16-byte chunks of the V^T tile per thread
    __shared__ __align__(16) uint16_t ks[2][kFwdBN * KP];
    __shared__ __align__(16) uint16_t vs[2][D * kVtPitch];

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int c32 = lane % 32, h = lane / 32;
    // LDS row j of the K tile holds key swap23(j) (bits 2 and 3 of the row number exchanged), i.e. row
    // i of a 32-key S^T block is key 16(i/16) + 8((i/4)%2) + 4((i/8)%2) + i%4.  In the accumulator
    // layout (register 4g+t of half h = row 8g+4h+t) registers 8G..8G+7 of a lane then hold the 8
    // CONSECUTIVE keys 16G + 8h .. +7: the P fragment of a P.V MFMA is a run of registers and its V^T
    // operand a single 16-byte LDS read, while the K-tile reads stay linear and conflict-free.
    const int item = xcd_contiguous_item(blockIdx.x, n_qtiles * n_heads);
    if (item >= n_qtiles * n_heads) return;
    const int bh = item / n_qtiles;
    const int Tq = ragged_rows(seq_len, bh / H, geo.Tq), P = geo.P, L = P + Tq;
    const int m0 = (n_qtiles - 1 - item % n_qtiles) * BM;  // longest rows first inside a head
    if (m0 >= Tq) return;  // ragged batch: this sequence ends before the tile (whole workgroup)
    const int mw = m0 + wave * 32;                          // first query of this wave
    const int m = mw + c32;                            // this lane's query
    const uint16_t* qh = q + (size_t)bh * geo.q_rows * D;
    const uint16_t* kh = k + (size_t)bh * geo.kv_rows * D;
    const uint16_t* vth = vt + (size_t)bh * D * Tp;
    const bool want_out = out != nullptr;

    bf16x8 qf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        uint4 x = make_uint4(0, 0, 0, 0);
        if (m < Tq) x = *reinterpret_cast<const uint4*>(qh + (size_t)m * D + kb * 16 + h * 8);
        qf[kb] = __builtin_bit_cast(bf16x8, x);
    }

    f32x16 o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;  // l_run: this half-wave's share of the row sum

    u32x4 kreg[KCH], vreg[VCH];
    auto fetch = [&](int n0) {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int c = tid + i * THREADS;
            const int r = c / (D / 8), cc = c % (D / 8);
            kreg[i] = u32x4{0u, 0u, 0u, 0u};
            if (n0 + r < L) kreg[i] = *reinterpret_cast<const u32x4*>(kh + (size_t)(n0 + r) * D + cc * 8);
        }
        if (want_out) {
#pragma unroll
            for (int i = 0; i < VCH; ++i) {
                const int c = tid + i * THREADS;
                const int d = c / (kFwdBN / 8), cc = c % (kFwdBN / 8);
                vreg[i] = *reinterpret_cast<const u32x4*>(vth + (size_t)d * Tp + n0 + cc * 8);
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < KCH; ++i) {
            const int c = tid + i * THREADS;
            const int r = c / (D / 8), cc = c % (D / 8);
            const int lr = (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1);  // swap23
            *reinterpret_cast<u32x4*>(&ks[buf][lr * KP + cc * 8]) = kreg[i];
        }
        if (want_out) {
#pragma unroll
            for (int i = 0; i < VCH; ++i) {
                const int c = tid + i * THREADS;
                const int d = c / (kFwdBN / 8), cc = c % (kFwdBN / 8);
                *reinterpret_cast<u32x4*>(&vs[buf][d * kVtPitch + cc * 8]) = vreg[i];
            }
        }
    };

    const int n_end = min(L, P + m0 + BM);  // the workgroup's last query sees rows up to P + m0 + BM - 1
    fetch(0);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int n0 = 0; n0 < n_end; n0 += kFwdBN, buf ^= 1) {
        const bool more = n0 + kFwdBN < n_end;
        if (more) fetch(n0 + kFwdBN);

        if (n0 <= P + mw + 31) {  // otherwise every key of the tile is in this wave's future
            // S^T = K . Q^T : two 32-key blocks x this wave's 32 queries
            f32x16 s[2];
            {
                bf16x8 ka[2][KB];  // every A fragment of the tile is requested before the first MFMA
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        ka[nb][kb] = *reinterpret_cast<const bf16x8*>(
                            &ks[buf][(nb * 32 + c32) * KP + kb * 16 + h * 8]);
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[nb][r] = 0.f;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
                        s[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[nb][kb], qf[kb], s[nb], 0, 0, 0);
                // LDS reads run ahead of the matrix pipe: 4 in flight, then one read per MFMA
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
                for (int i = 0; i < 2 * KB - 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            }
            // causal mask (diagonal tiles only), row max on the raw products
            if ((n0 + kFwdBN - 1 > P + mw) || (n0 + kFwdBN > L)) {
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int n = n0 + nb * 32 + (r / 8) * 16 + h * 8 + (r % 8);  // key of register r
                        if (n > P + m || n >= L) s[nb][r] = -INFINITY;
                    }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[nb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, kWave)) * scale_log2e;
            const float m_new = fmaxf(m_run, mx);  // finite: key 0 is visible to every query
            const bool grew = m_new > m_run;
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);  // exp2(-inf) = 0 on the first tile
            m_run = m_new;
            float psum = 0.f;
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s[nb][r], scale_log2e, -m_new));
                    s[nb][r] = p;
                    psum += p;
                }
            l_run = l_run * corr + psum;

            if (want_out) {
                if (__any(grew)) {  // wave-uniform: the running max settles after a few tiles
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) o[db][r] *= corr;
                }
                // O^T += V^T . P^T, 16 keys per MFMA: half h contracts keys 16G + 8h .. +7 (G = kk % 2)
                bf16x8 va[4][DB];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        va[kk][db] = *reinterpret_cast<const bf16x8*>(
                            &vs[buf][(db * 32 + c32) * kVtPitch + kk * 16 + h * 8]);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const int nb = kk / 2, r0 = (kk % 2) * 8;
                    bf16x8 pf;
#pragma unroll
                    for (int t = 0; t < 8; ++t) pf[t] = (__bf16)s[nb][r0 + t];
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[kk][db], pf, o[db], 0, 0, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 1);
#pragma unroll
                for (int i = 0; i < 4 * DB - 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 1);
            }
        }
        if (more) stage(buf ^ 1);  // that buffer was last read before the previous barrier
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (m < Tq) {
        if (h == 0) lse[(size_t)bh * geo.q_rows + m] = (m_run + log2f(l_tot)) * kLn2;
        if (want_out) {
            const float inv = 1.f / l_tot;
            uint16_t* orow = out + ((size_t)bh * geo.q_rows + m) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    bf16x4 y;
#pragma unroll
                    for (int t = 0; t < 4; ++t) y[t] = (__bf16)(o[db][g * 4 + t] * inv);
                    *reinterpret_cast<bf16x4*>(orow + db * 32 + g * 8 + h * 4) = y;
                }
        }
    }
}

// ------------------------------------------------------------------ column mass
template <int D>
__global__ __launch_bounds__(kMfmaThreads) void colsum_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const float* __restrict__ lse,
    float* __restrict__ head_imp, ScoreGeom geo, float scale_log2e, int n_ktiles, int n_heads,
    const int32_t* __restrict__ seq_len, int H)
{
    constexpr int KB = D / 16;
    constexpr int QP = D + 8;
    __shared__ __align__(16) uint16_t qs[2][kColBM * QP];
    __shared__ __align__(16) float lse2[2][kColBM];  // row log-sum-exp in base-2 units

    const int tid = threadIdx.x, wave = tid / kWave, lane = tid % kWave;
    const int c32 = lane % 32, h = lane / 32;
    const int item = xcd_contiguous_item(blockIdx.x, n_ktiles * n_heads);
    if (item >= n_ktiles * n_heads) return;
    const int bh = item / n_ktiles;
    const int Tq = ragged_rows(seq_len, bh / H, geo.Tq), P = geo.P, L = P + Tq;
    const int n0 = (item % n_ktiles) * kColBN;  // low key tiles (most query tiles) first inside a head
    if (n0 >= L) return;  // ragged batch: this sequence ends before the tile (whole workgroup)
    const int n = n0 + wave * 32 + c32;  // this lane's key
    const uint16_t* qh = q + (size_t)bh * geo.q_rows * D;
    const uint16_t* kh = k + (size_t)bh * geo.kv_rows * D;
    const float* lh = lse + (size_t)bh * geo.q_rows;

    bf16x8 kf[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        uint4 x = make_uint4(0, 0, 0, 0);
        if (n < L) x = *reinterpret_cast<const uint4*>(kh + (size_t)n * D + kb * 16 + h * 8);
        kf[kb] = __builtin_bit_cast(bf16x8, x);
    }

    constexpr int QCH = kColBM * (D / 8) / kMfmaThreads;  // 16-byte chunks of the Q tile per thread
    u32x4 qreg[QCH];
    float lreg = 0.f;
    auto fetch = [&](int m0) {
#pragma unroll
        for (int i = 0; i < QCH; ++i) {
            const int c = tid + i * kMfmaThreads;
            const int r = c / (D / 8), cc = c % (D / 8);
            qreg[i] = u32x4{0u, 0u, 0u, 0u};
            if (m0 + r < Tq) qreg[i] = *reinterpret_cast<const u32x4*>(qh + (size_t)(m0 + r) * D + cc * 8);
        }
        if (tid < kColBM) lreg = (m0 + tid < Tq) ? lh[m0 + tid] * kLog2e : INFINITY;
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < QCH; ++i) {
            const int c = tid + i * kMfmaThreads;
            const int r = c / (D / 8), cc = c % (D / 8);
            *reinterpret_cast<u32x4*>(&qs[buf][r * QP + cc * 8]) = qreg[i];
        }
        if (tid < kColBM) lse2[buf][tid] = lreg;
    };

    float col = 0.f;
    const int m_begin = (max(n0 - P, 0) / kColBM) * kColBM;  // first query tile that sees key n0 (query m sees n <= P + m)
    fetch(m_begin);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int m0 = m_begin; m0 < Tq; m0 += kColBM, buf ^= 1) {
        const bool more = m0 + kColBM < Tq;
        if (more) fetch(m0 + kColBM);

        if (P + m0 + kColBM - 1 >= n0 + wave * 32) {  // else no query of the tile sees this wave's keys
            constexpr int MB = kColBM / 32;  // 32-query blocks per tile
#pragma unroll
            for (int mp = 0; mp < MB; mp += 2) {  // two blocks at a time: two independent MFMA chains
                f32x16 s[2];
                bf16x8 qa[2][KB];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
                        qa[mb][kb] = *reinterpret_cast<const bf16x8*>(
                            &qs[buf][((mp + mb) * 32 + c32) * QP + kb * 16 + h * 8]);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[mb][r] = 0.f;
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
                        s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[mb][kb], kf[kb], s[mb], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
                for (int i = 0; i < 2 * KB - 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);

                // p = exp(s - lse_row), summed down the column.  Only blocks that touch the diagonal need
                // the causal mask; the others take the three-instruction path (fma, exp, add).
                const int mq = m0 + mp * 32;                     // first query of this pair of blocks
                const bool diag = P + mq < n0 + wave * 32 + 31;  // some (query, key) pair is masked
                if (diag) {
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const float4 l4 =
                                *reinterpret_cast<const float4*>(&lse2[buf][(mp + mb) * 32 + g * 8 + h * 4]);
                            const float lr[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                            for (int t = 0; t < 4; ++t) {
                                const float p = __builtin_amdgcn_exp2f(fmaf(s[mb][g * 4 + t], scale_log2e, -lr[t]));
                                const int mm = mq + mb * 32 + g * 8 + h * 4 + t;
                                col += (P + mm >= n) ? p : 0.f;  // rows beyond Tq carry lse = +inf, so p = 0
                            }
                        }
                } else {
                    float c0 = 0.f, c1 = 0.f;  // two chains keep the adds off the exp latency
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const float4 l4 =
                                *reinterpret_cast<const float4*>(&lse2[buf][(mp + mb) * 32 + g * 8 + h * 4]);
                            c0 += __builtin_amdgcn_exp2f(fmaf(s[mb][g * 4 + 0], scale_log2e, -l4.x));
                            c1 += __builtin_amdgcn_exp2f(fmaf(s[mb][g * 4 + 1], scale_log2e, -l4.y));
                            c0 += __builtin_amdgcn_exp2f(fmaf(s[mb][g * 4 + 2], scale_log2e, -l4.z));
                            c1 += __builtin_amdgcn_exp2f(fmaf(s[mb][g * 4 + 3], scale_log2e, -l4.w));
                        }
                    col += c0 + c1;
                }
            }
        }
        if (more) stage(buf ^ 1);
        __syncthreads();
    }
    col += __shfl_xor(col, 32, kWave);
    if (h == 0 && n < L) head_imp[(size_t)bh * geo.imp_rows + n] = col;
}

template <int D>
static int launch_mfma(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse,
                       float* head_imp, uint16_t* vt, int B, int H, ScoreGeom geo, const int32_t* seq_len, float scale,
                       int forced_waves, hipStream_t stream)
{
    const float sl = scale * kLog2e;
    const int Tq = geo.Tq, L = geo.L;
    const int Lp = padded_T(L);
    const int BH = B * H;
    if (out != nullptr) {
        hipLaunchKernelGGL(vt_transpose_kernel, dim3(Lp / 64, D / 64, BH), dim3(256), 0, stream, v, vt, L, Lp, D,
                           geo.kv_rows, seq_len, H);
        int rc = status_from_hip(hipGetLastError());
        if (rc != EC_OK) return rc;
    }
    // 8-wave workgroups (256 queries) halve the LDS staging per flop, which pays once the key loop is long
    // (measured crossover between 2048 and 3072 keys); 4-wave ones balance shorter prompts better
    int waves = forced_waves;
    if (waves != 4 && waves != 8) waves = (L >= 2560 && (long long)BH * ((Tq + 255) / 256) >= 512) ? 8 : 4;
    if (waves == 8)
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, 8>), dim3(xcd_grid(((Tq + 255) / 256) * BH)), dim3(512), 0,
                           stream, q, k, vt, out, lse, geo, Lp, sl, (Tq + 255) / 256, BH, seq_len, H);
    else
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, 4>), dim3(xcd_grid(((Tq + 127) / 128) * BH)), dim3(256), 0,
                           stream, q, k, vt, out, lse, geo, Lp, sl, (Tq + 127) / 128, BH, seq_len, H);
    int rc = status_from_hip(hipGetLastError());
    if (rc != EC_OK) return rc;
    hipLaunchKernelGGL((colsum_mfma_kernel<D>), dim3(xcd_grid(((L + kColBN - 1) / kColBN) * BH)),
                       dim3(kMfmaThreads), 0, stream, q, k, lse, head_imp, geo, sl, (L + kColBN - 1) / kColBN, BH,
                       seq_len, H);
    return status_from_hip(hipGetLastError());
}

// bytes of workspace the V^T copy needs (T = number of key rows)
size_t score_mfma_vt_bytes(int B, int H, int T, int D) { return (size_t)B * H * D * padded_T(T) * sizeof(uint16_t); }

// Per-head importance into head_imp [B,H,L]; out may be NULL (then vt is not touched).
int score_mfma_dispatch(const void* q, const void* k, const void* v, void* out, float* lse, float* head_imp,
                        void* vt, int B, int H, ScoreGeom geo, const int32_t* seq_len, int D, int dt, float scale,
                        int forced_waves, hipStream_t stream)
{
    if (dt != EC_BF16) return EC_EUNSUPPORTED;
    if (D == 128)
        return launch_mfma<128>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)out, lse,
                                head_imp, (uint16_t*)vt, B, H, geo, seq_len, scale, forced_waves, stream);
    if (D == 64)
        return launch_mfma<64>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)out, lse,
                               head_imp, (uint16_t*)vt, B, H, geo, seq_len, scale, forced_waves, stream);
    return EC_EUNSUPPORTED;
}

}  // namespace ec
