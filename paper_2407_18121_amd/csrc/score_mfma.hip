// ec_prefill_score / ec_chunk_score, matrix-core path for bf16 inputs (Sec. 3.3, Eq. 1 and I_n = sum_m A_mn).
// Geometry (ScoreGeom): Tq queries over L = P + Tq key rows, query m sees rows n <= P + m; the first-turn
// prompt pass is P = 0.
//
// Two kernels, neither of which stores the T x T matrix:
//   attn_fwd     : one workgroup = 128 or 256 queries (4 or 8 waves x 32), key tiles of 64 double-
//                  buffered in LDS.  The score tile is computed TRANSPOSED, S^T = K.Q^T, with
//                  v_mfma_f32_32x32x16_bf16: in the accumulator layout a lane then owns one query
//                  (column) and 16 keys (rows), so the row max / row sum of the online softmax are
//                  in-lane reductions plus one exchange between the two half-waves, the rescale
//                  factor is a per-lane scalar, and the fp32 accumulators -- rounded to bf16 -- are
//                  directly the B operand of O^T += V^T.P^T (the contraction index is permuted the
//                  same way on both operands).  V tiles are staged as they lie in memory and transposed
//                  by the LDS transpose read on their way to the registers, so no V^T copy is made.
//                  Emits out (optional) and the row log-sum-exp.
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
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr int kMfmaThreads = 256;
constexpr int kFwdBN = 64;   // keys per LDS tile
constexpr int kSplitMaxWorkgroups = 256;  // launches of at most this many workgroups split one workgroup's loop over two wave groups
constexpr int kColBM = 64;   // queries per LDS tile in colsum (128 measured slower: it halves the occupancy)

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

// Buffer descriptor over `bytes` bytes at p (raw: no stride, 32-bit data format).  Loads through it whose byte
// offset is at or beyond `bytes` return zeros instead of touching memory.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t tile_rsrc(const void* p, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}
// The whole offset travels in the vector operand: the bounds check of this hardware generation does not see
// the scalar offset.
__device__ __forceinline__ u32x4 buffer_load_16(__amdgpu_buffer_rsrc_t rsrc, int byte_offset)
{
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_offset, 0, 0));
}

// ------------------------------------------------------------------ forward
// Double-buffered: the global loads of key tile i+1 are issued before tile i is consumed and land
// in the other LDS buffer after it, so there is one barrier per tile and the HBM/L2 latency is
// hidden behind the MFMA + softmax work of the current tile.
// KSPLIT = 2 (short prompts that give the chip one workgroup per compute unit or less): the 8 waves form two
// groups of 4 that share the workgroup's 128 queries and take alternate key tiles, each group staging its own
// tiles; their (max, sum, O) are merged through LDS at the end.  The key loop of a workgroup, which is what
// bounds such launches, is half as long, and every SIMD has two waves.
template <int D, int WAVES, int KSPLIT>
__global__ __launch_bounds__(WAVES * kWave, 2) void attn_fwd_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
    uint16_t* __restrict__ out, float* __restrict__ lse, ScoreGeom geo, float scale_log2e, int n_qtiles,
    int n_heads, const int32_t* __restrict__ seq_len, int H)
{
    constexpr int GW = WAVES / KSPLIT;  // waves of one group: one per 32 queries
    constexpr int THREADS = GW * kWave; // threads that stage one tile together
    constexpr int BM = GW * 32;      // queries per workgroup
    constexpr int KB = D / 16;       // contraction blocks of Q.K
    constexpr int DB = D / 32;       // 32-row blocks of O^T
    constexpr int KP = D + 8;        // K tile pitch in elements (272 B for D=128: conflict-free b128)
    constexpr int KCH = kFwdBN * (D / 8) / THREADS;  // 16-byte chunks of the K tile per thread
    constexpr int VP = D + 32;       // V tile pitch in elements (320 B for D=128: the transposed b64 reads measure conflict-free)
    constexpr int VCH = kFwdBN * (D / 8) / THREADS;  // 16-byte chunks of the V tile per thread
    __shared__ __align__(16) uint16_t ks_all[KSPLIT][2][kFwdBN * KP];
    __shared__ __align__(16) uint16_t vs_all[KSPLIT][2][kFwdBN * VP];

    const int lane = threadIdx.x % kWave;
    const int wave_wg = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int grp = wave_wg / GW;    // scalar: which key tiles (tile number mod KSPLIT)
    const int wave = wave_wg % GW;   // scalar: which 32 queries; tile skips branch instead of masking
    const int tid = threadIdx.x % THREADS;
    uint16_t (*ks)[kFwdBN * KP] = ks_all[grp];
    uint16_t (*vs)[kFwdBN * VP] = vs_all[grp];
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
    const uint16_t* vh = v + (size_t)bh * geo.kv_rows * D;
    const bool want_out = out != nullptr;
    // V rows sit in LDS as they are in memory (key-major); the operand of O^T += V^T.P^T needs, per lane, 8
    // keys of ONE feature.  ds_read_b64_tr_b16 does that transposition on the way out of LDS: in a group of
    // 16 lanes, lane r points at 4 consecutive features of key r/4 (features 4(r%4).. of the group's 16),
    // and lane j receives feature j of keys 0..3.  Two such reads (keys +0..3, +4..7) make one 8-key
    // fragment.  Groups 0,1 (half h = 0) take keys 0..7 of a 16-key contraction block, groups 2,3 keys 8..15.
    const int vt_lane = ((lane / 32) * 8 + (lane % 16) / 4) * VP + ((lane / 16) % 2) * 16 + (lane % 4) * 4;

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
    // l_run: this half-wave's share of the row sum.  A group that does not start at key 0 can meet a tile in
    // which a query sees no key at all; a finite floor for the running maximum keeps exp2(-inf - m) at zero
    // there instead of exp2(-inf + inf).
    float m_run = (KSPLIT == 1) ? -INFINITY : -1e30f, l_run = 0.f;

    // K and V tiles are fetched through buffer descriptors that end at the sequence's last row: a 16-byte
    // chunk beyond it comes back as zeros from the address unit itself (no compare, no branch, and 0 * padding
    // stays 0 for V), and the per-thread offset is one add per tile.
    const __amdgpu_buffer_rsrc_t k_rsrc = tile_rsrc(kh, L * D * 2);
    const __amdgpu_buffer_rsrc_t v_rsrc = tile_rsrc(vh, L * D * 2);
    u32x4 kreg[KCH], vreg[VCH];
    auto fetch = [&](int n0) {
        const int off = n0 * (D * 2) + tid * 16;  // chunk c = tid + i THREADS of the tile sits 16 c bytes into it
#pragma unroll
        for (int i = 0; i < KCH; ++i) kreg[i] = buffer_load_16(k_rsrc, off + i * THREADS * 16);
        if (want_out) {
#pragma unroll
            for (int i = 0; i < VCH; ++i) vreg[i] = buffer_load_16(v_rsrc, off + i * THREADS * 16);
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
                const int r = c / (D / 8), cc = c % (D / 8);
                *reinterpret_cast<u32x4*>(&vs[buf][r * VP + cc * 8]) = vreg[i];
            }
        }
    };

    const int n_end = min(L, P + m0 + BM);  // the workgroup's last query sees rows up to P + m0 + BM - 1
    const int n_iter = ((n_end + kFwdBN - 1) / kFwdBN + KSPLIT - 1) / KSPLIT;  // same for both groups: one barrier each
    fetch(grp * kFwdBN);
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int it = 0; it < n_iter; ++it, buf ^= 1) {
        const int n0 = (it * KSPLIT + grp) * kFwdBN;
        const bool more = n0 + KSPLIT * kFwdBN < n_end;
        if (more) fetch(n0 + KSPLIT * kFwdBN);

        if (n0 < n_end && n0 <= P + mw + 31) {  // otherwise every key of the tile is in this wave's future
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
            {   // the other half-wave holds the other 32 keys of each query: exchange through the lane-swap
                // instruction (a shuffle would go through LDS and its latency sits on the critical path)
                const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
                mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2e;
            }
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
                // O^T += V^T . P^T, 16 keys per MFMA: half h contracts keys 16 kk + 8h .. +7
                bf16x8 va[4][DB];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const uint16_t* src = &vs[buf][vt_lane + (kk * 16) * VP + db * 32];
                        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)src);
                        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(src + 4 * VP));
                        va[kk][db] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    }
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
                __builtin_amdgcn_sched_group_barrier(0x100, 8, 1);
#pragma unroll
                for (int i = 0; i < 4 * DB - 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 4, 1);
            }
        }
        if (more) stage(buf ^ 1);  // that buffer was last read before the previous barrier
        __syncthreads();
    }

    if (KSPLIT == 2) {
        // group 1 hands its state over through the K tile area (all tile reads ended at the last barrier);
        // word j of thread t sits at j * THREADS + t: consecutive lanes, consecutive words
        static_assert(KSPLIT == 1 || sizeof(ks_all) >= sizeof(float) * THREADS * (2 + DB * 16), "hand-over area");
        float* xch = reinterpret_cast<float*>(&ks_all[0][0][0]);
        if (grp == 1) {
            xch[0 * THREADS + tid] = m_run;
            xch[1 * THREADS + tid] = l_run;
            if (want_out) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) xch[(2 + db * 16 + r) * THREADS + tid] = o[db][r];
            }
        }
        __syncthreads();
        if (grp == 1) return;
        const float m1 = xch[0 * THREADS + tid], l1 = xch[1 * THREADS + tid];
        const float m_all = fmaxf(m_run, m1);  // group 0 has seen key 0: a real maximum
        const float f0 = __builtin_amdgcn_exp2f(m_run - m_all), f1 = __builtin_amdgcn_exp2f(m1 - m_all);
        l_run = l_run * f0 + l1 * f1;
        m_run = m_all;
        if (want_out) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    o[db][r] = o[db][r] * f0 + xch[(2 + db * 16 + r) * THREADS + tid] * f1;
        }
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
// One workgroup = 4 waves x NB blocks of 32 keys; the K fragments of a wave's keys stay in registers and every
// Q fragment read from LDS feeds NB matrix instructions.  Work advances in steps of 32 queries.  The
// exponentials of a step are issued between the matrix instructions of the NEXT step (the score block of a
// step is kept "pending" for one step), so that the vector and transcendental work of one block runs while
// the matrix pipe computes the following one.
// QSPLIT = 2 (launches of one workgroup per compute unit or less): 8 waves in two groups of 4 that own the same
// keys and take alternate query tiles, each group staging its own tiles; group 1's column sums are added to
// group 0's through LDS at the end (always in that order).
template <int D, int NB, bool PIPE, int MINW, int QSPLIT>
__global__ __launch_bounds__(kMfmaThreads * QSPLIT, MINW) void colsum_mfma_kernel(
    const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const float* __restrict__ lse,
    float* __restrict__ head_imp, ScoreGeom geo, float scale_log2e, int n_ktiles, int n_heads,
    const int32_t* __restrict__ seq_len, int H)
{
    constexpr int KB = D / 16;
    constexpr int QP = D + 8;
    constexpr int KEYS_W = 32 * NB;                   // keys per wave
    constexpr int BN = (kMfmaThreads / kWave) * KEYS_W;  // keys per workgroup
    __shared__ __align__(16) uint16_t qs_all[QSPLIT][2][kColBM * QP];
    __shared__ __align__(16) float lse2_all[QSPLIT][2][kColBM];  // row log-sum-exp in base-2 units
    __shared__ float col_xch[QSPLIT == 2 ? BN : 1];

    const int tid = threadIdx.x % kMfmaThreads, lane = tid % kWave;  // tid: thread within its group
    const int wave_wg = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int grp = wave_wg / (kMfmaThreads / kWave);   // scalar: which query tiles (tile number mod QSPLIT)
    const int wave = wave_wg % (kMfmaThreads / kWave);  // scalar: which keys; conditions on it branch, not mask
    uint16_t (*qs)[kColBM * QP] = qs_all[grp];
    float (*lse2)[kColBM] = lse2_all[grp];
    const int c32 = lane % 32, h = lane / 32;
    const int item = xcd_contiguous_item(blockIdx.x, n_ktiles * n_heads);
    if (item >= n_ktiles * n_heads) return;
    const int bh = item / n_ktiles;
    const int Tq = ragged_rows(seq_len, bh / H, geo.Tq), P = geo.P, L = P + Tq;
    const int n0 = (item % n_ktiles) * BN;  // low key tiles (most query tiles) first inside a head
    if (n0 >= L) return;  // ragged batch: this sequence ends before the tile (whole workgroup)
    const int nw = n0 + wave * KEYS_W;  // first key of this wave
    const uint16_t* qh = q + (size_t)bh * geo.q_rows * D;
    const uint16_t* kh = k + (size_t)bh * geo.kv_rows * D;
    const float* lh = lse + (size_t)bh * geo.q_rows;

    bf16x8 kf[NB][KB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int n = nw + nb * 32 + c32;  // this lane's key in block nb
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            uint4 x = make_uint4(0, 0, 0, 0);
            if (n < L) x = *reinterpret_cast<const uint4*>(kh + (size_t)n * D + kb * 16 + h * 8);
            kf[nb][kb] = __builtin_bit_cast(bf16x8, x);
        }
    }

    constexpr int QCH = kColBM * (D / 8) / kMfmaThreads;  // 16-byte chunks of the Q tile per thread
    u32x4 qreg[QCH];
    float lreg = 0.f;
    const __amdgpu_buffer_rsrc_t q_rsrc = tile_rsrc(qh, Tq * D * 2);  // queries beyond the sequence read as zeros
    auto fetch = [&](int m0) {
        const int off = m0 * (D * 2) + tid * 16;
#pragma unroll
        for (int i = 0; i < QCH; ++i) qreg[i] = buffer_load_16(q_rsrc, off + i * kMfmaThreads * 16);
        // no arithmetic on the loaded value here: using it would wait for every load just issued
        if (tid < kColBM) lreg = (m0 + tid < Tq) ? lh[m0 + tid] : INFINITY;
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < QCH; ++i) {
            const int c = tid + i * kMfmaThreads;
            const int r = c / (D / 8), cc = c % (D / 8);
            *reinterpret_cast<u32x4*>(&qs[buf][r * QP + cc * 8]) = qreg[i];
        }
        if (tid < kColBM) lse2[buf][tid] = lreg * kLog2e;
    };

    // PIPE: a step's score block stays "pending" for one step and its exponentials are issued between the
    // matrix instructions of the next one.  Two register sets, A and B, take turns: the first step of a query
    // tile computes into A while B is pending, the second into B while A is pending, so no block is ever
    // copied.  B's initial values make its exponentials exact zeros (rows with lse = +inf carry no mass).
    f32x16 sA[NB], sB[NB];
    float lA[16], lB[16];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sA[nb][r] = sB[nb][r] = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) lA[r] = lB[r] = INFINITY;
    int mq_pend = 0x3fffffff;  // first query of the step pending in B between tiles
    float col[NB][2];  // two chains per key keep the adds off the exp latency
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) col[nb][0] = col[nb][1] = 0.f;

    // exponentials of a block with the causal mask (steps that touch the diagonal, and the last one)
    auto exp_masked = [&](const f32x16 (&sx)[NB], const float (&lx)[16], int mq) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int n = nw + nb * 32 + c32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = __builtin_amdgcn_exp2f(fmaf(sx[nb][r], scale_log2e, -lx[r]));
                const int mm = mq + (r / 4) * 8 + h * 4 + (r % 4);
                col[nb][r & 1] += (P + mm >= n) ? p : 0.f;
            }
        }
    };
    auto exp_plain = [&](const f32x16 (&sx)[NB], const float (&lx)[16]) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                col[nb][r & 1] += __builtin_amdgcn_exp2f(fmaf(sx[nb][r], scale_log2e, -lx[r]));
    };
    // S = Q.K^T of the 32 queries of step st into sn, their log-sum-exp into ln
    auto load_q = [&](int buf, int st, bf16x8 (&qa)[KB], float (&ln)[16]) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
            qa[kb] = *reinterpret_cast<const bf16x8*>(&qs[buf][(st * 32 + c32) * QP + kb * 16 + h * 8]);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const float4 l4 = *reinterpret_cast<const float4*>(&lse2[buf][st * 32 + g * 8 + h * 4]);
            ln[g * 4 + 0] = l4.x;
            ln[g * 4 + 1] = l4.y;
            ln[g * 4 + 2] = l4.z;
            ln[g * 4 + 3] = l4.w;
        }
    };
    auto mfmas = [&](const bf16x8 (&qa)[KB], f32x16 (&sn)[NB]) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sn[nb][r] = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                sn[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[kb], kf[nb][kb], sn[nb], 0, 0, 0);
    };
    // one pipelined step: sn, ln <- step st of the tile; the pending block (sp, lp, first query mqp) is retired
    auto piped_step = [&](int buf, int st, f32x16 (&sn)[NB], float (&ln)[16], const f32x16 (&sp)[NB],
                          const float (&lp)[16], int mqp) {
        bf16x8 qa[KB];
        load_q(buf, st, qa, ln);
        if (P + mqp < nw + KEYS_W - 1) {  // some (query, key) pair of the pending step is masked
            exp_masked(sp, lp, mqp);
            mfmas(qa, sn);
        } else {
            mfmas(qa, sn);
            exp_plain(sp, lp);
            // issue order: LDS reads run ahead, then per matrix instruction two elements' worth of vector
            // work (scale-and-shift, exponential, add) of the pending block
            __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
            for (int i = 0; i < NB * KB; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
            }
        }
    };

    const int m_begin = (max(n0 - P, 0) / kColBM) * kColBM;  // first query tile that sees key n0 (query m sees n <= P + m)
    const int n_iter = ((Tq - m_begin + kColBM - 1) / kColBM + QSPLIT - 1) / QSPLIT;  // same for both groups
    fetch(m_begin + grp * kColBM);  // a tile beyond the sequence reads as zero queries with lse = +inf: no mass
    stage(0);
    __syncthreads();
    int buf = 0;
    for (int it = 0; it < n_iter; ++it, buf ^= 1) {
        const int m0 = m_begin + (it * QSPLIT + grp) * kColBM;
        const bool more = m0 + QSPLIT * kColBM < Tq;
        if (more) fetch(m0 + QSPLIT * kColBM);

        if (PIPE) {
            // a tile takes part as soon as one of its queries sees one of this wave's keys (wave-uniform); a
            // step of it that sees none is masked away like the diagonal
            if (P + m0 + kColBM - 1 >= nw) {
                static_assert(kColBM == 64, "two steps per query tile");
                piped_step(buf, 0, sA, lA, sB, lB, mq_pend);
                piped_step(buf, 1, sB, lB, sA, lA, m0);
                mq_pend = m0 + 32;
            }
        } else {
#pragma unroll
            for (int st = 0; st < kColBM / 32; ++st) {
                const int mq = m0 + st * 32;  // first query of this step
                if (mq < Tq && P + mq + 31 >= nw) {  // else no query of the step sees any of this wave's keys (wave-uniform)
                    // no pending block: this step's exponentials follow its own matrix instructions; other
                    // waves of the SIMD fill the matrix pipe meanwhile
                    bf16x8 qa[KB];
                    load_q(buf, st, qa, lA);
                    mfmas(qa, sA);
                    if (P + mq < nw + KEYS_W - 1)  // some (query, key) pair of the step is masked
                        exp_masked(sA, lA, mq);
                    else
                        exp_plain(sA, lA);
                }
            }
        }
        if (more) stage(buf ^ 1);
        __syncthreads();
    }
    if (PIPE) exp_masked(sB, lB, mq_pend);
    float csum[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        csum[nb] = col[nb][0] + col[nb][1];
        csum[nb] += __shfl_xor(csum[nb], 32, kWave);
    }
    if (QSPLIT == 2) {
        if (grp == 1 && h == 0) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) col_xch[wave * KEYS_W + nb * 32 + c32] = csum[nb];
        }
        __syncthreads();
        if (grp == 1) return;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) csum[nb] += col_xch[wave * KEYS_W + nb * 32 + c32];
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int n = nw + nb * 32 + c32;
        if (h == 0 && n < L) head_imp[(size_t)bh * geo.imp_rows + n] = csum[nb];
    }
}

template <int D>
static int launch_mfma(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out, float* lse,
                       float* head_imp, int B, int H, ScoreGeom geo, const int32_t* seq_len, float scale,
                       int forced_waves, hipStream_t stream)
{
    const float sl = scale * kLog2e;
    const int Tq = geo.Tq, L = geo.L;
    const int BH = B * H;
    // 8-wave workgroups (256 queries) halve the LDS staging per flop, which pays once the key loop is long
    // (measured crossover between 2048 and 2304 keys); 4-wave ones balance shorter prompts better
    int waves = forced_waves;
    if (waves != 4 && waves != 8) waves = (L >= 2176 && (long long)BH * ((Tq + 255) / 256) >= 512) ? 8 : 4;
    const int qt128 = (Tq + 127) / 128;
    if (waves == 8)
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, 8, 1>), dim3(xcd_grid(((Tq + 255) / 256) * BH)), dim3(512), 0,
                           stream, q, k, v, out, lse, geo, sl, (Tq + 255) / 256, BH, seq_len, H);
    else if (forced_waves == 0 && (long long)qt128 * BH <= kSplitMaxWorkgroups && L >= 4 * kFwdBN)
        // a workgroup per compute unit or less: the launch lasts as long as its longest key loop
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, 8, 2>), dim3(xcd_grid(qt128 * BH)), dim3(512), 0, stream, q, k,
                           v, out, lse, geo, sl, qt128, BH, seq_len, H);
    else
        hipLaunchKernelGGL((attn_fwd_mfma_kernel<D, 4, 1>), dim3(xcd_grid(qt128 * BH)), dim3(256), 0, stream, q, k,
                           v, out, lse, geo, sl, qt128, BH, seq_len, H);
    int rc = status_from_hip(hipGetLastError());
    if (rc != EC_OK) return rc;
    // 64 keys per wave halve the LDS reads per matrix instruction; 32 keep twice as many workgroups for
    // shapes that would otherwise leave compute units idle
    const int kt256 = (L + 255) / 256, kt128 = (L + 127) / 128;
#define EC_COLSUM(NB_, PIPE_, MINW_, KT_, QS_)                                                                   \
    hipLaunchKernelGGL((colsum_mfma_kernel<D, NB_, PIPE_, MINW_, QS_>), dim3(xcd_grid(KT_ * BH)),                \
                       dim3(kMfmaThreads * QS_), 0, stream, q, k, lse, head_imp, geo, sl, KT_, BH, seq_len, H)
    // measured (B4 H32 T8192 / B8 H32 T2048): 64 keys per wave with the pending-block pipeline 1165 / 223 us,
    // 32 keys per wave without it at four waves per SIMD 1272 / 202 us
    if ((long long)kt256 * BH >= 4096 || (L >= 6144 && (long long)kt256 * BH >= 1024))  // B2 H32 T8192: 1762 / 1802 us
        EC_COLSUM(2, true, 2, kt256, 1);
    else if ((long long)kt128 * BH <= kSplitMaxWorkgroups && Tq >= 4 * kColBM)
        EC_COLSUM(1, false, 2, kt128, 2);  // the launch lasts as long as the first key tile's loop over the queries
    else
        EC_COLSUM(1, false, 4, kt128, 1);
#undef EC_COLSUM
    return status_from_hip(hipGetLastError());
}

// Per-head importance into head_imp [B,H,L]; out may be NULL (then v is not read).
int score_mfma_dispatch(const void* q, const void* k, const void* v, void* out, float* lse, float* head_imp,
                        int B, int H, ScoreGeom geo, const int32_t* seq_len, int D, int dt, float scale,
                        int forced_waves, hipStream_t stream)
{
    if (dt != EC_BF16) return EC_EUNSUPPORTED;
    if (D == 128)
        return launch_mfma<128>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)out, lse,
                                head_imp, B, H, geo, seq_len, scale, forced_waves, stream);
    if (D == 64)
        return launch_mfma<64>((const uint16_t*)q, (const uint16_t*)k, (const uint16_t*)v, (uint16_t*)out, lse,
                               head_imp, B, H, geo, seq_len, scale, forced_waves, stream);
    return EC_EUNSUPPORTED;
}

}  // namespace ec
