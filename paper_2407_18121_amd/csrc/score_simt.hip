// ec_prefill_score / ec_chunk_score, vector-ALU path (fp32 arithmetic throughout).
// Geometry (ScoreGeom): Tq queries over L = P + Tq key rows, query m sees rows n <= P + m.
//
// Used for fp32 inputs, where the contraction must be true fp32 (the matrix-core
// bf16 path lives in score_mfma.hip), and as a fallback for shapes that path does
// not cover.  Two passes, neither of which stores the T x T matrix (Sec. 3.3,
// Eq. 1 and I_n = sum_m A_mn):
//   pass 1  attn_fwd : per 64-query tile, stream key tiles with an online softmax,
//                      emit out (optional) and the row log-sum-exp.
//   pass 2  colsum   : per 32-key tile, stream the query tiles at or below the
//                      diagonal, recompute s, p = exp(s - lse_row), sum p down each
//                      key column.  One workgroup owns a column, so there are no
//                      atomics and the result is deterministic.
// Then the head mean for the layer-wise score (G == 1).
#include "ec_common.h"

namespace ec {

constexpr int kSimtThreads = 256;
constexpr int kBM = 64;  // query rows per tile
constexpr int kBN = 32;  // key columns per tile
constexpr int kDC = 32;  // head-dim chunk staged in LDS

struct alignas(16) SimtSmem {
    float qt[kDC][kBM + 4];  // transposed Q chunk: [d][row]
    float kt[kDC][kBN + 4];  // transposed K chunk: [d][col]
};

template <int DT> __device__ __forceinline__ void load4(const void* base, size_t elem_off, float* f)
{
    if constexpr (DT == EC_F32) {
        const float4 x = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(base) + elem_off);
        f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w;
    } else {
        const uint2 x = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(base) + elem_off);
        f[0] = __uint_as_float(x.x << 16);
        f[1] = __uint_as_float(x.x & 0xffff0000u);
        f[2] = __uint_as_float(x.y << 16);
        f[3] = __uint_as_float(x.y & 0xffff0000u);
    }
}

// s[i][j] = sum_d Q[m0 + ty*4 + i][d] * K[n0 + tx*2 + j][d]   (unscaled)
// Query rows at or beyond Tq and key rows at or beyond L read as zero.
template <int DT, int D>
__device__ __forceinline__ void s_tile(const void* qh, const void* kh, int m0, int n0, int Tq, int L,
                                       SimtSmem& sm, float s[4][2])
{
    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
#pragma unroll
    for (int i = 0; i < 4; ++i) s[i][0] = s[i][1] = 0.f;
    for (int d0 = 0; d0 < D; d0 += kDC) {
        __syncthreads();
        for (int u = tid; u < kBM * (kDC / 4); u += kSimtThreads) {
            const int r = u % kBM, c = u / kBM;
            float f[4] = {0.f, 0.f, 0.f, 0.f};
            if (m0 + r < Tq) load4<DT>(qh, (size_t)(m0 + r) * D + d0 + c * 4, f);
#pragma unroll
            for (int i = 0; i < 4; ++i) sm.qt[c * 4 + i][r] = f[i];
        }
        for (int u = tid; u < kBN * (kDC / 4); u += kSimtThreads) {
            const int r = u % kBN, c = u / kBN;
            float f[4] = {0.f, 0.f, 0.f, 0.f};
            if (n0 + r < L) load4<DT>(kh, (size_t)(n0 + r) * D + d0 + c * 4, f);
#pragma unroll
            for (int i = 0; i < 4; ++i) sm.kt[c * 4 + i][r] = f[i];
        }
        __syncthreads();
#pragma unroll 8
        for (int dd = 0; dd < kDC; ++dd) {
            const float4 a = *reinterpret_cast<const float4*>(&sm.qt[dd][ty * 4]);
            const float2 b = *reinterpret_cast<const float2*>(&sm.kt[dd][tx * 2]);
            s[0][0] = fmaf(a.x, b.x, s[0][0]); s[0][1] = fmaf(a.x, b.y, s[0][1]);
            s[1][0] = fmaf(a.y, b.x, s[1][0]); s[1][1] = fmaf(a.y, b.y, s[1][1]);
            s[2][0] = fmaf(a.z, b.x, s[2][0]); s[2][1] = fmaf(a.z, b.y, s[2][1]);
            s[3][0] = fmaf(a.w, b.x, s[3][0]); s[3][1] = fmaf(a.w, b.y, s[3][1]);
        }
    }
}

__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, dpp_mov<kDppQuadXor1>(x));
    x = fmaxf(x, dpp_mov<kDppQuadXor2>(x));
    x = fmaxf(x, dpp_mov<kDppRowHalfMirror>(x));
    x = fmaxf(x, dpp_mov<kDppRowMirror>(x));
    return x;
}

template <int DT, int D>
__global__ __launch_bounds__(kSimtThreads) void attn_fwd_simt_kernel(
    const void* __restrict__ q, const void* __restrict__ k, const void* __restrict__ v,
    void* __restrict__ out, float* __restrict__ lse, ScoreGeom geo, float scale_log2e,
    const int32_t* __restrict__ seq_len, int H)
{
    constexpr int CPT = D / 16;  // output columns per thread
    const int Tq = ragged_rows(seq_len, blockIdx.y / H, geo.Tq), P = geo.P, L = P + Tq;
    __shared__ SimtSmem sm;
    __shared__ float ps[kBM][kBN + 1];
    __shared__ __align__(16) float vs[kBN][D];

    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int bh = blockIdx.y;
    const int m0 = (gridDim.x - 1 - blockIdx.x) * kBM;  // longest rows first
    if (m0 >= Tq) return;  // ragged batch: this sequence ends before the tile (whole workgroup)
    using E = typename Elem<DT>::type;
    const E* qh = reinterpret_cast<const E*>(q) + (size_t)bh * geo.q_rows * D;
    const E* kh = reinterpret_cast<const E*>(k) + (size_t)bh * geo.kv_rows * D;
    const E* vh = reinterpret_cast<const E*>(v) + (size_t)bh * geo.kv_rows * D;

    float m_run[4], l_run[4], o[4][CPT];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        m_run[i] = -INFINITY;
        l_run[i] = 0.f;
#pragma unroll
        for (int c = 0; c < CPT; ++c) o[i][c] = 0.f;
    }

    const int n_end = min(L, P + m0 + kBM);  // causal: keys up to the last query of the tile
    for (int n0 = 0; n0 < n_end; n0 += kBN) {
        float s[4][2];
        s_tile<DT, D>(qh, kh, m0, n0, Tq, L, sm, s);
        // stage V tile (rows beyond L read as zero)
        for (int u = tid; u < kBN * (D / 4); u += kSimtThreads) {
            const int r = u / (D / 4), c = u % (D / 4);
            float f[4] = {0.f, 0.f, 0.f, 0.f};
            if (n0 + r < L) load4<DT>(vh, (size_t)(n0 + r) * D + c * 4, f);
            *reinterpret_cast<float4*>(&vs[r][c * 4]) = make_float4(f[0], f[1], f[2], f[3]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + ty * 4 + i;
            float sv[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + tx * 2 + j;
                sv[j] = (n <= P + m && n < L) ? s[i][j] * scale_log2e : -INFINITY;
            }
            const float mt = row16_max(fmaxf(sv[0], sv[1]));
            const float m_new = fmaxf(m_run[i], mt);
            float corr = 1.f, p0 = 0.f, p1 = 0.f;
            if (m_new > -INFINITY) {
                corr = exp2f(m_run[i] - m_new);
                p0 = exp2f(sv[0] - m_new);
                p1 = exp2f(sv[1] - m_new);
            }
            const float rs = group_sum<16>(p0 + p1);
            l_run[i] = l_run[i] * corr + rs;
            m_run[i] = m_new;
#pragma unroll
            for (int c = 0; c < CPT; ++c) o[i][c] *= corr;
            ps[ty * 4 + i][tx * 2] = p0;
            ps[ty * 4 + i][tx * 2 + 1] = p1;
        }
        __syncthreads();
        if (out != nullptr) {
            for (int n = 0; n < kBN; ++n) {
                float vv[CPT];
#pragma unroll
                for (int c = 0; c < CPT; c += 4) {
                    const float4 x = *reinterpret_cast<const float4*>(&vs[n][tx * CPT + c]);
                    vv[c] = x.x; vv[c + 1] = x.y; vv[c + 2] = x.z; vv[c + 3] = x.w;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = ps[ty * 4 + i][n];
#pragma unroll
                    for (int c = 0; c < CPT; ++c) o[i][c] = fmaf(p, vv[c], o[i][c]);
                }
            }
        }
        // the next s_tile starts with a barrier, which also protects ps/vs
    }

#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= Tq) continue;
        if (tx == 0) lse[(size_t)bh * geo.q_rows + m] = (m_run[i] + log2f(l_run[i])) * kLn2;
        if (out != nullptr) {
            const float inv = 1.f / l_run[i];
            E* orow = reinterpret_cast<E*>(out) + ((size_t)bh * geo.q_rows + m) * D + tx * CPT;
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const float r = o[i][c] * inv;
                if constexpr (DT == EC_F32)
                    orow[c] = r;
                else
                    orow[c] = f32_to_bf16(r);
            }
        }
    }
}

template <int DT, int D>
__global__ __launch_bounds__(kSimtThreads) void colsum_simt_kernel(
    const void* __restrict__ q, const void* __restrict__ k, const float* __restrict__ lse,
    float* __restrict__ head_imp, ScoreGeom geo, float scale_log2e, const int32_t* __restrict__ seq_len, int H)
{
    __shared__ SimtSmem sm;
    __shared__ float red[16][kBN];
    const int Tq = ragged_rows(seq_len, blockIdx.y / H, geo.Tq), P = geo.P, L = P + Tq;

    const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
    const int bh = blockIdx.y;
    const int n0 = blockIdx.x * kBN;  // low key tiles (most query tiles) are scheduled first
    if (n0 >= L) return;  // ragged batch: this sequence ends before the tile (whole workgroup)
    using E = typename Elem<DT>::type;
    const E* qh = reinterpret_cast<const E*>(q) + (size_t)bh * geo.q_rows * D;
    const E* kh = reinterpret_cast<const E*>(k) + (size_t)bh * geo.kv_rows * D;
    const float* lh = lse + (size_t)bh * geo.q_rows;

    float col[2] = {0.f, 0.f};
    for (int m0 = (max(n0 - P, 0) / kBM) * kBM; m0 < Tq; m0 += kBM) {  // query m sees keys n <= P + m
        float s[4][2];
        s_tile<DT, D>(qh, kh, m0, n0, Tq, L, sm, s);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + ty * 4 + i;
            if (m >= Tq) continue;
            const float l2 = lh[m] * kLog2e;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int n = n0 + tx * 2 + j;
                if (n <= P + m) col[j] += exp2f(s[i][j] * scale_log2e - l2);
            }
        }
    }
    red[ty][tx * 2] = col[0];
    red[ty][tx * 2 + 1] = col[1];
    __syncthreads();
    if (tid < kBN && n0 + tid < L) {
        float acc = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc += red[r][tid];
        head_imp[(size_t)bh * geo.imp_rows + n0 + tid] = acc;
    }
}

// score[b][n] = (1/H) sum_h head_imp[b][h][n], heads added in ascending order.
__global__ __launch_bounds__(64) void head_mean_kernel(const float* __restrict__ head_imp,
                                                        float* __restrict__ score, int H, int T)
{
    const int b = blockIdx.y;
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= T) return;
    // loads are issued 8 at a time; the additions keep ascending head order
    float acc = 0.f;
    int h = 0;
    for (; h + 8 <= H; h += 8) {
        float x[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = head_imp[((size_t)b * H + h + j) * T + n];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc += x[j];
    }
    for (; h < H; ++h) acc += head_imp[((size_t)b * H + h) * T + n];
    score[(size_t)b * T + n] = acc / (float)H;
}

int head_mean_launch(const float* head_imp, float* score, int B, int H, int T, hipStream_t stream)
{
    hipLaunchKernelGGL(head_mean_kernel, dim3((T + 63) / 64, B), dim3(64), 0, stream, head_imp, score, H, T);
    return status_from_hip(hipGetLastError());
}

// "Mean" importance metric: column mass over the number of queries that see the row (in place).
__global__ __launch_bounds__(256) void importance_mean_kernel(float* __restrict__ score, int Tq, int P, size_t rows)
{
    const int L = P + Tq;
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= L) return;
    const float seen = (float)(Tq - max(n - P, 0));
    for (size_t r = blockIdx.y; r < rows; r += gridDim.y) score[r * L + n] /= seen;
}

int importance_mean_launch(float* score, int B, int G, int Tq, int P, hipStream_t stream)
{
    const size_t rows = (size_t)B * G;
    const int L = P + Tq;
    hipLaunchKernelGGL(importance_mean_kernel, dim3((L + 255) / 256, (unsigned)(rows < 65535 ? rows : 65535)), dim3(256), 0,
                       stream, score, Tq, P, rows);
    return status_from_hip(hipGetLastError());
}

template <int DT, int D>
static int launch_simt(const void* q, const void* k, const void* v, void* out, float* lse,
                       float* head_imp, int B, int H, ScoreGeom geo, const int32_t* seq_len, float scale,
                       hipStream_t stream)
{
    const float sl = scale * kLog2e;
    dim3 g1((geo.Tq + kBM - 1) / kBM, B * H);
    hipLaunchKernelGGL((attn_fwd_simt_kernel<DT, D>), g1, dim3(kSimtThreads), 0, stream, q, k, v, out, lse,
                       geo, sl, seq_len, H);
    int rc = status_from_hip(hipGetLastError());
    if (rc != EC_OK) return rc;
    dim3 g2((geo.L + kBN - 1) / kBN, B * H);
    hipLaunchKernelGGL((colsum_simt_kernel<DT, D>), g2, dim3(kSimtThreads), 0, stream, q, k, lse, head_imp,
                       geo, sl, seq_len, H);
    return status_from_hip(hipGetLastError());
}

// Per-head importance into head_imp [B,H,L]; out may be NULL.
int score_simt_dispatch(const void* q, const void* k, const void* v, void* out, float* lse,
                        float* head_imp, int B, int H, ScoreGeom geo, const int32_t* seq_len, int D, int dt,
                        float scale, hipStream_t stream)
{
#define EC_SIMT_CASE(DT_, D_)                                                                     \
    if (dt == DT_ && D == D_)                                                                     \
        return launch_simt<DT_, D_>(q, k, v, out, lse, head_imp, B, H, geo, seq_len, scale, stream);
    EC_SIMT_CASE(EC_F32, 64)
    EC_SIMT_CASE(EC_F32, 128)
    EC_SIMT_CASE(EC_BF16, 64)
    EC_SIMT_CASE(EC_BF16, 128)
#undef EC_SIMT_CASE
    return EC_EUNSUPPORTED;
}

}  // namespace ec
