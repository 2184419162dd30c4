// C ABI of libelastic_cache: argument validation, workspace carving and dispatch.
// No allocation; every launch goes to the caller's stream.  The only state is the per-device address of
// the built-in scratch array of ec_decode_score_step_static, looked up once.
#include <cmath>
#include <mutex>

#include "ec_common.h"

namespace ec {
int decode_dispatch(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                    int32_t* pos, int B, int H, int G, int D, int cap, int cache_len, int evict_idx,
                    int32_t new_pos, float scale, int dt, void* out, int forced_waves, int forced_unroll,
                    int splits, bool strict, float* part, size_t part_floats, const int32_t* len_b,
                    const int32_t* evict_b, const int32_t* new_pos_b, hipStream_t stream);
size_t decode_part_floats(int B, int H, int cap, int D);
int decode_score_dispatch(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                          int32_t* pos, float* freq, int B, int H, int G, int D, int cap, int cache_len,
                          int32_t new_pos, float scale, int dt, void* out, float* raw, float* stats,
                          hipStream_t stream);
int evict_min_dispatch(void* k_cache, void* v_cache, int32_t* pos, float* freq, int B, int H, int G, int D, int cap,
                       int len, int protect_first, int protect_recent, int dt, int32_t* victim, hipStream_t stream);
int merge_dispatch(const void* k, const void* v, const int32_t* anchor_idx, const int32_t* weights,
                   const int32_t* src_pos, int B, int H, int G, int T, int src_rows, int D, int n_anchor, int dt,
                   int evict_only, void* k_cache, void* v_cache, int cap, int32_t* counts, int32_t* assign,
                   int32_t* pos, const int32_t* seq_len, const int32_t* n_anchor_b, hipStream_t stream);
int select_dispatch(const float* score, int B, int G, int T, int n_anchor, int protect_first,
                    int protect_last, int32_t* anchor_idx, const int32_t* seq_len, const int32_t* n_anchor_b,
                    hipStream_t stream);
int score_simt_dispatch(const void* q, const void* k, const void* v, void* out, float* lse,
                        float* head_imp, int B, int H, ScoreGeom geo, const int32_t* seq_len, int D, int dt,
                        float scale, hipStream_t stream);
int score_mfma_dispatch(const void* q, const void* k, const void* v, void* out, float* lse,
                        float* head_imp, int B, int H, ScoreGeom geo, const int32_t* seq_len, int D,
                        int dt, float scale, int forced_waves, hipStream_t stream);
int retention_step_launch(int32_t* n_seen_b, int32_t* cache_len_b, int32_t* evict_idx_b, int32_t* new_pos_b,
                          int32_t* pending_b, int B, int gamma_num, int gamma_den, int budget_mode, int fixed_len,
                          int trunc_mode, int recent, int n_tl, int protect_first, int flush_only, hipStream_t stream);
int importance_mean_launch(float* score, int B, int G, int Tq, int P, hipStream_t stream);
int head_mean_launch(const float* head_imp, float* score, int B, int H, int T, hipStream_t stream);
}  // namespace ec

// Scratch of ec_decode_score_step_static: one array per GPU the library runs on, held until the process
// ends.  The name below is only a host-side handle; the device address is looked up once per device.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device), or nullptr.
void* static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

bool shape_supported(int D, int dt) { return (D == 64 || D == 128) && (dt == EC_F32 || dt == EC_BF16); }

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// The softmax kernels take the row maximum before or after scaling depending on the path; a positive finite
// scale makes the two orders agree (zero, negative, infinite and NaN scales are rejected).
bool scale_ok(float scale) { return std::isfinite(scale) && scale > 0.f; }

// Scoring pass of either entry point: Tq queries over L = P + Tq rows, heads of k/v kv_rows rows apart.
int score_pass(const void* q, const void* k, const void* v, void* out, float* lse, float* score, int B, int H,
               int G, ec::ScoreGeom geo, const int32_t* seq_len, int D, int dt, float scale, void* ws,
               size_t ws_bytes, void* stream)
{
    if (!q || !k || !v || !score) return EC_EINVAL;
    if (B < 1 || H < 1 || geo.Tq < 1 || geo.P < 0 || D < 1) return EC_EINVAL;
    if (geo.kv_rows < geo.L) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (!scale_ok(scale)) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    const size_t need = ec_workspace_bytes(EC_FN_PREFILL_SCORE, B, H, geo.L, D, dt);
    if (need == (size_t)-1) return EC_EUNSUPPORTED;
    if (!ws || ws_bytes < need) return EC_EWORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);

    const size_t stat_bytes = align256((size_t)B * H * geo.L * sizeof(float));
    float* ws_imp = reinterpret_cast<float*>(ws);
    float* ws_lse = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + stat_bytes);
    float* lse_buf = lse ? lse : ws_lse;
    float* head_imp = (G == H) ? score : ws_imp;

    int rc;
    if (dt == EC_BF16)
        rc = ec::score_mfma_dispatch(q, k, v, out, lse_buf, head_imp, B, H, geo, seq_len, D, dt, scale, 0, s);
    else
        rc = ec::score_simt_dispatch(q, k, v, out, lse_buf, head_imp, B, H, geo, seq_len, D, dt, scale, s);
    if (rc != EC_OK) return rc;
    if (G == 1) rc = ec::head_mean_launch(head_imp, score, B, H, geo.L, s);
    return rc;
}

}  // namespace

extern "C" {

const char* ec_status_string(int status)
{
    switch (status) {
        case EC_OK: return "EC_OK";
        case EC_EINVAL: return "EC_EINVAL: invalid argument";
        case EC_EUNSUPPORTED: return "EC_EUNSUPPORTED: shape or type not covered";
        case EC_EWORKSPACE: return "EC_EWORKSPACE: workspace missing or too small";
        case EC_EDEVICE: return "EC_EDEVICE: HIP launch error";
        default: return "unknown ec_status";
    }
}

size_t ec_workspace_bytes(int fn, int B, int H, int T, int D, int dt)
{
    if (B < 1 || H < 1 || T < 1) return (size_t)-1;
    switch (fn) {
        case EC_FN_PREFILL_SCORE:
            if (!shape_supported(D, dt)) return (size_t)-1;
            // per-head importance [B,H,T] + row log-sum-exp [B,H,T], fp32
            return 2 * align256((size_t)B * H * T * sizeof(float));
        case EC_FN_SELECT_ANCHORS: return 0;
        case EC_FN_MERGE_COMPACT: return 0;
        case EC_FN_DECODE_STEP:
            if (!shape_supported(D, dt)) return (size_t)-1;
            // partial (max, sum, weighted V) of every split when one (batch, head) is divided over several
            // workgroups; 0 when the batch alone fills the chip
            return align256(ec::decode_part_floats(B, H, T, D) * sizeof(float));
        case EC_FN_DECODE_SCORE_STEP:
            if (!shape_supported(D, dt)) return (size_t)-1;
            // every row's scaled score [B,H,T] + softmax maximum and denominator [B,H,2], fp32
            return align256((size_t)B * H * T * sizeof(float)) + align256((size_t)B * H * 2 * sizeof(float));
        case EC_FN_EVICT_MIN: return 0;
        default: return (size_t)-1;
    }
}

int ec_prefill_score(const void* q, const void* k, const void* v, void* out, float* lse, float* score,
                     int B, int H, int G, int T, int D, int dt, float scale, void* ws, size_t ws_bytes,
                     void* stream)
{
    if (T < 1) return EC_EINVAL;
    return score_pass(q, k, v, out, lse, score, B, H, G, ec::ScoreGeom{T, 0, T, T, T, T}, nullptr, D, dt, scale, ws,
                      ws_bytes, stream);
}

int ec_prefill_score_varlen(const void* q, const void* k, const void* v, void* out, float* lse, float* score,
                            const int32_t* seq_len, int B, int H, int G, int T_max, int D, int dt, float scale,
                            void* ws, size_t ws_bytes, void* stream)
{
    if (T_max < 1 || !seq_len) return EC_EINVAL;
    return score_pass(q, k, v, out, lse, score, B, H, G, ec::ScoreGeom{T_max, 0, T_max, T_max, T_max, T_max}, seq_len,
                      D, dt, scale, ws, ws_bytes, stream);
}

int ec_chunk_score(const void* q, const void* k, const void* v, void* out, float* lse, float* score, int B,
                   int H, int G, int T_new, int P, int kv_rows, int D, int dt, float scale, void* ws,
                   size_t ws_bytes, void* stream)
{
    if (T_new < 1 || P < 0 || (long long)P + T_new > 0x7fffffffLL / 2) return EC_EINVAL;
    return score_pass(q, k, v, out, lse, score, B, H, G, ec::ScoreGeom{T_new, P, P + T_new, kv_rows, T_new, P + T_new},
                      nullptr, D, dt, scale, ws, ws_bytes, stream);
}

int ec_importance_mean(float* score, int B, int G, int T_new, int P, void* stream)
{
    if (!score) return EC_EINVAL;
    if (B < 1 || G < 1 || T_new < 1 || P < 0 || (long long)P + T_new > 0x7fffffffLL / 2) return EC_EINVAL;
    return ec::importance_mean_launch(score, B, G, T_new, P, reinterpret_cast<hipStream_t>(stream));
}

int ec_select_anchors(const float* score, int B, int G, int T, int n_anchor, int protect_first,
                      int protect_last, int32_t* anchor_idx, void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    if (!score || !anchor_idx) return EC_EINVAL;
    if (B < 1 || G < 1 || T < 1 || n_anchor < 1 || n_anchor > T) return EC_EINVAL;
    if (protect_first < 0 || protect_last < 0) return EC_EINVAL;
    if ((long long)protect_first + protect_last > n_anchor) return EC_EINVAL;
    if (T > 65536) return EC_EUNSUPPORTED;
    return ec::select_dispatch(score, B, G, T, n_anchor, protect_first, protect_last, anchor_idx, nullptr, nullptr,
                               reinterpret_cast<hipStream_t>(stream));
}

int ec_select_anchors_varlen(const float* score, const int32_t* seq_len, const int32_t* n_anchor_b, int B, int G,
                             int T_max, int n_max, int protect_first, int protect_last, int32_t* anchor_idx,
                             void* ws, size_t ws_bytes, void* stream)
{
    (void)ws;
    (void)ws_bytes;
    if (!score || !anchor_idx || !seq_len || !n_anchor_b) return EC_EINVAL;
    if (B < 1 || G < 1 || T_max < 1 || n_max < 1 || n_max > T_max) return EC_EINVAL;
    if (protect_first < 0 || protect_last < 0) return EC_EINVAL;
    if (T_max > 65536) return EC_EUNSUPPORTED;
    return ec::select_dispatch(score, B, G, T_max, n_max, protect_first, protect_last, anchor_idx, seq_len,
                               n_anchor_b, reinterpret_cast<hipStream_t>(stream));
}

int ec_merge_compact(const void* k, const void* v, const int32_t* anchor_idx, int B, int H, int G, int T,
                     int D, int n_anchor, int dt, int merge_mode, void* k_cache, void* v_cache, int cap,
                     int32_t* counts, int32_t* assign, int32_t* pos, void* stream)
{
    return ec_remerge_compact(k, v, T, nullptr, nullptr, anchor_idx, B, H, G, T, D, n_anchor, dt, merge_mode,
                              k_cache, v_cache, cap, counts, assign, pos, stream);
}

int ec_remerge_compact(const void* k, const void* v, int src_rows, const int32_t* weights,
                       const int32_t* src_pos, const int32_t* anchor_idx, int B, int H, int G, int L, int D,
                       int n_anchor, int dt, int merge_mode, void* k_cache, void* v_cache, int cap,
                       int32_t* counts, int32_t* assign, int32_t* pos, void* stream)
{
    if (merge_mode != EC_MERGE_MEAN && merge_mode != EC_MERGE_EVICT) return EC_EINVAL;
    if (!k || !v || !anchor_idx || !k_cache || !v_cache) return EC_EINVAL;
    if (k == k_cache || v == v_cache || k == v_cache || v == k_cache) return EC_EINVAL;  // out of place only
    if (B < 1 || H < 1 || L < 1 || D < 1 || cap < 1 || src_rows < L) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (n_anchor < 1 || n_anchor > L || n_anchor > cap) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    return ec::merge_dispatch(k, v, anchor_idx, weights, src_pos, B, H, G, L, src_rows, D, n_anchor, dt,
                              merge_mode == EC_MERGE_EVICT, k_cache, v_cache, cap, counts, assign, pos, nullptr,
                              nullptr, reinterpret_cast<hipStream_t>(stream));
}

int ec_merge_compact_varlen(const void* k, const void* v, const int32_t* anchor_idx, const int32_t* seq_len,
                            const int32_t* n_anchor_b, int B, int H, int G, int T_max, int D, int n_max, int dt,
                            int merge_mode, void* k_cache, void* v_cache, int cap, int32_t* counts,
                            int32_t* assign, int32_t* pos, void* stream)
{
    if (merge_mode != EC_MERGE_MEAN && merge_mode != EC_MERGE_EVICT) return EC_EINVAL;
    if (!k || !v || !anchor_idx || !k_cache || !v_cache || !seq_len || !n_anchor_b) return EC_EINVAL;
    if (k == k_cache || v == v_cache || k == v_cache || v == k_cache) return EC_EINVAL;
    if (B < 1 || H < 1 || T_max < 1 || D < 1 || cap < 1) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (n_max < 1 || n_max > T_max || n_max > cap) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    return ec::merge_dispatch(k, v, anchor_idx, nullptr, nullptr, B, H, G, T_max, T_max, D, n_max, dt,
                              merge_mode == EC_MERGE_EVICT, k_cache, v_cache, cap, counts, assign, pos, seq_len,
                              n_anchor_b, reinterpret_cast<hipStream_t>(stream));
}

int ec_evict_index(int64_t n_seen, int len_after_append, int gamma_num, int gamma_den, int budget_mode,
                   int fixed_len, int trunc_mode, int recent, int n_tl, int protect_first)
{
    if (n_seen < 1 || len_after_append < 1 || protect_first < 0) return -2;
    if (budget_mode != EC_BUDGET_RATIO && budget_mode != EC_BUDGET_FIXED) return -2;
    if (trunc_mode != EC_TRUNC_RECENT && trunc_mode != EC_TRUNC_ABS) return -2;
    int64_t keep;
    if (budget_mode == EC_BUDGET_RATIO) {
        if (gamma_den < 1 || gamma_num < 0 || gamma_num > gamma_den) return -2;
        const int64_t prod = (int64_t)gamma_num * n_seen;
        keep = prod / gamma_den + ((prod % gamma_den) ? 1 : 0);
    } else {
        if (fixed_len < 1) return -2;
        keep = fixed_len;
    }
    if (len_after_append <= keep) return -1;
    int64_t victim;
    if (trunc_mode == EC_TRUNC_RECENT) {
        if (recent < 0) return -2;
        victim = (int64_t)len_after_append - 1 - recent;
    } else {
        if (n_tl < 0) return -2;
        victim = n_tl;
    }
    if (victim < protect_first) victim = protect_first;
    if (victim >= (int64_t)len_after_append - 1) return -1;
    return (int)victim;
}

int ec_retention_step_varlen(int32_t* n_seen_b, int32_t* cache_len_b, int32_t* evict_idx_b, int32_t* new_pos_b,
                             int32_t* pending_b, int B, int gamma_num, int gamma_den, int budget_mode, int fixed_len,
                             int trunc_mode, int recent, int n_tl, int protect_first, int flush_only, void* stream)
{
    if (!n_seen_b || !cache_len_b || !evict_idx_b || !new_pos_b || !pending_b || B < 1) return EC_EINVAL;
    if (budget_mode != EC_BUDGET_RATIO && budget_mode != EC_BUDGET_FIXED) return EC_EINVAL;
    if (trunc_mode != EC_TRUNC_RECENT && trunc_mode != EC_TRUNC_ABS) return EC_EINVAL;
    if (budget_mode == EC_BUDGET_RATIO && (gamma_den < 1 || gamma_num < 0 || gamma_num > gamma_den)) return EC_EINVAL;
    if (budget_mode == EC_BUDGET_FIXED && fixed_len < 1) return EC_EINVAL;
    if (protect_first < 0 || (trunc_mode == EC_TRUNC_RECENT && recent < 0) || (trunc_mode == EC_TRUNC_ABS && n_tl < 0))
        return EC_EINVAL;
    return ec::retention_step_launch(n_seen_b, cache_len_b, evict_idx_b, new_pos_b, pending_b, B, gamma_num, gamma_den,
                                     budget_mode, fixed_len, trunc_mode, recent, n_tl, protect_first, flush_only ? 1 : 0,
                                     reinterpret_cast<hipStream_t>(stream));
}

namespace {
int decode_step_checked(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                        int32_t* pos, int B, int H, int G, int D, int cap, int cache_len, int evict_idx,
                        int32_t new_pos, float scale, int dt, void* out, void* ws, size_t ws_bytes, int waves,
                        int unroll, int splits, bool strict, void* stream)
{
    if (!q || !k_new || !v_new || !k_cache || !v_cache || !out) return EC_EINVAL;
    if (B < 1 || H < 1 || D < 1 || cap < 1) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (cache_len < 0 || cache_len >= cap) return EC_EINVAL;
    if (evict_idx < -1 || evict_idx > cache_len) return EC_EINVAL;
    if (!scale_ok(scale)) return EC_EINVAL;
    if (waves < 0 || unroll < 0 || splits < 0 || splits > 64) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    return ec::decode_dispatch(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, D, cap, cache_len, evict_idx,
                               new_pos, scale, dt, out, waves, unroll, splits, strict, reinterpret_cast<float*>(ws),
                               ws ? ws_bytes / sizeof(float) : 0, nullptr, nullptr, nullptr,
                               reinterpret_cast<hipStream_t>(stream));
}
}  // namespace

int ec_decode_step(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                   int32_t* pos, int B, int H, int G, int D, int cap, int cache_len, int evict_idx,
                   int32_t new_pos, float scale, int dt, void* out, void* ws, size_t ws_bytes, void* stream)
{
    return decode_step_checked(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, D, cap, cache_len, evict_idx, new_pos,
                               scale, dt, out, ws, ws_bytes, 0, 0, 0, false, stream);
}

int ec_decode_step_shaped(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                          int32_t* pos, int B, int H, int G, int D, int cap, int cache_len, int evict_idx,
                          int32_t new_pos, float scale, int dt, void* out, void* ws, size_t ws_bytes, int waves,
                          int unroll, int splits, void* stream)
{
    return decode_step_checked(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, D, cap, cache_len, evict_idx, new_pos,
                               scale, dt, out, ws, ws_bytes, waves, unroll, splits, true, stream);
}

int ec_decode_step_varlen(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                          int32_t* pos, const int32_t* cache_len_b, const int32_t* evict_idx_b,
                          const int32_t* new_pos_b, int B, int H, int G, int D, int cap, float scale, int dt,
                          void* out, void* ws, size_t ws_bytes, void* stream)
{
    if (!q || !k_new || !v_new || !k_cache || !v_cache || !out || !cache_len_b) return EC_EINVAL;
    if (B < 1 || H < 1 || D < 1 || cap < 1) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (pos && !new_pos_b) return EC_EINVAL;
    if (!scale_ok(scale)) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    // the lengths live on the device: the launch shape is chosen for the longest cache the buffers allow
    return ec::decode_dispatch(q, k_new, v_new, k_cache, v_cache, pos, B, H, G, D, cap, cap - 1, -1, 0, scale, dt, out,
                               0, 0, 0, false, reinterpret_cast<float*>(ws), ws ? ws_bytes / sizeof(float) : 0,
                               cache_len_b, evict_idx_b, new_pos_b, reinterpret_cast<hipStream_t>(stream));
}

int ec_decode_score_step(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                         int32_t* pos, float* freq, int B, int H, int G, int D, int cap, int cache_len,
                         int32_t new_pos, float scale, int dt, void* out, void* ws, size_t ws_bytes, void* stream)
{
    if (!q || !k_new || !v_new || !k_cache || !v_cache || !freq || !out) return EC_EINVAL;
    if (B < 1 || H < 1 || D < 1 || cap < 1) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (cache_len < 0 || cache_len >= cap) return EC_EINVAL;
    if (!scale_ok(scale)) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    const size_t need = ec_workspace_bytes(EC_FN_DECODE_SCORE_STEP, B, H, cap, D, dt);
    if (!ws || ws_bytes < need) return EC_EWORKSPACE;
    float* raw = reinterpret_cast<float*>(ws);
    float* stats = reinterpret_cast<float*>(reinterpret_cast<char*>(ws) + align256((size_t)B * H * cap * sizeof(float)));
    return ec::decode_score_dispatch(q, k_new, v_new, k_cache, v_cache, pos, freq, B, H, G, D, cap, cache_len, new_pos,
                                     scale, dt, out, raw, stats, reinterpret_cast<hipStream_t>(stream));
}

int ec_decode_score_step_static(const void* q, const void* k_new, const void* v_new, void* k_cache, void* v_cache,
                                int32_t* pos, float* freq, int B, int H, int G, int D, int cap, int cache_len,
                                int32_t new_pos, float scale, int dt, void* out, void* stream)
{
    if (B < 1 || H < 1 || cap < 1) return EC_EINVAL;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    const size_t need = ec_workspace_bytes(EC_FN_DECODE_SCORE_STEP, B, H, cap, D, dt);
    if (need == (size_t)-1 || need > kStaticScratchBytes) return EC_EWORKSPACE;  // beyond the built-in scratch
    void* ptr = static_scratch_ptr();
    if (!ptr) return EC_EDEVICE;
    // every word of the scratch the second kernel reads is written by the first one in the same call:
    // nothing has to start at zero
    return ec_decode_score_step(q, k_new, v_new, k_cache, v_cache, pos, freq, B, H, G, D, cap, cache_len, new_pos,
                                scale, dt, out, ptr, kStaticScratchBytes, stream);
}

int ec_evict_min(void* k_cache, void* v_cache, int32_t* pos, float* freq, int B, int H, int G, int D, int cap,
                 int len, int protect_first, int protect_recent, int dt, int32_t* victim, void* stream)
{
    if (!k_cache || !v_cache || !freq || !victim) return EC_EINVAL;
    if (B < 1 || H < 1 || D < 1 || cap < 1) return EC_EINVAL;
    if (G != 1 && G != H) return EC_EINVAL;
    if (len < 1 || len > cap) return EC_EINVAL;
    if (protect_first < 0 || protect_recent < 0 || (long long)protect_first + protect_recent >= len) return EC_EINVAL;
    if ((long long)B * H > 65535) return EC_EUNSUPPORTED;
    if (!shape_supported(D, dt)) return EC_EUNSUPPORTED;
    return ec::evict_min_dispatch(k_cache, v_cache, pos, freq, B, H, G, D, cap, len, protect_first, protect_recent, dt,
                                  victim, reinterpret_cast<hipStream_t>(stream));
}

}  // extern "C"
