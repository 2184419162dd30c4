// Internal helpers shared by the HIP translation units of libelastic_cache.
// gfx950 (CDNA4) only: 64-wide wavefronts, DPP row operations, 16-byte vector loads.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ec.h"

namespace ec {

constexpr int kWave = 64;

// Element access for the two storage types.  A "chunk" is the 16 bytes one lane
// moves per vector load: 4 fp32 or 8 bf16 values.
template <int DT> struct Elem;
template <> struct Elem<EC_F32> {
    using type = float;
    static constexpr int kBytes = 4;
    static constexpr int kPerChunk = 4;
};
template <> struct Elem<EC_BF16> {
    using type = uint16_t;
    static constexpr int kBytes = 2;
    static constexpr int kPerChunk = 8;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Unpack one 16-byte chunk into fp32 values.
template <int DT> __device__ __forceinline__ void unpack(const uint4& c, float* f);
template <> __device__ __forceinline__ void unpack<EC_F32>(const uint4& c, float* f)
{
    f[0] = __uint_as_float(c.x);
    f[1] = __uint_as_float(c.y);
    f[2] = __uint_as_float(c.z);
    f[3] = __uint_as_float(c.w);
}
template <> __device__ __forceinline__ void unpack<EC_BF16>(const uint4& c, float* f)
{
    f[0] = __uint_as_float(c.x << 16);
    f[1] = __uint_as_float(c.x & 0xffff0000u);
    f[2] = __uint_as_float(c.y << 16);
    f[3] = __uint_as_float(c.y & 0xffff0000u);
    f[4] = __uint_as_float(c.z << 16);
    f[5] = __uint_as_float(c.z & 0xffff0000u);
    f[6] = __uint_as_float(c.w << 16);
    f[7] = __uint_as_float(c.w & 0xffff0000u);
}

// Pack fp32 values into one 16-byte chunk of the storage type.
template <int DT> __device__ __forceinline__ uint4 pack(const float* f);
template <> __device__ __forceinline__ uint4 pack<EC_F32>(const float* f)
{
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                      __float_as_uint(f[3]));
}
template <> __device__ __forceinline__ uint4 pack<EC_BF16>(const float* f)
{
    uint4 c;
    c.x = (uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16);
    c.y = (uint32_t)f32_to_bf16(f[2]) | ((uint32_t)f32_to_bf16(f[3]) << 16);
    c.z = (uint32_t)f32_to_bf16(f[4]) | ((uint32_t)f32_to_bf16(f[5]) << 16);
    c.w = (uint32_t)f32_to_bf16(f[6]) | ((uint32_t)f32_to_bf16(f[7]) << 16);
    return c;
}

// 16-byte load of data that is read once: the non-temporal hint keeps the stream from displacing
// cache lines, which measurably raises the rate of large one-pass reads on this chip.
__device__ __forceinline__ uint4 load_stream(const uint4* p)
{
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- DPP cross-lane moves inside a row of 16 lanes (full rate, no LDS) ----
template <int CTRL> __device__ __forceinline__ float dpp_mov(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppRowMirror = 0x140;      // lane i <-> 15-i inside each 16 lanes

// Sum over aligned groups of LPR lanes (LPR in {8,16,32,64}); every lane gets the sum.
template <int LPR> __device__ __forceinline__ float group_sum(float x)
{
    x += dpp_mov<kDppQuadXor1>(x);
    x += dpp_mov<kDppQuadXor2>(x);
    x += dpp_mov<kDppRowHalfMirror>(x);
    if (LPR >= 16) x += dpp_mov<kDppRowMirror>(x);
    if (LPR >= 32) x += __shfl_xor(x, 16, kWave);
    if (LPR >= 64) x += __shfl_xor(x, 32, kWave);
    return x;
}

__device__ __forceinline__ float wave_max(float x)
{
    x = fmaxf(x, dpp_mov<kDppQuadXor1>(x));
    x = fmaxf(x, dpp_mov<kDppQuadXor2>(x));
    x = fmaxf(x, dpp_mov<kDppRowHalfMirror>(x));
    x = fmaxf(x, dpp_mov<kDppRowMirror>(x));
    x = fmaxf(x, __shfl_xor(x, 16, kWave));
    x = fmaxf(x, __shfl_xor(x, 32, kWave));
    return x;
}

// Geometry of one scoring pass.  Every head of k/v holds P rows of an existing compressed cache followed
// by the Tq rows of the chunk being encoded (L = P + Tq rows), heads kv_rows rows apart.  Query m of the
// chunk sees rows n <= P + m.  The first-turn pass over a bare prompt is P = 0, kv_rows = Tq.
// q, out and the row log-sum-exp have q_rows rows per head, the per-head importance imp_rows.  For a ragged
// batch (P = 0) Tq is the padded length all strides are built on and batch element b has seq_len[b] rows.
struct ScoreGeom {
    int Tq, P, L, kv_rows, q_rows, imp_rows;
};

// Rows of batch element b in a ragged batch (clamped into [0, t_max]); t_max for a dense one.
__device__ __forceinline__ int ragged_rows(const int32_t* __restrict__ seq_len, int b, int t_max)
{
    return seq_len ? min(max(seq_len[b], 0), t_max) : t_max;
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

inline int status_from_hip(hipError_t e) { return e == hipSuccess ? EC_OK : EC_EDEVICE; }

}  // namespace ec
