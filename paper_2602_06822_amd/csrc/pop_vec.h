// 16-byte vector traits for the weight rows: bf16 (8 elements) and float32 (4 elements).
#pragma once
#include "pop_internal.h"

namespace pop {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// bf16 rows: products of two bf16 values are exact in float32, so dot products accumulate in float32
// (v_dot2_f32_bf16).  float32 rows: dot products accumulate in float64 so that h keeps full float32
// accuracy even when the sum cancels; the kernels stay HBM-bound either way.
struct VecBF16 {
    typedef uint4 vec_t;
    typedef float acc_t;
    static constexpr int kElems = 8;
    static __device__ __forceinline__ vec_t zero() { return make_uint4(0, 0, 0, 0); }
    static __device__ __forceinline__ float dot(const vec_t &w, const vec_t &x, float acc)
    {
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.x), __builtin_bit_cast(bf16x2_t, x.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.y), __builtin_bit_cast(bf16x2_t, x.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.z), __builtin_bit_cast(bf16x2_t, x.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, w.w), __builtin_bit_cast(bf16x2_t, x.w), acc, false);
        return acc;
    }
    static __device__ __forceinline__ void axpy(float a, const vec_t &w, float (&acc)[8])
    {
        acc[0] = fmaf(a, bf16_lo(w.x), acc[0]);
        acc[1] = fmaf(a, bf16_hi(w.x), acc[1]);
        acc[2] = fmaf(a, bf16_lo(w.y), acc[2]);
        acc[3] = fmaf(a, bf16_hi(w.y), acc[3]);
        acc[4] = fmaf(a, bf16_lo(w.z), acc[4]);
        acc[5] = fmaf(a, bf16_hi(w.z), acc[5]);
        acc[6] = fmaf(a, bf16_lo(w.w), acc[6]);
        acc[7] = fmaf(a, bf16_hi(w.w), acc[7]);
    }
};

struct VecF32 {
    typedef float4 vec_t;
    typedef double acc_t;
    static constexpr int kElems = 4;
    static __device__ __forceinline__ vec_t zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    static __device__ __forceinline__ double dot(const vec_t &w, const vec_t &x, double acc)
    {
        acc = fma((double)w.x, (double)x.x, acc);
        acc = fma((double)w.y, (double)x.y, acc);
        acc = fma((double)w.z, (double)x.z, acc);
        acc = fma((double)w.w, (double)x.w, acc);
        return acc;
    }
    static __device__ __forceinline__ void axpy(float a, const vec_t &w, float (&acc)[8])
    {
        acc[0] = fmaf(a, w.x, acc[0]);
        acc[1] = fmaf(a, w.y, acc[1]);
        acc[2] = fmaf(a, w.z, acc[2]);
        acc[3] = fmaf(a, w.w, acc[3]);
    }
};

// ---- cross-lane sums in double (DPP moves on the two halves, no LDS).  The partial dot products of a bf16 row are
// float32 values whose sum can cancel; adding them up in double keeps the rounding of the cross-lane tree (a dozen
// levels at the magnitude of the full sum) out of h, so that only the few in-lane float32 adds remain.
template <int kCtrl>
__device__ __forceinline__ double dpp_move(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), kCtrl, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), kCtrl, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
// Sum over the 16 lanes of each DPP row, result in every lane of the row.
__device__ __forceinline__ double dpp_row_sum(double v)
{
    v += dpp_move<0xB1>(v);   // quad_perm 1,0,3,2
    v += dpp_move<0x4E>(v);   // quad_perm 2,3,0,1
    v += dpp_move<0x141>(v);  // row_half_mirror
    v += dpp_move<0x140>(v);  // row_mirror
    return v;
}
__device__ __forceinline__ double lane_value(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}
// Sum over the 64 lanes of the wave, same value in every lane (fixed order).
__device__ __forceinline__ double wave_total(double v)
{
    const double r = dpp_row_sum(v);
    return (lane_value(r, 0) + lane_value(r, 16)) + (lane_value(r, 32) + lane_value(r, 48));
}

// Four values per lane -> in every lane the sum over its row of 16 lanes of ONE of them: value id
// butterfly_value_id(lane).  Halving exchanges (each level sends half of what is left): 7 cross-lane moves of a
// double instead of 16, so that summing in double costs no more than the plain float32 row sums it replaces.
__device__ __forceinline__ double butterfly4_row_sum(const double (&v)[4], int lane)
{
    const bool o1 = lane & 1, o2 = lane & 2;
    double w[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const double send = o1 ? v[j] : v[j + 2], keep = o1 ? v[j + 2] : v[j];
        w[j] = keep + dpp_move<0xB1>(send);  // partner lane ^ 1
    }
    const double send = o2 ? w[0] : w[1], keep = o2 ? w[1] : w[0];
    double z = keep + dpp_move<0x4E>(send);  // partner lane ^ 2
    z += dpp_move<0x124>(z);                 // row_ror:4
    z += dpp_move<0x128>(z);                 // row_ror:8
    return z;
}
__device__ __forceinline__ int butterfly_value_id(int lane) { return ((lane & 1) << 1) | ((lane >> 1) & 1); }

// Dot products of one channel's gate and up rows with x (staged in LDS as vectors), lanes striding the row.
// Returns per-lane partial sums; the caller reduces across the wave.
template <class V, int U>
__device__ __forceinline__ void row_dot_gate_up(const typename V::vec_t *__restrict__ g,
                                                const typename V::vec_t *__restrict__ u,
                                                const typename V::vec_t *xs, int nvec, int lane,
                                                typename V::acc_t &ag, typename V::acc_t &au)
{
    typedef typename V::vec_t vec_t;
    const int group = kWave * U;
    const int nvec_full = nvec / group * group;
    ag = 0;
    au = 0;
    for (int c0 = 0; c0 < nvec_full; c0 += group) {
        vec_t wg[U], wu[U];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            wg[q] = g[c0 + q * kWave + lane];
            wu[q] = u[c0 + q * kWave + lane];
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            vec_t xv = xs[c0 + q * kWave + lane];
            ag = V::dot(wg[q], xv, ag);
            au = V::dot(wu[q], xv, au);
        }
    }
    for (int c = nvec_full + lane; c < nvec; c += kWave) {
        vec_t wg = g[c], wu = u[c], xv = xs[c];
        ag = V::dot(wg, xv, ag);
        au = V::dot(wu, xv, au);
    }
}

}  // namespace pop
