// Device-side helpers shared by the gfx950 kernels: Philox4x32-10, the
// uniform/Gumbel maps, and wavefront / workgroup reductions for 64-wide waves.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rsd {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr uint32_t kTagDraftGumbel = 0;
constexpr uint32_t kTagAcceptUniform = 1;
constexpr uint32_t kTagLastGumbel = 2;

// Loads of data that is read once and streamed (logit rows, K/V tiles) carry the non-temporal
// cache policy: on this chip a plain streaming read then runs at 7.1-7.2 TB/s where ordinary loads
// reach 6.2-6.3 TB/s (measured; register and memory-to-LDS loads alike).
constexpr int kStreamPolicy = 2;  // the NT bit of a memory-to-LDS load's cache-policy operand
__device__ __forceinline__ float4 load_stream(const float4 *p) {
    typedef float vf4 __attribute__((ext_vector_type(4)));
    const vf4 v = __builtin_nontemporal_load(reinterpret_cast<const vf4 *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// ---------------------------------------------------------------------------
// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  The key is
// wave-uniform, so its Weyl sequence lives in scalar registers; each round is
// two 32x32->64 multiplies and two three-way xors on the vector side.
// ---------------------------------------------------------------------------
struct PhiloxKey {
    uint32_t k0, k1;
};

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               PhiloxKey key) {
    uint32_t k0 = key.k0, k1 = key.k1;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return make_uint4(c0, c1, c2, c3);
}

__device__ __forceinline__ PhiloxKey make_key(uint64_t seed) {
    PhiloxKey k;
    k.k0 = (uint32_t)seed;
    k.k1 = (uint32_t)(seed >> 32);
    return k;
}

__device__ __forceinline__ uint32_t counter_word3(uint32_t tag, uint32_t step) {
    return (tag & 0xFu) | (step << 4);
}

// u = (2*(w >> 9) + 1) * 2^-24: odd 24-bit grid, exact in fp32, never 0 or 1.
__device__ __forceinline__ float uniform_from_word(uint32_t w) {
    return (float)((w >> 8) | 1u) * 5.9604644775390625e-08f;
}

// Standard Gumbel variate -log(-log u) through the hardware log2 (two v_log_f32 and two
// multiplies).  Against fp64 over the whole 24-bit grid of u the largest absolute error is
// 1.6e-6, no worse than the library logf path.
__device__ __forceinline__ float gumbel_from_word(uint32_t w) {
    const float u = uniform_from_word(w);
    const float t = __builtin_amdgcn_logf(u) * -kLn2;  // -ln u > 0
    return __builtin_amdgcn_logf(t) * -kLn2;
}

// ---------------------------------------------------------------------------
// Wavefront reductions (all 64 lanes receive the result).  The fp32 sum and max
// use DPP lane permutes inside each row of 16 lanes (no LDS traffic), then
// combine the four rows through scalar lane reads; the order is fixed.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

__device__ __forceinline__ float read_lane(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_move<0xB1>(v));   // quad_perm [1,0,3,2]
    v = fmaxf(v, dpp_move<0x4E>(v));   // quad_perm [2,3,0,1]
    v = fmaxf(v, dpp_move<0x124>(v));  // row_ror 4
    v = fmaxf(v, dpp_move<0x128>(v));  // row_ror 8
    return fmaxf(fmaxf(read_lane(v, 0), read_lane(v, 16)), fmaxf(read_lane(v, 32), read_lane(v, 48)));
}

__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x124>(v);
    v += dpp_move<0x128>(v);
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// (value, index) ordering used by every selection: larger value first, on
// equal values the lower index first.  NaN never beats anything.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
    return (v > bv) || (v == bv && i < bi);
}

__device__ __forceinline__ void wave_argmax(float &v, int &i) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float ov = __shfl_xor(v, o, kWave);
        const int oi = __shfl_xor(i, o, kWave);
        if (better(ov, oi, v, i)) {
            v = ov;
            i = oi;
        }
    }
}

// Online (max, sum of 2^(x - max)) pair and its merge.
struct MaxSum {
    float m;  // running maximum (log2 domain), -inf when empty
    float s;  // sum of 2^(x - m)
};

__device__ __forceinline__ MaxSum merge(MaxSum a, MaxSum b) {
    const float m = fmaxf(a.m, b.m);
    if (m == -INFINITY) return MaxSum{-INFINITY, 0.f};
    MaxSum r;
    r.m = m;
    r.s = a.s * __builtin_amdgcn_exp2f(a.m - m) + b.s * __builtin_amdgcn_exp2f(b.m - m);
    return r;
}

__device__ __forceinline__ MaxSum wave_merge(MaxSum v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        MaxSum other;
        other.m = __shfl_xor(v.m, o, kWave);
        other.s = __shfl_xor(v.s, o, kWave);
        v = merge(v, other);
    }
    return v;
}

// The same merge without LDS traffic: the maximum and the rescaled sums go through the DPP
// reductions (one exponential per lane).  All lanes receive the result; fixed order.
__device__ __forceinline__ MaxSum wave_merge_dpp(MaxSum v) {
    const float m = wave_max(v.m);
    if (m == -INFINITY) return MaxSum{-INFINITY, 0.f};  // (uniform)
    return MaxSum{m, wave_sum(v.s * __builtin_amdgcn_exp2f(v.m - m))};
}

// Workgroup-wide merge of (max,sum) pairs.  `scratch` holds one pair per wave.
// Every thread returns the merged pair.  Contains two barriers.
template <int THREADS>
__device__ __forceinline__ MaxSum block_merge(MaxSum v, MaxSum *scratch) {
    constexpr int NW = THREADS / kWave;
    v = wave_merge(v);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[wave] = v;
    __syncthreads();
    float m = scratch[0].m;
#pragma unroll 1
    for (int w = 1; w < NW; ++w) m = fmaxf(m, scratch[w].m);
    MaxSum r{m, 0.f};
    if (m > -INFINITY) {
#pragma unroll 1
        for (int w = 0; w < NW; ++w) r.s += scratch[w].s * __builtin_amdgcn_exp2f(scratch[w].m - m);
    }
    __syncthreads();
    return r;
}

// Workgroup-wide sum of fp32 partials: fp32 inside a wave (fixed DPP order), fp64 across
// the waves in wave order.  Two barriers.
template <int THREADS>
__device__ __forceinline__ double block_sum(float part, double *scratch) {
    constexpr int NW = THREADS / kWave;
    const float v = wave_sum(part);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[wave] = (double)v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) r += scratch[w];
    __syncthreads();
    return r;
}

// Workgroup-wide arg-max with the `better` ordering.  Two barriers.
template <int THREADS>
__device__ __forceinline__ void block_argmax(float &v, int &i, float *sv, int *si) {
    constexpr int NW = THREADS / kWave;
    wave_argmax(v, i);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) {
        sv[wave] = v;
        si[wave] = i;
    }
    __syncthreads();
    float bv = sv[0];
    int bi = si[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        if (better(sv[w], si[w], bv, bi)) {
            bv = sv[w];
            bi = si[w];
        }
    }
    __syncthreads();
    v = bv;
    i = bi;
}

// Wave-wide arg-max with the `better` ordering through DPP reductions (no LDS traffic): the
// maximum first, then the lowest index among the lanes that hold it.
template <int CTRL>
__device__ __forceinline__ int dpp_move_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false);
}
__device__ __forceinline__ int wave_min_int(int v) {
    v = min(v, dpp_move_i<0xB1>(v));
    v = min(v, dpp_move_i<0x4E>(v));
    v = min(v, dpp_move_i<0x124>(v));
    v = min(v, dpp_move_i<0x128>(v));
    return min(min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16)),
               min(__builtin_amdgcn_readlane(v, 32), __builtin_amdgcn_readlane(v, 48)));
}
__device__ __forceinline__ void wave_argmax_dpp(float &v, int &i) {
    const float m = wave_max(v);
    i = wave_min_int(v == m ? i : INT_MAX);
    v = m;
}

// Two workgroup-wide arg-maxima at once (one barrier; the scratch arrays are written once per
// call, so a kernel that calls this again has to put a barrier of its own in between).
template <int THREADS>
__device__ __forceinline__ void block_argmax_pair(float &v0, int &i0, float &v1, int &i1, float *sv, int *si) {
    constexpr int NW = THREADS / kWave;
    static_assert(NW <= kWave, "one lane per wave");
    wave_argmax_dpp(v0, i0);
    wave_argmax_dpp(v1, i1);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x & (kWave - 1);
    if (lane == 0) {
        sv[wave] = v0;
        si[wave] = i0;
        sv[NW + wave] = v1;
        si[NW + wave] = i1;
    }
    __syncthreads();
    v0 = lane < NW ? sv[lane] : -INFINITY;
    i0 = lane < NW ? si[lane] : INT_MAX;
    v1 = lane < NW ? sv[NW + lane] : -INFINITY;
    i1 = lane < NW ? si[NW + lane] : INT_MAX;
    wave_argmax_dpp(v0, i0);
    wave_argmax_dpp(v1, i1);
}

// z c - m in fp32 with c = c2h + c2l: the first fused multiply-add rounds once at the size of the
// result, the second adds the part of c that a float cannot hold (c2l > 0, so a logit of -inf
// stays -inf).  neg_m = -inf turns any finite z into -inf (entries outside the row).
__device__ __forceinline__ float exponent_of(float z, float c2h, float c2l, float neg_m) {
    return fmaf(z, c2l, fmaf(z, c2h, neg_m));
}

// fp64 sum over the 64 lanes in a fixed order (all lanes active, all receive the result).
template <int CTRL>
__device__ __forceinline__ double dpp_move_d(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double read_lane_d(double v, int lane) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_move_d<0xB1>(v);
    v += dpp_move_d<0x4E>(v);
    v += dpp_move_d<0x124>(v);
    v += dpp_move_d<0x128>(v);
    return (read_lane_d(v, 0) + read_lane_d(v, 16)) + (read_lane_d(v, 32) + read_lane_d(v, 48));
}

// Hardware log2 (one instruction).  The operand is scaled out of the denormal range first,
// which the instruction would read as zero.
__device__ __forceinline__ float fast_ln(float x) {
    const bool tiny = x < 0x1p-100f;
    const float l2 = __builtin_amdgcn_logf(tiny ? x * 0x1p100f : x) - (tiny ? 100.f : 0.f);
    return l2 * kLn2;
}

// c = log2(e) / T in fp64 and as a pair of floats with a strictly positive low part (so that a
// logit of -inf keeps its sign through both fused multiply-adds of exponent_of).
struct ScalePair {
    double c2e;
    float c2h, c2l;
};

}  // namespace rsd
