// Top-k / nucleus (top-p) filtering of logit rows (Sec. 4, experiment setup: nucleus sampling
// with p = 0.95; last step of Alg. 4 and Alg. 9: candidates filtered to -inf are dropped).
//
// One 1024-thread workgroup owns one row and keeps its unnormalised probabilities
// e_x = exp((z_x - max) / T) in registers.  Both filters ask for the largest threshold t with
// F(t) >= target, where F(t) = sum over {x : e_x >= t} of a weight (1 for top-k, e_x for top-p)
// is a non-increasing step function: the threshold is found by bisection on the bit pattern of
// t (positive floats order like their bit patterns): workgroup-wide sums over the registers
// until few entries are left between the bounds, then one wave finishes on those alone.  The
// summation order is fixed, so a row always gives the same result.  No sort; entries equal to
// the threshold are all kept.
#include <hip/hip_runtime.h>
#include <math.h>

#include "../../include/rsd.h"
#include "rsd_device.hpp"

namespace rsd {

struct FilterLogitsArgs {
    const float *logits;
    int64_t ld;
    float *out;
    int64_t out_ld;
    int V;
    float c2;     // log2(e) / T
    int top_k;    // 0: off
    float top_p;  // >= 1: off
    int *kept;    // [R] or null
};

constexpr int kFilterThreads = 1024;
constexpr float kMinNormal = 1.17549435e-38f;
constexpr uint32_t kMinNormalBits = 0x00800000u;
constexpr int kFilterCand = 1024;  // entries between the bounds when one wave takes over the search

template <int CH>
__global__ __launch_bounds__(kFilterThreads) void prob_filter_kernel(FilterLogitsArgs a) {
    __shared__ double s_sum[kFilterThreads / kWave];
    __shared__ __align__(16) float s_part[2 * kFilterThreads / kWave];  // wave partials: masses, then counts
    __shared__ float s_max[kFilterThreads / kWave];
    __shared__ int s_woff[kFilterThreads / kWave];
    __shared__ float s_cand[kFilterCand];
    __shared__ uint32_t s_cut;
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const float *zrow = a.logits + (int64_t)row * a.ld;
    const float4 *z4 = reinterpret_cast<const float4 *>(zrow);
    const int V = a.V, nfull = V >> 2;

    // entry (j, q) of this thread is vocabulary index 4 * (j * 1024 + tid) + q; a chunk that
    // straddles the end of the row is read entry by entry
    auto load_chunk = [&](int c) -> float4 {
        float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        if (c < nfull) {
            t = z4[c];
        } else if (c == nfull) {
            if (4 * c + 0 < V) t.x = zrow[4 * c + 0];
            if (4 * c + 1 < V) t.y = zrow[4 * c + 1];
            if (4 * c + 2 < V) t.z = zrow[4 * c + 2];
        }
        return t;
    };
    float e[CH * 4];  // raw logits first, then exp((z - max) / T)
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const float4 t = load_chunk(j * kFilterThreads + tid);
        e[4 * j + 0] = t.x; e[4 * j + 1] = t.y; e[4 * j + 2] = t.z; e[4 * j + 3] = t.w;
        mx = fmaxf(mx, fmaxf(fmaxf(t.x, t.y), fmaxf(t.z, t.w)));
    }
    // row maximum of the raw logits (the scale is positive)
    mx = wave_max(mx);
    if (lane == 0) s_max[wave] = mx;
    __syncthreads();
    mx = s_max[0];
#pragma unroll
    for (int w = 1; w < kFilterThreads / kWave; ++w) mx = fmaxf(mx, s_max[w]);
    __syncthreads();
    const float mref = (mx == -INFINITY || mx == INFINITY) ? 0.f : mx * a.c2;
#pragma unroll
    for (int i = 0; i < CH * 4; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(e[i], a.c2, -mref));
        // -inf and NaN never count; neither do probabilities below the smallest normal number
        // (1e-38 of the row maximum), so that every threshold tried is a normal number
        // (the rounded reference can leave the maximum a hair above 1: clamp, the search assumes e <= 1)
        e[i] = (e[i] > -INFINITY && p >= kMinNormal) ? fminf(p, 1.f) : 0.f;
    }

    // (mass, count) of the entries with e >= t; every thread gets the workgroup's values.
    // fp32 inside a thread and a wave (fixed order), fp64 across the waves.
    auto tail_sums = [&](uint32_t t_bits, double &mass, double &cnt) {
        const float t = __uint_as_float(t_bits);
        // the count is a population count of the compare mask (scalar unit, whole wave at once);
        // only the mass costs vector adds
        float pm = 0.f;
        int wc = 0;
#pragma unroll
        for (int i = 0; i < CH * 4; ++i) {
            const bool ge = e[i] >= t;
            wc += __builtin_popcountll(__ballot(ge));
            pm += ge ? e[i] : 0.f;
        }
        pm = wave_sum(pm);
        const float pc = (float)wc;
        if (lane == 0) {
            s_part[wave] = pm;
            s_part[kFilterThreads / kWave + wave] = pc;
        }
        __syncthreads();
        // 16 wave partials each, fetched as 16-byte broadcast reads and added in fp64 in wave order
        mass = 0.0;
        cnt = 0.0;
#pragma unroll
        for (int w4 = 0; w4 < kFilterThreads / kWave / 4; ++w4) {
            const float4 pm4 = reinterpret_cast<const float4 *>(s_part)[w4];
            const float4 pc4 = reinterpret_cast<const float4 *>(s_part)[kFilterThreads / kWave / 4 + w4];
            mass += (double)pm4.x; mass += (double)pm4.y; mass += (double)pm4.z; mass += (double)pm4.w;
            cnt += (double)pc4.x; cnt += (double)pc4.y; cnt += (double)pc4.z; cnt += (double)pc4.w;
        }
        __syncthreads();
    };
    // Largest bit pattern t in [smallest normal, 0x3F800000] with F(t) >= target (F = count or mass of the entries
    // >= t), or 0 when even the smallest pattern falls short.  Bisection over the whole row until at
    // most kFilterCand entries lie between the two bounds; those are then compacted into LDS in index
    // order and one wave finishes the bisection on them alone.
    auto threshold = [&](double target, bool by_count) -> uint32_t {
        uint32_t lo = kMinNormalBits, hi = 0x3F800001u;  // e <= 1, so F(hi) = 0; invariant F(lo) >= target > F(hi)
        double f_lo, c_lo, f_hi = 0.0, c_hi = 0.0, m, c;
        tail_sums(lo, m, c);
        f_lo = by_count ? c : m;
        c_lo = c;
        if (f_lo < target) return 0u;
        while (hi - lo > 1u && c_lo - c_hi > (double)kFilterCand) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            tail_sums(mid, m, c);
            const double f = by_count ? c : m;
            if (f >= target) { lo = mid; f_lo = f; c_lo = c; } else { hi = mid; f_hi = f; c_hi = c; }
        }
        if (hi - lo <= 1u) return lo;
        // compaction: thread-local count, exclusive scan over the workgroup, ordered writes
        const float flo = __uint_as_float(lo), fhi = __uint_as_float(hi);
        int mine = 0;
#pragma unroll
        for (int i = 0; i < CH * 4; ++i) mine += (e[i] >= flo && e[i] < fhi) ? 1 : 0;
        int incl = mine;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int up = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += up;
        }
        if (lane == kWave - 1) s_woff[wave] = incl;
        __syncthreads();
        int base = 0;
        for (int w = 0; w < wave; ++w) base += s_woff[w];
        int pos = base + incl - mine;
#pragma unroll
        for (int i = 0; i < CH * 4; ++i)
            if (e[i] >= flo && e[i] < fhi && pos < kFilterCand) s_cand[pos++] = e[i];
        __syncthreads();
        if (wave == 0) {
            const int ncand = (int)(c_lo - c_hi + 0.5);
            float cv[kFilterCand / kWave];
#pragma unroll
            for (int q = 0; q < kFilterCand / kWave; ++q) {
                const int idx = q * kWave + lane;
                cv[q] = idx < ncand ? s_cand[idx] : 0.f;   // 0 < every threshold tried: never counted
            }
            uint32_t l2 = lo, h2 = hi;
            while (h2 - l2 > 1u) {
                const uint32_t mid = l2 + ((h2 - l2) >> 1);
                const float t = __uint_as_float(mid);
                // the candidates together hold a small part of the row's mass (or a count below
                // 2^24), so fp32 is ample here; lane-permute reduction, fixed order
                float part = 0.f;
#pragma unroll
                for (int q = 0; q < kFilterCand / kWave; ++q)
                    part += (cv[q] >= t) ? (by_count ? 1.f : cv[q]) : 0.f;
                part = wave_sum(part);
                if (f_hi + (double)part >= target) l2 = mid; else h2 = mid;
            }
            if (lane == 0) s_cut = l2;
        }
        __syncthreads();
        const uint32_t r = s_cut;
        __syncthreads();
        return r;
    };
    auto mass_at_least = [&](uint32_t t_bits, bool by_count) -> double {
        double m, c;
        tail_sums(t_bits, m, c);
        return by_count ? c : m;
    };

    uint32_t cut = kMinNormalBits;  // keep every entry with e >= cut (bit pattern): all positive ones so far
    if (a.top_k > 0) {
        const uint32_t t = threshold((double)a.top_k, true);
        if (t != 0u) cut = t;  // fewer than k positive entries: keep them all
#pragma unroll
        for (int i = 0; i < CH * 4; ++i) e[i] = (e[i] >= __uint_as_float(cut)) ? e[i] : 0.f;
    }
    if (a.top_p < 1.f) {
        const double total = mass_at_least(kMinNormalBits, false);
        // a target that rounding could push above the total would empty the row: cap it
        const double target = fmin((double)a.top_p * total, total);
        const uint32_t t = threshold(target, false);
        if (t > cut) cut = t;
    }
    const float cutf = __uint_as_float(cut);
    float nkept = 0.f;
    float *orow = a.out + (int64_t)row * a.out_ld;
    float4 *o4 = reinterpret_cast<float4 *>(orow);
    // the logits are read a second time (they were not kept in registers; the row is still in
    // L2) just before the same thread overwrites them, so `out` may be `logits` itself
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = j * kFilterThreads + tid;
        const float4 t = load_chunk(c);
        const float zq[4] = {t.x, t.y, t.z, t.w};
        float r[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool keep = e[4 * j + q] >= cutf && e[4 * j + q] > 0.f;
            r[q] = keep ? zq[q] : -INFINITY;
            nkept += keep ? 1.f : 0.f;
        }
        if (c < nfull) {
            o4[c] = make_float4(r[0], r[1], r[2], r[3]);
        } else if (c == nfull) {
            for (int q = 0; q < 3; ++q)
                if (4 * c + q < V) orow[4 * c + q] = r[q];
        }
    }
    if (a.kept) {
        const double n = block_sum<kFilterThreads>(nkept, s_sum);
        if (tid == 0) a.kept[row] = (int)(n + 0.5);
    }
}

}  // namespace rsd

using namespace rsd;

extern "C" int32_t rsd_filter_logits(const float *logits, int64_t ld, int32_t R, int32_t V,
                                     float inv_temperature, int32_t top_k, float top_p, float *out,
                                     int64_t out_ld, int32_t *kept, void *stream) {
    if (!logits || !out) return RSD_ERR_NULL;
    if (R < 0 || V < 1 || V > RSD_VOCAB_MAX || ld < V || out_ld < V || top_k < 0 ||
        !(inv_temperature > 0.f) || !(top_p > 0.f))
        return RSD_ERR_SHAPE;
    auto misaligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
    if (misaligned(logits) || misaligned(out) || ld % 4 || out_ld % 4) return RSD_ERR_SHAPE;
    if (R == 0) return RSD_OK;
    FilterLogitsArgs a;
    a.logits = logits; a.ld = ld; a.out = out; a.out_ld = out_ld; a.V = V;
    a.c2 = inv_temperature * kLog2e; a.top_k = top_k; a.top_p = top_p; a.kept = kept;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int need = (V >> 2) + ((V & 3) ? 1 : 0);  // float4 chunks of a row, a ragged tail included
    const int chunks = (need + kFilterThreads - 1) / kFilterThreads;
    if (chunks <= 2)
        hipLaunchKernelGGL(prob_filter_kernel<2>, dim3(R), dim3(kFilterThreads), 0, st, a);
    else if (chunks <= 8)
        hipLaunchKernelGGL(prob_filter_kernel<8>, dim3(R), dim3(kFilterThreads), 0, st, a);
    else if (chunks <= 13)
        hipLaunchKernelGGL(prob_filter_kernel<13>, dim3(R), dim3(kFilterThreads), 0, st, a);
    else
        hipLaunchKernelGGL(prob_filter_kernel<16>, dim3(R), dim3(kFilterThreads), 0, st, a);
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}
