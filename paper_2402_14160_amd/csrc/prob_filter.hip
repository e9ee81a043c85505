// Top-k / nucleus (top-p) filtering of logit rows (Sec. 4, experiment setup: nucleus sampling
// with p = 0.95; last step of Alg. 4 and Alg. 9: candidates filtered to -inf are dropped).
//
// One workgroup owns one row and keeps its unnormalised probabilities
// e_x = exp((z_x - max) / T) in registers.  Both filters ask for the largest threshold t with
// F(t) >= target, where F(t) = sum over {x : e_x >= t} of a weight (1 for top-k, e_x for top-p)
// is a non-increasing step function.  The threshold is found by bisection on the bit pattern of
// t (positive floats order like their bit patterns), starting between the row's smallest
// positive entry (whose F, the total, comes out of the exponential pass) and 1: workgroup-wide
// sums over the registers until few entries are left between the bounds; those are compacted
// into LDS and every wave then probes its own threshold on them (a 17-way split per round)
// until one entry is left.  The summation order is fixed, so a row always gives the same
// result.  No sort; entries equal to the threshold are all kept.
#include <hip/hip_runtime.h>
#include <math.h>

#include <type_traits>

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
constexpr uint32_t kAboveOneBits = 0x3F800001u;  // e <= 1, so nothing is >= this
constexpr int kFilterCand = 1024;  // entries between the bounds when the per-wave probes take over
// A top-k larger than the number of entries that fp32 tells apart from zero goes on below the
// fp32 range, 126 binary orders of magnitude at a time, at most this many times (entries more
// than 126 * 17 = 2142 log2 units below the row maximum are never kept).
constexpr int kUnderflowBands = 16;

// sum of lanes 0..15 of a wave (one DPP row), the same in every lane; fixed order
__device__ __forceinline__ float row0_sum(float v) {
    v += dpp_move<0xB1>(v);
    v += dpp_move<0x4E>(v);
    v += dpp_move<0x124>(v);
    v += dpp_move<0x128>(v);
    return read_lane(v, 0);
}

// CH: float4 chunks per thread; RAGGED: V is not a multiple of 4 (the last chunk is then read
// and written entry by entry).  Up to 8 chunks per thread the kernel fits 64 registers, so two
// workgroups share a CU and one row's loads and stores overlap the other's arithmetic.
// BANDS: top-k without top-p, the one case that may have to rank entries below the fp32 range
// (kept out of the other instantiations, whose register budget it would strain).
template <int CH, bool RAGGED, bool BANDS>
__global__ __launch_bounds__(kFilterThreads, CH <= 8 ? 8 : 4) void prob_filter_kernel(FilterLogitsArgs a) {
    constexpr int kWaves = kFilterThreads / kWave;
    static_assert(kWaves <= 16, "the wave partials are combined inside one row of 16 lanes");
    __shared__ float s_part[2][2 * kWaves];  // wave partials (masses, then counts), double-buffered
    __shared__ float s_max[kWaves];
    __shared__ uint32_t s_min[kWaves];
    __shared__ int s_woff[kWaves];
    __shared__ float s_cand[kFilterCand];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const float *zrow = a.logits + (int64_t)row * a.ld;
    const float4 *z4 = reinterpret_cast<const float4 *>(zrow);
    const int V = a.V, nfull = V >> 2;
    int flip = 0;  // which half of s_part the next workgroup-wide sum uses

    // entry (j, q) of this thread is vocabulary index 4 * (j * 1024 + tid) + q; a chunk that
    // straddles the end of the row is read entry by entry
    auto load_chunk = [&](int j, int th) -> float4 {
        const int c = j * kFilterThreads + th;
        float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        if (c < nfull) {
            t = (z4 + j * kFilterThreads)[th];  // uniform base, one lane offset for every j
        } else if (RAGGED && c == nfull) {
            if (4 * c + 0 < V) t.x = zrow[4 * c + 0];
            if (4 * c + 1 < V) t.y = zrow[4 * c + 1];
            if (4 * c + 2 < V) t.z = zrow[4 * c + 2];
        }
        return t;
    };
    float e[CH * 4];  // raw logits first, then exp((z - max) / T)
    float mx = -INFINITY;
    // (with the bands the lane index is live through the whole kernel and the register allocator
    // would reload it from scratch before every load below, which drains the loads one by one: a
    // copy it takes for a new value keeps the reloads out of this loop)
    int tid_a = tid;
    if constexpr (BANDS) asm volatile("" : "+v"(tid_a));
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const float4 t = load_chunk(j, tid_a);
        e[4 * j + 0] = t.x; e[4 * j + 1] = t.y; e[4 * j + 2] = t.z; e[4 * j + 3] = t.w;
        mx = fmaxf(mx, fmaxf(fmaxf(t.x, t.y), fmaxf(t.z, t.w)));
    }
    // row maximum of the raw logits (the scale is positive)
    mx = wave_max(mx);
    if (lane == 0) s_max[wave] = mx;
    __syncthreads();
    mx = s_max[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, s_max[w]);
    const float mref = (mx == -INFINITY || mx == INFINITY) ? 0.f : mx * a.c2;

    // wave partials (mass, count) -> workgroup totals in every thread: one barrier, then lanes
    // 0..15 of each wave fetch one partial each and add them inside their DPP row (fp32, fixed
    // order).  The two halves of s_part alternate, so the next call's writes cannot overtake
    // this call's reads.
    auto combine = [&](float pm, float pc, float &mass, float &cnt) {
        if (lane == 0) {
            s_part[flip][wave] = pm;
            s_part[flip][kWaves + wave] = pc;
        }
        __syncthreads();
        const float m = lane < kWaves ? s_part[flip][lane] : 0.f;
        const float c = lane < kWaves ? s_part[flip][kWaves + lane] : 0.f;
        mass = row0_sum(m);
        cnt = row0_sum(c);
        flip ^= 1;
    };

    // exponentials; their total, the number of positive ones and the smallest positive one
    // come out of the same pass
    float total, npos;
    uint32_t min_bits;
    {
        float pm = 0.f;
        int wc = 0;
        uint32_t mb = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < CH * 4; ++i) {
            const float p = __builtin_amdgcn_exp2f(fmaf(e[i], a.c2, -mref));
            // -inf and NaN never count (their p is 0 or NaN); neither do probabilities below the
            // smallest normal number (1e-38 of the row maximum), so that every threshold tried is
            // a normal number.  The rounded reference can leave the maximum a hair above 1:
            // clamp, the search assumes e <= 1.
            const bool pos = p >= kMinNormal;
            e[i] = pos ? __builtin_amdgcn_fmed3f(p, 0.f, 1.f) : 0.f;
            pm += e[i];
            wc += __builtin_popcountll(__builtin_amdgcn_ballot_w64(pos));
            mb = min(mb, __float_as_uint(e[i]) - 1u);  // zero wraps to the largest value
        }
        pm = wave_sum(pm);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mb = min(mb, (uint32_t)__shfl_xor((int)mb, o, kWave));
        if (lane == 0) s_min[wave] = mb;
        combine(pm, (float)wc, total, npos);
        mb = s_min[0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) mb = min(mb, s_min[w]);
        min_bits = mb + 1u;  // meaningful when npos > 0
    }
    // (a lane index the compiler takes for a new value wherever the row is read again, so that
    // the first pass's addresses and bounds are recomputed there instead of being held in
    // registers through the search)
    int tid_w = tid;
    if constexpr (BANDS) asm volatile("" : "+v"(tid_w));  // (the bands read the row inside the search)

    // (mass, count) of the entries with e >= t; every thread gets the workgroup's values.
    // The count is a population count of the compare mask (scalar unit, whole wave at once);
    // only the mass costs vector adds, and a search by count skips it.
    auto tail_sums = [&](uint32_t t_bits, auto by_count, float &mass, float &cnt) {
        const float t = __uint_as_float(t_bits);
        float pm = 0.f;
        int wc = 0;
#pragma unroll
        for (int i = 0; i < CH * 4; ++i) {
            const bool ge = e[i] >= t;
            wc += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ge));
            if (!decltype(by_count)::value) pm += ge ? e[i] : 0.f;
        }
        if (!decltype(by_count)::value) pm = wave_sum(pm);
        combine(pm, (float)wc, mass, cnt);
    };

    // Largest bit pattern t in [lo, 1] with F(t) >= target, given F(lo) = f_lo >= target and the
    // count c_lo of the entries >= lo.  Bisection over the whole row until at most kFilterCand
    // entries lie between the two bounds; those are compacted into LDS in index order and every
    // wave then evaluates F at its own threshold inside the bounds (kWaves + 1 intervals per
    // round) until one entry is left between them: that entry is the threshold.
    auto search = [&](float target, auto by_count, uint32_t lo, float f_lo, float c_lo) -> uint32_t {
        constexpr bool kByCount = decltype(by_count)::value;
        uint32_t hi = kAboveOneBits;  // invariant F(lo) >= target > F(hi)
        float f_hi = 0.f, c_hi = 0.f, m, c;
        while (hi - lo > 1u && c_lo - c_hi > (float)kFilterCand) {
            const uint32_t mid = lo + ((hi - lo) >> 1);
            tail_sums(mid, by_count, m, c);
            const float f = kByCount ? c : m;
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
        const int ncand = (int)(c_lo - c_hi + 0.5f);
        float cv[kFilterCand / kWave];
#pragma unroll
        for (int q = 0; q < kFilterCand / kWave; ++q) {
            const int idx = q * kWave + lane;
            cv[q] = idx < ncand ? s_cand[idx] : 0.f;  // 0 < every threshold tried: never counted
        }
        // F(t) = f_hi + the candidates >= t.  The candidates hold a small part of the row's mass
        // (or a count below 2^24), so fp32 is ample.
        float n_lo = (float)ncand, n_hi = 0.f;  // candidates >= lo, >= hi
        while (hi - lo > 1u && n_lo - n_hi > 1.5f) {
            const uint32_t span = hi - lo;
            auto probe = [&](int w) -> uint32_t {  // lo <= probe(w) < hi, non-decreasing in w
                return lo + (uint32_t)(((uint64_t)(w + 1) * span) / (uint32_t)(kWaves + 1));
            };
            const float t = __uint_as_float(probe(wave));
            float part = 0.f;
            int wc = 0;
#pragma unroll
            for (int q = 0; q < kFilterCand / kWave; ++q) {
                const bool ge = cv[q] >= t;
                wc += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ge));
                if (!kByCount) part += ge ? cv[q] : 0.f;
            }
            part = kByCount ? (float)wc : wave_sum(part);
            if (lane == 0) {
                s_part[flip][wave] = f_hi + part;
                s_part[flip][kWaves + wave] = (float)wc;
            }
            __syncthreads();
            // F does not increase with t: the probes that still reach the target are the first n_ok
            const bool ok = lane < kWaves && s_part[flip][lane < kWaves ? lane : 0] >= target;
            const int n_ok = __builtin_popcountll(__ballot(ok));
            const uint32_t new_lo = n_ok > 0 ? probe(n_ok - 1) : lo;
            const uint32_t new_hi = n_ok < kWaves ? probe(n_ok) : hi;
            if (n_ok > 0) n_lo = s_part[flip][kWaves + n_ok - 1];
            if (n_ok < kWaves) n_hi = s_part[flip][kWaves + n_ok];
            lo = new_lo;
            hi = new_hi;
            flip ^= 1;
        }
        if (hi - lo > 1u && n_lo - n_hi > 0.5f) {
            // one candidate c in [lo, hi): F(c) = F(lo) >= target > F(hi) = F(c + 1 ulp)
            const float flo2 = __uint_as_float(lo), fhi2 = __uint_as_float(hi);
            float best = 0.f;
#pragma unroll
            for (int q = 0; q < kFilterCand / kWave; ++q)
                best = fmaxf(best, (cv[q] >= flo2 && cv[q] < fhi2) ? cv[q] : 0.f);
            best = wave_max(best);
            if (best > 0.f) lo = __float_as_uint(best);
        }
        return lo;
    };

    uint32_t cut = kMinNormalBits;  // keep every entry with e >= cut (bit pattern): all positive ones so far
    // The cut lies this many log2 units below the fp32 range: an entry is kept when
    // 2^(log2 of its relative probability + shift) >= cut.  Once a band below the range has been
    // looked at (top-k alone, see below) the registers no longer hold band 0, and the decision
    // is worked out again from the logits when the row is written.
    float shift = 0.f;
    bool stale = false;
    if (npos > 0.5f) {
        if (a.top_k > 0) {
            // The row is ranked band by band: band 0 is what fp32 tells apart from zero (the
            // values in the registers); when top-k alone wants more entries than that, the
            // relative probabilities in [2^-126 (s+1), 2^-126 s) are worked out again from the
            // logits, scaled up by 2^(126 s).  A band that fits is taken whole, the one that
            // does not is searched.
            const bool deeper = BANDS && !(a.top_p < 1.f);  // with top-p the bands below carry no mass and go anyway
            float have = 0.f, cnt = npos, base = 0.f;
            uint32_t band_min = min_bits;
            for (int band = 0;; ++band) {
                if (have + cnt > (float)a.top_k) {  // the cut falls inside this band
                    cut = search((float)a.top_k - have, std::true_type{}, band_min, cnt, cnt);
                    shift = base;
                    break;
                }
                if (cnt > 0.5f) {  // the whole band is kept
                    have += cnt;
                    cut = kMinNormalBits;
                    shift = base;
                }
                if (!BANDS || !deeper || band == kUnderflowBands || have >= (float)a.top_k) break;
                base += 126.f;
                stale = true;
                int wc = 0;
                uint32_t mb = 0xFFFFFFFFu;
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const float4 t = load_chunk(j, tid_w);
                    const float zq[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float pb = __builtin_amdgcn_exp2f(fmaf(zq[q], a.c2, -mref) + base);
                        const bool in_band = pb >= kMinNormal && pb < 1.f;
                        e[4 * j + q] = in_band ? pb : 0.f;
                        wc += __builtin_popcountll(__builtin_amdgcn_ballot_w64(in_band));
                        mb = min(mb, __float_as_uint(e[4 * j + q]) - 1u);
                    }
                }
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) mb = min(mb, (uint32_t)__shfl_xor((int)mb, o, kWave));
                __syncthreads();  // the previous round's s_min has been read
                if (lane == 0) s_min[wave] = mb;
                float unused;
                combine(0.f, (float)wc, unused, cnt);
                mb = s_min[0];
#pragma unroll
                for (int w = 1; w < kWaves; ++w) mb = min(mb, s_min[w]);
                band_min = mb + 1u;
            }
            if (a.top_p < 1.f) {  // (then the cut lies in band 0)
#pragma unroll
                for (int i = 0; i < CH * 4; ++i) e[i] = (e[i] >= __uint_as_float(cut)) ? e[i] : 0.f;
                if (cut != kMinNormalBits) {
                    min_bits = cut;  // every surviving entry is >= cut
                    tail_sums(cut, std::false_type{}, total, npos);
                }
            }
        }
        if (a.top_p < 1.f) {
            // a target that rounding could push above the total would empty the row: cap it
            const float target = fminf(a.top_p * total, total);
            const uint32_t t = search(target, std::false_type{}, min_bits, total, npos);
            if (t > cut) cut = t;
        }
    }
    const float cutf = __uint_as_float(cut);
    int wkept = 0;
    float *orow = a.out + (int64_t)row * a.out_ld;
    float4 *o4 = reinterpret_cast<float4 *>(orow);
    // the logits are read a second time (they were not kept in registers; the row is still in
    // L2) just before the same thread overwrites them, so `out` may be `logits` itself
    const bool below_range = BANDS && stale;  // uniform
    asm volatile("" : "+v"(tid_w));
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = j * kFilterThreads + tid_w;
        const float4 t = load_chunk(j, tid_w);
        const float zq[4] = {t.x, t.y, t.z, t.w};
        float r[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // cutf > 0: the dropped entries (e = 0) fail.  After a look below the fp32 range the
            // entry's scaled probability is worked out again (infinite for the bands above the
            // cut's, zero or NaN for what is never kept).
            bool keep = e[4 * j + q] >= cutf;
            if (below_range) keep = __builtin_amdgcn_exp2f(fmaf(zq[q], a.c2, -mref) + shift) >= cutf;
            r[q] = keep ? zq[q] : -INFINITY;
            wkept += __builtin_popcountll(__builtin_amdgcn_ballot_w64(keep));
        }
        if (c < nfull) {
            (o4 + j * kFilterThreads)[tid_w] = make_float4(r[0], r[1], r[2], r[3]);
        } else if (RAGGED && c == nfull) {
            for (int q = 0; q < 3; ++q)
                if (4 * c + q < V) orow[4 * c + q] = r[q];
        }
    }
    if (a.kept) {
        if (lane == 0) s_woff[wave] = wkept;
        __syncthreads();
        if (tid == 0) {
            int n = 0;
            for (int w = 0; w < kWaves; ++w) n += s_woff[w];
            a.kept[row] = n;
        }
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
    const bool ragged = (V & 3) != 0;
    const bool bands = top_k > 0 && !(top_p < 1.f);
#define RSD_LAUNCH_FILTER(CH)                                                                                 \
    do {                                                                                                      \
        if (bands && ragged)                                                                                  \
            hipLaunchKernelGGL((prob_filter_kernel<CH, true, true>), dim3(R), dim3(kFilterThreads), 0, st, a);   \
        else if (bands)                                                                                       \
            hipLaunchKernelGGL((prob_filter_kernel<CH, false, true>), dim3(R), dim3(kFilterThreads), 0, st, a);  \
        else if (ragged)                                                                                      \
            hipLaunchKernelGGL((prob_filter_kernel<CH, true, false>), dim3(R), dim3(kFilterThreads), 0, st, a);  \
        else                                                                                                  \
            hipLaunchKernelGGL((prob_filter_kernel<CH, false, false>), dim3(R), dim3(kFilterThreads), 0, st, a); \
    } while (0)
    if (chunks <= 2)
        RSD_LAUNCH_FILTER(2);
    else if (chunks <= 8)
        RSD_LAUNCH_FILTER(8);
    else if (chunks <= 13)
        RSD_LAUNCH_FILTER(13);
    else
        RSD_LAUNCH_FILTER(16);
#undef RSD_LAUNCH_FILTER
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}
