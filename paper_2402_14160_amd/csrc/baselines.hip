// Baseline verifiers of one level of K draft tokens drawn i.i.d. from the draft distribution
// (Sec. 2, tree-based speculative decoding): K-SEQ of SpecTr and multi-round rejection sampling of
// SpecInfer, on the same logit rows and with the same position-indexed randomness as recursive
// rejection sampling, so that acceptance can be compared method against method on one workload.
//
// One workgroup verifies one (target row, draft row) pair and streams the two rows from memory
// at every pass (the rows of a level are few; nothing is kept resident).  With
//   e_t(x) = 2^(zt(x) c - m_t),  e_d(x) = 2^(zd(x) c - m_d),  St = sum e_t,  Sd = sum e_d:
//  K-SEQ:        Theta_k = min(1, q(x_k) / (gamma p(x_k)));  beta = sum_x min(p, q / gamma);
//                all rejected -> draw from [q - min(p, q / gamma) (1 - (1 - beta)^K) / beta]^+.
//  multi-round:  u = e_t, A_1 = St;  Theta_k = (u(x_k) / A_k) / p(x_k);
//                u <- max(u - (A_k / Sd) e_d, 0), A_{k+1} = sum u;  all rejected -> draw from u.
// The drafted tokens are followed in fp64 by one lane each (and left out of the fp32 sums once);
// everything else is fp32 per entry with sums combined in fp64 in a fixed order.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>

#include "../../include/rsd.h"
#include "rsd_device.hpp"

namespace rsd {

constexpr int kBaseThreads = 512;
constexpr int kBaseWaves = kBaseThreads / kWave;

struct BaseArgs {
    const float *zt, *zd;
    int64_t ld;
    int R, V, K, method;
    double gamma;      // K-SEQ
    float inv_t;
    ScalePair sc;
    const int *drafts;  // [R, K]
    const int *seq_id, *node_id;
    uint64_t seed;
    uint32_t step;
    int *accepted, *token;
    float *theta;
    uint32_t *flags;
};

struct BaseShared {
    double red[3][kBaseWaves];
    MaxSum ms[kBaseWaves];
    float sv[2 * kBaseWaves];
    int si[2 * kBaseWaves];
    int tok[RSD_K_MAX];
    double du[RSD_K_MAX], de[RSD_K_MAX];   // fp64 exponentials of the drafted tokens
    double gam[RSD_K_MAX];                  // multi-round: gamma_k of stage k (0: skipped)
    float theta[RSD_K_MAX];
    int accepted;
    uint32_t flags;
};

// Workgroup-wide sums of up to three fp32 partials (fp32 inside a wave, fp64 across waves, fixed order).
__device__ __forceinline__ void block_sum3(float a, float b, float c, BaseShared &sh, double out[3]) {
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    a = wave_sum(a); b = wave_sum(b); c = wave_sum(c);
    __syncthreads();  // (the scratch may still be read from the previous call)
    if (lane == 0) { sh.red[0][wave] = (double)a; sh.red[1][wave] = (double)b; sh.red[2][wave] = (double)c; }
    __syncthreads();
    out[0] = out[1] = out[2] = 0.0;
#pragma unroll
    for (int w = 0; w < kBaseWaves; ++w) { out[0] += sh.red[0][w]; out[1] += sh.red[1][w]; out[2] += sh.red[2][w]; }
}

__device__ __forceinline__ bool is_draft(int x, const int *tok, int K) {
    bool hit = false;
    for (int i = 0; i < K; ++i) hit |= tok[i] == x;
    return hit;
}

__global__ __launch_bounds__(kBaseThreads) void baseline_verify_kernel(BaseArgs a) {
    __shared__ BaseShared sh;
    const int r = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int K = a.K, V = a.V;
    const float *zt = a.zt + (int64_t)r * a.ld, *zd = a.zd + (int64_t)r * a.ld;
    const uint32_t seq = a.seq_id ? (uint32_t)a.seq_id[r] : 0u;
    const uint32_t node = a.node_id ? (uint32_t)a.node_id[r] : (uint32_t)r;
    const float c2h = a.sc.c2h, c2l = a.sc.c2l;
    if (tid < K) sh.tok[tid] = min(max(a.drafts[(int64_t)r * K + tid], 0), V - 1);
    if (tid == 0) { sh.accepted = -1; sh.flags = 0; }
    // ---- row maxima of the raw logits ------------------------------------------------------
    float mt = -INFINITY, md = -INFINITY;
    for (int x = tid; x < V; x += kBaseThreads) {
        mt = fmaxf(mt, zt[x]);
        md = fmaxf(md, zd[x]);
    }
    mt = wave_max(mt);
    md = wave_max(md);
    if (lane == 0) sh.ms[wave] = MaxSum{mt, md};
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kBaseWaves; ++w) { mt = fmaxf(mt, sh.ms[w].m); md = fmaxf(md, sh.ms[w].s); }
    const float m_t = (mt == -INFINITY) ? 0.f : mt * c2h, m_d = (md == -INFINITY) ? 0.f : md * c2h;
    // the drafted tokens in fp64 (lane k follows draft k; equal tokens are equal copies)
    double tU = 0.0, tE = 0.0;
    bool first = false;  // this lane holds the first copy of its token: it stands for the token in sums
    if (tid < K) {
        const int x = sh.tok[tid];
        tU = exp2((double)zt[x] * a.sc.c2e - (double)m_t);
        tE = exp2((double)zd[x] * a.sc.c2e - (double)m_d);
        first = true;
        for (int i = 0; i < tid; ++i) first = first && sh.tok[i] != x;
        sh.du[tid] = tU;
        sh.de[tid] = tE;
    }
    // ---- sums (drafted tokens left out of the fp32 part) -----------------------------------
    float st = 0.f, sd = 0.f;
    for (int x = tid; x < V; x += kBaseThreads) {
        const bool dr = is_draft(x, sh.tok, K);
        st += dr ? 0.f : __builtin_amdgcn_exp2f(exponent_of(zt[x], c2h, c2l, -m_t));
        sd += dr ? 0.f : __builtin_amdgcn_exp2f(exponent_of(zd[x], c2h, c2l, -m_d));
    }
    double sums[3];
    block_sum3(st, sd, 0.f, sh, sums);
    double St = sums[0], Sd = sums[1];
    for (int i = 0; i < K; ++i) {  // every thread, same order
        bool fst = true;
        for (int j = 0; j < i; ++j) fst = fst && sh.tok[j] != sh.tok[i];
        if (fst) { St += sh.du[i]; Sd += sh.de[i]; }
    }
    if (tid == 0 && (!(St > 0.0) || !isfinite(St) || !(Sd > 0.0) || !isfinite(Sd))) sh.flags |= RSD_FLAG_NONFINITE;

    double kseq_c = 0.0;       // K-SEQ: (1 - (1 - beta)^K) / beta
    const double ratio = St / Sd;  // e_d * ratio is p on the scale of e_t
    if (a.method == RSD_BASELINE_KSEQ) {
        // beta * St = sum_x min(e_d St / Sd, e_t / gamma)
        const float rf = (float)ratio, ig = (float)(1.0 / a.gamma);
        float part = 0.f;
        for (int x = tid; x < V; x += kBaseThreads) {
            if (is_draft(x, sh.tok, K)) continue;
            const float et = __builtin_amdgcn_exp2f(exponent_of(zt[x], c2h, c2l, -m_t));
            const float ed = __builtin_amdgcn_exp2f(exponent_of(zd[x], c2h, c2l, -m_d));
            part += fminf(ed * rf, et * ig);
        }
        block_sum3(part, 0.f, 0.f, sh, sums);
        double bsum = sums[0];
        for (int i = 0; i < K; ++i) {
            bool fst = true;
            for (int j = 0; j < i; ++j) fst = fst && sh.tok[j] != sh.tok[i];
            if (fst) bsum += fmin(sh.de[i] * ratio, sh.du[i] / a.gamma);
        }
        const double beta = bsum / St;
        kseq_c = beta > 0.0 ? (1.0 - pow(1.0 - beta, (double)K)) / beta : (double)K;
        if (tid < K) {
            const double p = tE * ratio * a.gamma;
            sh.theta[tid] = (p > 0.0) ? (float)fmin(1.0, tU / p) : 1.f;
        }
    } else {
        // multi-round: K stages, each re-reading the rows and replaying the chain so far
        double A = St;
        for (int k = 0; k < K; ++k) {
            if (tid == k) {
                const double p = tE / Sd;
                sh.theta[k] = (p > 0.0) ? (float)fmin(1.0, tU / (A * p)) : 1.f;
            }
            const double gam = A / Sd;
            const float gh = (float)gam, gl = (float)(gam - (double)(float)gam);
            float part = 0.f;
            for (int x = tid; x < V; x += kBaseThreads) {
                if (is_draft(x, sh.tok, K)) continue;
                float u = __builtin_amdgcn_exp2f(exponent_of(zt[x], c2h, c2l, -m_t));
                const float ed = __builtin_amdgcn_exp2f(exponent_of(zd[x], c2h, c2l, -m_d));
                for (int j = 0; j < k; ++j) {
                    const double gj = sh.gam[j];
                    const float hj = (float)gj, lj = (float)(gj - (double)hj);
                    u = fmaxf(fmaf(-lj, ed, fmaf(-hj, ed, u)), 0.f);
                }
                part += fmaxf(fmaf(-gl, ed, fmaf(-gh, ed, u)), 0.f);
            }
            const double cnew = fmax(tU - gam * tE, 0.0);
            block_sum3(part, 0.f, 0.f, sh, sums);
            __syncthreads();
            if (tid < K) sh.du[tid] = cnew;   // (du now carries the candidates' next values)
            __syncthreads();
            double S = sums[0];
            for (int i = 0; i < K; ++i) {
                bool fst = true;
                for (int j = 0; j < i; ++j) fst = fst && sh.tok[j] != sh.tok[i];
                if (fst) S += sh.du[i];
            }
            const bool ok = S > 0.0 && isfinite(S);
            if (ok) {
                tU = cnew;
                A = S;
            }
            if (tid == 0) {
                sh.gam[k] = ok ? gam : 0.0;
                if (!ok) sh.flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
            }
            __syncthreads();
        }
    }
    __syncthreads();
    // ---- accept / reject in order -------------------------------------------------------------
    if (tid == 0) {
        const PhiloxKey key = make_key(a.seed);
        for (int k = 0; k < K; ++k) {
            const uint4 w = philox4x32_10((uint32_t)k >> 2, node, seq, counter_word3(kTagAcceptUniform, a.step), key);
            const uint32_t sel = (uint32_t)k & 3u;
            const float u = uniform_from_word(sel == 0 ? w.x : (sel == 1 ? w.y : (sel == 2 ? w.z : w.w)));
            if (u < sh.theta[k]) {
                sh.accepted = k;
                break;
            }
        }
    }
    if (a.theta && tid < K) a.theta[(int64_t)r * K + tid] = sh.theta[tid];
    __syncthreads();
    const int acc = sh.accepted;
    if (acc >= 0) {
        if (tid == 0) {
            a.accepted[r] = acc;
            a.token[r] = sh.tok[acc];
            // (flags of stages behind the accepted draft do not matter: their residuals were not used)
            if (a.flags) a.flags[r] = sh.flags & RSD_FLAG_NONFINITE;
        }
        return;
    }
    // ---- all rejected: Gumbel-max over the residual -------------------------------------------
    const PhiloxKey key = make_key(a.seed);
    const uint32_t c3 = counter_word3(kTagLastGumbel, a.step);
    float bv = -INFINITY, av = -INFINITY;
    int bi = INT_MAX, ai = INT_MAX;
    bool negative = false;
    for (int x = tid; x < V; x += kBaseThreads) {
        const uint4 w = philox4x32_10((uint32_t)x >> 2, node, seq, c3, key);
        const uint32_t sel = (uint32_t)x & 3u;
        const float gum = gumbel_from_word(sel == 0 ? w.x : (sel == 1 ? w.y : (sel == 2 ? w.z : w.w)));
        double res, alt;  // residual and the fallback (the target itself / the last kept q^(k)), up to one factor
        if (is_draft(x, sh.tok, K)) {
            const double U0 = exp2((double)zt[x] * a.sc.c2e - (double)m_t);
            const double E = exp2((double)zd[x] * a.sc.c2e - (double)m_d);
            if (a.method == RSD_BASELINE_KSEQ) {
                const double raw = U0 - fmin(E * ratio, U0 / a.gamma) * kseq_c;
                negative |= raw < -1e-5 * U0;
                res = fmax(raw, 0.0);
                alt = U0;
            } else {
                double U = U0;
                for (int j = 0; j < K; ++j) U = fmax(U - sh.gam[j] * E, 0.0);
                res = U;
                alt = U0;
            }
        } else {
            float u = __builtin_amdgcn_exp2f(exponent_of(zt[x], c2h, c2l, -m_t));
            const float ed = __builtin_amdgcn_exp2f(exponent_of(zd[x], c2h, c2l, -m_d));
            alt = (double)u;
            if (a.method == RSD_BASELINE_KSEQ) {
                const float raw = fmaf(-fminf(ed * (float)ratio, u * (float)(1.0 / a.gamma)), (float)kseq_c, u);
                negative |= raw < -1e-5f * u;
                res = (double)fmaxf(raw, 0.f);
            } else {
                for (int j = 0; j < K; ++j) {
                    const double gj = sh.gam[j];
                    const float hj = (float)gj, lj = (float)(gj - (double)hj);
                    u = fmaxf(fmaf(-lj, ed, fmaf(-hj, ed, u)), 0.f);
                }
                res = (double)u;
            }
        }
        const float s = fast_ln((float)res) + gum, s2 = fast_ln((float)alt) + gum;
        if (better(s, x, bv, bi)) { bv = s; bi = x; }
        if (better(s2, x, av, ai)) { av = s2; ai = x; }
    }
    const unsigned long long neg_any = __ballot(negative);
    if (lane == 0 && neg_any) atomicOr(&sh.flags, RSD_FLAG_DEGENERATE_RESIDUAL);
    block_argmax_pair<kBaseThreads>(bv, bi, av, ai, sh.sv, sh.si);
    __syncthreads();
    if (tid == 0) {
        uint32_t flags = sh.flags;
        int tokn = bi;
        if (!(bv > -INFINITY)) {  // empty residual: the fallback distribution
            flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
            tokn = ai;
        }
        a.accepted[r] = -1;
        a.token[r] = tokn == INT_MAX ? 0 : tokn;
        if (a.flags) a.flags[r] = flags;
    }
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace rsd

using namespace rsd;

extern "C" int32_t rsd_baseline_verify(const float *draft_logits, const float *target_logits, int64_t ld,
                                       int32_t R, int32_t V, const int32_t *drafts, int32_t K,
                                       int32_t method, float gamma, float inv_temperature,
                                       const int32_t *seq_id, const int32_t *node_id, uint64_t seed,
                                       uint32_t step, int32_t *accepted, int32_t *token, float *theta,
                                       uint32_t *flags, void *stream) {
    if (!draft_logits || !target_logits || !drafts || !accepted || !token) return RSD_ERR_NULL;
    if (R < 0 || V < 1 || ld < V || K < 1 || K > RSD_K_MAX || !(inv_temperature > 0.f) ||
        !aligned16(draft_logits) || !aligned16(target_logits))
        return RSD_ERR_SHAPE;
    if (method != RSD_BASELINE_KSEQ && method != RSD_BASELINE_MULTIROUND) return RSD_ERR_UNSUPPORTED;
    if (method == RSD_BASELINE_KSEQ && !(gamma >= 1.f && gamma <= (float)K)) return RSD_ERR_SHAPE;
    if (R == 0) return RSD_OK;
    BaseArgs a{};
    a.zt = target_logits; a.zd = draft_logits; a.ld = ld; a.R = R; a.V = V; a.K = K; a.method = method;
    a.gamma = (double)gamma; a.inv_t = inv_temperature;
    a.sc.c2e = (double)inv_temperature * 1.4426950408889634;
    a.sc.c2h = (float)a.sc.c2e;
    if ((double)a.sc.c2h >= a.sc.c2e) a.sc.c2h = nextafterf(a.sc.c2h, 0.f);
    a.sc.c2l = (float)(a.sc.c2e - (double)a.sc.c2h);
    a.drafts = drafts; a.seq_id = seq_id; a.node_id = node_id; a.seed = seed; a.step = step;
    a.accepted = accepted; a.token = token; a.theta = theta; a.flags = flags;
    hipLaunchKernelGGL(baseline_verify_kernel, dim3(R), dim3(kBaseThreads), 0, (hipStream_t)stream, a);
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}
