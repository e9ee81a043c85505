// Recursive rejection sampling over the draft tree (Sec. 3.1; Sec. 3.2.2; Alg. 6).
//
// A sibling group (the children x_1..x_K of one node) is verified by one
// workgroup.  The residual distributions q^(k) of Eq. (2) are never stored:
// with e_t(x) = 2^(zt(x) - max zt), e_d(x) = 2^(zd(x) - max zd) (log2 domain),
//   q^(1)(x)   = e_t(x) / s_t
//   p^(k)(x)   = e_d(x) / s_k          for x not in {x_1..x_{k-1}}, else 0
//   q^(k+1)(x) = max(q^(k)(x) - p^(k)(x), 0) / S_k,   S_k = sum_x max(q^(k) - p^(k), 0)
// The resident variants keep u(x) = q^(k)(x) * A_k and e_d(x) on chip (registers, and LDS
// for the larger vocabularies) and update u in place at every stage; the streaming variant
// (largest vocabularies) re-reads the two rows at every stage and evaluates the short
// per-entry chain from the scalars (s_t, s_1.., S_1..) found so far.  Either way only the
// scalars go to memory, and the last-token pass re-evaluates the chain from them.
// s_k sums the draft row without the removed tokens directly (no 1 - p
// cancellation).  Sums are accumulated per lane in fp32, across waves in fp64
// in a fixed order, so results do not depend on scheduling.
//
// ALL_GROUPS runs three kernels (plan, groups, walk + last token), PATH one persistent
// workgroup per sequence.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>

#include "../../include/rsd.h"
#include "rsd_device.hpp"

namespace rsd {

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;

constexpr int kGroupThreads = 512;   // streaming variant (any vocabulary size)
constexpr int kRegThreads = 512;     // register-resident variant: 2 waves per SIMD, 256 VGPRs each
// resident variant with most of the draft row in LDS (larger vocabularies): 12 waves, three per
// SIMD, so that a thread has 168 registers
constexpr int kLdsThreads = 768;
constexpr int kLdsChunks = 17;       // float4 chunks per thread: 52224 entries
constexpr int kLdsChunksInLds = 12;  // of which in LDS: 12 * 768 * 16 B = 144 KB
constexpr int kGroupWavesMax = 16;
constexpr int kFinalThreads = 512;
constexpr int kFinalSplitsMax = 8;

// Per (sequence, node) record produced by the group pass, kept in workspace.
struct GroupRec {
    float mt2;      // max of target row, log2 domain
    float md2;      // max of draft row, log2 domain
    float inv_st;   // 1 / sum_x 2^(zt2 - mt2)
    int K;          // number of verified children (<= RSD_K_MAX); 0 for a leaf
    uint32_t flags;
    int pad[3];
    int kid[RSD_K_MAX];      // child node ids in stored order
    int tok[RSD_K_MAX];      // their tokens
    float inv_s[RSD_K_MAX];  // 1 / s_k (draft mass left at stage k); 0 marks a skipped stage
    float inv_S[RSD_K_MAX];  // 1 / S_k (1 for a skipped stage)
    float theta[RSD_K_MAX];
};

struct RrsArgs {
    const float *zd;
    const float *zt;
    int B, N, V;
    float inv_t;   // 1/T
    float c2;      // log2(e)/T
    const int *tokens;
    const int *parent;
    const int *n_nodes;
    const int *seq_id;
    uint64_t seed;
    uint32_t step;
    int *accepted_nodes;
    int *accepted_tokens;
    int depth_max;
    int *n_accepted;
    int *last_token;
    int *final_node;
    float *theta;
    float *uniforms;
    uint32_t *flags;
    // workspace
    GroupRec *rec;              // [B, N]
    unsigned long long *fkey;   // [B, 2] packed (score, token) maxima: residual / fallback
    int *fdone;                 // [B]
    int *kcount;                // [B, N] number of children of every node
    int2 *work;                 // [B, N] non-leaf nodes {b * N + node, nodes of the tree}, most children first
    int *wq;                    // [0] number of work items
};

__device__ __forceinline__ int removal_stage(int x, const int *tok, int K) {
    int rs = K;
    for (int i = K - 1; i >= 0; --i)
        if (tok[i] == x) rs = i;
    return rs;
}

__device__ __forceinline__ float uniform_f(float v) {
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(v)));
}

// The group's scalars pulled into (scalar) registers once per pass so that the
// per-entry chain indexes them statically.
struct ChainRegs {
    float mt2, md2, inv_st;
    float is[RSD_K_MAX];
    float iS[RSD_K_MAX];
};

__device__ __forceinline__ ChainRegs load_chain(const GroupRec &g) {
    ChainRegs r;
    r.mt2 = uniform_f(g.mt2);
    r.md2 = uniform_f(g.md2);
    r.inv_st = uniform_f(g.inv_st);
#pragma unroll
    for (int j = 0; j < RSD_K_MAX; ++j) {
        r.is[j] = uniform_f(g.inv_s[j]);
        r.iS[j] = uniform_f(g.inv_S[j]);
    }
    return r;
}

// q^(nst+1) for four entries none of which is a child token.
__device__ __forceinline__ void chain4(const float et[4], const float ed[4], const ChainRegs &r,
                                       int nst, float q[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = et[i] * r.inv_st;
#pragma unroll
    for (int j = 0; j < RSD_K_MAX - 1; ++j) {
        if (j < nst) {  // wave-uniform; keeps the scalar arrays statically indexed
#pragma unroll
            for (int i = 0; i < 4; ++i) q[i] = fmaxf(q[i] - ed[i] * r.is[j], 0.f) * r.iS[j];
        }
    }
}

// q^(nst+1)(x) when x may be the child token removed at stage rs (rs = K: never).
__device__ __forceinline__ float chain1_masked(float et, float ed, int rs, const ChainRegs &r,
                                               int nst) {
    float q = et * r.inv_st;
#pragma unroll
    for (int j = 0; j < RSD_K_MAX - 1; ++j) {
        if (j < nst) {
            const float p = (rs < j) ? 0.f : ed * r.is[j];
            q = fmaxf(q - p, 0.f) * r.iS[j];
        }
    }
    return q;
}

// Bit i set: this thread's i-th chunk (c = c_lo + tid + i*THREADS) holds a child token.
template <int THREADS>
__device__ __forceinline__ uint64_t child_chunk_mask(const GroupRec &g, int c_lo, int c_hi) {
    uint64_t m = 0;
    for (int i = 0; i < g.K; ++i) {
        const int cc = g.tok[i] >> 2;
        if (cc >= c_lo && cc < c_hi) {
            const int rel = cc - c_lo;
            if (rel % THREADS == (int)threadIdx.x) m |= 1ull << (rel / THREADS);
        }
    }
    return m;
}

struct GroupShared {
    GroupRec g;
    MaxSum ms[kGroupWavesMax];
    double red[kGroupWavesMax];
    double red2[kGroupWavesMax];
    float czt[RSD_K_MAX];   // raw target / draft logits of the child tokens (resident variant)
    float czd[RSD_K_MAX];
    double ce[RSD_K_MAX];   // draft exponentials of the child tokens (fp64)
    double sred[2][kGroupWavesMax];  // stage sums of the resident variant, alternating
    unsigned long long cmask[RSD_NODES_MAX / kWave];  // per-wave ballots of the child scan
    int cur;
    int done;
};

// Pass 0: maxima and sums of both rows.  The draft sum leaves out every child token.
template <int THREADS>
__device__ void group_lse_pass(const float *zt, const float *zd, int V, float c2, GroupShared &sh) {
    const int nchunk = V >> 2;
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const uint64_t hits = child_chunk_mask<THREADS>(sh.g, 0, nchunk);
    MaxSum at{-INFINITY, 0.f}, ad{-INFINITY, 0.f};
    int it = 0;
#pragma unroll 2
    for (int c = threadIdx.x; c < nchunk; c += THREADS, ++it) {
        const float4 t = zt4[c];
        const float4 d = zd4[c];
        const float a[4] = {t.x * c2, t.y * c2, t.z * c2, t.w * c2};
        const float e[4] = {d.x * c2, d.y * c2, d.z * c2, d.w * c2};
        const float mt = fmaxf(fmaxf(a[0], a[1]), fmaxf(a[2], a[3]));
        const float md = fmaxf(fmaxf(e[0], e[1]), fmaxf(e[2], e[3]));
        if (mt > at.m) { at.s *= exp2f(at.m - mt); at.m = mt; }
        if (md > ad.m) { ad.s *= exp2f(ad.m - md); ad.m = md; }
        if (at.m > -INFINITY)
            at.s += (exp2f(a[0] - at.m) + exp2f(a[1] - at.m)) + (exp2f(a[2] - at.m) + exp2f(a[3] - at.m));
        if (ad.m > -INFINITY) {
            if (!((hits >> it) & 1ull)) {
                ad.s += (exp2f(e[0] - ad.m) + exp2f(e[1] - ad.m)) + (exp2f(e[2] - ad.m) + exp2f(e[3] - ad.m));
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (removal_stage((c << 2) + i, sh.g.tok, sh.g.K) == sh.g.K) ad.s += exp2f(e[i] - ad.m);
            }
        }
    }
    at = block_merge<THREADS>(at, sh.ms);
    ad = block_merge<THREADS>(ad, sh.ms);
    if (threadIdx.x == 0) {
        sh.g.mt2 = at.m;
        sh.g.md2 = ad.m;
        sh.g.inv_st = 1.f / at.s;
        // draft mass still available at stage k: the rest plus the children not yet removed
        double e[RSD_K_MAX];
        for (int i = 0; i < sh.g.K; ++i) e[i] = exp2((double)zd[sh.g.tok[i]] * (double)c2 - (double)ad.m);
        double s = (double)ad.s;
        for (int k = RSD_K_MAX - 1; k >= 0; --k) {
            if (k < sh.g.K) {
                s += e[k];
                sh.g.inv_s[k] = (float)(1.0 / s);
            } else {
                sh.g.inv_s[k] = 0.f;
            }
            sh.g.inv_S[k] = 1.f;
        }
        if (!(at.s > 0.f) || !isfinite(at.s) || !(s > 0.0) || !isfinite(s)) sh.g.flags |= RSD_FLAG_NONFINITE;
    }
    __syncthreads();
}

// Stage pass: S = sum_x max(q^(nst+1)(x) - p^(nst+1)(x), 0).
template <int THREADS>
__device__ double group_residual_mass(const float *zt, const float *zd, int V, float c2, int nst,
                                      GroupShared &sh) {
    const int nchunk = V >> 2;
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const GroupRec &g = sh.g;
    const ChainRegs cr = load_chain(g);
    const float inv_s = uniform_f(g.inv_s[nst]);
    const uint64_t hits = child_chunk_mask<THREADS>(g, 0, nchunk);
    float part = 0.f;
    int it = 0;
#pragma unroll 2
    for (int c = threadIdx.x; c < nchunk; c += THREADS, ++it) {
        const float4 t = zt4[c];
        const float4 d = zd4[c];
        const float et[4] = {exp2f(fmaf(t.x, c2, -cr.mt2)), exp2f(fmaf(t.y, c2, -cr.mt2)),
                             exp2f(fmaf(t.z, c2, -cr.mt2)), exp2f(fmaf(t.w, c2, -cr.mt2))};
        const float ed[4] = {exp2f(fmaf(d.x, c2, -cr.md2)), exp2f(fmaf(d.y, c2, -cr.md2)),
                             exp2f(fmaf(d.z, c2, -cr.md2)), exp2f(fmaf(d.w, c2, -cr.md2))};
        float r[4];
        if (!((hits >> it) & 1ull)) {
            float q[4];
            chain4(et, ed, cr, nst, q);
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = fmaxf(q[i] - ed[i] * inv_s, 0.f);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rs = removal_stage((c << 2) + i, g.tok, g.K);
                const float p = (rs < nst) ? 0.f : ed[i] * inv_s;
                r[i] = fmaxf(chain1_masked(et[i], ed[i], rs, cr, nst) - p, 0.f);
            }
        }
        part += (r[0] + r[1]) + (r[2] + r[3]);
    }
    return block_sum<THREADS>(part, sh.red);
}

// Threshold of child k (Eq. (3)) from the scalars found so far, in fp64.
__device__ double child_theta(const float *zt, const float *zd, float c2, int k, const GroupRec &g) {
    const int x = g.tok[k];
    const double et = exp2((double)zt[x] * (double)c2 - (double)g.mt2);
    const double ed = exp2((double)zd[x] * (double)c2 - (double)g.md2);
    double q = et * (double)g.inv_st;
    for (int j = 0; j < k; ++j)  // x_k is not removed before stage k
        q = fmax(q - ed * (double)g.inv_s[j], 0.0) * (double)g.inv_S[j];
    const double p = ed * (double)g.inv_s[k];
    if (!(p > 0.0)) return 1.0;
    return fmin(1.0, q / p);
}

// Children of `node` in stored order, into sh.g (kid, tok, K): the first RSD_NODES_MAX threads
// test one node each, wave ballots give every match its rank.  All threads of the workgroup
// take part; ends with a barrier.  The halves can be called apart: fetch_candidate only issues
// this thread's loads (its parent and token), fetch_child_logits the two logits of its token
// when it is a child (sh.czt / sh.czd then hold them by rank), rank_children consumes them.
struct ChildCandidate {
    int parent, token;
    float zt, zd;
};

__device__ __forceinline__ ChildCandidate fetch_candidate(const RrsArgs &a, int b, int node, int n, int j) {
    const int *par = a.parent + (int64_t)b * a.N;
    const int *tok = a.tokens + (int64_t)b * a.N;
    ChildCandidate c{-2, 0, 0.f, 0.f};  // -2: not a node of this tree (a parent is >= -1)
    if (j > node && j < n) {
        c.parent = par[j];
        c.token = tok[j];
    }
    return c;
}

// (the first use of the candidate: clamps its token so that it never indexes outside the row)
__device__ __forceinline__ void fetch_child_logits(const float *zt, const float *zd, int V, int node,
                                                   ChildCandidate &c) {
    c.token = min(max(c.token, 0), V - 1);
    if (c.parent == node) {
        c.zt = zt[c.token];
        c.zd = zd[c.token];
    }
}

__device__ __forceinline__ void rank_children(const RrsArgs &a, int node, ChildCandidate cand, GroupShared &sh,
                                              int j) {
    const int lane = j & (kWave - 1), wave = j / kWave;
    const bool match = cand.parent == node;
    const int t = cand.token;
    const unsigned long long mask = __ballot(match);
    if (wave < RSD_NODES_MAX / kWave && lane == 0) sh.cmask[wave] = mask;
    __syncthreads();
    if (match) {
        int rank = __popcll(mask & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) rank += __popcll(sh.cmask[w]);
        if (rank < RSD_K_MAX) {
            sh.g.kid[rank] = j;
            sh.g.tok[rank] = t;
            sh.czt[rank] = cand.zt;
            sh.czd[rank] = cand.zd;
        }
    }
    if (j == 0) {
        int total = 0;
        for (int w = 0; w < RSD_NODES_MAX / kWave; ++w) total += __popcll(sh.cmask[w]);
        sh.g.K = min(total, RSD_K_MAX);
        sh.g.flags = 0;
    }
    __syncthreads();
}

__device__ __forceinline__ void scan_children(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    ChildCandidate c = fetch_candidate(a, b, node, n, threadIdx.x);
    c.token = min(max(c.token, 0), a.V - 1);
    rank_children(a, node, c, sh, threadIdx.x);
}

template <int THREADS>
__device__ void process_group(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    scan_children(a, b, node, n, sh);
    const int K = sh.g.K;
    if (K == 0) return;
    const float *zt = a.zt + ((int64_t)b * a.N + node) * a.V;
    const float *zd = a.zd + ((int64_t)b * a.N + node) * a.V;
    group_lse_pass<THREADS>(zt, zd, a.V, a.c2, sh);
    for (int k = 0; k < K; ++k) {
        if (threadIdx.x == 0) sh.g.theta[k] = (float)child_theta(zt, zd, a.c2, k, sh.g);
        if (k == K - 1) break;
        __syncthreads();
        const double S = group_residual_mass<THREADS>(zt, zd, a.V, a.c2, k, sh);
        if (threadIdx.x == 0) {
            if (S > 0.0 && isfinite(S)) {
                sh.g.inv_S[k] = (float)(1.0 / S);
            } else {  // keep q^(k): no subtraction, no rescale
                sh.g.inv_s[k] = 0.f;
                sh.g.inv_S[k] = 1.f;
                sh.g.flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
            }
        }
        __syncthreads();
    }
    __syncthreads();
}


// Resident variant for vocabularies up to T * 4 * CH entries: both logit rows are read from
// memory once; each thread keeps its share of the target-side value u(x) (q^(k) = u / A_k) in
// registers and its share of the draft exponentials e_d(x) in registers (chunks CL..CH-1) and,
// for the larger vocabularies, in LDS (chunks 0..CL-1, a slot of its own per thread and chunk,
// so no barrier guards them).  A stage is
//     S = sum_x max(u - gamma_k * e_d, 0);   u <- max(u - gamma_k * e_d, 0);   A_{k+1} = S
// with gamma_k = A_k / s_k: three to five ALU operations per entry, one wave reduction and a
// single barrier.  Every thread carries the scalars; lane t < K follows child token t in fp64.
template <int T, int CH, int CL>
__device__ void process_group_reg(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    constexpr int NW = T / kWave;
    constexpr int CR = CH - CL;  // chunks of e_d held in registers
    static_assert(NW <= kGroupWavesMax && CL >= 0 && CL < CH, "");
    __shared__ float4 s_ed[CL > 0 ? CL * T : 1];
    // (a copy of the thread index that the compiler takes for a new value in every call: what
    // derives from it -- chunk addresses, LDS slots, lane masks -- is then worked out here, next
    // to its use, instead of being kept in registers from one group to the next)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int wave = tid / kWave;
    const bool lane0 = (tid & (kWave - 1)) == 0;
    const float *zt = a.zt + ((int64_t)b * a.N + node) * a.V;
    const float *zd = a.zd + ((int64_t)b * a.N + node) * a.V;
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const int nchunk = a.V >> 2;
    const float c2 = a.c2;
    const int last = nchunk - 1;  // the caller checks V >= 4
    // The children's lookup is requested first and the rows right after it, before the lookup
    // is used: its dependent steps (the children's own logits, two barriers) then run under
    // the rows' memory latency.  Every row load is unconditional (a chunk past the end of the
    // row reads the row's last chunk instead and is set to -inf when it is scaled), so that
    // the loads form one straight line and a wait can name exactly the loads it needs.  A node
    // without children (the end of a path) costs one row pair that is not used.
    ChildCandidate cand = fetch_candidate(a, b, node, n, tid);
    float ut[CH * 4], edr[CR * 4];
    // chunk j of e_d, wherever it lives (j is a constant once the loops are unrolled)
    auto ed_get = [&](int j) -> float4 {
        if (j < CL) return s_ed[j * T + tid];
        const int r = j < CL ? 0 : 4 * (j - CL);
        return make_float4(edr[r], edr[r + 1], edr[r + 2], edr[r + 3]);
    };
    auto ed_put = [&](int j, float4 v) {
        if (j < CL) {
            s_ed[j * T + tid] = v;
        } else {
            const int r = j < CL ? 0 : 4 * (j - CL);
            edr[r] = v.x; edr[r + 1] = v.y; edr[r + 2] = v.z; edr[r + 3] = v.w;
        }
    };
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = min(j * T + tid, last);
        const float4 t = zt4[c];
        ut[4 * j + 0] = t.x; ut[4 * j + 1] = t.y; ut[4 * j + 2] = t.z; ut[4 * j + 3] = t.w;
        if (j >= CL) ed_put(j, zd4[c]);
    }
    // (the candidate is consumed from here on: its wait and the children's own logit loads come
    // after every row load has been issued)
    asm volatile("" : "+v"(cand.parent), "+v"(cand.token));
    fetch_child_logits(zt, zd, a.V, node, cand);
    // chunks 0..CL-1 of the draft row go from memory straight into this thread's LDS slots (no
    // registers, raw logits; 64 lanes x 16 bytes land contiguously, which is the slot layout;
    // issued last, so that the wait above counts register loads only)
    if constexpr (CL > 0) {
#pragma unroll
        for (int j = 0; j < CL; ++j)
            __builtin_amdgcn_global_load_lds((global_void *)(zd4 + min(j * T + tid, last)),
                                             (lds_void *)(s_ed + j * T + wave * kWave), 16, 0, 0);
    }
    // The row maxima and the children's ranks share their barriers: every wave first reduces
    // its part of the two rows (scaled in place) and takes the ballot of its candidates, then
    // one barrier publishes both, and the ranks are written while the maxima are combined.
    float mt = -INFINITY, md = -INFINITY;
    // the LDS part of the draft row: wait for this wave's memory-to-LDS loads (the slots are the
    // wave's own, so no barrier)
    if constexpr (CL > 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // scaling: x * c2 + 0 for a chunk of the row, x * c2 - inf = -inf for a chunk past its end
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const float bias = (j * T + tid <= last) ? 0.f : -INFINITY;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            ut[4 * j + e] = fmaf(ut[4 * j + e], c2, bias);
            mt = fmaxf(mt, ut[4 * j + e]);
        }
        float4 d = ed_get(j);
        d.x = fmaf(d.x, c2, bias); d.y = fmaf(d.y, c2, bias); d.z = fmaf(d.z, c2, bias); d.w = fmaf(d.w, c2, bias);
        md = fmaxf(md, fmaxf(fmaxf(d.x, d.y), fmaxf(d.z, d.w)));
        ed_put(j, d);
    }
    mt = wave_max(mt);
    md = wave_max(md);
    const int lane = tid & (kWave - 1);
    const bool match = cand.parent == node;
    const unsigned long long cmask = __ballot(match);
    if (lane0) {
        sh.ms[wave] = MaxSum{mt, md};
        if (wave < RSD_NODES_MAX / kWave) sh.cmask[wave] = cmask;
    }
    __syncthreads();
    if (match) {
        int rank = __popcll(cmask & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) rank += __popcll(sh.cmask[w]);
        if (rank < RSD_K_MAX) {
            sh.g.kid[rank] = tid;
            sh.g.tok[rank] = cand.token;
            sh.czt[rank] = cand.zt;
            sh.czd[rank] = cand.zd;
        }
    }
    if (tid == 0) {
        int total = 0;
        for (int w = 0; w < RSD_NODES_MAX / kWave; ++w) total += __popcll(sh.cmask[w]);
        sh.g.K = min(total, RSD_K_MAX);
        sh.g.flags = 0;
    }
#pragma unroll
    for (int w = 0; w < NW; ++w) { mt = fmaxf(mt, sh.ms[w].m); md = fmaxf(md, sh.ms[w].s); }
    __syncthreads();
    const int K = sh.g.K;
    if (K == 0) return;
    // bit (4 j + e) set: this thread's entry (j, e) is a child token
    static_assert(CH * 4 <= 128, "element mask holds 128 entries");
    uint64_t elmask[2] = {0, 0};
    for (int i = 0; i < K; ++i) {
        const int x = sh.g.tok[i], c = x >> 2;
        if (c % T == tid) {
            const int bit = ((c / T) << 2) | (x & 3);
            if (bit < 64) elmask[0] |= 1ull << bit; else elmask[1] |= 1ull << (bit - 64);
        }
    }
    // children: lane t < K follows its token's two logits in fp64
    double cu = 0.0, ce = 0.0;
    if (tid < K) {
        cu = (double)sh.czt[tid] * (double)c2;
        ce = (double)sh.czd[tid] * (double)c2;
    }
    const float mt_use = (mt == -INFINITY) ? 0.f : mt, md_use = (md == -INFINITY) ? 0.f : md;
    // exponentials in place; the draft sum leaves out every child token
    float st = 0.f, sd = 0.f;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        float4 d = ed_get(j);
        d.x = __builtin_amdgcn_exp2f(d.x - md_use);
        d.y = __builtin_amdgcn_exp2f(d.y - md_use);
        d.z = __builtin_amdgcn_exp2f(d.z - md_use);
        d.w = __builtin_amdgcn_exp2f(d.w - md_use);
        ed_put(j, d);
#pragma unroll
        for (int e = 0; e < 4; ++e) ut[4 * j + e] = __builtin_amdgcn_exp2f(ut[4 * j + e] - mt_use);
        st += (ut[4 * j] + ut[4 * j + 1]) + (ut[4 * j + 2] + ut[4 * j + 3]);
        const float dv[4] = {d.x, d.y, d.z, d.w};
        float dsum[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            dsum[e] = ((elmask[(4 * j + e) >> 6] >> ((4 * j + e) & 63)) & 1ull) ? 0.f : dv[e];
        sd += (dsum[0] + dsum[1]) + (dsum[2] + dsum[3]);
    }
    st = wave_sum(st);
    sd = wave_sum(sd);
    if (tid < K) {
        cu = exp2(cu - (double)mt_use);
        ce = exp2(ce - (double)md_use);
        sh.ce[tid] = ce;
    }
    if (lane0) {
        sh.red[wave] = (double)st;
        sh.red2[wave] = (double)sd;
    }
    __syncthreads();
    double St = 0.0, Sd = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { St += sh.red[w]; Sd += sh.red2[w]; }
    // draft mass still available at stage k: the rest plus the children not yet removed.  Lane
    // k writes 1 / s_k into the record; the stage loop below works the same number out in every
    // thread (same order of additions), so no barrier stands between the two.
    if (tid < RSD_K_MAX) {
        double s = Sd;
        for (int i = K - 1; i >= tid; --i) s += sh.ce[i];
        const double inv = (tid < K) ? 1.0 / s : 0.0;
        sh.g.inv_s[tid] = (float)inv;
        sh.g.inv_S[tid] = 1.f;
        if (tid == 0) {
            sh.g.mt2 = mt_use;
            sh.g.md2 = md_use;
            sh.g.inv_st = (float)(1.0 / St);
            if (!(St > 0.0) || !isfinite(St) || !(s > 0.0) || !isfinite(s)) sh.g.flags |= RSD_FLAG_NONFINITE;
        }
    }
    double A = St;  // q^(k) = u / A
    for (int k = 0; k < K; ++k) {
        double s_k = Sd;
        for (int i = K - 1; i >= k; --i) s_k += sh.ce[i];
        const double inv_sk = 1.0 / s_k;
        if (tid == k) {  // threshold of child k (Eq. (3))
            const double p = ce * inv_sk;
            sh.g.theta[k] = (p > 0.0) ? (float)fmin(1.0, cu / (A * p)) : 1.f;
        }
        if (k == K - 1) break;
        const float gamma = (float)(inv_sk * A);
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const float4 d = ed_get(j);
            part += fmaxf(fmaf(-gamma, d.x, ut[4 * j + 0]), 0.f);
            part += fmaxf(fmaf(-gamma, d.y, ut[4 * j + 1]), 0.f);
            part += fmaxf(fmaf(-gamma, d.z, ut[4 * j + 2]), 0.f);
            part += fmaxf(fmaf(-gamma, d.w, ut[4 * j + 3]), 0.f);
        }
        part = wave_sum(part);
        double *red = sh.sred[k & 1];
        if (lane0) red[wave] = (double)part;
        __syncthreads();
        double S = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) S += red[w];
        const bool ok = S > 0.0 && isfinite(S);
        if (ok) {
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const float4 d = ed_get(j);
                ut[4 * j + 0] = fmaxf(fmaf(-gamma, d.x, ut[4 * j + 0]), 0.f);
                ut[4 * j + 1] = fmaxf(fmaf(-gamma, d.y, ut[4 * j + 1]), 0.f);
                ut[4 * j + 2] = fmaxf(fmaf(-gamma, d.z, ut[4 * j + 2]), 0.f);
                ut[4 * j + 3] = fmaxf(fmaf(-gamma, d.w, ut[4 * j + 3]), 0.f);
            }
            if (tid < K) cu = fmax(cu - (double)gamma * ce, 0.0);
            if (tid == 0) sh.g.inv_S[k] = (float)(A / S);
            A = S;
        } else if (tid == 0) {  // keep q^(k): no subtraction, no rescale
            sh.g.inv_s[k] = 0.f;
            sh.g.inv_S[k] = 1.f;
            sh.g.flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
        }
        // x_k leaves the draft distribution either way
        if (tid == k) ce = 0.0;
        if ((elmask[0] | elmask[1]) != 0ull) {
            const int xk = sh.g.tok[k], ck = xk >> 2;
            const int target = (ck % T == tid) ? (((ck / T) << 2) | (xk & 3)) : -1;
            if (target >= 0) {
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    if ((target >> 2) == j) {
                        float4 d = ed_get(j);
                        if ((target & 3) == 0) d.x = 0.f;
                        if ((target & 3) == 1) d.y = 0.f;
                        if ((target & 3) == 2) d.z = 0.f;
                        if ((target & 3) == 3) d.w = 0.f;
                        ed_put(j, d);
                    }
                }
            }
        }
    }
    __syncthreads();
}

// CH == 0: streaming variant; else the resident variant with CH chunks per thread, CL of them in LDS
template <int THREADS, int CH, int CL>
__device__ __forceinline__ void verify_group(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    if constexpr (CH > 0)
        process_group_reg<THREADS, CH, CL>(a, b, node, n, sh);
    else
        process_group<THREADS>(a, b, node, n, sh);
}

// ---------------------------------------------------------------------------
// Last-token sampling (Alg. 6, last lines): arg-max over x of log r(x) + G(x)
// for entries [x_lo, x_hi) of one node.  r = q^(K+1) (unnormalised) when the
// node's K children were all rejected, or the target row itself for a leaf.
// Tracks a second arg-max over q^(K) used when the last residual is empty.
// ---------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long pack_key(float v, int idx) {
    uint32_t bits = __float_as_uint(v);
    bits = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return ((unsigned long long)bits << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)idx);
}

// Hardware exp2 / log2 (one instruction each).  The logarithm's operand is scaled out of the
// denormal range first, which the instruction would read as zero.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_ln(float x) {
    const bool tiny = x < 0x1p-100f;
    const float l2 = __builtin_amdgcn_logf(tiny ? x * 0x1p100f : x) - (tiny ? 100.f : 0.f);
    return l2 * kLn2;
}

template <int THREADS>
__device__ void final_sample_range(const RrsArgs &a, int b, int node, const GroupRec &g, int c_lo,
                                   int c_hi, float &best_v, int &best_i, float &alt_v, int &alt_i) {
    const float *zt = a.zt + ((int64_t)b * a.N + node) * a.V;
    const float *zd = a.zd + ((int64_t)b * a.N + node) * a.V;
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const uint32_t seq = a.seq_id ? (uint32_t)a.seq_id[b] : (uint32_t)b;
    const PhiloxKey key = make_key(a.seed);
    const uint32_t c3 = counter_word3(kTagLastGumbel, a.step);
    const int K = g.K;
    best_v = -INFINITY; best_i = INT_MAX; alt_v = -INFINITY; alt_i = INT_MAX;
    if (K == 0) {
        for (int c = c_lo + (int)threadIdx.x; c < c_hi; c += THREADS) {
            const float4 t = zt4[c];
            const uint4 rnd = philox4x32_10((uint32_t)c, (uint32_t)node, seq, c3, key);
            const uint32_t wd[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
            const float tz[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float s = tz[i] * a.inv_t + gumbel_from_word(wd[i]);
                if (better(s, (c << 2) + i, best_v, best_i)) { best_v = s; best_i = (c << 2) + i; }
            }
        }
        return;
    }
    const ChainRegs cr = load_chain(g);
    const float inv_s_last = uniform_f(g.inv_s[K - 1]);
    const uint64_t hits = child_chunk_mask<THREADS>(g, c_lo, c_hi);
    int it = 0;
    for (int c = c_lo + (int)threadIdx.x; c < c_hi; c += THREADS, ++it) {
        const float4 t = zt4[c];
        const float4 d = zd4[c];
        const uint4 rnd = philox4x32_10((uint32_t)c, (uint32_t)node, seq, c3, key);
        const uint32_t wd[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
        const float et[4] = {fast_exp2(fmaf(t.x, a.c2, -cr.mt2)), fast_exp2(fmaf(t.y, a.c2, -cr.mt2)),
                             fast_exp2(fmaf(t.z, a.c2, -cr.mt2)), fast_exp2(fmaf(t.w, a.c2, -cr.mt2))};
        const float ed[4] = {fast_exp2(fmaf(d.x, a.c2, -cr.md2)), fast_exp2(fmaf(d.y, a.c2, -cr.md2)),
                             fast_exp2(fmaf(d.z, a.c2, -cr.md2)), fast_exp2(fmaf(d.w, a.c2, -cr.md2))};
        float q[4], r[4];
        if (!((hits >> it) & 1ull)) {
            chain4(et, ed, cr, K - 1, q);                                      // q^(K)
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = fmaxf(q[i] - ed[i] * inv_s_last, 0.f);  // ~ q^(K+1)
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rs = removal_stage((c << 2) + i, g.tok, K);
                q[i] = chain1_masked(et[i], ed[i], rs, cr, K - 1);
                r[i] = fmaxf(q[i] - ((rs < K - 1) ? 0.f : ed[i] * inv_s_last), 0.f);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float gum = gumbel_from_word(wd[i]);
            const float s = fast_ln(r[i]) + gum;
            const float s2 = fast_ln(q[i]) + gum;
            if (better(s, (c << 2) + i, best_v, best_i)) { best_v = s; best_i = (c << 2) + i; }
            if (better(s2, (c << 2) + i, alt_v, alt_i)) { alt_v = s2; alt_i = (c << 2) + i; }
        }
    }
}

// ---------------------------------------------------------------------------
// ALL_GROUPS, kernel 0 (one workgroup): count the children of every node and list the
// non-leaf nodes, those with the most children first, as work items for kernel 1.
// ---------------------------------------------------------------------------
constexpr int kPlanThreads = 1024;

constexpr int kPlanLds = 8192;  // nodes whose child counts fit the workgroup's LDS

__global__ __launch_bounds__(kPlanThreads) void rrs_plan_kernel(RrsArgs a) {
    __shared__ int hist[RSD_K_MAX + 1];
    __shared__ int offs[RSD_K_MAX + 1];
    __shared__ int s_k[kPlanLds];
    const int tid = threadIdx.x;
    const int total = a.B * a.N;
    // the counts are accumulated in LDS when they fit (LDS atomics instead of global ones)
    const bool in_lds = total <= kPlanLds;
    int *cnt = in_lds ? s_k : a.kcount;
    for (int i = tid; i < total; i += kPlanThreads) cnt[i] = 0;
    if (tid <= RSD_K_MAX) hist[tid] = 0;
    // the last kernel's per-sequence maxima and arrival counters start at zero
    for (int i = tid; i < a.B; i += kPlanThreads) {
        a.fkey[2 * i] = 0ull;
        a.fkey[2 * i + 1] = 0ull;
        a.fdone[i] = 0;
    }
    __syncthreads();
    for (int i = tid; i < total; i += kPlanThreads) {
        const int b = i / a.N, j = i - b * a.N;
        const int n = min(max(a.n_nodes[b], 1), a.N);
        if (j >= 1 && j < n) {
            const int p = a.parent[i];
            if (p >= 0 && p < j) atomicAdd(&cnt[b * a.N + p], 1);
        }
    }
    __syncthreads();
    for (int i = tid; i < total; i += kPlanThreads) {
        const int c = cnt[i];
        if (in_lds) a.kcount[i] = c;
        const int k = min(c, RSD_K_MAX);
        if (k > 0) atomicAdd(&hist[k], 1);
    }
    __syncthreads();
    if (tid == 0) {
        int running = 0;
        for (int k = RSD_K_MAX; k >= 1; --k) {
            offs[k] = running;
            running += hist[k];
        }
        a.wq[0] = running;
    }
    __syncthreads();
    for (int i = tid; i < total; i += kPlanThreads) {
        const int k = min(cnt[i], RSD_K_MAX);
        if (k > 0) {
            const int b = i / a.N;
            a.work[atomicAdd(&offs[k], 1)] = make_int2(i, min(max(a.n_nodes[b], 1), a.N));
        }
    }
}

// ---------------------------------------------------------------------------
// ALL_GROUPS, kernel 1: persistent workgroups go through the work list (largest groups
// first) in rounds of gridDim.x items, forwards in even rounds and backwards in odd ones, so
// that a workgroup that drew a large group in one round draws a small one in the next.  The
// assignment is static: the next item's entry is read while the current group is verified.
// ---------------------------------------------------------------------------
template <int THREADS, int CH, int CL>
__global__ __launch_bounds__(THREADS) void rrs_group_kernel(RrsArgs a) {
    __shared__ GroupShared sh;
    const int count = a.wq[0];
    const int G = gridDim.x, g = blockIdx.x;
    auto item_of_round = [&](int r) { return r * G + ((r & 1) ? G - 1 - g : g); };
    // (every lane reads the same entry through an offset the compiler cannot see is zero: the
    // value then stays in a vector register, and its wait at the first use, one round later)
    int lane_zero = 0;
    asm volatile("" : "+v"(lane_zero));
    int idx = item_of_round(0);
    int2 ent = make_int2(0, 1);
    if (idx < count) ent = a.work[idx + lane_zero];
    for (int r = 0; idx < count; ++r) {
        const int i = __builtin_amdgcn_readfirstlane(ent.x), n = __builtin_amdgcn_readfirstlane(ent.y);
        const int nidx = item_of_round(r + 1);
        // (an entry past the end of the list is never used: any entry will do, and the load
        // stays unconditional)
        int2 nent = a.work[min(nidx, count - 1) + lane_zero];
        const int b = i / a.N, node = i - b * a.N;
        verify_group<THREADS, CH, CL>(a, b, node, n, sh);
        GroupRec *out = a.rec + i;
        const int words = sizeof(GroupRec) / 4;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(&sh.g);
        uint32_t *dst = reinterpret_cast<uint32_t *>(out);
        for (int w = threadIdx.x; w < words; w += THREADS) dst[w] = src[w];
        if (a.theta) {
            // children beyond the supported group size are not verified: mark them
            const int *par = a.parent + (int64_t)b * a.N;
            const int last = sh.g.K > 0 ? sh.g.kid[sh.g.K - 1] : node;
            for (int j = last + 1 + (int)threadIdx.x; j < n; j += THREADS)
                if (par[j] == node) a.theta[(int64_t)b * a.N + j] = NAN;
            if ((int)threadIdx.x < sh.g.K)
                a.theta[(int64_t)b * a.N + sh.g.kid[threadIdx.x]] = sh.g.theta[threadIdx.x];
        }
        __syncthreads();  // sh is reused by the next item
        ent = nent;
        idx = nidx;
    }
}

// The uniform that decides child `node` of sequence b (Alg. 6: U ~ Uniform(0, 1) per tested token).
__device__ __forceinline__ float accept_uniform(const RrsArgs &a, int b, int node) {
    const uint32_t seq = a.seq_id ? (uint32_t)a.seq_id[b] : (uint32_t)b;
    const uint4 r = philox4x32_10(0u, (uint32_t)node, seq, counter_word3(kTagAcceptUniform, a.step),
                                  make_key(a.seed));
    return uniform_from_word(r.x);
}

// The walk of one sequence by one wave (ALL_GROUPS): at every node the wave reads the node's
// verified record with all its lanes at once, lane k draws the uniform of child k, and a ballot
// names the first accepted child -- one memory round trip per level.  Returns the node the walk
// ends at; `g` receives that node's record (K = 0 for a leaf).  With `write` set (one workgroup per
// sequence) the accepted path goes to the outputs.
struct WalkResult {
    int node, nacc;
    uint32_t flags;
};

__device__ __forceinline__ WalkResult walk_tree(const RrsArgs &a, int b, int lane, bool write, GroupRec &g) {
    constexpr int W_K = offsetof(GroupRec, K) / 4, W_FLAGS = offsetof(GroupRec, flags) / 4;
    constexpr int W_KID = offsetof(GroupRec, kid) / 4, W_TOK = offsetof(GroupRec, tok) / 4;
    constexpr int W_INVS = offsetof(GroupRec, inv_s) / 4, W_THETA = offsetof(GroupRec, theta) / 4;
    constexpr int kWords = sizeof(GroupRec) / 4;
    static_assert(kWords <= 2 * kWave && RSD_K_MAX <= kWave, "a record is two words per lane at most");
    // word w of the record sits in lane w % 64, register w / 64
    auto word = [&](uint32_t r0, uint32_t r1, int w) -> uint32_t {
        const uint32_t lo = (uint32_t)__shfl((int)r0, w & (kWave - 1), kWave);
        const uint32_t hi = (uint32_t)__shfl((int)r1, w & (kWave - 1), kWave);
        return w < kWave ? lo : hi;
    };
    int cur = 0, nacc = 0;
    uint32_t flags = 0, r0 = 0, r1 = 0;
    bool leaf = true;
    for (int guard = 0; guard < a.N; ++guard) {
        const int64_t i = (int64_t)b * a.N + cur;
        const int kc = a.kcount[i];
        const uint32_t *src = reinterpret_cast<const uint32_t *>(a.rec + i);
        // (the record of a leaf was never written: what is read is not used)
        r0 = src[lane];
        r1 = (lane + kWave < kWords) ? src[lane + kWave] : 0u;
        leaf = kc == 0;
        if (leaf) break;
        const int K = (int)word(r0, r1, W_K);
        if (K == 0) { leaf = true; break; }
        const uint32_t gflags = word(r0, r1, W_FLAGS);
        flags |= gflags & RSD_FLAG_NONFINITE;
        const int kid = (int)word(r0, r1, W_KID + min(lane, RSD_K_MAX - 1));
        const float theta = __uint_as_float(word(r0, r1, W_THETA + min(lane, RSD_K_MAX - 1)));
        const float inv_s = __uint_as_float(word(r0, r1, W_INVS + min(lane, RSD_K_MAX - 1)));
        const bool ok = lane < K && accept_uniform(a, b, kid) < theta;
        const unsigned long long acc = __ballot(ok);
        const int took = acc ? __ffsll((long long)acc) - 1 : -1;
        // degenerate stages matter only if their residual was used
        if (gflags & RSD_FLAG_DEGENERATE_RESIDUAL) {
            const int used = took < 0 ? K - 1 : took;
            if (__ballot(lane < used && inv_s == 0.f)) flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
        }
        if (took < 0) break;
        const int next = __shfl(kid, took, kWave);
        const int next_tok = (int)word(r0, r1, W_TOK + took);  // (lane exchanges stay outside divergent code)
        if (write && lane == 0 && nacc < a.depth_max) {
            a.accepted_nodes[(int64_t)b * a.depth_max + nacc] = next;
            if (a.accepted_tokens) a.accepted_tokens[(int64_t)b * a.depth_max + nacc] = next_tok;
        }
        ++nacc;
        cur = next;
    }
    uint32_t *dst = reinterpret_cast<uint32_t *>(&g);
    if (leaf) {
        if (lane == 0) g.K = 0;  // sample from the target row itself
    } else {
        dst[lane] = r0;
        if (lane + kWave < kWords) dst[lane + kWave] = r1;
    }
    return WalkResult{cur, nacc, flags};
}

// ALL_GROUPS, kernel 2: the walk and the last token.  The vocabulary of a sequence is split over
// gridDim.x workgroups (more of them for small batches; one per sequence, with no atomics at all,
// once the batch fills the chip); every one of them walks the tree itself (the walk is a few
// dependent reads of records that the previous kernel wrote), workgroup 0 of the sequence writes
// the path.
__global__ __launch_bounds__(kFinalThreads) void rrs_final_kernel(RrsArgs a) {
    __shared__ GroupRec g;
    __shared__ float s_v[2 * kFinalThreads / kWave];
    __shared__ int s_i[2 * kFinalThreads / kWave];
    __shared__ int s_last;
    __shared__ int s_node;
    __shared__ uint32_t s_flags;
    const int b = blockIdx.y;
    const int split = blockIdx.x;
    const int tid = threadIdx.x;
    const bool writer = split == 0;
    const int n = min(max(a.n_nodes[b], 1), a.N);
    if (writer) {
        for (int j = tid; j < a.N; j += kFinalThreads) {
            if (a.uniforms) a.uniforms[(int64_t)b * a.N + j] = (j < n) ? accept_uniform(a, b, j) : 0.f;
            if (a.theta && (j == 0 || j >= n)) a.theta[(int64_t)b * a.N + j] = NAN;
        }
    }
    if (tid < kWave) {
        const WalkResult w = walk_tree(a, b, tid, writer, g);
        if (writer) {
            // slots of the path that the walk did not reach
            for (int j = w.nacc + tid; j < a.depth_max; j += kWave) {
                a.accepted_nodes[(int64_t)b * a.depth_max + j] = -1;
                if (a.accepted_tokens) a.accepted_tokens[(int64_t)b * a.depth_max + j] = -1;
            }
        }
        if (tid == 0) {
            s_node = w.node;
            s_flags = w.flags;
            if (writer) {
                a.n_accepted[b] = w.nacc;
                if (a.final_node) a.final_node[b] = w.node;
            }
        }
    }
    __syncthreads();
    const int node = s_node;
    const int nchunk = a.V >> 2;
    const int nsplit = gridDim.x;
    const int per = (nchunk + nsplit - 1) / nsplit;
    const int c_lo = min(split * per, nchunk), c_hi = min(c_lo + per, nchunk);
    float bv, av;
    int bi, ai;
    final_sample_range<kFinalThreads>(a, b, node, g, c_lo, c_hi, bv, bi, av, ai);
    block_argmax_pair<kFinalThreads>(bv, bi, av, ai, s_v, s_i);
    if (nsplit > 1) {
        if (threadIdx.x == 0) {
            if (bi != INT_MAX) atomicMax(&a.fkey[2 * b], pack_key(bv, bi));
            if (ai != INT_MAX) atomicMax(&a.fkey[2 * b + 1], pack_key(av, ai));
            __threadfence();
            s_last = (atomicAdd(&a.fdone[b], 1) == nsplit - 1);
        }
        __syncthreads();
        if (!s_last) return;
    }
    if (threadIdx.x == 0) {
        unsigned long long k0 = (bi != INT_MAX) ? pack_key(bv, bi) : 0ull;
        unsigned long long k1 = (ai != INT_MAX) ? pack_key(av, ai) : 0ull;
        if (nsplit > 1) {
            __threadfence();
            k0 = atomicMax(&a.fkey[2 * b], 0ull);
            k1 = atomicMax(&a.fkey[2 * b + 1], 0ull);
        }
        uint32_t flags = s_flags;
        const unsigned long long ninf = pack_key(-INFINITY, 0) >> 32;
        unsigned long long use = k0;
        if ((k0 >> 32) <= ninf) {  // empty last residual: fall back to q^(K)
            if (g.K > 0) flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
            use = (g.K > 0) ? k1 : k0;
        }
        a.last_token[b] = (use == 0ull) ? 0 : (int)(0xFFFFFFFFu - (uint32_t)(use & 0xFFFFFFFFull));
        if (a.flags) a.flags[b] = flags;
    }
}

// ---------------------------------------------------------------------------
// PATH mode: one persistent workgroup per sequence verifies only the groups on
// the accepted path, then draws the last token.
// ---------------------------------------------------------------------------
template <int THREADS, int CH, int CL>
__global__ __launch_bounds__(THREADS) void rrs_path_kernel(RrsArgs a) {
    __shared__ GroupShared sh;
    __shared__ float s_v[2 * THREADS / kWave];
    __shared__ int s_i[2 * THREADS / kWave];
    __shared__ int s_nacc;
    __shared__ uint32_t s_flags;
    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int n = min(max(a.n_nodes[b], 1), a.N);
    for (int j = tid; j < a.N; j += THREADS) {
        if (a.uniforms) a.uniforms[(int64_t)b * a.N + j] = (j < n) ? accept_uniform(a, b, j) : 0.f;
        if (a.theta) a.theta[(int64_t)b * a.N + j] = NAN;
    }
    for (int j = tid; j < a.depth_max; j += THREADS) {
        a.accepted_nodes[(int64_t)b * a.depth_max + j] = -1;
        if (a.accepted_tokens) a.accepted_tokens[(int64_t)b * a.depth_max + j] = -1;
    }
    if (tid == 0) {
        sh.cur = 0;
        sh.done = 0;
        s_nacc = 0;
        s_flags = 0;
    }
    __syncthreads();
    for (int guard = 0; guard < a.N; ++guard) {
        const int cur = sh.cur;
        verify_group<THREADS, CH, CL>(a, b, cur, n, sh);
        const int K = sh.g.K;
        if (K == 0) break;
        if (tid == 0) {
            uint32_t flags = s_flags | (sh.g.flags & RSD_FLAG_NONFINITE);
            int took = -1;
            for (int k = 0; k < K; ++k) {
                if (a.theta) a.theta[(int64_t)b * a.N + sh.g.kid[k]] = sh.g.theta[k];
                if (accept_uniform(a, b, sh.g.kid[k]) < sh.g.theta[k]) {
                    took = k;
                    break;
                }
            }
            if (sh.g.flags & RSD_FLAG_DEGENERATE_RESIDUAL) {
                const int used = took < 0 ? K - 1 : took;
                for (int j = 0; j < used; ++j)
                    if (sh.g.inv_s[j] == 0.f) flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
            }
            s_flags = flags;
            if (took >= 0) {
                const int nacc = s_nacc;
                if (nacc < a.depth_max) {
                    a.accepted_nodes[(int64_t)b * a.depth_max + nacc] = sh.g.kid[took];
                    if (a.accepted_tokens)
                        a.accepted_tokens[(int64_t)b * a.depth_max + nacc] = sh.g.tok[took];
                }
                s_nacc = nacc + 1;
                sh.cur = sh.g.kid[took];
            } else {
                sh.done = 1;
            }
        }
        __syncthreads();
        if (sh.done) break;
    }
    // last token at sh.cur with record sh.g (K = 0 for a leaf)
    const int node = sh.cur;
    float bv, av;
    int bi, ai;
    final_sample_range<THREADS>(a, b, node, sh.g, 0, a.V >> 2, bv, bi, av, ai);
    block_argmax_pair<THREADS>(bv, bi, av, ai, s_v, s_i);
    if (tid == 0) {
        uint32_t flags = s_flags;
        int tokn = bi;
        if (!(bv > -INFINITY)) {
            if (sh.g.K > 0) {
                flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
                tokn = ai;
            }
        }
        if (tokn == INT_MAX) tokn = 0;
        a.last_token[b] = tokn;
        a.n_accepted[b] = s_nacc;
        if (a.final_node) a.final_node[b] = node;
        if (a.flags) a.flags[b] = flags;
    }
}

static size_t align_up(size_t x, size_t al) { return (x + al - 1) / al * al; }
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace rsd

using namespace rsd;

extern "C" size_t rsd_recursive_reject_workspace_bytes(int32_t B, int32_t N_max, int32_t) {
    if (B <= 0 || N_max <= 0) return 0;
    return align_up((size_t)B * N_max * sizeof(GroupRec), 256) + align_up((size_t)B * 16, 256) +
           align_up((size_t)B * 4, 256) + 3 * align_up((size_t)B * N_max * 4, 256) + 256;
}

extern "C" int32_t rsd_recursive_reject(const float *draft_logits, const float *target_logits,
                                        int32_t B, int32_t N_max, int32_t V, float inv_temperature,
                                        const int32_t *tokens, const int32_t *parent,
                                        const int32_t *n_nodes, const int32_t *seq_id, int32_t mode,
                                        uint64_t seed, uint32_t step, int32_t *accepted_nodes,
                                        int32_t *accepted_tokens, int32_t depth_max,
                                        int32_t *n_accepted, int32_t *last_token, int32_t *final_node,
                                        float *theta, float *uniforms, uint32_t *flags,
                                        void *workspace, size_t workspace_bytes, void *stream) {
    if (!draft_logits || !target_logits || !tokens || !parent || !n_nodes || !accepted_nodes ||
        !n_accepted || !last_token)
        return RSD_ERR_NULL;
    if (B < 0 || N_max < 1 || N_max > RSD_NODES_MAX || V < 4 || (V & 3) || V > 131072 || depth_max < 1 ||
        !(inv_temperature > 0.f) || !aligned16(draft_logits) || !aligned16(target_logits))
        return RSD_ERR_SHAPE;
    if (mode != RSD_MODE_PATH && mode != RSD_MODE_ALL_GROUPS) return RSD_ERR_UNSUPPORTED;
    if (B == 0) return RSD_OK;
    const size_t need = rsd_recursive_reject_workspace_bytes(B, N_max, V);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return RSD_ERR_WORKSPACE;
    char *ws = static_cast<char *>(workspace);
    RrsArgs a{};
    a.zd = draft_logits; a.zt = target_logits; a.B = B; a.N = N_max; a.V = V;
    a.inv_t = inv_temperature;
    a.c2 = (float)((double)inv_temperature * 1.4426950408889634);
    a.tokens = tokens; a.parent = parent; a.n_nodes = n_nodes; a.seq_id = seq_id;
    a.seed = seed; a.step = step; a.accepted_nodes = accepted_nodes;
    a.accepted_tokens = accepted_tokens; a.depth_max = depth_max; a.n_accepted = n_accepted;
    a.last_token = last_token; a.final_node = final_node; a.theta = theta; a.uniforms = uniforms;
    a.flags = flags;
    size_t off = 0;
    a.rec = reinterpret_cast<GroupRec *>(ws + off); off += align_up((size_t)B * N_max * sizeof(GroupRec), 256);
    a.fkey = reinterpret_cast<unsigned long long *>(ws + off); off += align_up((size_t)B * 16, 256);
    a.fdone = reinterpret_cast<int *>(ws + off); off += align_up((size_t)B * 4, 256);
    a.kcount = reinterpret_cast<int *>(ws + off); off += align_up((size_t)B * N_max * 4, 256);
    a.work = reinterpret_cast<int2 *>(ws + off); off += 2 * align_up((size_t)B * N_max * 4, 256);
    a.wq = reinterpret_cast<int *>(ws + off);
    hipStream_t st = (hipStream_t)stream;
    // Rows of up to 32768 entries fit the register-resident variant (128 data registers per
    // thread); up to 52224 entries (the 50k vocabularies) the variant that keeps most of the
    // draft row in LDS; beyond that the rows are streamed from memory at every stage.
    const bool reg16 = V <= kRegThreads * 4 * 16;
    const bool lds13 = !reg16 && V <= kLdsThreads * 4 * kLdsChunks;
    if (mode == RSD_MODE_PATH) {
        if (reg16)
            hipLaunchKernelGGL((rrs_path_kernel<kRegThreads, 16, 0>), dim3(B), dim3(kRegThreads), 0, st, a);
        else if (lds13)
            hipLaunchKernelGGL((rrs_path_kernel<kLdsThreads, kLdsChunks, kLdsChunksInLds>), dim3(B),
                               dim3(kLdsThreads), 0, st, a);
        else
            hipLaunchKernelGGL((rrs_path_kernel<kGroupThreads, 0, 0>), dim3(B), dim3(kGroupThreads), 0, st, a);
    } else {
        static int n_cu = 0;
        if (n_cu == 0) {
            int dev = 0, cus = 0;
            if (hipGetDevice(&dev) != hipSuccess ||
                hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
                cus = 256;
            n_cu = cus;
        }
        const long items_max = (long)B * N_max;
        const int grid = (int)(items_max < n_cu ? items_max : n_cu);
        hipLaunchKernelGGL(rrs_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, a);
        if (reg16)
            hipLaunchKernelGGL((rrs_group_kernel<kRegThreads, 16, 0>), dim3(grid), dim3(kRegThreads), 0, st, a);
        else if (lds13)
            hipLaunchKernelGGL((rrs_group_kernel<kLdsThreads, kLdsChunks, kLdsChunksInLds>), dim3(grid),
                               dim3(kLdsThreads), 0, st, a);
        else
            hipLaunchKernelGGL((rrs_group_kernel<kGroupThreads, 0, 0>), dim3(2 * grid), dim3(kGroupThreads), 0, st, a);
        // enough workgroups to fill the chip, but no more: every split costs two device-wide fences
        int fsplits = 256 / (B > 0 ? B : 1);
        fsplits = fsplits < 1 ? 1 : (fsplits > kFinalSplitsMax ? kFinalSplitsMax : fsplits);
        hipLaunchKernelGGL(rrs_final_kernel, dim3(fsplits, B), dim3(kFinalThreads), 0, st, a);
    }
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}
