// Recursive rejection sampling over the draft tree (Sec. 3.1; Sec. 3.2.2; Alg. 6).
//
// A sibling group (the children x_1..x_K of one node) is verified by one
// workgroup.  The residual distributions q^(k) of Eq. (2) are never stored: with
//   e_t(x) = 2^(zt(x) c - m_t),  e_d(x) = 2^(zd(x) c - m_d),  c = log2(e) / T,
// the kernels carry u(x) = q^(k)(x) A_k, starting from u = e_t, A_1 = sum_x e_t(x), and a stage is
//   gamma_k = A_k / s_k,          s_k = sum of e_d over the tokens not yet removed,
//   u <- max(u - gamma_k e_d, 0), A_{k+1} = S_k = sum_x u(x),   then e_d(x_k) <- 0,
// so that Theta_k = (u(x_k) / A_k) / (e_d(x_k) / s_k) (Eq. (3)).  Only the gamma_k go to memory;
// the last-token pass re-evaluates the chain from them.
//
// Precision.  A stage whose residual mass S_k is a small fraction of A_k cancels the leading
// digits of u - gamma e_d at the probable tokens, so what Theta of the later siblings sees is the
// absolute error of the big entries divided by that fraction.  Three measures keep it near 1e-7:
//  * exponents are z c - m formed by fused multiply-adds with c split into two floats, rounded
//    once at the size of the result (a probable token has a result near zero);
//  * the child tokens and every entry within 2^-4 of its row's maximum are followed in fp64
//    (exponentials from the raw logits), by one lane each, and are zero in the fp32 arrays;
//  * gamma is applied as a pair of floats once the residual mass has shrunk below 1/16.
// Sums are accumulated per lane in fp32 (entries below 2^-4 only), across lanes in a fixed order
// and across waves in fp64, so results do not depend on scheduling.
//
// ALL_GROUPS runs three kernels (plan, groups, walk + last token), PATH one persistent
// workgroup per sequence.
//
// Memory.  A row pair (2 V floats) fills half a CU's vector registers, so one group is resident per
// CU, and the CU's vector memory path needs 4096 cycles for it (64 B/clk), about a sixth of what a
// group takes.  The group kernel of ALL_GROUPS therefore fetches the next item's rows while it
// works on the current one, into whatever is free: the target row memory-to-LDS, spread over the
// exponent and exponential passes; half of the draft row into registers the passes leave free,
// spread over the exponential pass; the rest of the draft row into the registers of the current
// rows right after their last use.  The variant that keeps draft chunks in LDS has no room to
// stage and only does the last of the three.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>
#include <stddef.h>

#include <type_traits>

#include "../../include/rsd.h"
#include "rsd_device.hpp"

namespace rsd {

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;

constexpr int kStreamThreads = 512;  // streaming variant (any vocabulary size)
// Resident variants <threads, float4 chunks per thread, of which in LDS>:
//  up to 8192 entries:   256 threads, 8 chunks in registers (small vocabularies)
//  up to 32768 entries:  512 threads, both rows in registers (2 x 64 per thread)
//  up to 51200 entries:  512 threads, 18 of the 25 draft chunks in LDS (144 KB)
constexpr int kSmallThreads = 256, kSmallChunks = 8;
constexpr int kRegThreads = 512, kRegChunks = 16, kRegChunksInLds = 0;
constexpr int kLdsThreads = 512, kLdsChunks = 25, kLdsChunksInLds = 18;
constexpr int kGroupWavesMax = 16;
constexpr int kFinalThreads = 512;
constexpr int kFinalSplitsMax = 8;
constexpr float kHeavy = 4.f;   // entries with exponent >= -kHeavy are followed in fp64
constexpr int kCandCap = 48;    // such entries per wave: lanes 16..63 (lanes 0..15 of wave 0: the children)

// Per (sequence, node) record produced by the group pass, kept in workspace.
struct GroupRec {
    float mt2;      // exponent offset of the target row (about its maximum, log2 domain)
    float md2;      // the same for the draft row
    int K;          // number of verified children (<= RSD_K_MAX); 0 for a leaf
    uint32_t flags;
    int kid[RSD_K_MAX];      // child node ids in stored order
    int tok[RSD_K_MAX];      // their tokens
    float theta[RSD_K_MAX];
    double gam[RSD_K_MAX];   // gamma_k of stage k (0 marks a skipped stage: q^(k+1) = q^(k))
};
static_assert(offsetof(GroupRec, gam) % 8 == 0, "");

struct RrsArgs {
    const float *zd;
    const float *zt;
    int B, N, V;
    float inv_t;   // 1/T
    float c2h;     // c = log2(e)/T as a pair of floats: c2h < c <= c2h + c2l, c2l > 0
    float c2l;
    double c2e;    // c in fp64
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
    int *wq;                    // [0] number of work items, [1] next item to hand out
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

// The stage scalars of a group pulled into (scalar) registers once per pass so that the
// per-entry chain indexes them statically: gamma_j as a pair of floats.
struct ChainRegs {
    float mt2, md2;
    float gh[RSD_K_MAX];
    float gl[RSD_K_MAX];
};

__device__ __forceinline__ ChainRegs load_chain(const GroupRec &g) {
    ChainRegs r;
    r.mt2 = uniform_f(g.mt2);
    r.md2 = uniform_f(g.md2);
#pragma unroll
    for (int j = 0; j < RSD_K_MAX; ++j) {
        const double gam = g.gam[j];
        const float hi = (float)gam;
        r.gh[j] = uniform_f(hi);
        r.gl[j] = uniform_f((float)(gam - (double)hi));
    }
    return r;
}

// u after the first nst stages for four entries none of which is followed in fp64.
__device__ __forceinline__ void chain4(float u[4], const float ed[4], const ChainRegs &r, int nst) {
#pragma unroll
    for (int j = 0; j < RSD_K_MAX - 1; ++j) {
        if (j < nst) {  // wave-uniform; keeps the scalar arrays statically indexed
#pragma unroll
            for (int i = 0; i < 4; ++i) u[i] = fmaxf(fmaf(-r.gl[j], ed[i], fmaf(-r.gh[j], ed[i], u[i])), 0.f);
        }
    }
}

// The same chain in fp64 from the raw logits, for an entry that the draft distribution loses
// after stage rs (rs = K: never).  Returns u after nst stages.
__device__ __forceinline__ double chain1_f64(double U, double E, int rs, const GroupRec &g, int nst) {
    for (int j = 0; j < nst; ++j) U = fmax(U - g.gam[j] * (j <= rs ? E : 0.0), 0.0);
    return U;
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
    float czt[RSD_K_MAX];   // raw target / draft logits of the child tokens
    float czd[RSD_K_MAX];
    double ce[RSD_K_MAX];   // draft exponentials of the child tokens (fp64)
    double th[RSD_K_MAX][4];  // per child: u, A, s, e_d at its own stage
    double sred[2][kGroupWavesMax];  // stage sums, alternating
    unsigned long long cmask[RSD_NODES_MAX / kWave];  // per-wave ballots of the child scan
    int cur;
    int done;
    int next_idx;   // work queue: the item this workgroup takes next
    int2 next_ent;
};

// Children of `node` in stored order: thread j < RSD_NODES_MAX tests node j, wave ballots give
// every match its rank.  The halves can be called apart: fetch_candidate only issues this
// thread's loads (its parent and token), fetch_child_logits the two logits of its token when it
// is a child (sh.czt / sh.czd then hold them by rank).
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

// Publishes the ranks of the matching candidates (kid, tok, czt, czd by rank) and K.  Every
// thread of the workgroup calls it; two barriers.
__device__ __forceinline__ void rank_children(int node, const ChildCandidate &cand, GroupShared &sh, int j) {
    const int lane = j & (kWave - 1), wave = j / kWave;
    const bool match = cand.parent == node;
    const unsigned long long mask = __ballot(match);
    if (wave < RSD_NODES_MAX / kWave && lane == 0) sh.cmask[wave] = mask;
    __syncthreads();
    if (match) {
        int rank = __popcll(mask & ((1ull << lane) - 1ull));
        for (int w = 0; w < wave; ++w) rank += __popcll(sh.cmask[w]);
        if (rank < RSD_K_MAX) {
            sh.g.kid[rank] = j;
            sh.g.tok[rank] = cand.token;
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

// ---------------------------------------------------------------------------
// Streaming variant (vocabularies that no resident variant holds): the rows are read from
// memory at every stage and the chain is re-evaluated per entry from the gammas found so far.
// Only the child tokens are followed in fp64 here.
// ---------------------------------------------------------------------------
template <int THREADS>
__device__ void process_group_stream(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    constexpr int NW = THREADS / kWave;
    static_assert(THREADS >= RSD_NODES_MAX && NW <= kGroupWavesMax, "");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const float *zt = a.zt + ((int64_t)b * a.N + node) * a.V;
    const float *zd = a.zd + ((int64_t)b * a.N + node) * a.V;
    ChildCandidate cand = fetch_candidate(a, b, node, n, tid);
    fetch_child_logits(zt, zd, a.V, node, cand);
    rank_children(node, cand, sh, tid);
    const int K = sh.g.K;
    if (K == 0) return;
    const int nchunk = a.V >> 2;
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const float c2h = a.c2h, c2l = a.c2l;
    // pass A: row maxima of the raw logits
    float mt = -INFINITY, md = -INFINITY;
    for (int c = tid; c < nchunk; c += THREADS) {
        const float4 t = zt4[c], d = zd4[c];
        mt = fmaxf(mt, fmaxf(fmaxf(t.x, t.y), fmaxf(t.z, t.w)));
        md = fmaxf(md, fmaxf(fmaxf(d.x, d.y), fmaxf(d.z, d.w)));
    }
    mt = wave_max(mt);
    md = wave_max(md);
    if (lane == 0) sh.ms[wave] = MaxSum{mt, md};
    __syncthreads();
#pragma unroll
    for (int w = 0; w < NW; ++w) { mt = fmaxf(mt, sh.ms[w].m); md = fmaxf(md, sh.ms[w].s); }
    const float m_t = (mt == -INFINITY) ? 0.f : mt * c2h, m_d = (md == -INFINITY) ? 0.f : md * c2h;
    const uint64_t hits = child_chunk_mask<THREADS>(sh.g, 0, nchunk);
    // children: lane k < K of wave 0 follows child k in fp64
    double tU = 0.0, tE = 0.0;
    if (tid < K) {
        tU = exp2((double)sh.czt[tid] * a.c2e - (double)m_t);
        tE = exp2((double)sh.czd[tid] * a.c2e - (double)m_d);
        sh.ce[tid] = tE;
    }
    // pass B: sums without the child tokens
    float st = 0.f, sd = 0.f;
    {
        int it = 0;
        for (int c = tid; c < nchunk; c += THREADS, ++it) {
            const float4 t = zt4[c], d = zd4[c];
            const float tz[4] = {t.x, t.y, t.z, t.w}, dz[4] = {d.x, d.y, d.z, d.w};
            const bool hit = (hits >> it) & 1ull;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool child = hit && removal_stage((c << 2) + i, sh.g.tok, K) < K;
                st += child ? 0.f : __builtin_amdgcn_exp2f(exponent_of(tz[i], c2h, c2l, -m_t));
                sd += child ? 0.f : __builtin_amdgcn_exp2f(exponent_of(dz[i], c2h, c2l, -m_d));
            }
        }
    }
    st = wave_sum(st);
    sd = wave_sum(sd);
    double su = (double)st;
    if (wave == 0) su += wave_sum_f64(tU);
    if (lane == 0) {
        sh.red[wave] = su;
        sh.red2[wave] = (double)sd;
    }
    __syncthreads();
    double St = 0.0, Sd = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { St += sh.red[w]; Sd += sh.red2[w]; }
    if (tid == 0) {
        sh.g.mt2 = m_t;
        sh.g.md2 = m_d;
        double s0 = Sd;
        for (int i = 0; i < K; ++i) s0 += sh.ce[i];
        if (!(St > 0.0) || !isfinite(St) || !(s0 > 0.0) || !isfinite(s0)) sh.g.flags |= RSD_FLAG_NONFINITE;
    }
    for (int i = tid; i < RSD_K_MAX; i += THREADS) sh.g.gam[i] = 0.0;
    __syncthreads();
    double A = St;
    for (int k = 0; k < K; ++k) {
        double s_k = Sd;
        for (int i = K - 1; i >= k; --i) s_k += sh.ce[i];
        const double gam = A / s_k;
        if (tid == k) {  // threshold of child k (Eq. (3))
            const double p = tE / s_k;
            sh.g.theta[k] = (p > 0.0) ? (float)fmin(1.0, tU / (A * p)) : 1.f;
        }
        if (k == K - 1) {
            if (tid == 0) sh.g.gam[k] = gam;
            break;
        }
        const ChainRegs cr = load_chain(sh.g);
        const float gh = uniform_f((float)gam), gl = uniform_f((float)(gam - (double)(float)gam));
        float part = 0.f;
        int it = 0;
        for (int c = tid; c < nchunk; c += THREADS, ++it) {
            const float4 t = zt4[c], d = zd4[c];
            const float tz[4] = {t.x, t.y, t.z, t.w}, dz[4] = {d.x, d.y, d.z, d.w};
            float u[4], e[4];
            const bool hit = (hits >> it) & 1ull;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const bool child = hit && removal_stage((c << 2) + i, sh.g.tok, K) < K;
                u[i] = child ? 0.f : __builtin_amdgcn_exp2f(exponent_of(tz[i], c2h, c2l, -m_t));
                e[i] = child ? 0.f : __builtin_amdgcn_exp2f(exponent_of(dz[i], c2h, c2l, -m_d));
            }
            chain4(u, e, cr, k);
#pragma unroll
            for (int i = 0; i < 4; ++i) part += fmaxf(fmaf(-gl, e[i], fmaf(-gh, e[i], u[i])), 0.f);
        }
        const double cnew = fmax(tU - gam * tE, 0.0);
        part = wave_sum(part);
        double wsum = (double)part;
        if (wave == 0) wsum += wave_sum_f64(tid < K ? cnew : 0.0);
        double *red = sh.sred[k & 1];
        if (lane == 0) red[wave] = wsum;
        __syncthreads();
        double S = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) S += red[w];
        if (S > 0.0 && isfinite(S)) {
            tU = cnew;
            if (tid == 0) sh.g.gam[k] = gam;
            A = S;
        } else if (tid == 0) {  // keep q^(k): no subtraction
            sh.g.gam[k] = 0.0;
            sh.g.flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
        }
        if (tid == k) tE = 0.0;  // x_k leaves the draft distribution either way
        __syncthreads();         // gam[k] is read by the next stage's chain
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------
// Resident variant for vocabularies up to T * 4 * CH entries: both logit rows are read from
// memory once; each thread keeps its share of u(x) in registers and its share of e_d(x) in
// registers (chunks CL..CH-1) and in LDS (chunks 0..CL-1, a slot of its own per thread and
// chunk, so no barrier guards them).  Lane k < K of wave 0 follows child token k in fp64; lanes
// 16..63 of every wave follow the heavy entries that the wave met (see the file header).  A
// stage is three to four ALU operations per entry, one wave reduction and a single barrier.
// ---------------------------------------------------------------------------
// Issues the loads of one group's row pair and nothing else: the target row into ut, the draft
// row into edr (chunks CL..CH-1) and, for CL > 0, straight from memory into this thread's LDS
// slots (chunks 0..CL-1; no registers, raw logits; 64 lanes x 16 bytes land contiguously,
// which is the slot layout).  Every load is unconditional (a chunk past the end of the row
// reads the row's last chunk instead and gets the exponent -inf), so that the loads form one
// straight line and a wait can name exactly the loads it needs.
// `chunk_mask` is -1, or 0 to make every load read the row's first chunk (a request nobody uses:
// the loads stay unconditional and cost no traffic).
// TARGET false: the draft row only (the target row comes another way).  Draft chunks below P
// go to pf, the registers they are prefetched into in steady state; P_DONE: they are there already.
template <int T, int CH, int CL, bool TARGET = true, int P = 0, bool P_DONE = false>
__device__ __forceinline__ void issue_row_loads(const float *zt, const float *zd, int V, int tid,
                                                float (&ut)[CH * 4], float (&edr)[(CH - CL) * 4],
                                                float4 *s_ed, int chunk_mask, float (&pf)[(P > 0 ? P : 1) * 4]) {
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const int last = (V >> 2) - 1;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = min(j * T + tid, last) & chunk_mask;
        if constexpr (TARGET) {
            const float4 t = load_stream(zt4 + c);
            ut[4 * j + 0] = t.x; ut[4 * j + 1] = t.y; ut[4 * j + 2] = t.z; ut[4 * j + 3] = t.w;
        }
        if (j >= CL && j < P) {
            if constexpr (!P_DONE) {
                const float4 d = load_stream(zd4 + c);
                pf[4 * j] = d.x; pf[4 * j + 1] = d.y; pf[4 * j + 2] = d.z; pf[4 * j + 3] = d.w;
            }
        } else if (j >= CL) {
            const float4 d = load_stream(zd4 + c);
            const int r = 4 * (j - CL);
            edr[r] = d.x; edr[r + 1] = d.y; edr[r + 2] = d.z; edr[r + 3] = d.w;
        }
    }
    if constexpr (CL > 0) {
        const int wave = tid / kWave;
#pragma unroll
        for (int j = 0; j < CL; ++j)
            __builtin_amdgcn_global_load_lds((global_void *)(zd4 + (min(j * T + tid, last) & chunk_mask)),
                                             (lds_void *)(s_ed + j * T + wave * kWave), 16, 0, kStreamPolicy);
    }
}

// What the ALL_GROUPS work loop hands through a group: in, thread 0's next queue index and that
// item's entry; out, the next item as every thread knows it, its children lookup and -- in ut,
// edr and the LDS slots -- its rows, requested as soon as the current group has read its own
// for the last time.
struct NextGroup {
    int idx;      // in (thread 0): queue index of the next item; out: the same for every thread
    int2 ent;     // in (thread 0): that item's work entry {group, tree size}
    int claim;    // in/out (thread 0): the queue index asked for at the start of this group; it is
                  // waited for before the next rows are requested, not behind them
    bool has;     // out: there is a next item
    int b, node, n;
    ChildCandidate cand;
};

// The next group's target row is staged in LDS while the current group is worked on, when LDS has
// the room (no draft chunks there): one memory-to-LDS load per chunk, spread over the exponent
// pass and the exponential pass, so that the CU's vector memory path (64 B/clk: a row pair takes
// it 4096 cycles) is busy under arithmetic instead of in front of it.
template <int CL, bool PIPE>
constexpr bool stages_next_row() { return PIPE && CL == 0; }

// Workgroup barrier for threads that talk through LDS only.  __syncthreads() also waits for
// every memory-to-LDS load in flight, which would end the staging at the first barrier.
template <bool LDS_ONLY>
__device__ __forceinline__ void group_barrier() {
    if constexpr (LDS_ONLY)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    else
        __syncthreads();
}

// ... and P chunks of its draft row are prefetched into registers that the passes leave free, one
// load per chunk of the exponential pass.
template <int T, int CH, int CL, bool PIPE>
constexpr int prefetched_draft_chunks() { return !stages_next_row<CL, PIPE>() ? 0 : (T == 512 && CH == 16) ? 8 : CH / 2; }

template <int T, int CH, int CL, bool PIPE>
__device__ __forceinline__ void compute_group_res(const RrsArgs &a, int node, ChildCandidate cand,
                                                  float (&ut)[CH * 4], float (&edr)[(CH - CL) * 4],
                                                  float (&pf)[(prefetched_draft_chunks<T, CH, CL, PIPE>() > 0 ? prefetched_draft_chunks<T, CH, CL, PIPE>() : 1) * 4],
                                                  float4 *s_ed, float4 *s_nt, GroupShared &sh, NextGroup &nx, int count) {
    constexpr bool STAGE = stages_next_row<CL, PIPE>();
    constexpr int P = prefetched_draft_chunks<T, CH, CL, PIPE>();
    constexpr int NW = T / kWave;
    static_assert(NW <= kGroupWavesMax && CL >= 0 && CL < CH && T >= RSD_NODES_MAX, "");
    static_assert(CH * 4 <= 128, "the child mask holds 128 entries");
    // heavy entries met by each wave: their two raw logits (three scalar arrays rather than one
    // of records: a record would need its fields in consecutive registers when it is stored)
    __shared__ float s_trk_zt[NW * kCandCap];
    __shared__ float s_trk_zd[NW * kCandCap];
    // (a copy of the thread index that the compiler takes for a new value in every call: what
    // derives from it -- chunk addresses, LDS slots, lane masks -- is then worked out here, next
    // to its use, instead of being kept in registers from one group to the next)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int wave = tid / kWave;
    const int lane = tid & (kWave - 1);
    const bool lane0 = lane == 0;
    const int nchunk = a.V >> 2;
    const float c2h = a.c2h, c2l = a.c2l;
    const int last = nchunk - 1;  // the caller checks V >= 4
    // chunk j of e_d, wherever it lives (j is a constant once the loops are unrolled)
    auto ed_get = [&](int j) -> float4 {
        if (j < CL) return s_ed[j * T + tid];
        const int r = j < CL ? 0 : 4 * (j - CL);
        return make_float4(edr[r], edr[r + 1], edr[r + 2], edr[r + 3]);
    };
    // chunk j of the raw draft row as the group finds it (the prefetched chunks are still in pf)
    auto ed_raw = [&](int j) -> float4 {
        if (j < P) return make_float4(pf[4 * j], pf[4 * j + 1], pf[4 * j + 2], pf[4 * j + 3]);
        return ed_get(j);
    };
    auto ed_put = [&](int j, float4 v) {
        if (j < CL) {
            s_ed[j * T + tid] = v;
        } else {
            const int r = j < CL ? 0 : 4 * (j - CL);
            edr[r] = v.x; edr[r + 1] = v.y; edr[r + 2] = v.z; edr[r + 3] = v.w;
        }
    };
    // Row maxima of the raw logits (a chunk past the end repeats real entries of the row, so it
    // needs no mask here) and the children's ranks share their barriers.
    if constexpr (CL > 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float mt = -INFINITY, md = -INFINITY;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        mt = fmaxf(mt, fmaxf(fmaxf(ut[4 * j], ut[4 * j + 1]), fmaxf(ut[4 * j + 2], ut[4 * j + 3])));
        const float4 d = ed_raw(j);
        md = fmaxf(md, fmaxf(fmaxf(d.x, d.y), fmaxf(d.z, d.w)));
        if (j % 3 == 2) __builtin_amdgcn_sched_barrier(0);  // (bounds how far ahead chunks are read)
    }
    mt = wave_max(mt);
    md = wave_max(md);
    const bool match = cand.parent == node;
    const unsigned long long cmask = __ballot(match);
    if (lane0) {
        sh.ms[wave] = MaxSum{mt, md};
        if (wave < RSD_NODES_MAX / kWave) sh.cmask[wave] = cmask;
    }
    if constexpr (PIPE) {
        if (tid == 0) {
            sh.next_idx = nx.idx;
            sh.next_ent = nx.ent;
        }
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
    if constexpr (PIPE) {
        nx.idx = sh.next_idx;
        nx.has = nx.idx < count;
        const int gi = sh.next_ent.x;
        nx.n = sh.next_ent.y;
        nx.b = gi / a.N;
        nx.node = gi - nx.b * a.N;
    }
    // (without a next item the entry names the current group, and the requests all go to the first
    // chunk of its rows)
    const int nmask = (PIPE && nx.has) ? -1 : 0;
    const float4 *nzt4 = reinterpret_cast<const float4 *>(a.zt + ((int64_t)nx.b * a.N + nx.node) * a.V);
    const float4 *nzd4 = reinterpret_cast<const float4 *>(a.zd + ((int64_t)nx.b * a.N + nx.node) * a.V);
    // its children's lookup is asked for now and used at the end of this group (their own logits)
    if constexpr (PIPE) nx.cand = fetch_candidate(a, nx.b, nx.node, nx.n, tid);
    // (No group of the work list is empty.  If one were, the passes below would run on it to no
    // effect -- no child lane, no stage, no threshold -- and the next item's rows are still asked for.)
    if constexpr (!PIPE) {
        if (K == 0) return;
    }
    // bit (4 j + e) set: this thread's entry (j, e) is a child token
    uint64_t elmask[2] = {0, 0};
    for (int i = 0; i < K; ++i) {
        const int x = sh.g.tok[i], c = x >> 2;
        if (c % T == tid) {
            const int bit = ((c / T) << 2) | (x & 3);
            if (bit < 64) elmask[0] |= 1ull << bit; else elmask[1] |= 1ull << (bit - 64);
        }
    }
    const float m_t = (mt == -INFINITY) ? 0.f : mt * c2h, m_d = (md == -INFINITY) ? 0.f : md * c2h;
    // Exponents in place first.  Child tokens and heavy entries leave the fp32 arrays (exponent
    // -inf); the heavy ones go to this wave's list with their raw logits.
    int ncand = 0;  // (wave-uniform)
    // chunk c of the next item's target row, memory to LDS (this thread's slot)
    auto stage_chunk = [&](int c) {
        __builtin_amdgcn_global_load_lds((global_void *)(nzt4 + (min(c * T + tid, last) & nmask)),
                                         (lds_void *)(s_nt + c * T + wave * kWave), 16, 0, kStreamPolicy);
    };
    // (chunk numbers are worked out again here rather than kept from the load loop)
    int tid_x = tid;
    asm volatile("" : "+v"(tid_x));
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        if constexpr (STAGE) {
            if (j < CH / 2) stage_chunk(j);
        }
        const bool inrow = j * T + tid_x <= last;
        const float bt = inrow ? -m_t : -INFINITY, bd = inrow ? -m_d : -INFINITY;
        const float4 dr = ed_raw(j);
        const float tz[4] = {ut[4 * j], ut[4 * j + 1], ut[4 * j + 2], ut[4 * j + 3]};
        const float dz[4] = {dr.x, dr.y, dr.z, dr.w};
        float at[4], ad[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            at[e] = exponent_of(tz[e], c2h, c2l, bt);
            ad[e] = exponent_of(dz[e], c2h, c2l, bd);
        }
        const float amax = fmaxf(fmaxf(fmaxf(at[0], at[1]), fmaxf(at[2], at[3])),
                                 fmaxf(fmaxf(ad[0], ad[1]), fmaxf(ad[2], ad[3])));
        const uint32_t cbits = (uint32_t)(elmask[(4 * j) >> 6] >> ((4 * j) & 63)) & 0xFu;
        if (__ballot(amax >= -kHeavy || cbits != 0u) != 0ull) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool child = (cbits >> e) & 1u;
                const bool push = !child && (at[e] >= -kHeavy || ad[e] >= -kHeavy);
                const unsigned long long bal = __ballot(push);
                bool drop = child;
                if (bal != 0ull) {
                    const int slot = ncand + __popcll(bal & ((1ull << lane) - 1ull));
                    if (push && slot < kCandCap) {
                        s_trk_zt[wave * kCandCap + slot] = tz[e];
                        s_trk_zd[wave * kCandCap + slot] = dz[e];
                        drop = true;
                    }
                    ncand += __popcll(bal);
                }
                if (drop) {
                    at[e] = -INFINITY;
                    ad[e] = -INFINITY;
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) ut[4 * j + e] = at[e];
        ed_put(j, make_float4(ad[0], ad[1], ad[2], ad[3]));
    }
    // ... then the exponentials and the sums of what stays in fp32, one straight line
    float st = 0.f, sd = 0.f;
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        if constexpr (STAGE) {
            if (CH / 2 + j < CH) stage_chunk(CH / 2 + j);
            if (j < P) {
                const float4 nd = load_stream(nzd4 + (min(j * T + tid, last) & nmask));
                pf[4 * j] = nd.x; pf[4 * j + 1] = nd.y; pf[4 * j + 2] = nd.z; pf[4 * j + 3] = nd.w;
            }
        }
        float4 d = ed_get(j);
        d.x = __builtin_amdgcn_exp2f(d.x);
        d.y = __builtin_amdgcn_exp2f(d.y);
        d.z = __builtin_amdgcn_exp2f(d.z);
        d.w = __builtin_amdgcn_exp2f(d.w);
        ed_put(j, d);
#pragma unroll
        for (int e = 0; e < 4; ++e) ut[4 * j + e] = __builtin_amdgcn_exp2f(ut[4 * j + e]);
        st += (ut[4 * j] + ut[4 * j + 1]) + (ut[4 * j + 2] + ut[4 * j + 3]);
        sd += (d.x + d.y) + (d.z + d.w);
        if (j % 3 == 2) __builtin_amdgcn_sched_barrier(0);  // (bounds how far ahead chunks are read)
    }
    ncand = min(ncand, kCandCap);
    __builtin_amdgcn_wave_barrier();
    // the entries this lane follows in fp64: child `lane` (wave 0, lanes < K) or heavy entry lane - 16
    const bool is_child = wave == 0 && lane < K;
    const bool is_cand = lane >= 16 && lane - 16 < ncand;
    const bool tracked = ncand > 0 || wave == 0;  // (wave-uniform)
    double tU = 0.0, tE = 0.0;
    if (tracked) {
        float fzt = -INFINITY, fzd = -INFINITY;
        if (is_child) {
            fzt = sh.czt[lane];
            fzd = sh.czd[lane];
        } else if (is_cand) {
            fzt = s_trk_zt[wave * kCandCap + lane - 16];
            fzd = s_trk_zd[wave * kCandCap + lane - 16];
        }
        // (one copy of the fp64 exponential in the code, run twice: its temporaries would
        // otherwise push the resident rows out of their registers)
        double x = (double)fzt * a.c2e - (double)m_t;
#pragma unroll 1
        for (int i = 0; i < 2; ++i) {
            asm volatile("" : "+v"(x));
            const double r = (is_child || is_cand) ? exp2(x) : 0.0;
            if (i == 0) {
                tU = r;
                x = (double)fzd * a.c2e - (double)m_d;
            } else {
                tE = r;
            }
        }
        if (is_child) sh.ce[lane] = tE;
    }
    st = wave_sum(st);
    sd = wave_sum(sd);
    {
        double su = (double)st, se = (double)sd;
        if (tracked) {
            su += wave_sum_f64(tU);
            se += wave_sum_f64(is_child ? 0.0 : tE);
        }
        if (lane0) {
            sh.red[wave] = su;
            sh.red2[wave] = se;
        }
    }
    group_barrier<STAGE>();
    double St = 0.0, Sd = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { St += sh.red[w]; Sd += sh.red2[w]; }
    if (tid == 0) {
        sh.g.mt2 = m_t;
        sh.g.md2 = m_d;
        double s0 = Sd;
        for (int i = 0; i < K; ++i) s0 += sh.ce[i];
        if (!(St > 0.0) || !isfinite(St) || !(s0 > 0.0) || !isfinite(s0)) sh.g.flags |= RSD_FLAG_NONFINITE;
    }
    double A = St;  // q^(k) = u / A
    // Stage k < K - 1 needs A_{k+1} = sum_x max(u - gamma_k e_d, 0) and, only if a stage follows it,
    // the rows after the subtraction.  So the subtraction of stage k - 1 is applied inside the
    // pass of stage k (one read-modify-write of u and one read of e_d per stage instead of two
    // passes), the first stage only sums, and the last subtraction -- whose result nobody reads:
    // the last-token pass works from the raw rows -- is never made.  A stage that is skipped
    // (its residual has no mass) leaves a pending subtraction of zero.
    float uh = 0.f, ul = 0.f;  // pending subtraction: gamma_{k-1} as a pair of floats
    // Draft mass still available at stage k: the rest plus the children not yet removed.  Lane k of
    // every wave works out s_k and its reciprocal before the stages, so that a stage starts with a
    // lane read and a product instead of a chain of additions and a division.
    double sk_lane = Sd;
    for (int i = K - 1; i >= min(lane, K); --i) sk_lane += sh.ce[i];
    const double rsk_lane = 1.0 / sk_lane;
    auto stage = [&](auto first_tag, int k) {
        constexpr bool FIRST = decltype(first_tag)::value;
        const double s_k = read_lane_d(sk_lane, k);
        const double gam = A * read_lane_d(rsk_lane, k);
        if (tid == k) {  // what child k's threshold needs, divided once after the loop
            sh.th[k][0] = tU; sh.th[k][1] = A; sh.th[k][2] = s_k; sh.th[k][3] = tE;
        }
        const float gh = (float)gam;
        // small residual mass: gamma as a pair of floats (A_1 = St: never at the first stage)
        const bool fine = !FIRST && A < St * 0.0625;
        const float gl = fine ? (float)(gam - (double)gh) : 0.f;
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const float4 d = ed_get(j);
            const float de[4] = {d.x, d.y, d.z, d.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (FIRST) {
                    part += fmaxf(fmaf(-gh, de[e], ut[4 * j + e]), 0.f);
                } else {
                    const float u = fmaxf(fmaf(-ul, de[e], fmaf(-uh, de[e], ut[4 * j + e])), 0.f);
                    ut[4 * j + e] = u;
                    part += fmaxf(fmaf(-gl, de[e], fmaf(-gh, de[e], u)), 0.f);
                }
            }
            if (CL > 0 && j % 3 == 2) __builtin_amdgcn_sched_barrier(0);  // (bounds how far ahead chunks are read)
        }
        const double cnew = fmax(tU - gam * tE, 0.0);  // (zero in lanes that follow no entry)
        const double wsum = wave_sum_f64((double)part + cnew);
        double *red = sh.sred[k & 1];
        if (lane0) red[wave] = wsum;
        group_barrier<STAGE>();
        double S = 0.0;
#pragma unroll
        for (int w = 0; w < NW; ++w) S += red[w];
        const bool ok = S > 0.0 && isfinite(S);
        uh = ok ? gh : 0.f;
        ul = ok ? gl : 0.f;
        if (ok) {
            tU = cnew;
            if (tid == 0) sh.g.gam[k] = gam;
            A = S;
        } else if (tid == 0) {  // keep q^(k): no subtraction
            sh.g.gam[k] = 0.0;
            sh.g.flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
        }
        // x_k leaves the draft distribution either way
        if (tid == k) tE = 0.0;
    };
    if (K >= 2) {
        stage(std::true_type{}, 0);
#pragma unroll 1
        for (int k = 1; k < K - 1; ++k) stage(std::false_type{}, k);
    }
    if (K > 0) {  // the last child: its threshold's inputs and gamma_K (the last-token pass subtracts it)
        const int k = K - 1;
        const double s_k = read_lane_d(sk_lane, k);
        if (tid == k) {
            sh.th[k][0] = tU; sh.th[k][1] = A; sh.th[k][2] = s_k; sh.th[k][3] = tE;
        }
        if (tid == 0) sh.g.gam[k] = A * read_lane_d(rsk_lane, k);
    }
    // Nothing reads this group's rows any more: the next group's are requested here, under the
    // thresholds, the record's way to memory and the queue.
    if constexpr (PIPE) {
        asm volatile("" : "+v"(nx.claim));
        const int64_t row = ((int64_t)nx.b * a.N + nx.node) * a.V;
        fetch_child_logits(a.zt + row, a.zd + row, a.V, nx.node, nx.cand);
        issue_row_loads<T, CH, CL, !STAGE, P, true>(a.zt + row, a.zd + row, a.V, tid, ut, edr, s_ed, nmask, pf);
    }
    if (tid < K) {  // threshold of child `tid` (Eq. (3)): (u / A) / (e_d / s); the lane's own values
        const double p = sh.th[tid][3] / sh.th[tid][2];
        sh.g.theta[tid] = (p > 0.0) ? (float)fmin(1.0, sh.th[tid][0] / (sh.th[tid][1] * p)) : 1.f;
    }
    group_barrier<STAGE>();
}

// The resident variant on rows that it loads itself: one row pair per call, nothing overlapped
// beyond the children's lookup.
template <int T, int CH, int CL>
__device__ void process_group_res(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    constexpr int CR = CH - CL;  // chunks of e_d held in registers
    __shared__ float4 s_ed[CL > 0 ? CL * T : 1];
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const float *zt = a.zt + ((int64_t)b * a.N + node) * a.V;
    const float *zd = a.zd + ((int64_t)b * a.N + node) * a.V;
    // The children's lookup is requested first and the rows right after it, before the lookup
    // is used: its dependent steps (the children's own logits, two barriers) then run under
    // the rows' memory latency.
    ChildCandidate cand = fetch_candidate(a, b, node, n, tid);
    float ut[CH * 4], edr[CR * 4];
    float pf[4];  // (no prefetch here)
    issue_row_loads<T, CH, CL>(zt, zd, a.V, tid, ut, edr, s_ed, -1, pf);
    // (the candidate is consumed from here on: its wait and the children's own logit loads come
    // after every row load has been issued)
    asm volatile("" : "+v"(cand.parent), "+v"(cand.token));
    fetch_child_logits(zt, zd, a.V, node, cand);
    NextGroup nx{};
    compute_group_res<T, CH, CL, false>(a, node, cand, ut, edr, pf, s_ed, nullptr, sh, nx, 0);
}

// CH == 0: streaming variant; else the resident variant with CH chunks per thread, CL of them in LDS
template <int THREADS, int CH, int CL>
__device__ __forceinline__ void verify_group(const RrsArgs &a, int b, int node, int n, GroupShared &sh) {
    if constexpr (CH > 0)
        process_group_res<THREADS, CH, CL>(a, b, node, n, sh);
    else
        process_group_stream<THREADS>(a, b, node, n, sh);
}

// ---------------------------------------------------------------------------
// Last-token sampling (Alg. 6, last lines): arg-max over x of log r(x) + G(x)
// for entries [x_lo, x_hi) of one node.  r = u after all K stages (q^(K+1) up to a
// factor) when the node's K children were all rejected, or the target row itself for
// a leaf.  Tracks a second arg-max over q^(K) used when the last residual is empty.
// ---------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long pack_key(float v, int idx) {
    uint32_t bits = __float_as_uint(v);
    bits = (bits & 0x80000000u) ? ~bits : (bits | 0x80000000u);
    return ((unsigned long long)bits << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)idx);
}

constexpr int kFinalHeavyCap = 256;  // fp64 entries per workgroup that get a thread of their own

struct FinalShared {
    int count;
    int x[kFinalHeavyCap];
};

// Scores of one entry with the chain in fp64 from the raw logits (child tokens, heavy entries).
__device__ __forceinline__ void final_scores_f64(const RrsArgs &a, const GroupRec &g, const float *zt,
                                                 const float *zd, int x, uint32_t node, uint32_t seq,
                                                 float &s_res, float &s_alt) {
    const int K = g.K;
    const int rs = removal_stage(x, g.tok, K);
    const double U0 = exp2((double)zt[x] * a.c2e - (double)g.mt2);
    const double E = exp2((double)zd[x] * a.c2e - (double)g.md2);
    const double UK = chain1_f64(U0, E, rs, g, K - 1);
    const double R = fmax(UK - g.gam[K - 1] * (K - 1 <= rs ? E : 0.0), 0.0);
    const uint4 rnd = philox4x32_10((uint32_t)x >> 2, node, seq, counter_word3(kTagLastGumbel, a.step),
                                    make_key(a.seed));
    const uint32_t sel = (uint32_t)x & 3u;
    const float gum = gumbel_from_word(sel == 0 ? rnd.x : (sel == 1 ? rnd.y : (sel == 2 ? rnd.z : rnd.w)));
    s_res = (float)log(R) + gum;
    s_alt = (float)log(UK) + gum;
}

// Every thread of the workgroup calls this (one barrier inside when the node has children).
template <int THREADS>
__device__ void final_sample_range(const RrsArgs &a, int b, int node, const GroupRec &g, int c_lo,
                                   int c_hi, FinalShared &fs, float &best_v, int &best_i, float &alt_v,
                                   int &alt_i) {
    const float *zt = a.zt + ((int64_t)b * a.N + node) * a.V;
    const float *zd = a.zd + ((int64_t)b * a.N + node) * a.V;
    const float4 *zt4 = reinterpret_cast<const float4 *>(zt);
    const float4 *zd4 = reinterpret_cast<const float4 *>(zd);
    const uint32_t seq = a.seq_id ? (uint32_t)a.seq_id[b] : (uint32_t)b;
    const PhiloxKey key = make_key(a.seed);
    const uint32_t c3 = counter_word3(kTagLastGumbel, a.step);
    const int K = g.K;
    best_v = -INFINITY; best_i = INT_MAX; alt_v = -INFINITY; alt_i = INT_MAX;
    // The range is walked in batches of kBatch chunks per thread whose loads are all requested
    // before the first is used: one memory round trip per batch instead of one per chunk.
    constexpr int kBatch = 4;
    const int c_last = c_hi - 1;  // (callers pass c_lo < c_hi or an empty range)
    if (K == 0) {
        for (int c0 = c_lo + (int)threadIdx.x; c0 < c_hi; c0 += kBatch * THREADS) {
            float4 tb[kBatch];
#pragma unroll
            for (int r = 0; r < kBatch; ++r) tb[r] = load_stream(zt4 + min(c0 + r * THREADS, c_last));
#pragma unroll
            for (int r = 0; r < kBatch; ++r) {
                const int c = c0 + r * THREADS;
                if (c >= c_hi) break;
                const float4 t = tb[r];
                const uint4 rnd = philox4x32_10((uint32_t)c, (uint32_t)node, seq, c3, key);
                const uint32_t wd[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
                const float tz[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float s = tz[i] * a.inv_t + gumbel_from_word(wd[i]);
                    if (better(s, (c << 2) + i, best_v, best_i)) { best_v = s; best_i = (c << 2) + i; }
                }
            }
        }
        return;
    }
    if (threadIdx.x == 0) fs.count = 0;
    __syncthreads();
    const ChainRegs cr = load_chain(g);
    const float gh_last = uniform_f((float)g.gam[K - 1]);
    const float gl_last = uniform_f((float)(g.gam[K - 1] - (double)(float)g.gam[K - 1]));
    const uint64_t hits = child_chunk_mask<THREADS>(g, c_lo, c_hi);
    int it = 0;
    for (int c0 = c_lo + (int)threadIdx.x; c0 < c_hi; c0 += kBatch * THREADS) {
        float4 tb[kBatch], db[kBatch];
#pragma unroll
        for (int r = 0; r < kBatch; ++r) {
            const int c = min(c0 + r * THREADS, c_last);
            tb[r] = load_stream(zt4 + c);
            db[r] = load_stream(zd4 + c);
        }
#pragma unroll
        for (int r = 0; r < kBatch; ++r, ++it) {
            const int c = c0 + r * THREADS;
            if (c >= c_hi) break;
            const float4 t = tb[r];
            const float4 d = db[r];
            const uint4 rnd = philox4x32_10((uint32_t)c, (uint32_t)node, seq, c3, key);
            const uint32_t wd[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
            const float tz[4] = {t.x, t.y, t.z, t.w}, dz[4] = {d.x, d.y, d.z, d.w};
            float u[4], e[4];
            bool f64[4];
            const bool hit = (hits >> it) & 1ull;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float at = exponent_of(tz[i], a.c2h, a.c2l, -cr.mt2);
                const float ad = exponent_of(dz[i], a.c2h, a.c2l, -cr.md2);
                // child tokens and heavy entries get the chain in fp64, from a thread of their own
                f64[i] = at >= -kHeavy || ad >= -kHeavy || (hit && removal_stage((c << 2) + i, g.tok, K) < K);
                u[i] = __builtin_amdgcn_exp2f(at);
                e[i] = __builtin_amdgcn_exp2f(ad);
            }
            chain4(u, e, cr, K - 1);  // ~ q^(K)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int x = (c << 2) + i;
                float s, s2;
                if (!f64[i]) {
                    const float gum = gumbel_from_word(wd[i]);
                    s2 = fast_ln(u[i]) + gum;
                    s = fast_ln(fmaxf(fmaf(-gl_last, e[i], fmaf(-gh_last, e[i], u[i])), 0.f)) + gum;
                } else {
                    const int slot = atomicAdd(&fs.count, 1);
                    if (slot < kFinalHeavyCap) {
                        fs.x[slot] = x;
                        continue;
                    }
                    final_scores_f64(a, g, zt, zd, x, (uint32_t)node, seq, s, s2);  // (list full: in place)
                }
                if (better(s, x, best_v, best_i)) { best_v = s; best_i = x; }
                if (better(s2, x, alt_v, alt_i)) { alt_v = s2; alt_i = x; }
            }
        }
    }
    __syncthreads();
    const int nlist = min(fs.count, kFinalHeavyCap);
    for (int t = threadIdx.x; t < nlist; t += THREADS) {
        const int x = fs.x[t];
        float s, s2;
        final_scores_f64(a, g, zt, zd, x, (uint32_t)node, seq, s, s2);
        if (better(s, x, best_v, best_i)) { best_v = s; best_i = x; }
        if (better(s2, x, alt_v, alt_i)) { alt_v = s2; alt_i = x; }
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
    for (int i = tid; i < total; i += kPlanThreads) {
        cnt[i] = 0;
        // thresholds of nodes that no group verifies (the root, padding, children beyond the
        // supported group size, nodes with an invalid parent) read NaN
        if (a.theta) a.theta[i] = NAN;
    }
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
        a.wq[1] = 0;
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
// ALL_GROUPS, kernel 1: persistent workgroups take items off the work list (largest groups
// first) through one atomic counter.  The first item of a workgroup is its own number; further
// ones come off the counter (which starts at zero and counts the items after the first G).  A
// workgroup asks for the number of the item after the next, and reads the next item's entry,
// while it verifies the current one, so no round trip is waited for inside the loop.  The
// resident variants also request the next item's rows as soon as the current group has read
// its own for the last time (the rows live in the same registers and LDS slots).
// ---------------------------------------------------------------------------
__device__ __forceinline__ void write_group_record(const RrsArgs &a, int i, int b, const GroupShared &sh, int threads) {
    GroupRec *out = a.rec + i;
    const int words = sizeof(GroupRec) / 4;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(&sh.g);
    uint32_t *dst = reinterpret_cast<uint32_t *>(out);
    for (int w = threadIdx.x; w < words; w += threads) dst[w] = src[w];
    if (a.theta && (int)threadIdx.x < sh.g.K)
        a.theta[(int64_t)b * a.N + sh.g.kid[threadIdx.x]] = sh.g.theta[threadIdx.x];
}

template <int THREADS, int CH, int CL>
__global__ __launch_bounds__(THREADS) void rrs_group_kernel(RrsArgs a) {
    __shared__ GroupShared sh;
    const int count = a.wq[0];
    const int G = gridDim.x;
    int lane_zero = 0;
    asm volatile("" : "+v"(lane_zero));
    int idx = blockIdx.x;
    if (idx >= count) return;
    int2 ent = a.work[idx + lane_zero];
    int idx1 = 0;  // (thread 0) the next item
    if (threadIdx.x == 0) idx1 = G + atomicAdd(&a.wq[1], 1);
    if constexpr (CH > 0) {
        constexpr int CR = CH - CL;  // chunks of e_d held in registers
        constexpr bool STAGE = stages_next_row<CL, true>();
        __shared__ float4 s_ed[CL > 0 ? CL * THREADS : 1];
        __shared__ float4 s_nt[STAGE ? CH * THREADS : 1];  // the next item's target row (raw logits)
        constexpr int P = prefetched_draft_chunks<THREADS, CH, CL, true>();
        float ut[CH * 4], edr[CR * 4], pf[(P > 0 ? P : 1) * 4];
        int i = __builtin_amdgcn_readfirstlane(ent.x), n = __builtin_amdgcn_readfirstlane(ent.y);
        int b = i / a.N, node = i - b * a.N;
        // first item: the children's lookup is requested first and the rows right after it
        ChildCandidate cand = fetch_candidate(a, b, node, n, threadIdx.x);
        {
            const int64_t row = ((int64_t)b * a.N + node) * a.V;
            issue_row_loads<THREADS, CH, CL, true, P, false>(a.zt + row, a.zd + row, a.V, threadIdx.x, ut, edr, s_ed, -1, pf);
        }
        {
            // (the candidate is consumed from here on: the children's own logit loads come
            // after every row load has been issued)
            asm volatile("" : "+v"(cand.parent), "+v"(cand.token));
            const int64_t row = ((int64_t)b * a.N + node) * a.V;
            fetch_child_logits(a.zt + row, a.zd + row, a.V, node, cand);
        }
        while (true) {
            NextGroup nx{};
            if (threadIdx.x == 0) {
                nx.idx = idx1;
                // (past the end of the list the "next item" is the current one over again: what
                // is requested for it then goes to this group's own rows, a different place for
                // every workgroup, and is never used)
                nx.ent = make_int2(i, n);
                if (idx1 < count) nx.ent = a.work[idx1];
                nx.claim = atomicAdd(&a.wq[1], 1);  // (G is added where the value is first needed)
            }
            compute_group_res<THREADS, CH, CL, true>(a, node, cand, ut, edr, pf, s_ed, s_nt, sh, nx, count);
            write_group_record(a, i, b, sh, THREADS);
            idx1 = G + nx.claim;
            group_barrier<STAGE>();  // sh is reused by the next item
            if (!nx.has) break;
            if constexpr (STAGE) {
                // The staged row moves to the registers.  Its loads are older than the CH - P
                // loads of the draft row that followed them, and loads complete in order.
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"(CH - P) : "memory");
                int tid = threadIdx.x;
                asm volatile("" : "+v"(tid));
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const float4 t = s_nt[j * THREADS + tid];
                    ut[4 * j + 0] = t.x; ut[4 * j + 1] = t.y; ut[4 * j + 2] = t.z; ut[4 * j + 3] = t.w;
                }
            }
            const int gi = nx.b * a.N + nx.node;
            i = __builtin_amdgcn_readfirstlane(gi);
            n = __builtin_amdgcn_readfirstlane(nx.n);
            b = __builtin_amdgcn_readfirstlane(nx.b);
            node = __builtin_amdgcn_readfirstlane(nx.node);
            cand = nx.cand;
        }
        // (the requests made for a next item that does not exist land before the workgroup gives
        // up its LDS and registers)
        asm volatile("s_waitcnt vmcnt(0)");
    } else {
        while (idx < count) {
            const int i = __builtin_amdgcn_readfirstlane(ent.x), n = __builtin_amdgcn_readfirstlane(ent.y);
            int idx2 = 0;
            int2 nent = make_int2(0, 1);
            if (threadIdx.x == 0) {
                nent = a.work[min(idx1, count - 1)];
                idx2 = G + atomicAdd(&a.wq[1], 1);
            }
            const int b = i / a.N, node = i - b * a.N;
            verify_group<THREADS, CH, CL>(a, b, node, n, sh);
            write_group_record(a, i, b, sh, THREADS);
            if (threadIdx.x == 0) {
                sh.next_idx = idx1;
                sh.next_ent = nent;
                idx1 = idx2;
            }
            __syncthreads();
            idx = sh.next_idx;
            ent = sh.next_ent;
            __syncthreads();  // sh is reused by the next item
        }
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
    constexpr int W_GAM = offsetof(GroupRec, gam) / 4, W_THETA = offsetof(GroupRec, theta) / 4;
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
        // (the high word of a stage's gamma: zero only for a skipped stage)
        const uint32_t gam_hi = word(r0, r1, W_GAM + 2 * min(lane, RSD_K_MAX - 1) + 1);
        const bool ok = lane < K && accept_uniform(a, b, kid) < theta;
        const unsigned long long acc = __ballot(ok);
        const int took = acc ? __ffsll((long long)acc) - 1 : -1;
        // degenerate stages matter only if their residual was used
        if (gflags & RSD_FLAG_DEGENERATE_RESIDUAL) {
            const int used = took < 0 ? K - 1 : took;
            if (__ballot(lane < used && gam_hi == 0u)) flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
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
    __shared__ FinalShared fs;
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
    final_sample_range<kFinalThreads>(a, b, node, g, c_lo, c_hi, fs, bv, bi, av, ai);
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
    __shared__ FinalShared fs;
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
                    if (sh.g.gam[j] == 0.0) flags |= RSD_FLAG_DEGENERATE_RESIDUAL;
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
    final_sample_range<THREADS>(a, b, node, sh.g, 0, a.V >> 2, fs, bv, bi, av, ai);
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
    // c = log2(e) / T in fp64 and as a pair of floats with a strictly positive low part
    a.c2e = (double)inv_temperature * 1.4426950408889634;
    a.c2h = (float)a.c2e;
    if ((double)a.c2h >= a.c2e) a.c2h = nextafterf(a.c2h, 0.f);
    a.c2l = (float)(a.c2e - (double)a.c2h);
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
    // Which variant holds a row (see the constants at the top of this file).
    const bool small = V <= kSmallThreads * 4 * kSmallChunks;
    const bool reg = !small && V <= kRegThreads * 4 * kRegChunks;
    const bool lds = !small && !reg && V <= kLdsThreads * 4 * kLdsChunks;
    if (mode == RSD_MODE_PATH) {
        if (small)
            hipLaunchKernelGGL((rrs_path_kernel<kSmallThreads, kSmallChunks, 0>), dim3(B), dim3(kSmallThreads), 0, st, a);
        else if (reg)
            hipLaunchKernelGGL((rrs_path_kernel<kRegThreads, kRegChunks, kRegChunksInLds>), dim3(B),
                               dim3(kRegThreads), 0, st, a);
        else if (lds)
            hipLaunchKernelGGL((rrs_path_kernel<kLdsThreads, kLdsChunks, kLdsChunksInLds>), dim3(B),
                               dim3(kLdsThreads), 0, st, a);
        else
            hipLaunchKernelGGL((rrs_path_kernel<kStreamThreads, 0, 0>), dim3(B), dim3(kStreamThreads), 0, st, a);
    } else {
        int dev = 0, n_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
            n_cu = 256;
        const long items_max = (long)B * N_max;
        // persistent workgroups: as many as are resident at once (two per CU where two fit)
        auto grid_for = [&](int per_cu) { return (int)(items_max < (long)per_cu * n_cu ? items_max : (long)per_cu * n_cu); };
        hipLaunchKernelGGL(rrs_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, a);
        if (small)
            hipLaunchKernelGGL((rrs_group_kernel<kSmallThreads, kSmallChunks, 0>), dim3(grid_for(4)),
                               dim3(kSmallThreads), 0, st, a);
        else if (reg)
            hipLaunchKernelGGL((rrs_group_kernel<kRegThreads, kRegChunks, kRegChunksInLds>), dim3(grid_for(1)),
                               dim3(kRegThreads), 0, st, a);
        else if (lds)
            hipLaunchKernelGGL((rrs_group_kernel<kLdsThreads, kLdsChunks, kLdsChunksInLds>), dim3(grid_for(1)),
                               dim3(kLdsThreads), 0, st, a);
        else
            hipLaunchKernelGGL((rrs_group_kernel<kStreamThreads, 0, 0>), dim3(grid_for(2)), dim3(kStreamThreads), 0, st, a);
        // enough workgroups to fill the chip, but no more: every split costs two device-wide fences
        int fsplits = 256 / (B > 0 ? B : 1);
        fsplits = fsplits < 1 ? 1 : (fsplits > kFinalSplitsMax ? kFinalSplitsMax : fsplits);
        hipLaunchKernelGGL(rrs_final_kernel, dim3(fsplits, B), dim3(kFinalThreads), 0, st, a);
    }
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}
