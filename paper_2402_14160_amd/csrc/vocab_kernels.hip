// Vocabulary-wide passes of the drafting side: log-softmax normaliser,
// Gumbel-Top-k (Alg. 4) and the Stochastic Beam Search step (Alg. 9).
//
// One workgroup owns one logit row.  The row is read once from HBM with
// 16-byte coalesced loads; each lane's four consecutive entries share one
// Philox block.  The perturbed scores stay in registers, so selecting the k
// winners needs no second pass over memory.
#include <hip/hip_runtime.h>
#include <limits.h>
#include <math.h>

#include <mutex>

#include "../../include/rsd.h"
#include "rsd_device.hpp"

namespace rsd {

// ---------------------------------------------------------------------------
// lse[r] = log sum_x exp(z[r,x] / T)      (Eq. (5): phi = z/T - lse)
// ---------------------------------------------------------------------------
template <int THREADS>
__global__ __launch_bounds__(THREADS) void lse_kernel(const float *__restrict__ logits, int64_t ld,
                                                      int V, float c2, float *__restrict__ lse) {
    __shared__ MaxSum s_ms[THREADS / kWave];
    const int row = blockIdx.x;
    const float *zrow = logits + (int64_t)row * ld;
    const float4 *z4 = reinterpret_cast<const float4 *>(zrow);
    const int nchunk = V >> 2;
    MaxSum acc{-INFINITY, 0.f};
#pragma unroll 4
    for (int c = threadIdx.x; c < nchunk; c += THREADS) {
        const float4 z = load_stream(z4 + c);
        const float a0 = z.x * c2, a1 = z.y * c2, a2 = z.z * c2, a3 = z.w * c2;
        const float mx = fmaxf(fmaxf(a0, a1), fmaxf(a2, a3));
        if (mx > acc.m) {
            acc.s *= exp2f(acc.m - mx);
            acc.m = mx;
        }
        if (acc.m > -INFINITY)
            acc.s += (exp2f(a0 - acc.m) + exp2f(a1 - acc.m)) + (exp2f(a2 - acc.m) + exp2f(a3 - acc.m));
    }
    const int tail = (nchunk << 2) + threadIdx.x;
    if (tail < V) {
        const float a = zrow[tail] * c2;
        if (a > acc.m) {
            acc.s *= exp2f(acc.m - a);
            acc.m = a;
        }
        if (acc.m > -INFINITY) acc.s += exp2f(a - acc.m);
    }
    acc = block_merge<THREADS>(acc, s_ms);
    if (threadIdx.x == 0) lse[row] = (acc.m + log2f(acc.s)) * kLn2;
}

// ---------------------------------------------------------------------------
// Gumbel-Top-k row kernel.
// ---------------------------------------------------------------------------
struct TopkArgs {
    const float *logits;
    int64_t ld;
    int V;
    int k_max;
    const int *k_per_row;  // [R] or null
    const int *seq_id;     // indexed by row / rows_per_seq, or null
    const int *node_id;    // [R] or null
    const int *n_live;     // [R / rows_per_seq] or null: rows w >= n_live[b] are dead (SBS)
    int rows_per_seq;      // 1 for Gumbel-Top-k; W_in for SBS
    int seq_default_is_b;  // null seq_id means: 0 (Gumbel-Top-k) or b (SBS)
    int node_default_is_w; // null node_id means: row (Gumbel-Top-k) or w (SBS)
    float inv_t;
    uint64_t seed;
    uint32_t step;
    int *tokens;       // [R, k_max]
    float *perturbed;  // [R, k_max] or null
    float *logprob;    // [R, k_max] or null
    float *lse;        // [R] or null
    int *count;        // [R] or null
    // Row segments (SBS on few rows): nseg > 1 workgroups share a row, each takes a contiguous
    // range of chunks and writes its own candidate list at index row * nseg + seg of tokens /
    // perturbed / logprob / count -- scores and logits NOT yet reduced by the row normaliser,
    // whose per-segment (max, sum) pair goes to seg_ms; `lse` is then left to the consumer.
    int nseg;
    MaxSum *seg_ms;    // [R * nseg] when nseg > 1 or raw_lists
    // SBS: the lists keep the raw logit of every candidate in `logprob` and scores that are not
    // reduced by the row normaliser, whose (max, sum) pair always goes to seg_ms: the consumer
    // recomputes what it needs from exact inputs.
    int raw_lists;
};

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kCandMax = 1024;

// Without the normaliser and up to 8 chunks per thread the kernel is held to 64 registers: two
// workgroups then share a CU, and one row's load, reduction and selection phases run under the
// other's Philox arithmetic (with the normaliser the same limit spills too much to pay).
template <int CH, bool WANT_LSE>
__global__ __launch_bounds__(kTopkThreads, (CH <= 8 && !WANT_LSE) ? 8 : 4) void gumbel_topk_kernel(TopkArgs a) {
    __shared__ MaxSum s_ms[kTopkWaves];
    __shared__ float s_wmax[kTopkWaves];
    __shared__ int s_cnt;
    __shared__ float s_cval[kCandMax];
    __shared__ int s_cidx[kCandMax];
    __shared__ float s_av[kTopkWaves];
    __shared__ int s_ai[kTopkWaves];
    __shared__ float s_outv[RSD_K_MAX];
    __shared__ int s_outi[RSD_K_MAX];
    __shared__ int s_nout;

    const int nseg = a.nseg;
    const int row = blockIdx.x / nseg;
    const int seg = blockIdx.x - row * nseg;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int b = row / a.rows_per_seq;
    const int w = row - b * a.rows_per_seq;
    const bool dead = a.n_live != nullptr && w >= a.n_live[b];

    int k = a.k_per_row ? a.k_per_row[row] : a.k_max;
    k = min(max(k, 0), a.k_max);
    if (dead) k = 0;
    const uint32_t seq = a.seq_id ? (uint32_t)a.seq_id[a.rows_per_seq > 1 ? b : row]
                                  : (a.seq_default_is_b ? (uint32_t)b : 0u);
    const uint32_t node = a.node_id ? (uint32_t)a.node_id[row]
                                    : (a.node_default_is_w ? (uint32_t)w : (uint32_t)row);
    const PhiloxKey key = make_key(a.seed);
    const uint32_t c3 = counter_word3(kTagDraftGumbel, a.step);

    const float *zrow = a.logits + (int64_t)row * a.ld;
    const float4 *z4 = reinterpret_cast<const float4 *>(zrow);
    const int V = a.V;
    // chunks of four entries that lie fully inside the row (a dead row is read like any other --
    // it is memory of the same tensor -- so that the loads below do not wait for n_live; its k = 0
    // keeps it out of every output)
    const int nfull = V >> 2;
    const float inv_t = a.inv_t;
    // this workgroup's chunk range [c0, c1) of the row; the ragged tail goes with the last segment
    const int per = (nfull + nseg - 1) / nseg;
    const int c0 = min(seg * per, nfull), c1 = min(c0 + per, nfull);
    const bool has_tail = seg == nseg - 1;

    // Entry (j, e) of this thread is vocabulary index 4 * (c0 + j * 1024 + tid) + e; one extra slot
    // holds the up to three entries of a ragged tail (threads 0..2).
    float val[CH * 4 + 1];
    MaxSum acc{-INFINITY, 0.f};
    // all loads first (the row streams in while the first Philox blocks are computed) ...
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = c0 + j * kTopkThreads + tid;
        float4 t = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
        if (c < c1) t = load_stream(z4 + c);
        val[j * 4 + 0] = t.x; val[j * 4 + 1] = t.y; val[j * 4 + 2] = t.z; val[j * 4 + 3] = t.w;
    }
    // ... then one chunk at a time, so that only one Philox block is live
#pragma unroll
    for (int j = 0; j < CH; ++j) {
        const int c = c0 + j * kTopkThreads + tid;
        if (c < c1) {
            const uint4 r = philox4x32_10((uint32_t)c, node, seq, c3, key);
            const float s0 = val[j * 4 + 0] * inv_t, s1 = val[j * 4 + 1] * inv_t;
            const float s2 = val[j * 4 + 2] * inv_t, s3 = val[j * 4 + 3] * inv_t;
            val[j * 4 + 0] = s0 + gumbel_from_word(r.x);
            val[j * 4 + 1] = s1 + gumbel_from_word(r.y);
            val[j * 4 + 2] = s2 + gumbel_from_word(r.z);
            val[j * 4 + 3] = s3 + gumbel_from_word(r.w);
            if (WANT_LSE) {
                const float mx2 = fmaxf(fmaxf(s0, s1), fmaxf(s2, s3)) * kLog2e;
                if (mx2 > acc.m) {
                    acc.s *= __builtin_amdgcn_exp2f(acc.m - mx2);
                    acc.m = mx2;
                }
                if (acc.m > -INFINITY)
                    acc.s += (__builtin_amdgcn_exp2f(fmaf(s0, kLog2e, -acc.m)) +
                              __builtin_amdgcn_exp2f(fmaf(s1, kLog2e, -acc.m))) +
                             (__builtin_amdgcn_exp2f(fmaf(s2, kLog2e, -acc.m)) +
                              __builtin_amdgcn_exp2f(fmaf(s3, kLog2e, -acc.m)));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    {
        float vt = -INFINITY;
        const int x = (nfull << 2) + tid;
        if (!dead && has_tail && tid < (V & 3)) {
            const uint4 r = philox4x32_10((uint32_t)nfull, node, seq, c3, key);
            const uint32_t wd = tid == 0 ? r.x : (tid == 1 ? r.y : r.z);
            const float s = zrow[x] * inv_t;
            vt = s + gumbel_from_word(wd);
            if (WANT_LSE) {
                const float s2 = s * kLog2e;
                if (s2 > acc.m) {
                    acc.s *= __builtin_amdgcn_exp2f(acc.m - s2);
                    acc.m = s2;
                }
                if (acc.m > -INFINITY) acc.s += __builtin_amdgcn_exp2f(s2 - acc.m);
            }
        }
        val[CH * 4] = vt;
    }
    // vocabulary index of register slot i
    auto slot_index = [&](int i) { return i < CH * 4 ? (((c0 + (i >> 2) * kTopkThreads + tid) << 2) | (i & 3)) : (nfull << 2) + tid; };

    // ---- per-wave partials, one barrier, then every wave finishes both reductions itself ----
    float tmax = -INFINITY;
#pragma unroll
    for (int e = 0; e < CH * 4 + 1; ++e) tmax = fmaxf(tmax, val[e]);
    const float wmax = wave_max(tmax);
    if (WANT_LSE) acc = wave_merge_dpp(acc);
    if (lane == 0) {
        s_wmax[wave] = wmax;
        if (WANT_LSE) s_ms[wave] = acc;
    }
    if (tid == 0) {
        s_cnt = 0;
        s_nout = 0;
    }
    __syncthreads();
    // row normaliser
    float lse_nat = 0.f;
    if (WANT_LSE) {
        acc = wave_merge_dpp(lane < kTopkWaves ? s_ms[lane] : MaxSum{-INFINITY, 0.f});
        lse_nat = (acc.m + log2f(acc.s)) * kLn2;
    }
    // threshold: the k-th largest wave maximum (ranks of the 16 maxima, ties by wave index)
    const float mine = lane < kTopkWaves ? s_wmax[lane] : -INFINITY;
    int mrank = 0;
#pragma unroll
    for (int o = 0; o < kTopkWaves; ++o) {
        const float ov = read_lane(mine, o);
        mrank += (ov > mine) || (ov == mine && o < lane);
    }
    const uint64_t hit = __builtin_amdgcn_ballot_w64(lane < kTopkWaves && mrank == max(k, 1) - 1);
    const float tau = read_lane(mine, hit ? __builtin_ctzll(hit) : 0);

    // ---- gather everything at or above the threshold ---------------------
    if (k > 0 && tmax >= tau && tmax > -INFINITY) {
#pragma unroll
        for (int i = 0; i < CH * 4 + 1; ++i) {
            const float v = val[i];
            if (v >= tau && v > -INFINITY) {
                const int slot = atomicAdd(&s_cnt, 1);
                if (slot < kCandMax) {
                    s_cval[slot] = v;
                    s_cidx[slot] = slot_index(i);
                }
            }
        }
    }
    __syncthreads();
    const int ncand = s_cnt;

    if (ncand <= kCandMax) {
        // ---- wave 0 picks the k best candidates in order -----------------
        if (wave == 0 && ncand <= kWave) {
            // one candidate per lane: its rank among them is its place in the output
            const float v = lane < ncand ? s_cval[lane] : -INFINITY;
            const int i = lane < ncand ? s_cidx[lane] : INT_MAX;
            int rank = 0;
            for (int t = 0; t < ncand; ++t)
                rank += better(read_lane(v, t), __builtin_amdgcn_readlane(i, t), v, i);
            if (lane < ncand && rank < k) {
                s_outv[rank] = v;
                s_outi[rank] = i;
            }
            if (lane == 0) s_nout = min(k, ncand);  // (every candidate is finite)
        } else if (wave == 0) {
            for (int r = 0; r < k; ++r) {
                float bv = -INFINITY;
                int bi = INT_MAX, bslot = -1;
                for (int s = lane; s < ncand; s += kWave) {
                    const float v = s_cval[s];
                    const int i = s_cidx[s];
                    if (better(v, i, bv, bi)) {
                        bv = v;
                        bi = i;
                        bslot = s;
                    }
                }
                float wv = bv;
                int wi = bi;
                wave_argmax(wv, wi);
                if (!(wv > -INFINITY)) break;
                if (bslot >= 0 && bi == wi) s_cval[bslot] = -INFINITY;
                if (lane == 0) {
                    s_outv[r] = wv;
                    s_outi[r] = wi;
                    s_nout = r + 1;
                }
                __threadfence_block();
            }
        }
        __syncthreads();
    } else {
        // ---- rare: too many candidates (many equal or -inf scores); k rounds of
        // workgroup-wide arg-max over the register-resident scores ---------
        for (int r = 0; r < k; ++r) {
            float bv = -INFINITY;
            int bi = INT_MAX;
#pragma unroll
            for (int i = 0; i < CH * 4 + 1; ++i) {
                const int x = slot_index(i);
                if (better(val[i], x, bv, bi)) {
                    bv = val[i];
                    bi = x;
                }
            }
            block_argmax<kTopkThreads>(bv, bi, s_av, s_ai);
            if (!(bv > -INFINITY)) break;
#pragma unroll
            for (int i = 0; i < CH * 4 + 1; ++i)
                if (slot_index(i) == bi) val[i] = -INFINITY;
            if (tid == 0) {
                s_outv[r] = bv;
                s_outi[r] = bi;
                s_nout = r + 1;
            }
        }
        __syncthreads();
    }

    // ---- outputs ----------------------------------------------------------
    const int nout = s_nout;
    const int64_t orow = (int64_t)row * nseg + seg;  // list index: the row, or the row's segment
    const bool raw = a.raw_lists != 0;
    const float sub = (nseg > 1 || raw) ? 0.f : lse_nat;  // segments leave the normaliser to the consumer
    if (tid < a.k_max) {
        const int64_t o = orow * a.k_max + tid;
        if (tid < nout) {
            const int t = s_outi[tid];
            a.tokens[o] = t;
            if (WANT_LSE) {
                if (a.perturbed) a.perturbed[o] = s_outv[tid] - sub;
                if (a.logprob) a.logprob[o] = raw ? zrow[t] : zrow[t] * a.inv_t - sub;
            }
        } else {
            a.tokens[o] = -1;
            if (a.perturbed) a.perturbed[o] = -INFINITY;
            if (a.logprob) a.logprob[o] = -INFINITY;
        }
    }
    if (tid == 0) {
        if (a.count) a.count[orow] = nout;
        if (WANT_LSE && (nseg > 1 || raw)) a.seg_ms[orow] = dead ? MaxSum{-INFINITY, 0.f} : acc;
        if (WANT_LSE && nseg == 1 && !raw && a.lse) a.lse[row] = dead ? 0.f : lse_nat;
    }
}

// ---------------------------------------------------------------------------
// SBS: combine the per-row top-W lists of one sequence (Alg. 9, last steps).
// Only each row's W best perturbed scores can be among the global top-W since
// T(u, .) is increasing within a row (Theorem 3.2's argument).
// ---------------------------------------------------------------------------
struct SbsSelectArgs {
    const int *row_tok;      // [B*W_in*nseg, W]
    const float *row_pert;   // [B*W_in*nseg, W]  z/T + G in fp32 (ranks a row's candidates)
    const float *row_z;      // [B*W_in*nseg, W]  the candidates' raw logits
    const int *row_cnt;      // [B*W_in*nseg]
    const MaxSum *seg_ms;    // [B*W_in*nseg] (max, sum) of every list's share of the row, log2 domain
    const float *sum_logprob;   // [B, W_in]
    const float *trunc_gumbel;  // [B, W_in]
    const int *n_in;
    const int *seq_id;       // [B] or null (= b)
    const int *node_id;      // [B, W_in] or null (= w)
    uint64_t seed;
    uint32_t step;
    float inv_t;
    int W_in, W, V, nseg;
    int *tokens;
    int *parent;
    float *sum_out;
    float *gum_out;
    int *n_out;
    float *lse;  // [B, W_in] or null
};

// One thread per candidate slot (row w, segment sg, position j): W_in * nseg * W <= 256.  With
// segments, every slot of a row is a candidate (a superset of the row's top W, which is all
// that can matter) and the row's W best by fp32 score go on.  For those the truncated Gumbel
// of Eq. (11) is worked out in fp64 from exact inputs: the candidate's raw logit and the Gumbel
// variate of its own Philox word, so that the distance Phi~ - Z to the row maximum -- which
// Eq. (11) amplifies by exp(psi - Phi~) -- carries no fp32 rounding (within a row the
// normaliser and the parent's sum cancel in it).
__global__ __launch_bounds__(256) void sbs_select_kernel(SbsSelectArgs a) {
    __shared__ __align__(16) double s_psi[256];
    __shared__ __align__(16) double s_rel[256];
    __shared__ __align__(16) int s_key[256];
    __shared__ __align__(16) int s_key2[256];
    __shared__ float s_rpert[256];
    __shared__ double s_lse[RSD_K_MAX];  // per row
    __shared__ MaxSum s_sms[RSD_K_MAX * 8];
    const int b = blockIdx.x;
    const int t = threadIdx.x;
    const int nseg = a.nseg;
    const int per_row = nseg * a.W;
    const int w = t / per_row;
    const int sg = (t - w * per_row) / a.W;
    const int j = t - w * per_row - sg * a.W;
    const int n = min(max(a.n_in[b], 0), a.W_in);
    // Everything a slot needs comes from global memory in one round of independent loads (the
    // lists were written by other CUs a moment ago, so every dependent round trip costs
    // microseconds); slots beyond a list's count read initialised padding.
    const bool slot = t < a.W_in * per_row;
    const int row = b * a.W_in + (slot ? w : 0);
    const int list = row * nseg + (slot ? sg : 0);
    const int cnt = a.row_cnt[list];
    const int tok_in = a.row_tok[(int64_t)list * a.W + j % a.W];
    const float pert_in = a.row_pert[(int64_t)list * a.W + j % a.W];
    const float z_in = a.row_z[(int64_t)list * a.W + j % a.W];
    const MaxSum ms_in = a.seg_ms[list];
    const float sigma_in = a.sum_logprob[row], gamma_in = a.trunc_gumbel[row];
    const uint32_t seq = a.seq_id ? (uint32_t)a.seq_id[b] : (uint32_t)b;
    const uint32_t node = a.node_id ? (uint32_t)a.node_id[row] : (uint32_t)(slot ? w : 0);
    const bool row_live = slot && w < n;
    if (slot && j == 0) s_sms[w * nseg + sg] = row_live ? ms_in : MaxSum{-INFINITY, 0.f};
    const int slots = a.W_in * a.W;  // entries of the table that the last ranking runs over
    if (t < ((slots + 3) & ~3)) {
        s_psi[t] = -INFINITY;
        s_rel[t] = -INFINITY;
        s_key2[t] = INT_MAX;
    }
    bool live = row_live && j < cnt;
    if (nseg > 1) {  // (token array of the row ranking below)
        s_rpert[t] = live ? pert_in : -INFINITY;
        s_key[t] = live ? tok_in : INT_MAX;
    }
    __syncthreads();
    // With segments a row has nseg * W candidates, of which only its W best by perturbed score
    // can be selected: rank inside the row first (fp32), so that the fp64 part below and the
    // ranking over all rows handle W_in * W entries, as without segments.
    int place = j;  // position inside the row's list of (at most) W
    if (nseg > 1) {
        const int base = w * per_row;
        int rr = 0;
        if (live) {
            for (int o = 0; o < per_row; ++o) {
                const float op = s_rpert[base + o];
                const int ot = s_key[base + o];
                rr += (int)((op > pert_in) | ((op == pert_in) & (ot < tok_in)));
            }
        }
        live = live && rr < a.W;
        place = rr;
    }
    if (t < a.W_in) {
        double lse = 0.0;
        MaxSum ms{-INFINITY, 0.f};
        for (int g = 0; g < nseg; ++g) ms = merge(ms, s_sms[t * nseg + g]);
        if (t < n) lse = ((double)ms.m + log2((double)ms.s)) * 0.6931471805599453;
        s_lse[t] = lse;
        if (a.lse) a.lse[b * a.W_in + t] = (float)lse;
    }
    // the candidate's score relative to its row: z/T + G in fp64, G from the candidate's own word
    double rel = -INFINITY, s = 0.0;
    int tok = -1;
    if (live) {
        tok = tok_in;
        const uint4 r = philox4x32_10((uint32_t)tok >> 2, node, seq, counter_word3(kTagDraftGumbel, a.step),
                                      make_key(a.seed));
        const uint32_t sel = (uint32_t)tok & 3u;
        const uint32_t wd = sel == 0 ? r.x : (sel == 1 ? r.y : (sel == 2 ? r.z : r.w));
        const double u = (double)((wd >> 8) | 1u) * 5.9604644775390625e-08;
        s = (double)z_in * (double)a.inv_t;
        rel = s - log(-log(u));
        s_rel[w * a.W + place] = rel;
    }
    __syncthreads();
    double psi = -INFINITY, phi = -INFINITY;
    if (live) {
        double top = -INFINITY;  // the row's maximum: it is among the row's candidates
        for (int o = 0; o < a.W; ++o) top = fmax(top, s_rel[w * a.W + o]);
        const double sigma = (double)sigma_in;
        const double gamma = (double)gamma_in;
        const double shift = sigma - s_lse[w];
        phi = s + shift;
        const double d = rel - top;  // Phi~ - Z <= 0
        if (!(d < 0.0)) {
            psi = gamma;
        } else {
            const double log1m = d > -0.6931471805599453 ? log(-expm1(d)) : log1p(-exp(d));
            const double v = gamma - (rel + shift) + log1m;
            psi = gamma - (fmax(v, 0.0) + log1p(exp(-fabs(v))));
        }
    }
    // compact table of W_in * W entries: entry w * W + place (the others were initialised dead)
    const int mykey = live ? (w * a.V + tok) : INT_MAX;
    if (live) {
        s_psi[w * a.W + place] = psi;
        s_key2[w * a.W + place] = mykey;
    }
    __syncthreads();
    // rank of this candidate among all (the table is padded to a multiple of four entries:
    // 16-byte LDS reads)
    int total = 0, rank = 0;
    for (int o = 0; o < slots; o += 4) {
        const double2 p01 = *reinterpret_cast<const double2 *>(&s_psi[o]);
        const double2 p23 = *reinterpret_cast<const double2 *>(&s_psi[o + 2]);
        const int4 k4 = *reinterpret_cast<const int4 *>(&s_key2[o]);
        const double op[4] = {p01.x, p01.y, p23.x, p23.y};
        const int ok[4] = {k4.x, k4.y, k4.z, k4.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // bitwise on purpose: no branches inside the loop
            const bool olive = ok[q] != INT_MAX;
            total += olive ? 1 : 0;
            rank += (int)(olive & ((op[q] > psi) | ((op[q] == psi) & (ok[q] < mykey))));
        }
    }
    if (live && rank < a.W) {  // (the rank of a slot that is not live is never used)
        const int o = b * a.W + rank;
        a.tokens[o] = tok;
        a.parent[o] = w;
        a.sum_out[o] = (float)phi;
        a.gum_out[o] = (float)psi;
    }
    const int nout = min(total, a.W);
    if (t >= nout && t < a.W) {
        const int o = b * a.W + t;
        a.tokens[o] = -1;
        a.parent[o] = -1;
        a.sum_out[o] = -INFINITY;
        a.gum_out[o] = -INFINITY;
    }
    if (t == 0) a.n_out[b] = nout;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int32_t launch_topk(const TopkArgs &a, int R, hipStream_t st) {
    if (R == 0) return RSD_OK;
    // the normaliser costs an exponential per entry: skip it when only tokens are wanted
    const bool want_lse = a.perturbed || a.logprob || a.lse;
    const int nseg = a.nseg;
    const int per = ((a.V >> 2) + nseg - 1) / nseg;                         // chunks of one segment
    const int chunks = per > 0 ? (per + kTopkThreads - 1) / kTopkThreads : 1;  // float4 chunks per thread
#define RSD_LAUNCH_TOPK(CH)                                                                          \
    do {                                                                                             \
        if (want_lse)                                                                                \
            hipLaunchKernelGGL((gumbel_topk_kernel<CH, true>), dim3(R * nseg), dim3(kTopkThreads), 0, st, a);  \
        else                                                                                         \
            hipLaunchKernelGGL((gumbel_topk_kernel<CH, false>), dim3(R * nseg), dim3(kTopkThreads), 0, st, a); \
    } while (0)
    if (chunks <= 2)
        RSD_LAUNCH_TOPK(2);
    else if (chunks <= 8)
        RSD_LAUNCH_TOPK(8);
    else if (chunks <= 13)
        RSD_LAUNCH_TOPK(13);
    else
        RSD_LAUNCH_TOPK(16);
#undef RSD_LAUNCH_TOPK
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}

}  // namespace rsd

using namespace rsd;

extern "C" int32_t rsd_log_softmax_lse(const float *logits, int64_t ld, int32_t R, int32_t V,
                                       float inv_temperature, float *lse, void *stream) {
    if (!logits || !lse) return RSD_ERR_NULL;
    if (R < 0 || V < 1 || ld < V || (ld & 3) || !aligned16(logits) || !(inv_temperature > 0.f))
        return RSD_ERR_SHAPE;
    if (R == 0) return RSD_OK;
    const float c2 = (float)((double)inv_temperature * 1.4426950408889634);
    hipLaunchKernelGGL(lse_kernel<256>, dim3(R), dim3(256), 0, (hipStream_t)stream, logits, ld, V, c2,
                       lse);
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}

extern "C" size_t rsd_gumbel_topk_workspace_bytes(int32_t, int32_t, int32_t) { return 0; }

extern "C" int32_t rsd_gumbel_topk(const float *logits, int64_t ld, int32_t R, int32_t V,
                                   int32_t k_max, const int32_t *k_per_row, float inv_temperature,
                                   const int32_t *seq_id, const int32_t *node_id, uint64_t seed,
                                   uint32_t step, int32_t *tokens, float *perturbed, float *logprob,
                                   float *lse, int32_t *count, void *, size_t, void *stream) {
    if (!logits || !tokens) return RSD_ERR_NULL;
    if (R < 0 || V < 1 || V > RSD_VOCAB_MAX || k_max < 1 || k_max > RSD_K_MAX || k_max > V ||
        ld < V || (ld & 3) || !aligned16(logits) || !(inv_temperature > 0.f))
        return RSD_ERR_SHAPE;
    TopkArgs a{};
    a.logits = logits; a.ld = ld; a.V = V; a.k_max = k_max; a.k_per_row = k_per_row;
    a.seq_id = seq_id; a.node_id = node_id; a.n_live = nullptr; a.rows_per_seq = 1;
    a.seq_default_is_b = 0; a.node_default_is_w = 0; a.inv_t = inv_temperature;
    a.seed = seed; a.step = step; a.tokens = tokens; a.perturbed = perturbed;
    a.logprob = logprob; a.lse = lse; a.count = count; a.nseg = 1; a.seg_ms = nullptr;
    return launch_topk(a, R, (hipStream_t)stream);
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Segments per row of one SBS step: split rows while the launch leaves most of the chip idle,
// as long as every candidate slot still has a thread in the select kernel and a segment keeps
// at least 4096 entries.
static int sbs_segments(int B, int W_in, int V, int W) {
    const long rows = (long)B * W_in;
    int s = 1;
    while (s < 8 && rows * (s * 2) <= 256 && (long)W_in * W * (s * 2) <= 256 && V / (s * 2) >= 4096 &&
           (V & 3) == 0)
        s *= 2;
    return s;
}

extern "C" size_t rsd_sbs_step_workspace_bytes(int32_t B, int32_t W_in, int32_t V, int32_t W) {
    if (B < 0 || W_in < 0 || W < 0) return 0;
    const size_t lists = (size_t)B * W_in * (size_t)sbs_segments(B, W_in, V > 0 ? V : 1, W > 0 ? W : 1);
    return 3 * align_up(lists * W * 4, 256) + align_up(lists * 4, 256) + align_up(lists * sizeof(MaxSum), 256);
}

// Shared by rsd_sbs_step and rsd_sbs_step_static: validation and the two launches on a scratch
// buffer `ws` (device memory, 16-byte aligned, at least rsd_sbs_step_workspace_bytes() long).
static int32_t sbs_check_args(const float *logits, const float *sum_logprob, const float *trunc_gumbel,
                              const int32_t *n_in, int32_t B, int32_t W_in, int32_t V, int32_t W,
                              float inv_temperature, const int32_t *tokens, const int32_t *parent,
                              const float *sum_logprob_out, const float *trunc_gumbel_out,
                              const int32_t *n_out) {
    if (!logits || !sum_logprob || !trunc_gumbel || !n_in || !tokens || !parent ||
        !sum_logprob_out || !trunc_gumbel_out || !n_out)
        return RSD_ERR_NULL;
    if (B < 0 || W_in < 1 || W_in > RSD_K_MAX || W < 1 || W > RSD_K_MAX || V < 1 ||
        V > RSD_VOCAB_MAX || W > V || !aligned16(logits) || !(inv_temperature > 0.f) || ((V & 3) && (int64_t)B * W_in > 1))
        return RSD_ERR_SHAPE;
    return RSD_OK;
}

static int32_t sbs_step_on(char *ws, const float *logits, const float *sum_logprob,
                           const float *trunc_gumbel, const int32_t *n_in, const int32_t *seq_id,
                           const int32_t *node_id, int32_t B, int32_t W_in, int32_t V, int32_t W,
                           float inv_temperature, uint64_t seed, uint32_t step, int32_t *tokens,
                           int32_t *parent, float *sum_logprob_out, float *trunc_gumbel_out,
                           int32_t *n_out, float *lse, hipStream_t stream) {
    const size_t rows = (size_t)B * W_in;
    const int nseg = sbs_segments(B, W_in, V, W);
    const size_t lists = rows * nseg;
    const size_t seg = align_up(lists * W * 4, 256);
    int *row_tok = reinterpret_cast<int *>(ws);
    float *row_pert = reinterpret_cast<float *>(ws + seg);
    float *row_logp = reinterpret_cast<float *>(ws + 2 * seg);
    int *row_cnt = reinterpret_cast<int *>(ws + 3 * seg);
    MaxSum *seg_ms = reinterpret_cast<MaxSum *>(ws + 3 * seg + align_up(lists * 4, 256));

    TopkArgs a{};
    a.logits = logits; a.ld = V; a.V = V; a.k_max = W; a.k_per_row = nullptr;
    a.seq_id = seq_id; a.node_id = node_id; a.n_live = n_in; a.rows_per_seq = W_in;
    a.seq_default_is_b = 1; a.node_default_is_w = 1; a.inv_t = inv_temperature;
    a.seed = seed; a.step = step; a.tokens = row_tok; a.perturbed = row_pert;
    a.logprob = row_logp; a.lse = nullptr; a.count = row_cnt; a.nseg = nseg; a.seg_ms = seg_ms;
    a.raw_lists = 1;
    const int32_t rc = launch_topk(a, (int)rows, stream);
    if (rc != RSD_OK) return rc;

    SbsSelectArgs s{};
    s.row_tok = row_tok; s.row_pert = row_pert; s.row_z = row_logp; s.row_cnt = row_cnt;
    s.seg_ms = seg_ms; s.nseg = nseg; s.lse = lse;
    s.seq_id = seq_id; s.node_id = node_id; s.seed = seed; s.step = step; s.inv_t = inv_temperature;
    s.sum_logprob = sum_logprob; s.trunc_gumbel = trunc_gumbel; s.n_in = n_in;
    s.W_in = W_in; s.W = W; s.V = V; s.tokens = tokens; s.parent = parent;
    s.sum_out = sum_logprob_out; s.gum_out = trunc_gumbel_out; s.n_out = n_out;
    hipLaunchKernelGGL(sbs_select_kernel, dim3(B), dim3(256), 0, stream, s);
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}

extern "C" int32_t rsd_sbs_step(const float *logits, const float *sum_logprob,
                                const float *trunc_gumbel, const int32_t *n_in,
                                const int32_t *seq_id, const int32_t *node_id, int32_t B,
                                int32_t W_in, int32_t V, int32_t W, float inv_temperature,
                                uint64_t seed, uint32_t step, int32_t *tokens, int32_t *parent,
                                float *sum_logprob_out, float *trunc_gumbel_out, int32_t *n_out,
                                float *lse, void *workspace, size_t workspace_bytes, void *stream) {
    const int32_t bad = sbs_check_args(logits, sum_logprob, trunc_gumbel, n_in, B, W_in, V, W, inv_temperature,
                                       tokens, parent, sum_logprob_out, trunc_gumbel_out, n_out);
    if (bad != RSD_OK) return bad;
    if (B == 0) return RSD_OK;
    const size_t need = rsd_sbs_step_workspace_bytes(B, W_in, V, W);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return RSD_ERR_WORKSPACE;
    return sbs_step_on(static_cast<char *>(workspace), logits, sum_logprob, trunc_gumbel, n_in, seq_id,
                       node_id, B, W_in, V, W, inv_temperature, seed, step, tokens, parent,
                       sum_logprob_out, trunc_gumbel_out, n_out, lse, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------
// The same step for callers that may not allocate: the per-row candidate lists live in a
// device array of this library instead of a caller's workspace.  Every GPU holds its own copy
// of the array at its own address, resolved once per device and kept.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[RSD_SBS_STATIC_SCRATCH_BYTES];

constexpr int kStaticDevicesMax = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kStaticDevicesMax];  // device address of `scratch` on device i, or null

extern "C" int32_t rsd_sbs_step_static(const float *logits, const float *sum_logprob,
                                       const float *trunc_gumbel, const int32_t *n_in,
                                       const int32_t *seq_id, const int32_t *node_id, int32_t B,
                                       int32_t W_in, int32_t V, int32_t W, float inv_temperature,
                                       uint64_t seed, uint32_t step, int32_t *tokens, int32_t *parent,
                                       float *sum_logprob_out, float *trunc_gumbel_out,
                                       int32_t *n_out, float *lse, void *stream) {
    const int32_t bad = sbs_check_args(logits, sum_logprob, trunc_gumbel, n_in, B, W_in, V, W, inv_temperature,
                                       tokens, parent, sum_logprob_out, trunc_gumbel_out, n_out);
    if (bad != RSD_OK) return bad;
    if (rsd_sbs_step_workspace_bytes(B, W_in, V, W) > (size_t)RSD_SBS_STATIC_SCRATCH_BYTES)
        return RSD_ERR_TOO_LARGE;
    if (B == 0) return RSD_OK;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticDevicesMax) return RSD_ERR_LAUNCH;
    void *ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            // (in host code the array's name is only a handle: the device address comes from here)
            void *p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RSD_ERR_LAUNCH;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    // Nothing in the buffer has to start at zero: the Gumbel kernel writes every list slot, count
    // and partial normaliser that the select kernel reads.
    return sbs_step_on(static_cast<char *>(ptr), logits, sum_logprob, trunc_gumbel, n_in, seq_id, node_id,
                       B, W_in, V, W, inv_temperature, seed, step, tokens, parent, sum_logprob_out,
                       trunc_gumbel_out, n_out, lse, (hipStream_t)stream);
}
