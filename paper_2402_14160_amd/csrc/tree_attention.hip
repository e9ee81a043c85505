// Tree-masked attention of the draft-tree tokens (Sec. 3.2.2, tree evaluation;
// mask of Alg. 5): every query row attends the cached prefix plus the tree
// nodes on its own root path.
//
// bf16 path (gfx950 MFMA, fp32 accumulate).  One workgroup = 4 waves owns 64
// "stacked" query rows of one (sequence, KV head): the N tree rows of the
// H_q/H_kv query heads that share the KV head are stacked so that K and V are
// read once per group.  Keys are streamed in tiles of 64 through LDS; each
// wave owns 16 query rows and computes, with v_mfma_f32_16x16x32_bf16,
//     S^T = K Q^T      (keys x queries)     then     O^T += V^T P^T.
// In this orientation a lane holds scores of ONE query, so the running softmax
// maximum and the rescale factor are per-lane scalars, and the fp32 scores of
// two 16-key tiles are, after conversion to bf16, already laid out as the B
// operand of the second product: P never goes through LDS.  K and V tiles go from
// global memory straight into LDS (global_load_lds, 16 bytes per lane, no staging
// registers), row-major, with the 16-byte chunks of every row XOR-swizzled by the row
// index so that all fragment reads are bank-conflict free without padding; the V^T
// operand is fetched with the gfx950 transposing LDS read (ds_read_b64_tr_b16), which
// hands each lane four keys of one head-dim column.  The tree mask is an ancestor bit-set per node (a node's
// set is its parent's set plus itself), applied only to the tree-key tiles.
//
// A long prefix can be split over several workgroups (flash-decoding style);
// a small second kernel merges the partial (max, sum, output) triples.
#include <hip/hip_runtime.h>
#include <type_traits>
#include <math.h>

#include "../../include/rsd.h"
#include "rsd_device.hpp"

namespace rsd {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr int kTile = 64;          // keys per LDS tile
constexpr int kRowsPerBlock = 64;  // stacked query rows per workgroup (4 waves x 16)
constexpr int kAttnThreads = 256;
constexpr int kAncWords = RSD_NODES_MAX / 64;

struct AttnArgs {
    const void *q, *kp, *vp, *kt, *vt;
    int B, Hq, Hkv, N, D, P_max;   // B: sequences per layer
    int L;                         // layers in this launch; a "batch index" below counts (layer, sequence) pairs
    int64_t lq, lp, lt, lo, ll;    // layer strides in elements: q, prefix K/V, tree K/V, out, lse_out
    int64_t sb, sh, sp;  // prefix strides in elements
    const int *plen;
    const int *nn;
    const int *par;
    float scale_log2;  // softmax scale * log2(e)
    int splits;     // prefix splits of this launch
    int ws_splits;  // split stride of the partial-result workspace (largest split count)
    int row_blocks;
    int row_base;   // first stacked row covered by this launch
    float *out;
    float *lse_out;
    float *ws_o;  // [B,Hq,N,splits,D]
    float *ws_m;  // [B,Hq,N,splits]  running max (log2 domain)
    float *ws_l;  // [B,Hq,N,splits]  running sum
};

// Workgroup -> (sequence, KV head, row block, prefix split).  The launch is one-dimensional
// and consecutive workgroup ids go round-robin to the 8 XCDs, each with its own L2.  The
// ids that land on one XCD are mapped to consecutive work items, so the row blocks (and
// splits) that stream the same K/V rows share an L2 and run at about the same time.
constexpr int kXcds = 8;

__device__ __forceinline__ void decode_block(const AttnArgs &a, int &b, int &kvh, int &rb, int &sp) {
    const int nblk = gridDim.x, i = blockIdx.x;
    const int per = nblk / kXcds, rem = nblk % kXcds;
    const int xcd = i % kXcds, slot = i / kXcds;
    int item = xcd * per + min(xcd, rem) + slot;
    sp = item % a.splits; item /= a.splits;
    rb = item % a.row_blocks; item /= a.row_blocks;
    kvh = item % a.Hkv;
    b = item / a.Hkv;
}

// Ancestor-or-self bit-sets of all nodes of one tree into `anc` ([n][kAncWords]).
// Parent values are clamped into [0, j-1], so the walk always terminates.
// The parent array goes to LDS first (one round trip): the walk up the tree is then a chain of
// LDS reads instead of one dependent global load per level.  Contains a barrier: every thread of
// the workgroup must call it.
__device__ __forceinline__ void build_ancestors(const int *gpar, int n, uint64_t *anc, int threads) {
    __shared__ int par[RSD_NODES_MAX];
    for (int i = threadIdx.x; i < n; i += threads) par[i] = gpar[i];
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += threads) {
        uint64_t w[kAncWords];
#pragma unroll
        for (int k = 0; k < kAncWords; ++k) w[k] = 0;
        int j = i;
        for (int guard = 0; guard <= n; ++guard) {
#pragma unroll
            for (int k = 0; k < kAncWords; ++k)
                if ((j >> 6) == k) w[k] |= 1ull << (j & 63);
            if (j <= 0) break;
            int p = par[j];
            p = min(max(p, 0), j - 1);
            j = p;
        }
#pragma unroll
        for (int k = 0; k < kAncWords; ++k) anc[i * kAncWords + k] = w[k];
    }
}

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;

// Swizzle of the 16-byte chunks of tile row r: chunk c is stored at position c ^ swz(r).
// For 16 chunks per row (D = 128) the four row bits are permuted so that (a) 16 consecutive
// rows give 16 different values (K fragments: one chunk of 16 or 32 consecutive rows),
// (b) 4 consecutive rows differ in the two high bits while rows 4 and 8 apart differ in the
// low bits (V fragments: four-row runs, two or four neighbouring chunks).
template <int D>
__device__ __forceinline__ int swz(int r) {
    if (D == 128) return ((r & 3) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1);
    return (r >> 1) & 7;  // 8 chunks per row: two rows span the 64 banks
}

// (The K/V tile loads carry the non-temporal cache policy, kStreamPolicy: every K/V byte is used by
// the workgroups of one (sequence, KV head) only, at about the same time.)
// One 64-row tile of K and of V from global memory into LDS.  Wave w, instruction it fills
// 64 consecutive chunk positions (4 or 8 rows); a lane fetches the chunk that belongs at its
// position.  Rows at or beyond `limit` re-read the last valid row (finite data; their scores
// are masked), so no lane is ever switched off and no LDS byte is left stale.
template <int D, int THREADS>
__device__ __forceinline__ void stage_tile(const __bf16 *ksrc, const __bf16 *vsrc, int64_t stride,
                                           int row0, int limit, __bf16 *kdst, __bf16 *vdst) {
    constexpr int DCH = D / 8;          // chunks per row
    constexpr int RPI = 64 / DCH;       // rows per wave instruction
    constexpr int NIT = kTile / (RPI * (THREADS / 64));
    static_assert(NIT >= 1, "tile smaller than one pass of the workgroup");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int rbase = (it * (THREADS / 64) + wave) * RPI;
        const int r = rbase + lane / DCH;
        const int c = (lane % DCH) ^ swz<D>(r);
        const int rs = min(row0 + r, limit - 1);
        const int64_t off = (int64_t)rs * stride + c * 8;
        __builtin_amdgcn_global_load_lds((global_void *)(ksrc + off), (lds_void *)(kdst + rbase * D), 16, 0, kStreamPolicy);
        __builtin_amdgcn_global_load_lds((global_void *)(vsrc + off), (lds_void *)(vdst + rbase * D), 16, 0, kStreamPolicy);
    }
}

// The same for a tile that lies wholly below `limit`: the per-thread part of the source offset
// (`lane_off` bytes: the thread's row within one pass of the workgroup and its swizzled chunk)
// never changes; `ksrc` / `vsrc` are the wave-uniform byte addresses of the tile's first row,
// `pass_bytes` the distance between the rows of consecutive passes, and the LDS destinations
// are computed from the scalar wave index `wave_s`.  Requires that `lane_off` fits 32 bits.
template <int D, int THREADS>
__device__ __forceinline__ uint32_t stage_lane_offset(int64_t stride) {
    constexpr int DCH = D / 8, RPI = 64 / DCH;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = wave * RPI + lane / DCH;  // the swizzle only sees r % 16, equal in every pass
    const int c = (lane % DCH) ^ swz<D>(r);
    return (uint32_t)((r * stride + c * 8) * 2);
}

template <int D, int THREADS>
__device__ __forceinline__ void stage_tile_full(const char *ksrc, const char *vsrc, int64_t pass_bytes,
                                                uint32_t lane_off, int wave_s, __bf16 *kdst, __bf16 *vdst) {
    constexpr int DCH = D / 8, RPI = 64 / DCH, WAVES = THREADS / 64;
    constexpr int NIT = kTile / (RPI * WAVES);
    static_assert((RPI * WAVES) % 16 == 0 || NIT == 1, "swizzle must repeat from pass to pass");
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int rbase = (it * WAVES + wave_s) * RPI;
        const char *kb = ksrc + it * pass_bytes;  // wave-uniform
        const char *vb = vsrc + it * pass_bytes;
        __builtin_amdgcn_global_load_lds((global_void *)(kb + lane_off), (lds_void *)(kdst + rbase * D), 16, 0, kStreamPolicy);
        __builtin_amdgcn_global_load_lds((global_void *)(vb + lane_off), (lds_void *)(vdst + rbase * D), 16, 0, kStreamPolicy);
    }
}

// Number of global->LDS load instructions one thread issues per staged tile (K and V).
template <int D, int THREADS>
constexpr int tile_loads_per_thread() { return 2 * (kTile / ((64 / (D / 8)) * (THREADS / 64))); }

// Wait until at most PENDING of this wave's global->LDS loads are still in flight (loads
// complete in issue order, so everything older than the newest PENDING has landed).
template <int PENDING>
__device__ __forceinline__ void wait_tile_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PENDING) : "memory"); }

// Transposing LDS read: within each block of 16 lanes, lane i supplies the address of four
// contiguous 16-bit elements and receives element (i % 4) of the loads of lanes
// i/4, 4 + i/4, 8 + i/4 and 12 + i/4.  Seen as a 4 x 16 tile (row k read by lanes 4k..4k+3,
// four columns each), lane i ends up with column i of all four rows.
__device__ __forceinline__ bf16x4 lds_read_tr(const __bf16 *p) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)(p));
}

// Sum of 16 probabilities as the matrix instruction will see them (after rounding to bf16), so
// that the row sum normalises exactly the weights that multiply V: with the unrounded sum a row
// dominated by one key is off by that key's rounding error (up to 2^-8 relative) whenever its
// exponential is not a power of two.  v_dot2_f32_bf16 adds two entries per instruction.
__device__ __forceinline__ float rounded_sum(const bf16x8 &p0, const bf16x8 &p1) {
    const bf16x2 ones = {(__bf16)1.f, (__bf16)1.f};
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const bf16x2 a = {p0[2 * e], p0[2 * e + 1]}, b = {p1[2 * e], p1[2 * e + 1]};
        s0 = __builtin_amdgcn_fdot2_f32_bf16(a, ones, s0, false);
        s1 = __builtin_amdgcn_fdot2_f32_bf16(b, ones, s1, false);
    }
    return s0 + s1;
}

template <int D>
__global__ __launch_bounds__(kAttnThreads, 2) void tree_attn_bf16_kernel(AttnArgs a) {
    constexpr int KS = D / 32;        // k-steps of the first product
    constexpr int DT = D / 16;        // output tiles of the second product
    extern __shared__ __align__(16) unsigned char smem[];
    __bf16 *Ks = reinterpret_cast<__bf16 *>(smem);          // [2][kTile][D], swizzled chunks
    __bf16 *Vs = Ks + 2 * kTile * D;                        // [2][kTile][D], swizzled chunks
    uint64_t *anc = reinterpret_cast<uint64_t *>(Vs + 2 * kTile * D);  // [N][kAncWords]

    int b, kvh, rb, sp;
    decode_block(a, b, kvh, rb, sp);
    const int layer = b / a.B, bs = b - layer * a.B;  // the tree and the prefix length are the sequence's
    const int n = min(max(a.nn[bs], 0), a.N);
    const int plen = min(max(a.plen[bs], 0), a.P_max);
    const int G = a.Hq / a.Hkv;
    const int rows = G * n;
    if (a.row_base + rb * kRowsPerBlock >= rows) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c16 = lane & 15, g = lane >> 4;
    const bool do_tree = (sp == a.splits - 1);

    // ---- this lane's query ------------------------------------------------
    const int R = a.row_base + rb * kRowsPerBlock + wave * 16 + c16;
    const bool qvalid = R < rows;
    const int hq = kvh * G + (qvalid ? R / n : 0);
    const int qi = qvalid ? R % n : 0;
    const __bf16 *qptr = reinterpret_cast<const __bf16 *>(a.q) + layer * a.lq + (((int64_t)bs * a.Hq + hq) * a.N + qi) * D;
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (qvalid) {
            qf[ks] = *reinterpret_cast<const bf16x8 *>(qptr + ks * 32 + g * 8);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[ks][e] = (__bf16)0.f;
        }
    }

    // ---- tile schedule ------------------------------------------------------
    const int Tp = (plen + kTile - 1) / kTile, Tt = (n + kTile - 1) / kTile;
    const int t0 = (int)((int64_t)Tp * sp / a.splits), t1 = (int)((int64_t)Tp * (sp + 1) / a.splits);
    const int npre = t1 - t0;
    const int ntiles = npre + (do_tree ? Tt : 0);

    const __bf16 *kp = reinterpret_cast<const __bf16 *>(a.kp) + layer * a.lp + (int64_t)bs * a.sb + (int64_t)kvh * a.sh;
    const __bf16 *vp = reinterpret_cast<const __bf16 *>(a.vp) + layer * a.lp + (int64_t)bs * a.sb + (int64_t)kvh * a.sh;
    const __bf16 *kt = reinterpret_cast<const __bf16 *>(a.kt) + layer * a.lt + ((int64_t)bs * a.Hkv + kvh) * a.N * D;
    const __bf16 *vt = reinterpret_cast<const __bf16 *>(a.vt) + layer * a.lt + ((int64_t)bs * a.Hkv + kvh) * a.N * D;

    // (a full prefix tile is staged from wave-uniform addresses plus one per-thread offset that
    // never changes; ragged and tree tiles take the general path)
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const bool lean_stage = a.sp < (1 << 24);  // per-thread byte offset fits 32 bits
    const uint32_t lane_off = stage_lane_offset<D, kAttnThreads>(lean_stage ? a.sp : 0);
    const int64_t pass_bytes = (int64_t)(kAttnThreads / 64) * (64 / (D / 8)) * a.sp * 2;
    const int64_t tile_bytes = (int64_t)kTile * a.sp * 2;
    int64_t pre_off = (int64_t)t0 * tile_bytes;  // byte offset of the next prefix tile (staged in order)
    auto stage = [&](int u) {  // tile u of this block's schedule into buffer u & 1
        const int buf = u & 1;
        __bf16 *kd = Ks + buf * kTile * D, *vd = Vs + buf * kTile * D;
        if (u < npre) {
            const int row0 = (t0 + u) * kTile;
            if (lean_stage && row0 + kTile <= plen)
                stage_tile_full<D, kAttnThreads>(reinterpret_cast<const char *>(kp) + pre_off,
                                                 reinterpret_cast<const char *>(vp) + pre_off, pass_bytes,
                                                 lane_off, wave_s, kd, vd);
            else
                stage_tile<D, kAttnThreads>(kp, vp, a.sp, row0, plen, kd, vd);
            pre_off += tile_bytes;
        } else {
            stage_tile<D, kAttnThreads>(kt, vt, D, (u - npre) * kTile, n, kd, vd);
        }
    };

    floatx4 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    if (ntiles > 0) stage(0);
    // (after the first tile and the query rows have been asked for: one round trip for all three)
    if (do_tree) build_ancestors(a.par + (int64_t)bs * a.N, n, anc, kAttnThreads);
    wait_tile_loads<0>();
    __syncthreads();

    // Full prefix tiles (nearly all of them) run a mask-free copy of the tile body; the ragged last
    // prefix tile and the tree tiles the masked one.  The running maximum m (of scale * score, in
    // log2 units) is only raised when some row of the wave exceeds it by more than kSlack16, so the
    // common tile has no rescale of the accumulators; p <= 2^kSlack16 keeps bf16's relative precision.
    constexpr float kSlack16 = 8.f;
    const int nfull = min(max(plen / kTile - t0, 0), npre);
    auto iteration = [&](int u, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int buf = u & 1;
        if (u + 1 < ntiles) stage(u + 1);  // lands while this tile is consumed

        // ---- S^T = K Q^T for the 64 keys of this tile ----------------------
        // lane (c16, g) reads chunk 4 ks + g of tile row 16 t + c16 (swizzle depends on c16 only)
        const __bf16 *kb = Ks + buf * kTile * D + c16 * D;
        const int ksw = swz<D>(c16);
        floatx4 s[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            s[t] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kb + t * 16 * D + (((ks * 4 + g) ^ ksw) << 3));
                s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[ks], s[t], 0, 0, 0);
            }
        }

        // ---- mask, online softmax (scores stay unscaled until the exponent) -----
        float mx = -INFINITY;
        if constexpr (MASKED) {
            const bool is_tree = u >= npre;
            const int row0 = is_tree ? (u - npre) * kTile : (t0 + u) * kTile;
            const int limit = is_tree ? n : plen;
            uint64_t vis = ~0ull;
            if (is_tree) vis = anc[qi * kAncWords + (u - npre)];
            if (row0 + kTile > limit) {
                const int nv = limit - row0;  // 1..63
                vis &= (nv >= 64) ? ~0ull : ((1ull << nv) - 1ull);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int kk = t * 16 + g * 4 + r;
                    const float v = ((vis >> kk) & 1ull) ? s[t][r] : -INFINITY;
                    s[t][r] = v;
                    mx = fmaxf(mx, v);
                }
            }
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t) mx = fmaxf(mx, fmaxf(fmaxf(s[t][0], s[t][1]), fmaxf(s[t][2], s[t][3])));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        mx *= a.scale_log2;  // (the scale is positive)
        if (__any(mx > m + kSlack16)) {  // (m = -inf at the start: any finite score raises it)
            const float m_new = fmaxf(m, mx);
            const float m_to = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = exp2f(m - m_to);
            m = m_new;
            l *= alpha;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
        }
        const float neg_ref = (m == -INFINITY) ? 0.f : -m;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int r = 0; r < 4; ++r) s[t][r] = __builtin_amdgcn_exp2f(fmaf(s[t][r], a.scale_log2, neg_ref));
        }

        // ---- O^T += V^T P^T ---------------------------------------------------
        bf16x8 pf[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[j][e] = (__bf16)s[2 * j + (e >> 2)][e & 3];
        }
        l += rounded_sum(pf[0], pf[1]);
        // lane (c16, g) of the A operand needs V[key][16 dt + c16] for the keys
        // 32 j + 16 a + 4 g + r (a = 0,1; r = 0..3): two transposing reads, in which this
        // lane loads row 32 j + 16 a + 4 g + c16 / 4, columns 16 dt + 4 (c16 % 4) .. + 3.
        const int vrow = g * 4 + (c16 >> 2);       // + 32 j + 16 a: the swizzle sees vrow only
        const __bf16 *vb = Vs + buf * kTile * D + vrow * D + (c16 & 1) * 4;
        const int vsw = swz<D>(vrow), vch = (c16 >> 1) & 1;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const int voff = ((dt * 2 + vch) ^ vsw) << 3;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const bf16x4 lo = lds_read_tr(vb + (j * 32) * D + voff);
                const bf16x4 hi = lds_read_tr(vb + (j * 32 + 16) * D + voff);
                const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[j], o[dt], 0, 0, 0);
            }
        }

        wait_tile_loads<0>();
        __syncthreads();
    };
    {
        int u = 0;
        for (; u < nfull; ++u) iteration(u, std::false_type{});
        for (; u < ntiles; ++u) iteration(u, std::true_type{});
    }

    // ---- epilogue -----------------------------------------------------------
    float lt = l + __shfl_xor(l, 16, kWave);
    lt += __shfl_xor(lt, 32, kWave);
    if (!qvalid) return;
    const int64_t orow = ((int64_t)b * a.Hq + hq) * a.N + qi;       // row of the partial-result workspace
    const int64_t orow_s = ((int64_t)bs * a.Hq + hq) * a.N + qi;   // row inside the layer
    if (a.splits == 1) {
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        float *dst = a.out + layer * a.lo + orow_s * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            float4 v = make_float4(o[dt][0] * inv, o[dt][1] * inv, o[dt][2] * inv, o[dt][3] * inv);
            *reinterpret_cast<float4 *>(dst + dt * 16 + g * 4) = v;
        }
        if (a.lse_out && g == 0) a.lse_out[layer * a.ll + orow_s] = (m + log2f(lt)) * kLn2;
    } else {
        float *dst = a.ws_o + (orow * a.ws_splits + sp) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            float4 v = make_float4(o[dt][0], o[dt][1], o[dt][2], o[dt][3]);
            *reinterpret_cast<float4 *>(dst + dt * 16 + g * 4) = v;
        }
        if (g == 0) {
            a.ws_m[orow * a.ws_splits + sp] = m;
            a.ws_l[orow * a.ws_splits + sp] = lt;
        }
    }
}


// ---------------------------------------------------------------------------
// Variant for many stacked rows (grouped-query attention): 4 waves x 32 query rows with
// v_mfma_f32_32x32x16_bf16.  Same orientation (S^T = K Q^T, O^T += V^T P^T); every K / V
// fragment read from LDS now feeds a 32 x 32 tile, halving LDS traffic per flop, and the
// wider row block re-reads K and V from L2 half as often.
// C layout of the 32x32 tile: lane l holds column l % 32 and rows 8 (r / 4) + 4 (l / 32) + r % 4
// for its registers r = 0..15; registers 8 m .. 8 m + 7 of a score tile are therefore the
// eight key slots lane group l / 32 feeds to the m-th 16-key step of the second product.
// ---------------------------------------------------------------------------
typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int kRowsPerBlock32 = 128;

__device__ __forceinline__ float max_across_halves(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float sum_across_halves(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D, int WAVES, int STAGES, bool EXACT>
__device__ __forceinline__ bool attn_w32_body(const AttnArgs &a, unsigned char *smem) {
    constexpr int THREADS = WAVES * 64;
    constexpr int RPB = WAVES * 32;  // stacked query rows per workgroup
    constexpr int LOADS = tile_loads_per_thread<D, THREADS>();
    static_assert(STAGES == 2 || STAGES == 3, "ring depth");
    constexpr int KS = D / 16;     // k-steps of the first product
    constexpr int DT = D / 32;     // 32-row output tiles of the second product
    constexpr float kRowSumLimit = 0x1p100f;  // fast pass: larger row sums send the block to the exact pass
    __bf16 *Ks = reinterpret_cast<__bf16 *>(smem);                         // [STAGES][kTile][D], swizzled
    __bf16 *Vs = Ks + STAGES * kTile * D;                                  // [STAGES][kTile][D], swizzled
    uint64_t *anc = reinterpret_cast<uint64_t *>(Vs + STAGES * kTile * D);  // [N][kAncWords]

    int b, kvh, rb, sp;
    decode_block(a, b, kvh, rb, sp);
    const int layer = b / a.B, bs = b - layer * a.B;  // the tree and the prefix length are the sequence's
    const int n = min(max(a.nn[bs], 0), a.N);
    const int plen = min(max(a.plen[bs], 0), a.P_max);
    const int G = a.Hq / a.Hkv;
    const int rows = G * n;
    if (a.row_base + rb * RPB >= rows) return false;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q32 = lane & 31, h = lane >> 5;
    const bool do_tree = (sp == a.splits - 1);

    const int R = a.row_base + rb * RPB + wave * 32 + q32;
    const bool qvalid = R < rows;
    const bool wave_active = a.row_base + rb * RPB + wave * 32 < rows;  // wave-uniform
    const int hq = kvh * G + (qvalid ? R / n : 0);
    const int qi = qvalid ? R % n : 0;
    const __bf16 *qptr = reinterpret_cast<const __bf16 *>(a.q) + layer * a.lq + (((int64_t)bs * a.Hq + hq) * a.N + qi) * D;
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        if (qvalid) {
            qf[ks] = *reinterpret_cast<const bf16x8 *>(qptr + ks * 16 + h * 8);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[ks][e] = (__bf16)0.f;
        }
    }

    const int Tp = (plen + kTile - 1) / kTile, Tt = (n + kTile - 1) / kTile;
    const int t0 = (int)((int64_t)Tp * sp / a.splits), t1 = (int)((int64_t)Tp * (sp + 1) / a.splits);
    const int npre = t1 - t0;
    const int ntiles = npre + (do_tree ? Tt : 0);

    const __bf16 *kp = reinterpret_cast<const __bf16 *>(a.kp) + layer * a.lp + (int64_t)bs * a.sb + (int64_t)kvh * a.sh;
    const __bf16 *vp = reinterpret_cast<const __bf16 *>(a.vp) + layer * a.lp + (int64_t)bs * a.sb + (int64_t)kvh * a.sh;
    const __bf16 *kt = reinterpret_cast<const __bf16 *>(a.kt) + layer * a.lt + ((int64_t)bs * a.Hkv + kvh) * a.N * D;
    const __bf16 *vt = reinterpret_cast<const __bf16 *>(a.vt) + layer * a.lt + ((int64_t)bs * a.Hkv + kvh) * a.N * D;

    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    const bool lean_stage = a.sp < (1 << 24);  // per-thread byte offset fits 32 bits
    const uint32_t lane_off = stage_lane_offset<D, THREADS>(lean_stage ? a.sp : 0);
    const int64_t pass_bytes = (int64_t)(THREADS / 64) * (64 / (D / 8)) * a.sp * 2;
    const int64_t tile_bytes = (int64_t)kTile * a.sp * 2;
    int64_t pre_off = (int64_t)t0 * tile_bytes;  // byte offset of the next prefix tile (staged in order)
    auto stage = [&](int u) {  // tile u of this block's schedule into ring buffer u % STAGES
        const int buf = u % STAGES;
        __bf16 *kd = Ks + buf * kTile * D, *vd = Vs + buf * kTile * D;
        if (u < npre) {
            const int row0 = (t0 + u) * kTile;
            if (lean_stage && row0 + kTile <= plen)
                stage_tile_full<D, THREADS>(reinterpret_cast<const char *>(kp) + pre_off,
                                            reinterpret_cast<const char *>(vp) + pre_off, pass_bytes,
                                            lane_off, wave_s, kd, vd);
            else
                stage_tile<D, THREADS>(kp, vp, a.sp, row0, plen, kd, vd);
            pre_off += tile_bytes;
        } else {
            stage_tile<D, THREADS>(kt, vt, D, (u - npre) * kTile, n, kd, vd);
        }
    };

    floatx16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    float m = -INFINITY, l = 0.f;  // running max of the raw scores times scale_log2, partial row sum

    // prologue: STAGES - 1 tiles in flight; tile 0 must have landed
#pragma unroll
    for (int u = 0; u < STAGES - 1; ++u)
        if (u < ntiles) stage(u);
    if (do_tree) build_ancestors(a.par + (int64_t)bs * a.N, n, anc, THREADS);
    if (ntiles > STAGES - 2 && STAGES > 2) {
        if (ntiles > 1) wait_tile_loads<(STAGES - 2) * LOADS>(); else wait_tile_loads<0>();
    } else {
        wait_tile_loads<0>();
    }
    __syncthreads();

    if (!EXACT && wave_active && ntiles > 0) {
        // fixed reference of the fast pass: the row maximum over the first tile (every valid row sees
        // at least one of its keys: a prefix tile is visible to all rows, tree tile 0 holds the root)
        const __bf16 *kb0 = Ks + q32 * D;
        const int ksw0 = swz<D>(q32);
        const bool is_tree = npre == 0;
        const int row0 = is_tree ? 0 : t0 * kTile;
        const int limit = is_tree ? n : plen;
        uint64_t vis = ~0ull;
        if (is_tree) vis = anc[qi * kAncWords];
        if (row0 + kTile > limit) vis &= (1ull << (limit - row0)) - 1ull;
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            floatx16 sv;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kk = t * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                sv[r] = ((vis >> kk) & 1ull) ? 0.f : -INFINITY;
            }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kb0 + t * 32 * D + (((ks * 2 + h) ^ ksw0) << 3));
                sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sv, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sv[r]);
        }
        mx = max_across_halves(mx) * a.scale_log2;
        m = (mx == -INFINITY) ? 0.f : mx;
    }

    // Full prefix tiles (nearly all of them) run the mask-free copy of the loop body in a loop of
    // their own; the ragged last prefix tile and the tree tiles follow in the masked copy.
    const int nfull = min(max(plen / kTile - t0, 0), npre);
    auto iteration = [&](int u, auto masked_tag) {
        constexpr bool MASKED = decltype(masked_tag)::value;
        const int buf = u % STAGES;
        // the buffer of tile u + STAGES - 1 was last read in iteration u - 1
        if (u + STAGES - 1 < ntiles) stage(u + STAGES - 1);

        if (wave_active) {
            // One 64-key tile is processed as two 32-key halves so that, inside this wave's own
            // instruction stream, the exponentials of one half issue in the shadow of the matrix
            // instructions of the other.  (Matrix and vector instructions overlap both inside a
            // wave and across the two waves of a SIMD; the halves give this wave independent work
            // of both kinds at every point, so it does not depend on what the other wave is at.)
            //   S0 = K0 Q^T | max(S0) | S1 = K1 Q^T || P0 = exp2(S0 - m) | max(S1) |
            //   O += V0^T P0 || P1 = exp2(S1 - m) | O += V1^T P1
            // The running maximum m is only raised when some row's new maximum exceeds it by more
            // than kSlack (in log2 units), so the common case has no branch and no rescale between
            // the matrix groups; p <= 2^kSlack keeps bf16's relative precision.
            constexpr float kSlack = 8.f;
            const __bf16 *kb = Ks + buf * kTile * D + q32 * D;
            const int ksw = swz<D>(q32);
            const bool is_tree = u >= npre;
            const int row0 = is_tree ? (u - npre) * kTile : (t0 + u) * kTile;
            const int limit = is_tree ? n : plen;
            uint64_t vis = ~0ull;
            if (MASKED) {
                if (is_tree) vis = anc[qi * kAncWords + (u - npre)];
                if (row0 + kTile > limit) vis &= (1ull << (limit - row0)) - 1ull;
            }
            auto half_max = [&](const floatx16 &sv) -> float {  // scaled row maximum of one half
                float mx = sv[0];
#pragma unroll
                for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sv[r]);
                return max_across_halves(mx) * a.scale_log2;
            };
            // Masked keys enter as -inf in the accumulator the first product starts from (lane
            // group h holds keys 32 t + 8 (r / 4) + 4 h + r % 4 of row q32 in register r of half t).
            auto mask_init = [&](floatx16 &sv, int t) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kk = t * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                    sv[r] = ((vis >> kk) & 1ull) ? 0.f : -INFINITY;
                }
            };
            floatx16 s0, s1;
            bf16x8 pf[4];
            // `first_half_pending`: P of the first half is already formed (kept as fp32 in s0) but
            // not yet multiplied into O, so it moves to the new reference as well
            auto raise_max = [&](float hm, bool first_half_pending) {
                if (__any(hm > m + kSlack)) {
                    const float m_new = fmaxf(m, hm);
                    const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m - m_new);
                    l *= alpha;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
                    if (first_half_pending) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            pf[0][e] = (__bf16)(s0[e] * alpha);
                            pf[1][e] = (__bf16)(s0[8 + e] * alpha);
                        }
                    }
                    m = m_new;
                }
            };
            auto half_exp = [&](floatx16 &sv, bf16x8 &p0, bf16x8 &p1) {
                const float mu = (m == -INFINITY) ? 0.f : m;
#pragma unroll
                for (int r = 0; r < 16; ++r) sv[r] = __builtin_amdgcn_exp2f(fmaf(sv[r], a.scale_log2, -mu));
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p0[e] = (__bf16)sv[e];
                    p1[e] = (__bf16)sv[8 + e];
                }
            };
            auto qk_half = [&](floatx16 &sv, int t) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    // lane (q32, h) reads chunk 2 ks + h of tile row 32 t + q32
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(kb + t * 32 * D + (((ks * 2 + h) ^ ksw) << 3));
                    sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], sv, 0, 0, 0);
                }
            };
            // transposing read: lane i of each 16-lane block loads row (key) i / 4 of the
            // 4-key run, four columns at 16 (block % 2) + 4 (i % 4)
            const int i16 = lane & 15;
            const int vrow = 4 * h + (i16 >> 2);                     // + 16 mm (+ 8 for the second run)
            const int vch = 2 * ((lane >> 4) & 1) + ((i16 >> 1) & 1);  // chunk within the 32-column tile
            const __bf16 *vb = Vs + buf * kTile * D + vrow * D + (i16 & 1) * 4;
            const int vsw_lo = swz<D>(vrow), vsw_hi = swz<D>(vrow + 8);
            auto pv_step = [&](int mm, const bf16x8 &p) {  // keys 16 mm .. 16 mm + 15
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const bf16x4 lo = lds_read_tr(vb + (16 * mm) * D + (((dt * 4 + vch) ^ vsw_lo) << 3));
                    const bf16x4 hi = lds_read_tr(vb + (16 * mm + 8) * D + (((dt * 4 + vch) ^ vsw_hi) << 3));
                    const bf16x8 vf = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p, o[dt], 0, 0, 0);
                }
            };

            if (MASKED) {
                mask_init(s0, 0);
                mask_init(s1, 1);
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) s0[r] = s1[r] = 0.f;
            }
            qk_half(s0, 0);
            if (EXACT) raise_max(half_max(s0), false);
            qk_half(s1, 1);
            half_exp(s0, pf[0], pf[1]);
            if (EXACT) raise_max(half_max(s1), true);
            l += rounded_sum(pf[0], pf[1]);  // (after the rescale, which forms this half's P again)
            pv_step(0, pf[0]);
            pv_step(1, pf[1]);
            half_exp(s1, pf[2], pf[3]);
            l += rounded_sum(pf[2], pf[3]);
            pv_step(2, pf[2]);
            pv_step(3, pf[3]);
        }

        // tile u + 1 must have landed; the STAGES - 2 newer tiles may still be in flight
        if (STAGES > 2 && u + STAGES - 1 < ntiles)
            wait_tile_loads<(STAGES - 2) * LOADS>();
        else
            wait_tile_loads<0>();
        __syncthreads();
    };
    int u = 0;
    for (; u < nfull; ++u) iteration(u, std::false_type{});
    for (; u < ntiles; ++u) iteration(u, std::true_type{});

    // ---- epilogue -------------------------------------------------------------------
    const float lt = sum_across_halves(l);
    if (!EXACT) {
        // every probability is at most its row sum: a row sum below the limit means that no
        // exponential (and no product with V of ordinary magnitude) overflowed
        if (__syncthreads_or(qvalid && !(lt < kRowSumLimit))) return true;  // workgroup-uniform
    }
    if (!qvalid) return false;
    const int64_t orow = ((int64_t)b * a.Hq + hq) * a.N + qi;       // row of the partial-result workspace
    const int64_t orow_s = ((int64_t)bs * a.Hq + hq) * a.N + qi;   // row inside the layer
    if (a.splits == 1) {
        const float inv = lt > 0.f ? 1.f / lt : 0.f;
        float *dst = a.out + layer * a.lo + orow_s * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const float4 v = make_float4(o[dt][4 * rq] * inv, o[dt][4 * rq + 1] * inv,
                                             o[dt][4 * rq + 2] * inv, o[dt][4 * rq + 3] * inv);
                *reinterpret_cast<float4 *>(dst + dt * 32 + 8 * rq + 4 * h) = v;
            }
        if (a.lse_out && h == 0) a.lse_out[layer * a.ll + orow_s] = (m + log2f(lt)) * kLn2;
    } else {
        float *dst = a.ws_o + (orow * a.ws_splits + sp) * D;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const float4 v = make_float4(o[dt][4 * rq], o[dt][4 * rq + 1], o[dt][4 * rq + 2], o[dt][4 * rq + 3]);
                *reinterpret_cast<float4 *>(dst + dt * 32 + 8 * rq + 4 * h) = v;
            }
        if (h == 0) {
            a.ws_m[orow * a.ws_splits + sp] = m;
            a.ws_l[orow * a.ws_splits + sp] = lt;
        }
    }
    return false;
}

// The 32-row kernel proper.  Fast pass with a fixed softmax reference per row, the row maximum
// over the first tile: no row maxima, no rescaling and no branch between the matrix groups of a
// tile.  A workgroup in which some row sum reaches 2^100 (scores about 100 log2 units above the
// reference) repeats its block with the exact running-maximum pass.
template <int D, int WAVES, int STAGES>
__global__ __launch_bounds__(WAVES * 64, WAVES == 4 ? 2 : 1) void tree_attn_bf16_w32_kernel(AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    if (attn_w32_body<D, WAVES, STAGES, false>(a, smem)) attn_w32_body<D, WAVES, STAGES, true>(a, smem);
}

// Merge the per-split partial results of the stacked rows [row_base, row_base + gridDim.x) of
// every (sequence, KV head) pair: one wave per row, `splits` partial results each.
__global__ __launch_bounds__(kWave) void tree_attn_merge_kernel(AttnArgs a) {
    const int R = a.row_base + blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int layer = b / a.B, bs = b - layer * a.B;
    const int n = min(max(a.nn[bs], 0), a.N);
    const int G = a.Hq / a.Hkv;
    if (R >= G * n) return;
    const int hq = kvh * G + R / n, i = R % n;
    const int splits = a.splits;  // at most 32: lane s holds split s
    const int64_t orow = ((int64_t)b * a.Hq + hq) * a.N + i;       // row of the partial-result workspace
    const int64_t orow_s = ((int64_t)bs * a.Hq + hq) * a.N + i;   // row inside the layer
    const int lane = threadIdx.x;
    const float wm = lane < splits ? a.ws_m[orow * a.ws_splits + lane] : -INFINITY;
    const float wl = lane < splits ? a.ws_l[orow * a.ws_splits + lane] : 0.f;
    // the partial outputs do not depend on the weights: the first four splits' values of this
    // lane's (at most two: D <= 128 on this path) columns are asked for in the same round trip
    const float *po = a.ws_o + orow * a.ws_splits * a.D;
    constexpr int kEarly = 4;
    float early[kEarly][2];
#pragma unroll
    for (int s = 0; s < kEarly; ++s) {
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int d = lane + c * kWave;
            early[s][c] = (s < splits && d < a.D) ? po[(int64_t)s * a.D + d] : 0.f;
        }
    }
    const float m = wave_max(wm);
    const float w = (wm == -INFINITY) ? 0.f : exp2f(wm - m);  // weight of this lane's split
    const float lsum = wave_sum(w * wl);
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int d = lane + c * kWave;
        float acc = 0.f;
#pragma unroll
        for (int s = 0; s < kEarly; ++s) acc += read_lane(w, s) * early[s][c];  // (w = 0 beyond the last split)
        if (d < a.D) {
            for (int s = kEarly; s < splits; ++s) acc += __shfl(w, s, kWave) * po[(int64_t)s * a.D + d];
            a.out[layer * a.lo + orow_s * a.D + d] = acc * inv;
        }
    }
    if (a.lse_out && lane == 0) a.lse_out[layer * a.ll + orow_s] = (m + log2f(lsum)) * kLn2;
}

// fp32 inputs (small configurations): one wave per query row, plain ALUs.
__global__ __launch_bounds__(kWave) void tree_attn_f32_kernel(AttnArgs a) {
    __shared__ uint64_t s_anc[kAncWords];
    __shared__ float s_p[kWave];
    __shared__ float s_q[256];
    const int i = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int layer = b / a.B, bs = b - layer * a.B;
    const int n = min(max(a.nn[bs], 0), a.N);
    if (i >= n) return;
    const int plen = min(max(a.plen[bs], 0), a.P_max);
    const int lane = threadIdx.x;
    const int D = a.D;
    const int kvh = hq / (a.Hq / a.Hkv);
    if (lane == 0) {
        uint64_t w[kAncWords];
        for (int k = 0; k < kAncWords; ++k) w[k] = 0;
        int j = i;
        const int *par = a.par + (int64_t)bs * a.N;
        for (int guard = 0; guard <= n; ++guard) {
            w[j >> 6] |= 1ull << (j & 63);
            if (j <= 0) break;
            j = min(max(par[j], 0), j - 1);
        }
        for (int k = 0; k < kAncWords; ++k) s_anc[k] = w[k];
    }
    const float *q = reinterpret_cast<const float *>(a.q) + layer * a.lq + (((int64_t)bs * a.Hq + hq) * a.N + i) * D;
    for (int d = lane; d < D; d += kWave) s_q[d] = q[d];
    __syncthreads();
    const float *kp = reinterpret_cast<const float *>(a.kp) + layer * a.lp + (int64_t)bs * a.sb + (int64_t)kvh * a.sh;
    const float *vp = reinterpret_cast<const float *>(a.vp) + layer * a.lp + (int64_t)bs * a.sb + (int64_t)kvh * a.sh;
    const float *kt = reinterpret_cast<const float *>(a.kt) + layer * a.lt + ((int64_t)bs * a.Hkv + kvh) * a.N * D;
    const float *vt = reinterpret_cast<const float *>(a.vt) + layer * a.lt + ((int64_t)bs * a.Hkv + kvh) * a.N * D;
    float m = -INFINITY, l = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};  // output dims lane, lane+64, lane+128, lane+192
    const int total = plen + n;
    for (int base = 0; base < total; base += kWave) {
        const int j = base + lane;
        float sc = -INFINITY;
        const float *krow = nullptr;
        if (j < plen) {
            krow = kp + (int64_t)j * a.sp;
        } else if (j < total) {
            const int node = j - plen;
            if ((s_anc[node >> 6] >> (node & 63)) & 1ull) krow = kt + (int64_t)node * D;
        }
        if (krow) {
            float dot = 0.f;
            for (int d = 0; d < D; ++d) dot = fmaf(s_q[d], krow[d], dot);
            sc = dot * a.scale_log2;
        }
        const float mx = wave_max(sc);
        const float m_new = fmaxf(m, mx);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = exp2f(m - m_use);
        const float p = exp2f(sc - m_use);
        l = l * alpha + wave_sum(p);
        m = m_new;
        __syncthreads();
        s_p[lane] = p;
        __syncthreads();
        const int cnt = min(kWave, total - base);
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] *= alpha;
        for (int jj = 0; jj < cnt; ++jj) {
            const float pj = s_p[jj];
            if (pj == 0.f) continue;
            const int key = base + jj;
            const float *vrow = key < plen ? vp + (int64_t)key * a.sp : vt + (int64_t)(key - plen) * D;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int d = lane + k * kWave;
                if (d < D) acc[k] = fmaf(pj, vrow[d], acc[k]);
            }
        }
    }
    const int64_t orow = ((int64_t)b * a.Hq + hq) * a.N + i;       // row of the partial-result workspace
    const int64_t orow_s = ((int64_t)bs * a.Hq + hq) * a.N + i;   // row inside the layer
    const float inv = l > 0.f ? 1.f / l : 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int d = lane + k * kWave;
        if (d < D) a.out[layer * a.lo + orow_s * D + d] = acc[k] * inv;
    }
    if (a.lse_out && lane == 0) a.lse_out[layer * a.ll + orow_s] = (m + log2f(l)) * kLn2;
}

static size_t align_up(size_t x, size_t al) { return (x + al - 1) / al * al; }
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// ---------------------------------------------------------------------------
// Launch plan.  The stacked rows of a (sequence, KV head) pair are covered by up to three
// launches: 256-row blocks (8 waves of 32 rows, one workgroup per compute unit: each staged K/V
// tile serves twice the rows), 128-row blocks (4 waves of 32 rows, two workgroups per compute
// unit; also taken for a remainder of at least 96 rows) and 64-row blocks (4 waves of 16 rows).
// Every kernel clips to the rows a sequence really has, so the launches write disjoint output
// rows.  Each launch splits the prefix on its own: only as far as it still fits the chip in one
// round.
// ---------------------------------------------------------------------------
enum AttnVariant { kV16 = 0, kV32x4 = 1, kV32x8 = 2 };
constexpr int kMaxSegments = 3;
constexpr int kMaxSplits = 32;

struct AttnSegment {
    int variant, row_base, row_blocks, splits;
};

static int plan_segments(int dtype, int B, int Hq, int Hkv, int N, int P_max, int requested,
                         AttnSegment seg[kMaxSegments]) {
    const int rows = (Hq / Hkv) * N;
    int nseg = 0, base = 0;
    const int full256 = rows / 256;
    if (full256 > 0) {
        seg[nseg++] = AttnSegment{kV32x8, 0, full256, 1};
        base = full256 * 256;
    }
    int full128 = (rows - base) / 128, rem = rows - base - full128 * 128;
    if (rem >= 96) {  // worth one more 128-row block
        ++full128;
        rem = 0;
    }
    if (full128 > 0) {
        seg[nseg++] = AttnSegment{kV32x4, base, full128, 1};
        base += full128 * 128;
    }
    if (rem > 0) seg[nseg++] = AttnSegment{kV16, base, (rem + 63) / 64, 1};
    const int tiles = (P_max + kTile - 1) / kTile;
    for (int i = 0; i < nseg; ++i) {
        int s = requested;
        if (dtype != RSD_DTYPE_BF16) s = 1;
        if (s <= 0) {
            // The number of splits that minimises the time of the launch in units of one tile of one
            // workgroup: the workgroups run in rounds over the chip's slots (one or two per CU); a
            // round takes tiles per split + about two tiles' worth of set-up, stretched when more
            // workgroups stream at once than HBM feeds at full speed (about 410 of the 16-row and
            // 128-row kernels, measured: a workgroup alone takes ~2 us per 32 KB tile, the chip
            // delivers ~205 tiles per us); the merge launch costs about five tiles once there is
            // more than one split.  A split of fewer than four tiles costs more in set-up and
            // merging than it gains.
            const long blocks = (long)seg[i].row_blocks * Hkv * B;
            const long slots = seg[i].variant == kV32x8 ? 256 : 512;
            const double fed = seg[i].variant == kV32x8 ? 1e9 : 410.0;  // (the 256-row kernel is bound by its arithmetic)
            int smax = tiles / 4 < kMaxSplits ? tiles / 4 : kMaxSplits;
            if (smax < 1) smax = 1;
            double best = 0.0;
            s = 1;
            for (int c = 1; c <= smax; ++c) {
                const double per = (double)tiles / c + 2.0;
                const long total = blocks * c, full_rounds = total / slots, last = total % slots;
                double cost = (double)full_rounds * per * ((double)slots > fed ? (double)slots / fed : 1.0);
                if (last > 0) cost += per * ((double)last > fed ? (double)last / fed : 1.0);
                if (c > 1) cost += 5.0;
                if (c == 1 || cost < best) {
                    best = cost;
                    s = c;
                }
            }
        }
        if (s > kMaxSplits) s = kMaxSplits;  // the merge holds one split per lane
        if (s > tiles) s = tiles;
        if (s < 1) s = 1;
        seg[i].splits = s;
    }
    return nseg;
}

static int max_splits(int dtype, int B, int Hq, int Hkv, int N, int P_max, int requested) {
    AttnSegment seg[kMaxSegments];
    const int nseg = plan_segments(dtype, B, Hq, Hkv, N, P_max, requested, seg);
    int s = 1;
    for (int i = 0; i < nseg; ++i) s = seg[i].splits > s ? seg[i].splits : s;
    return s;
}

template <int D>
static size_t attn_smem_bytes(int N, int stages) {
    return (size_t)stages * 2 * kTile * D * 2 + (size_t)N * kAncWords * 8;
}

// The dynamic-LDS limit of a kernel covers the largest tree; setting it is idempotent and cheap,
// so it is simply set at every launch (no state is kept between calls).
template <typename Kernel>
static hipError_t launch_attn(Kernel kernel, size_t smem_max, size_t smem, dim3 grid, int threads,
                              hipStream_t st, const AttnArgs &a) {
    const hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_max);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(kernel, grid, dim3(threads), smem, st, a);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_segment(const AttnSegment &sg, AttnArgs a, int pairs, hipStream_t st) {
    a.row_base = sg.row_base;
    a.row_blocks = sg.row_blocks;
    a.splits = sg.splits;
    const dim3 grid((unsigned)((long)sg.row_blocks * a.splits * a.Hkv * pairs));
    if (sg.variant == kV32x8)
        return launch_attn(tree_attn_bf16_w32_kernel<D, 8, 2>, attn_smem_bytes<D>(RSD_NODES_MAX, 2),
                           attn_smem_bytes<D>(a.N, 2), grid, 512, st, a);
    if (sg.variant == kV32x4)
        return launch_attn(tree_attn_bf16_w32_kernel<D, 4, 2>, attn_smem_bytes<D>(RSD_NODES_MAX, 2),
                           attn_smem_bytes<D>(a.N, 2), grid, 256, st, a);
    return launch_attn(tree_attn_bf16_kernel<D>, attn_smem_bytes<D>(RSD_NODES_MAX, 2),
                       attn_smem_bytes<D>(a.N, 2), grid, kAttnThreads, st, a);
}

}  // namespace rsd

using namespace rsd;

// Shared by the two entry points: L layers of B sequences each in one set of launches.  The
// launch plan (row blocks, prefix splits) is made for all L * B (layer, sequence) pairs, so a
// small batch that could not fill the chip in one layer does so over its layers.
static size_t attn_workspace_bytes(int32_t dtype, int32_t L, int32_t B, int32_t H_q, int32_t H_kv,
                                   int32_t N_max, int32_t D, int32_t P_max, int32_t num_splits) {
    if (L <= 0 || B <= 0 || H_q <= 0 || H_kv <= 0 || N_max <= 0 || D <= 0 || P_max < 0 || H_q % H_kv) return 0;
    if ((int64_t)L * B > 65535) return 0;
    const int s = max_splits(dtype, L * B, H_q, H_kv, N_max, P_max, num_splits);
    if (s <= 1) return 0;
    const size_t rows = (size_t)L * B * H_q * N_max;
    return align_up(rows * s * D * 4, 256) + 2 * align_up(rows * s * 4, 256);
}

static int32_t attn_launch(const void *q, const void *k_prefix, const void *v_prefix, const void *k_tree,
                           const void *v_tree, int32_t dtype, int32_t L, int64_t q_stride_l,
                           int64_t prefix_stride_l, int64_t tree_stride_l, int64_t out_stride_l,
                           int64_t lse_stride_l, int32_t B, int32_t H_q, int32_t H_kv, int32_t N_max,
                           int32_t D, int32_t P_max, int64_t prefix_stride_b, int64_t prefix_stride_h,
                           int64_t prefix_stride_p, const int32_t *prefix_len, const int32_t *n_nodes,
                           const int32_t *parent, float scale, int32_t num_splits, float *out,
                           float *lse_out, void *workspace, size_t workspace_bytes, void *stream) {
    if (!q || !k_tree || !v_tree || !prefix_len || !n_nodes || !parent || !out) return RSD_ERR_NULL;
    if (P_max > 0 && (!k_prefix || !v_prefix)) return RSD_ERR_NULL;
    if (B < 0 || L < 1 || H_q < 1 || H_kv < 1 || H_q % H_kv || N_max < 1 || N_max > RSD_NODES_MAX ||
        P_max < 0 || num_splits < 0 || (int64_t)L * B > 65535)
        return RSD_ERR_SHAPE;
    if (!(scale > 0.f) || !(scale < INFINITY)) return RSD_ERR_SHAPE;  // (row maxima are taken before scaling)
    if (dtype != RSD_DTYPE_BF16 && dtype != RSD_DTYPE_F32) return RSD_ERR_UNSUPPORTED;
    const int esz = dtype == RSD_DTYPE_BF16 ? 2 : 4;
    const int vec = 16 / esz;
    if (dtype == RSD_DTYPE_BF16 && D != 64 && D != 128) return RSD_ERR_UNSUPPORTED;
    if (dtype == RSD_DTYPE_F32 && (D < 1 || D > 256)) return RSD_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k_tree) || !aligned16(v_tree) || !aligned16(out) ||
        (P_max > 0 && (!aligned16(k_prefix) || !aligned16(v_prefix))))
        return RSD_ERR_SHAPE;
    if (P_max > 0 && dtype == RSD_DTYPE_BF16 &&
        (prefix_stride_b % vec || prefix_stride_h % vec || prefix_stride_p % vec || prefix_stride_p < D))
        return RSD_ERR_SHAPE;
    if (P_max > 0 && dtype == RSD_DTYPE_F32 && prefix_stride_p < D) return RSD_ERR_SHAPE;
    if (L > 1 && (q_stride_l % vec || prefix_stride_l % vec || tree_stride_l % vec || out_stride_l % 4 ||
                  q_stride_l < 0 || prefix_stride_l < 0 || tree_stride_l < 0 || out_stride_l < 0 || lse_stride_l < 0))
        return RSD_ERR_SHAPE;
    if (B == 0) return RSD_OK;

    AttnArgs a{};
    a.q = q; a.kp = k_prefix; a.vp = v_prefix; a.kt = k_tree; a.vt = v_tree;
    a.B = B; a.L = L; a.Hq = H_q; a.Hkv = H_kv; a.N = N_max; a.D = D; a.P_max = P_max;
    a.lq = q_stride_l; a.lp = prefix_stride_l; a.lt = tree_stride_l; a.lo = out_stride_l; a.ll = lse_stride_l;
    a.sb = prefix_stride_b; a.sh = prefix_stride_h; a.sp = prefix_stride_p;
    a.plen = prefix_len; a.nn = n_nodes; a.par = parent;
    a.scale_log2 = (float)((double)scale * 1.4426950408889634);
    a.out = out; a.lse_out = lse_out;
    hipStream_t st = (hipStream_t)stream;
    const int BL = B * L;  // (layer, sequence) pairs: the kernels' batch index

    if (dtype == RSD_DTYPE_F32) {
        a.splits = 1;
        hipLaunchKernelGGL(tree_attn_f32_kernel, dim3(N_max, H_q, BL), dim3(kWave), 0, st, a);
        return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
    }

    AttnSegment seg[kMaxSegments];
    const int nseg = plan_segments(dtype, BL, H_q, H_kv, N_max, P_max, num_splits, seg);
    a.ws_splits = 1;
    for (int i = 0; i < nseg; ++i) a.ws_splits = seg[i].splits > a.ws_splits ? seg[i].splits : a.ws_splits;
    if (a.ws_splits > 1) {
        const size_t need = attn_workspace_bytes(dtype, L, B, H_q, H_kv, N_max, D, P_max, num_splits);
        if (!workspace || workspace_bytes < need || !aligned16(workspace)) return RSD_ERR_WORKSPACE;
        const size_t rows = (size_t)BL * H_q * N_max;
        char *ws = static_cast<char *>(workspace);
        a.ws_o = reinterpret_cast<float *>(ws);
        a.ws_m = reinterpret_cast<float *>(ws + align_up(rows * a.ws_splits * D * 4, 256));
        a.ws_l = reinterpret_cast<float *>(ws + align_up(rows * a.ws_splits * D * 4, 256) +
                                           align_up(rows * a.ws_splits * 4, 256));
    }
    for (int i = 0; i < nseg; ++i) {
        const hipError_t err = D == 128 ? launch_segment<128>(seg[i], a, BL, st) : launch_segment<64>(seg[i], a, BL, st);
        if (err != hipSuccess) return RSD_ERR_LAUNCH;
    }
    const int rows_max = (H_q / H_kv) * N_max;
    for (int i = 0; i < nseg; ++i) {
        if (seg[i].splits <= 1) continue;
        const int row_end = (i + 1 < nseg) ? seg[i + 1].row_base : rows_max;
        a.row_base = seg[i].row_base;
        a.splits = seg[i].splits;
        hipLaunchKernelGGL(tree_attn_merge_kernel, dim3(row_end - seg[i].row_base, H_kv, BL), dim3(kWave), 0, st, a);
        if (hipGetLastError() != hipSuccess) return RSD_ERR_LAUNCH;
    }
    return RSD_OK;
}

extern "C" size_t rsd_tree_attention_workspace_bytes(int32_t dtype, int32_t B, int32_t H_q,
                                                     int32_t H_kv, int32_t N_max, int32_t D,
                                                     int32_t P_max, int32_t num_splits) {
    return attn_workspace_bytes(dtype, 1, B, H_q, H_kv, N_max, D, P_max, num_splits);
}

extern "C" int32_t rsd_tree_attention(const void *q, const void *k_prefix, const void *v_prefix,
                                      const void *k_tree, const void *v_tree, int32_t dtype,
                                      int32_t B, int32_t H_q, int32_t H_kv, int32_t N_max, int32_t D,
                                      int32_t P_max, int64_t prefix_stride_b,
                                      int64_t prefix_stride_h, int64_t prefix_stride_p,
                                      const int32_t *prefix_len, const int32_t *n_nodes,
                                      const int32_t *parent, float scale, int32_t num_splits,
                                      float *out, float *lse_out, void *workspace,
                                      size_t workspace_bytes, void *stream) {
    return attn_launch(q, k_prefix, v_prefix, k_tree, v_tree, dtype, 1, 0, 0, 0, 0, 0, B, H_q, H_kv, N_max, D,
                       P_max, prefix_stride_b, prefix_stride_h, prefix_stride_p, prefix_len, n_nodes, parent,
                       scale, num_splits, out, lse_out, workspace, workspace_bytes, stream);
}

extern "C" size_t rsd_tree_attention_layers_workspace_bytes(int32_t dtype, int32_t L, int32_t B,
                                                            int32_t H_q, int32_t H_kv, int32_t N_max,
                                                            int32_t D, int32_t P_max, int32_t num_splits) {
    return attn_workspace_bytes(dtype, L, B, H_q, H_kv, N_max, D, P_max, num_splits);
}

extern "C" int32_t rsd_tree_attention_layers(const void *q, const void *k_prefix, const void *v_prefix,
                                             const void *k_tree, const void *v_tree, int32_t dtype,
                                             int32_t L, int64_t q_stride_l, int64_t prefix_stride_l,
                                             int64_t tree_stride_l, int64_t out_stride_l,
                                             int64_t lse_stride_l, int32_t B, int32_t H_q, int32_t H_kv,
                                             int32_t N_max, int32_t D, int32_t P_max,
                                             int64_t prefix_stride_b, int64_t prefix_stride_h,
                                             int64_t prefix_stride_p, const int32_t *prefix_len,
                                             const int32_t *n_nodes, const int32_t *parent, float scale,
                                             int32_t num_splits, float *out, float *lse_out,
                                             void *workspace, size_t workspace_bytes, void *stream) {
    return attn_launch(q, k_prefix, v_prefix, k_tree, v_tree, dtype, L, q_stride_l, prefix_stride_l,
                       tree_stride_l, out_stride_l, lse_stride_l, B, H_q, H_kv, N_max, D, P_max,
                       prefix_stride_b, prefix_stride_h, prefix_stride_p, prefix_len, n_nodes, parent, scale,
                       num_splits, out, lse_out, workspace, workspace_bytes, stream);
}
