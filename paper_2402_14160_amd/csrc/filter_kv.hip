// FilterKVCache (Alg. 2 / Alg. 7 step 4): append the key/value rows of the root and of the
// accepted nodes to the cache.  A pure gather: (1 + n_accepted) * H_kv rows of D elements per
// sequence, for K and for V, so the launch is latency-bound; one workgroup per (sequence, head),
// one wave per row pair, 16-byte accesses.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/rsd.h"

namespace rsd {

struct FilterArgs {
    char *kc, *vc;              // cache, byte strides sb / sh / sp
    const char *kt, *vt;        // tree rows [B, H, N, D] contiguous
    int64_t sb, sh, sp;
    int B, H, N, cap, row_bytes, L;
    const int *plen, *acc, *nacc;
    int *new_len;
    uint32_t *flags;
};

// grid (H, B), 4 waves: wave w copies path slots w, w + 4, ...; slot 0 is the root, slot j >= 1
// the (j-1)-th accepted node
__global__ __launch_bounds__(256) void filter_kv_kernel(FilterArgs a) {
    const int h = blockIdx.x, b = blockIdx.y;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int plen = min(max(a.plen[b], 0), a.cap);
    const int nacc = min(max(a.nacc[b], 0), a.L);
    if (h == 0 && threadIdx.x == 0) {
        const int want = plen + 1 + nacc;
        a.new_len[b] = min(want, a.cap);
        if (a.flags) a.flags[b] = want > a.cap ? 1u : 0u;
    }
    for (int j = wave; j <= nacc; j += 4) {
        const int pos = plen + j;
        if (pos >= a.cap) break;  // dropped, reported through the flag
        int node = j == 0 ? 0 : a.acc[(int64_t)b * a.L + (j - 1)];
        node = min(max(node, 0), a.N - 1);  // an invalid id never leaves the tree buffers
        const int64_t src = (((int64_t)b * a.H + h) * a.N + node) * a.row_bytes;
        const int64_t dst = (int64_t)b * a.sb + (int64_t)h * a.sh + (int64_t)pos * a.sp;
        for (int off = lane * 16; off < a.row_bytes; off += 64 * 16) {
            *reinterpret_cast<uint4 *>(a.kc + dst + off) = *reinterpret_cast<const uint4 *>(a.kt + src + off);
            *reinterpret_cast<uint4 *>(a.vc + dst + off) = *reinterpret_cast<const uint4 *>(a.vt + src + off);
        }
    }
}

}  // namespace rsd

using namespace rsd;

extern "C" int32_t rsd_filter_kv_cache(void *k_cache, void *v_cache, const void *k_tree,
                                       const void *v_tree, int32_t dtype, int32_t B, int32_t H_kv,
                                       int32_t N_max, int32_t D, int32_t capacity,
                                       int64_t cache_stride_b, int64_t cache_stride_h,
                                       int64_t cache_stride_p, const int32_t *prefix_len,
                                       const int32_t *accepted_nodes, int32_t depth_max,
                                       const int32_t *n_accepted, int32_t *prefix_len_out,
                                       uint32_t *flags, void *stream) {
    if (!k_cache || !v_cache || !k_tree || !v_tree || !prefix_len || !n_accepted || !prefix_len_out)
        return RSD_ERR_NULL;
    if (depth_max > 0 && !accepted_nodes) return RSD_ERR_NULL;
    if (dtype != RSD_DTYPE_BF16 && dtype != RSD_DTYPE_F32) return RSD_ERR_UNSUPPORTED;
    const int esz = dtype == RSD_DTYPE_BF16 ? 2 : 4;
    if (B < 0 || H_kv < 1 || N_max < 1 || N_max > RSD_NODES_MAX || D < 1 || capacity < 0 ||
        depth_max < 0 || depth_max > RSD_NODES_MAX)
        return RSD_ERR_SHAPE;
    const int64_t row_bytes = (int64_t)D * esz;
    auto misaligned = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; };
    if (row_bytes % 16 || misaligned(k_cache) || misaligned(v_cache) || misaligned(k_tree) ||
        misaligned(v_tree) || (cache_stride_b * esz) % 16 || (cache_stride_h * esz) % 16 ||
        (cache_stride_p * esz) % 16 || cache_stride_p < D)
        return RSD_ERR_SHAPE;
    if (B == 0) return RSD_OK;
    FilterArgs a;
    a.kc = static_cast<char *>(k_cache);
    a.vc = static_cast<char *>(v_cache);
    a.kt = static_cast<const char *>(k_tree);
    a.vt = static_cast<const char *>(v_tree);
    a.sb = cache_stride_b * esz;
    a.sh = cache_stride_h * esz;
    a.sp = cache_stride_p * esz;
    a.B = B; a.H = H_kv; a.N = N_max; a.cap = capacity; a.row_bytes = (int)row_bytes; a.L = depth_max;
    a.plen = prefix_len; a.acc = accepted_nodes; a.nacc = n_accepted;
    a.new_len = prefix_len_out; a.flags = flags;
    hipLaunchKernelGGL(filter_kv_kernel, dim3(H_kv, B), dim3(256), 0,
                       static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? RSD_OK : RSD_ERR_LAUNCH;
}
