// Host-only entry points of the C ABI: version, status text, tree validation.
#include "../../include/rsd.h"

extern "C" int32_t rsd_version(void) { return 100; }

extern "C" const char *rsd_status_string(int32_t status) {
    switch (status) {
        case RSD_OK: return "ok";
        case RSD_ERR_NULL: return "a required pointer is NULL";
        case RSD_ERR_SHAPE: return "a size is out of range or a pointer/stride is misaligned";
        case RSD_ERR_TREE: return "tree violates the layout contract (root first, parent[i] < i)";
        case RSD_ERR_WORKSPACE: return "workspace missing, too small or not 16-byte aligned";
        case RSD_ERR_LAUNCH: return "the HIP runtime refused a launch";
        case RSD_ERR_UNSUPPORTED: return "request outside what the kernels implement";
        case RSD_ERR_TOO_LARGE: return "request needs more scratch than the library's fixed-size buffer holds";
        default: return "unknown status";
    }
}

extern "C" int32_t rsd_validate_tree(const int32_t *parent_host, int32_t n_nodes) {
    if (!parent_host) return RSD_ERR_NULL;
    if (n_nodes < 1 || n_nodes > RSD_NODES_MAX) return RSD_ERR_SHAPE;
    if (parent_host[0] != -1) return RSD_ERR_TREE;
    for (int32_t i = 1; i < n_nodes; ++i)
        if (parent_host[i] < 0 || parent_host[i] >= i) return RSD_ERR_TREE;
    return RSD_OK;
}
