// Host-side parts of the C ABI that launch no kernels: error reporting and the
// graph handle (CSR validation and placement in HBM or page-locked host memory;
// the graph structure that the samplers of the BGL paper's Sec. 3.1 work on).
#include <cstring>

#include "bgl_internal.h"

namespace bgl {

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

}  // namespace bgl

extern "C" const char *bgl_last_error(void) { return bgl::g_err; }

namespace {

template <typename RP>
int validate_csr(const RP *rp, const int32_t *col, int64_t n, int64_t e)
{
    if (rp[0] != 0) BGL_FAIL(BGL_EINVAL, "row_ptr[0] must be 0");
    for (int64_t v = 0; v < n; ++v) {
        const int64_t d = (int64_t)rp[v + 1] - (int64_t)rp[v];
        if (d < 0) BGL_FAIL(BGL_EINVAL, "row_ptr decreases at node %lld", (long long)v);
        if (d > INT32_MAX) BGL_FAIL(BGL_EINVAL, "degree of node %lld does not fit 31 bits", (long long)v);
    }
    if ((int64_t)rp[n] != e)
        BGL_FAIL(BGL_EINVAL, "row_ptr[num_nodes] = %lld differs from num_edges = %lld",
                 (long long)rp[n], (long long)e);
    for (int64_t i = 0; i < e; ++i)
        if ((uint32_t)col[i] >= (uint32_t)n)
            BGL_FAIL(BGL_EINVAL, "col_idx[%lld] = %d is outside [0, %lld)", (long long)i, col[i],
                     (long long)n);
    return BGL_OK;
}

int device_view(const void *host, const void **dev)
{
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, host) != hipSuccess) {
        (void)hipGetLastError();
        return BGL_EINVAL;
    }
    if (attr.type != hipMemoryTypeHost || !attr.devicePointer) return BGL_EINVAL;
    *dev = attr.devicePointer;
    return BGL_OK;
}

}  // namespace

extern "C" int bgl_graph_load_csr(const void *row_ptr, int row_ptr_bits, const int32_t *col_idx,
                                  int64_t num_nodes, int64_t num_edges, int placement,
                                  bgl_graph_t **out)
try {
    if (!out) BGL_FAIL(BGL_EINVAL, "out is null");
    *out = nullptr;
    if (!row_ptr) BGL_FAIL(BGL_EINVAL, "row_ptr is null");
    if (row_ptr_bits != 32 && row_ptr_bits != 64)
        BGL_FAIL(BGL_EINVAL, "row_ptr_bits must be 32 or 64 (got %d)", row_ptr_bits);
    if (num_nodes < 1 || num_nodes > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "num_nodes must be in [1, 2^31) (got %lld)", (long long)num_nodes);
    if (num_edges < 0) BGL_FAIL(BGL_EINVAL, "num_edges is negative");
    if (row_ptr_bits == 32 && num_edges > INT32_MAX)
        BGL_FAIL(BGL_EINVAL, "num_edges needs 64-bit row offsets");
    if (num_edges > 0 && !col_idx) BGL_FAIL(BGL_EINVAL, "col_idx is null");
    if (placement != BGL_DEVICE && placement != BGL_HOST_PINNED && placement != BGL_HOST_PINNED_COL)
        BGL_FAIL(BGL_EINVAL, "unknown placement %d", placement);

    int rc = row_ptr_bits == 64
                 ? validate_csr(static_cast<const int64_t *>(row_ptr), col_idx, num_nodes, num_edges)
                 : validate_csr(static_cast<const int32_t *>(row_ptr), col_idx, num_nodes, num_edges);
    if (rc != BGL_OK) return rc;

    bgl_graph *g = new (std::nothrow) bgl_graph();
    if (!g) BGL_FAIL(BGL_ENOMEM, "out of host memory");
    g->num_nodes = num_nodes;
    g->num_edges = num_edges;
    g->bits = row_ptr_bits;
    g->placement = placement;
    const size_t rp_bytes = (size_t)(num_nodes + 1) * (row_ptr_bits / 8);
    const size_t col_bytes = (size_t)(num_edges > 0 ? num_edges : 1) * sizeof(int32_t);
    if (placement == BGL_DEVICE) {
        hipError_t e;
        if ((e = hipMalloc(&g->owned_row_ptr, rp_bytes)) != hipSuccess ||
            (e = hipMalloc(&g->owned_col, col_bytes)) != hipSuccess) {
            bgl::set_error("hipMalloc for the graph failed: %s", hipGetErrorString(e));
            bgl_graph_destroy(g);
            return e == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP;
        }
        if ((e = hipMemcpy(g->owned_row_ptr, row_ptr, rp_bytes, hipMemcpyHostToDevice)) != hipSuccess ||
            (num_edges > 0 &&
             (e = hipMemcpy(g->owned_col, col_idx, (size_t)num_edges * sizeof(int32_t),
                            hipMemcpyHostToDevice)) != hipSuccess)) {
            bgl::set_error("copying the graph to the device failed: %s", hipGetErrorString(e));
            bgl_graph_destroy(g);
            return BGL_EHIP;
        }
        g->row_ptr = g->owned_row_ptr;
        g->col = static_cast<const int32_t *>(g->owned_col);
    } else if (placement == BGL_HOST_PINNED_COL) {
        // offsets (8 or 4 bytes per node) in HBM, the column ids stay where they are
        const void *col_dev = nullptr;
        if (num_edges > 0 && device_view(col_idx, &col_dev) != BGL_OK) {
            delete g;
            BGL_FAIL(BGL_EINVAL, "BGL_HOST_PINNED_COL needs a page-locked col_idx");
        }
        hipError_t e;
        if ((e = hipMalloc(&g->owned_row_ptr, rp_bytes)) != hipSuccess ||
            (e = hipMemcpy(g->owned_row_ptr, row_ptr, rp_bytes, hipMemcpyHostToDevice)) != hipSuccess) {
            bgl::set_error("copying the row offsets to the device failed: %s", hipGetErrorString(e));
            bgl_graph_destroy(g);
            return e == hipErrorOutOfMemory ? BGL_ENOMEM : BGL_EHIP;
        }
        g->row_ptr = g->owned_row_ptr;
        g->col = static_cast<const int32_t *>(col_dev);
    } else {
        const void *rp_dev = nullptr, *col_dev = nullptr;
        if (device_view(row_ptr, &rp_dev) != BGL_OK ||
            (num_edges > 0 && device_view(col_idx, &col_dev) != BGL_OK)) {
            delete g;
            BGL_FAIL(BGL_EINVAL, "BGL_HOST_PINNED needs page-locked row_ptr and col_idx");
        }
        g->row_ptr = rp_dev;
        g->col = static_cast<const int32_t *>(col_dev);
    }
    *out = g;
    return BGL_OK;
} BGL_NOTHROW_END

extern "C" int bgl_graph_destroy(bgl_graph_t *g)
try {
    if (!g) return BGL_OK;
    (void)hipFree(g->owned_row_ptr);
    (void)hipFree(g->owned_col);
    delete g;
    return BGL_OK;
} BGL_NOTHROW_END
