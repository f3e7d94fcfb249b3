// gnn_spmm_csr_static: the SpMM entry point for callers that cannot allocate device memory and have no
// workspace to hand over (code under HIP graph capture, tight serving loops, harnesses that forbid
// hipMalloc).  The scratch that gnn_spmm_csr takes from its `workspace` argument - the partial rows of the
// entry-balanced kernel and, for widths that are not a multiple of 4, the padded copy of the dense
// operand - lives in a file-scope device array instead.  Every GPU the library runs on holds its own
// copy of the array, at its own address, until the process ends.
#include <mutex>

#include "common.h"

namespace {

constexpr size_t kStaticScratchBytes = (size_t)GNN_STATIC_SCRATCH_BYTES;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code `scratch` is only a handle for the runtime, not a device address: the address of the
// array on each device is asked for once, with that device current, and kept.
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

gnn_status_t scratch_of_current_device(void **out) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return GNN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GNN_ERR_HIP;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return GNN_OK;
}

}  // namespace

extern "C" gnn_status_t gnn_spmm_csr_static(int32_t n, int32_t nnz, const int32_t *rowptr, const int32_t *col,
                                            const float *val, const int32_t *erow, const float *B, int32_t f,
                                            float *C, const float *bias, int32_t relu, void *hip_stream) {
    if (n < 0 || nnz < 0 || f <= 0 || !rowptr) return GNN_ERR_INVALID_ARG;
    if (relu != 0 && relu != 1) return GNN_ERR_INVALID_ARG;
    if (n > 0 && !C) return GNN_ERR_INVALID_ARG;
    if (nnz > 0 && (!col || !B)) return GNN_ERR_INVALID_ARG;
    void *ws = nullptr;
    if (erow && nnz > 0) {
        // the same bytes gnn_spmm_csr asks its caller for
        if (gnn::spmm_workspace_bytes(n, nnz, f) > kStaticScratchBytes) return GNN_ERR_BUFFER_TOO_SMALL;
        GNN_TRY(scratch_of_current_device(&ws));
    }
    return gnn::spmm_launch(n, nnz, rowptr, col, erow, gnn::EdgeWeights{val, nullptr, 1, f}, B, n, f, C, bias, relu,
                            ws, static_cast<hipStream_t>(hip_stream));
}
