// dbf_gemm_static: the prefill product with its scratch in a static device array, for callers that cannot
// allocate (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  The
// kernels are those of dbf_gemm; only where their scratch lives differs.
#include <mutex>

#include "dbf_kernels.h"

namespace {

// The scratch: one copy per GPU the library runs on, held until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress, never an address: everything below uses the looked-up pointer.
__device__ __align__(256) unsigned char scratch[DBF_GEMM_STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void* g_scratch_ptr[MAX_DEVICES] = {};  // device address of `scratch`, per device ordinal

// Address of this device's copy of the array (looked up once per device, with that device current).
hipError_t scratch_of(int device, void** out) {
    std::lock_guard<std::mutex> guard(g_lock);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace

extern "C" int dbf_gemm_static(const dbf_layer* L, const void* X_dev, void* Y_dev, int T, void* hip_stream) {
    if (!L || !X_dev || !Y_dev || T < 1) return DBF_EINVAL;
    if ((T + 63) / 64 > 65535) return DBF_EINVAL;
    if (L->n_in > DBF_INT_PATH_MAX_COLS || L->k > DBF_INT_PATH_MAX_COLS) return DBF_ESHAPE;  // (int32 sums: see dbf.h)
    const size_t need = dbf_gemm_i8_workspace_bytes_without_splits(L, T);  // (column splits only where they fit as well)
    if (need > DBF_GEMM_STATIC_BYTES) return DBF_EWORKSPACE;  // beyond the static scratch: use dbf_gemm
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return DBF_EHIP;
    }
    if (device != L->device || device < 0 || device >= MAX_DEVICES) return DBF_EINVAL;
    void* ws = nullptr;
    if (scratch_of(device, &ws) != hipSuccess) {
        (void)hipGetLastError();
        return DBF_EHIP;
    }
    if (dbf_gemm_i8_launch(L, X_dev, Y_dev, T, ws, DBF_GEMM_STATIC_BYTES, static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
        (void)hipGetLastError();
        return DBF_EHIP;
    }
    return DBF_OK;
}
