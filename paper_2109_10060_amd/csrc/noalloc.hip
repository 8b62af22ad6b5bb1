// ds_sliced_linear for callers that cannot allocate device memory: the m-tile list that the grouped
// kernels read (the only scratch of ds_sliced_linear) lives in a file-scope device array instead of a
// caller workspace.  Every call on a device shares that device's array, so calls that overlap in time on
// one device race; nothing in it has to start at zero (the list and its count are rewritten by every call).
#include <mutex>

#include "common.h"

namespace {

constexpr int MAX_TILES = DS_NOALLOC_MAX_TILES;
constexpr size_t SCRATCH_BYTES = 256 + (size_t)MAX_TILES * 16;   // count word (padded) + (group, row, slot, rows) records
constexpr int MAX_DEVICES = 64;

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

// the array's name is a host-side handle; its device address differs per GPU and is looked up once per device
void* g_scratch_ptr[MAX_DEVICES];
std::once_flag g_scratch_once[MAX_DEVICES];
hipError_t g_scratch_err[MAX_DEVICES];

int32_t scratch_for_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) DS_FAIL(DS_EHIP, "ds_sliced_linear_noalloc: hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES) DS_FAIL(DS_EUNSUPPORTED, "ds_sliced_linear_noalloc: device %d outside 0..%d", dev, MAX_DEVICES - 1);
    std::call_once(g_scratch_once[dev], [dev] {
        void* p = nullptr;
        g_scratch_err[dev] = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        g_scratch_ptr[dev] = g_scratch_err[dev] == hipSuccess ? p : nullptr;
    });
    if (g_scratch_err[dev] != hipSuccess || !g_scratch_ptr[dev])
        DS_FAIL(DS_EHIP, "ds_sliced_linear_noalloc: hipGetSymbolAddress: %s", hipGetErrorString(g_scratch_err[dev]));
    *out = g_scratch_ptr[dev];
    return DS_OK;
}

}  // namespace

extern "C" int32_t ds_sliced_linear_noalloc(const void* x, int64_t x_ld, const void* w, int64_t w_ld, int32_t N_full,
                                            int32_t K_full, const float* bias, const ds_groups* g, int32_t B,
                                            int32_t rows, int32_t act, const void* residual, int64_t r_ld, void* y,
                                            int32_t y_dtype, int64_t y_ld, void* stream) {
    const char* who = "ds_sliced_linear_noalloc";
    if (B < 0 || rows < 0) DS_FAIL(DS_EINVAL, "%s: negative size", who);
    if (!g) DS_FAIL(DS_EINVAL, "%s: null groups", who);
    if (g->T < 1 || g->T > DS_MAX_GROUPS) DS_FAIL(DS_EINVAL, "%s: T=%d outside 1..%d", who, g->T, DS_MAX_GROUPS);
    const size_t need = ds_sliced_linear_workspace(B, rows, g->T);
    if (ds_mtile_capacity(B, rows, g->T) > (size_t)MAX_TILES || need > SCRATCH_BYTES)
        DS_FAIL(DS_EWORKSPACE, "%s: B * rows = %lld needs %zu row tiles, the built-in scratch holds %d (use ds_sliced_linear)",
                who, (long long)B * rows, ds_mtile_capacity(B, rows, g->T), MAX_TILES);
    void* ws = nullptr;
    if (B > 0 && rows > 0) {
        const int32_t rc = scratch_for_current_device(&ws);
        if (rc) return rc;
    }
    ProfPause quiet;   // kernel timing would create events on first use
    return ds_sliced_linear(x, x_ld, w, w_ld, N_full, K_full, bias, g, B, rows, act, residual, r_ld, y, y_dtype, y_ld,
                            ws, SCRATCH_BYTES, stream);
}
