// rh_select_regions_noalloc: the selection of Sec. 3.3.1 for callers that cannot allocate.  The
// per-frame and per-segment tables that rh_select_regions keeps in a context's scratch memory
// live in a fixed device array here (every GPU the library runs on holds its own copy until the
// process ends), and no context is needed.
#include "rh_internal.h"
#include "rh_noalloc.h"

static __device__ __align__(256) uint32_t scratch[8 * RH_NOALLOC_MAX_FRAMES];
static void* g_scratch_ptr[RH_MAX_DEVICES];      // device address of `scratch` on each device, once known

extern "C" rh_status rh_select_regions_noalloc(const float* importance, int32_t F, int32_t mbh, int32_t mbw,
                                               const rh_segment* segs, int32_t nseg, int32_t mode, uint8_t* mask,
                                               uint32_t* list, uint32_t* n_sel, void* hip_stream)
{
    if (F < 1 || mbh < 1 || mbw < 1) return RH_E_SHAPE;
    if (F > RH_NOALLOC_MAX_FRAMES) return RH_E_CAPACITY;                 // beyond the fixed tables
    if ((uint64_t)F * (uint64_t)mbh * (uint64_t)mbw > 0x7FFFFFFFull) return RH_E_SHAPE;
    rh_status st;
    if (rh_check_select_args(importance, F, segs, nseg, mode, mask, list, n_sel, &st)) return st;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= RH_MAX_DEVICES) return RH_E_DEVICE;
    if (!g_scratch_ptr[dev]) {
        // the array's name is a host-side handle, not a device address: ask the runtime for the
        // address of this device's copy (the device is current)
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RH_E_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    uint32_t* base = (uint32_t*)g_scratch_ptr[dev];
    const size_t M = RH_NOALLOC_MAX_FRAMES;
    // every table entry the kernels read is written earlier in the same call (frames [0, F) and
    // segments [0, nseg)), so nothing of an earlier call's contents is used
    const rh_select_scratch sc = {(int32_t*)base, base + M, base + 5 * M, base + 6 * M, base + 7 * M};
    if (rh_enqueue_select((hipStream_t)hip_stream, sc, importance, F, mbh * mbw, segs, nseg, mode, mask, list, n_sel) != hipSuccess)
        return RH_E_DEVICE;
    return RH_OK;
}
