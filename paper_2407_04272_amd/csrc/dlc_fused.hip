// Host side of the fused compress kernel: which instantiation, how large a grid, the launch.
#include <algorithm>

#include "dlc_codec_dev.h"

namespace dlc {

const void* fused_kernel_64(const Geom& g);
const void* fused_kernel_128(const Geom& g);
const void* fused_kernel_256(const Geom& g);

static const void* fused_kernel(const Geom& g) {
    switch (g.S) {
        case 64: return fused_kernel_64(g);
        case 128: return fused_kernel_128(g);
        default: return fused_kernel_256(g);
    }
}

// Grid of the fused kernel for this geometry on the current device: as many work-groups as are resident
// at once (never more than there are items).  0: the fused kernel is not used, because a table's items
// would not all be resident together with room to spare (its progress argument needs that).
hipError_t fused_plan(const Geom& g, uint32_t* grid_out) {
    *grid_out = 0;
    if (g.K > kFusedMaxK) return hipSuccess;  // its LDS code tables are sized for alphabets up to that
    const void* fn = fused_kernel(g);
    const size_t sm = fused_lds_bytes(g.K);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sm);
    if (e != hipSuccess) return e;
    int per_cu = 0, dev = 0, cus = 0;
    if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, 256, sm)) != hipSuccess) return e;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    const uint64_t resident = (uint64_t)std::max(per_cu, 0) * (uint64_t)std::max(cus, 0);
    const uint64_t bpt = (g.G + 3) / 4, n_items = bpt * g.T;
    if (resident < 2 * bpt) return hipSuccess;
    *grid_out = (uint32_t)std::min<uint64_t>(resident, n_items);
    return hipSuccess;
}

hipError_t launch_fused(const Geom& g, const FixedLayout& F, const void* payload, const Ws& w, uint64_t epoch,
                        uint8_t* out, uint64_t capacity, hipStream_t s) {
    const uint32_t bpt = (g.G + 3) / 4, n_items = bpt * g.T;
    void* args[] = {(void*)&payload, (void*)&g, (void*)&F, (void*)&w.qp, (void*)&w.hist, (void*)&w.hist_view, (void*)&w.enc,
                    (void*)&w.lens, (void*)&w.tmeta, (void*)&w.ctrl, (void*)&w.arrive, (void*)&w.ready, (void*)&w.state,
                    (void*)&epoch, (void*)&out, (void*)&capacity, (void*)&bpt, (void*)&n_items, (void*)&w.word_start,
                    (void*)&w.word_end};
    return hipLaunchKernel(fused_kernel(g), dim3(w.fused_grid), dim3(256), args, fused_lds_bytes(g.K), s);
}

}  // namespace dlc
