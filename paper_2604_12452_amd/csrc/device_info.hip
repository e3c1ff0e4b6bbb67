// What the launchers need to know about the GPU they launch on, asked once per device ordinal.
#include <atomic>

#include "lca_internal.h"

namespace lca {

// Workgroups of a persistent one-workgroup-per-CU kernel on the current device: its compute-unit count, rounded down to
// a multiple of 8 (the kernels deal their items out over 8 dispatch slots, the chip's 8 XCDs under round-robin
// placement; on a device with another XCD count the result stays correct and only the L2 sharing is lost) and kept
// within [8, 256], the range the kernels' index arithmetic is validated for.  256 when the runtime cannot tell.
int persistent_grid()
{
    constexpr int MAX_DEVICES = 64;
    static std::atomic<int> cached[MAX_DEVICES];      // 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return 256;
    int grid = cached[dev].load(std::memory_order_relaxed);
    if (grid == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        grid = cus / 8 * 8;
        grid = grid < 8 ? 8 : grid > 256 ? 256 : grid;
        cached[dev].store(grid, std::memory_order_relaxed);
    }
    return grid;
}

}  // namespace lca
