// Per-device facts and one-time set-up shared by the library's translation units: the number
// of compute units (read from the device, not assumed) and the list of kernel instantiations
// whose dynamic LDS limit has to be raised once per device before their first launch.
#include <mutex>
#include <vector>

#include "common.h"

namespace cube3d {

int current_device()
{
    int d = 0;
    if (hipGetDevice(&d) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return d;
}

int num_compute_units()
{
    static std::mutex mu;
    static int cached[MAX_DEVICES] = {};
    const int d = current_device();
    if (d < 0 || d >= MAX_DEVICES) return DEFAULT_CUS;
    std::lock_guard<std::mutex> lock(mu);
    if (cached[d] == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, d) != hipSuccess || prop.multiProcessorCount < 1) {
            (void)hipGetLastError();
            return DEFAULT_CUS;
        }
        cached[d] = prop.multiProcessorCount;
    }
    return cached[d];
}

std::vector<KernelSetup> &kernel_setups()
{
    static std::vector<KernelSetup> list;
    return list;
}

int setup_all_kernels()
{
    for (KernelSetup fn : kernel_setups()) {
        const int rc = fn();
        if (rc != CUBE3D_OK) return rc;
    }
    return CUBE3D_OK;
}

}  // namespace cube3d
