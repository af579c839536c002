// What a kernel needs from a thread block against what the device grants one: checked on the host
// before a state is accepted, so that a configuration whose kernels cannot be launched as the
// library launches them is refused with an error instead of being tried on the GPU.
// Plain C++ (no HIP types) so that the rule itself can be unit-tested on a machine without a GPU.
#pragma once

#include <cstddef>
#include <string>

namespace cx {

struct KernelNeeds {
    const char* name;
    size_t static_lds_bytes;      // LDS the kernel declares (hipFuncAttributes::sharedSizeBytes)
    int max_threads_per_block;    // largest block the compiled kernel can run with (registers, launch bounds)
    int block_threads;            // block size the library launches it with
};
struct DeviceLimits {
    size_t lds_bytes_per_block;   // hipDeviceAttributeMaxSharedMemoryPerBlock
    int threads_per_block;        // hipDeviceAttributeMaxThreadsPerBlock
};

inline bool kernel_fits(const KernelNeeds& k, const DeviceLimits& d, std::string* why)
{
    if (k.static_lds_bytes > d.lds_bytes_per_block) {
        *why = std::string(k.name) + " needs " + std::to_string(k.static_lds_bytes) + " bytes of LDS per block, the device allows " +
               std::to_string(d.lds_bytes_per_block);
        return false;
    }
    if (k.block_threads > d.threads_per_block || k.block_threads > k.max_threads_per_block) {
        *why = std::string(k.name) + " is launched with " + std::to_string(k.block_threads) + " threads per block, the limit is " +
               std::to_string(k.block_threads > d.threads_per_block ? d.threads_per_block : k.max_threads_per_block);
        return false;
    }
    return true;
}

}  // namespace cx
