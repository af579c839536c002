// Host-only unit test of the rule that decides whether a kernel can be launched as the library
// launches it (csrc/launch_limits.hpp).  Built with g++ and run by tests/test_native_checks.py.
#include <cstdio>
#include <string>

#include "../../paper_2402_16801_amd/csrc/launch_limits.hpp"

static int failures = 0;
static void expect(bool cond, const char* what)
{
    if (!cond) { std::printf("FAILED: %s\n", what); ++failures; }
}

int main()
{
    using namespace cx;
    const DeviceLimits dev{65536, 1024};
    std::string why;
    expect(kernel_fits(KernelNeeds{"fits", 31000, 1024, 256}, dev, &why), "31 KB of LDS, 256 threads");
    expect(kernel_fits(KernelNeeds{"edge", 65536, 256, 256}, dev, &why), "exactly the limits");
    why.clear();
    // the shape of the two-lane step variant that was taken out: 128 environments x 142 dwords
    expect(!kernel_fits(KernelNeeds{"two_lanes", 128 * 142 * 4 + 2048, 1024, 256}, dev, &why), "72.7 KB of LDS on a 64 KB device");
    expect(why.find("two_lanes") != std::string::npos && why.find("LDS") != std::string::npos, "the message names the kernel and the resource");
    expect(kernel_fits(KernelNeeds{"two_lanes", 128 * 142 * 4 + 2048, 1024, 256}, DeviceLimits{163840, 1024}, &why), "the same on a 160 KB device");
    why.clear();
    expect(!kernel_fits(KernelNeeds{"wide", 1000, 256, 512}, dev, &why), "a block larger than the kernel was compiled for");
    expect(why.find("256") != std::string::npos, "the message gives the limit that binds");
    expect(!kernel_fits(KernelNeeds{"huge", 1000, 2048, 2048}, dev, &why), "a block larger than the device allows");
    std::printf(failures ? "launch_limits_test: %d failures\n" : "launch_limits_test: ok\n", failures);
    return failures ? 1 : 0;
}
