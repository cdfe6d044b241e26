// lnmod_misc.hip -- the plain device copy used as the bandwidth reference.
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st) {
    const int64_t nvec = static_cast<int64_t>(bytes / 16);
    if (nvec == 0) return hipSuccess;
    const int64_t pieces = nvec / (kCopyVecs * kWave);
    int64_t blocks = (pieces + kCopyWaves - 1) / kCopyWaves;
    const int64_t cap = static_cast<int64_t>(kNumCU) * 2;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(copy16_kernel<0>, dim3(static_cast<unsigned>(blocks)), dim3(kCopyWaves * kWave), 0, st,
                       static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), nvec);
    return hipGetLastError();
}

}  // namespace lnmod
