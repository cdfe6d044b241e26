// lnmod_misc.hip -- the plain device copy and the stream probes used as bandwidth references.
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

// Launch shapes: the best of a sweep over 64 ... 1024 blocks, 1 ... 8 waves per block and 1 ... 16
// vectors per step on 774 MB buffers (reads like many streams, writes few and long ones).
hipError_t launch_stream_probe(const void* a, const void* b, void* c, size_t bytes, int mode, hipStream_t st) {
    const int64_t nvec = static_cast<int64_t>(bytes / 16);
    if (nvec == 0) return hipSuccess;
    const u32x4* pa = static_cast<const u32x4*>(a);
    const u32x4* pb = static_cast<const u32x4*>(b);
    u32x4* pc = static_cast<u32x4*>(c);
    if (mode == kProbeAdd)
        hipLaunchKernelGGL((stream_probe_kernel<kProbeAdd, 4, 4>), dim3(kNumCU), dim3(4 * kWave), 0, st, pa, pb, pc, nvec);
    else if (mode == kProbeRead)
        hipLaunchKernelGGL((stream_probe_kernel<kProbeRead, 4, 4>), dim3(2 * kNumCU), dim3(4 * kWave), 0, st, pa, pb, pc, nvec);
    else
        hipLaunchKernelGGL((stream_probe_kernel<kProbeWrite, 1, 8>), dim3(kNumCU / 2), dim3(kWave), 0, st, pa, pb, pc, nvec);
    return hipGetLastError();
}

}  // namespace lnmod
