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

// Default launch shapes (blocks, waves per block, vectors per lane and step): the best of a sweep
// over 64 ... 1024 blocks, 1 ... 8 waves and 1 ... 16 vectors on 774 MB buffers (reads like many
// streams, writes few and long ones).
namespace {

template <int NR, int NW>
bool go_probe(const ProbeArgs& a, int blocks, int waves, int vecs, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(blocks)), block(static_cast<unsigned>(waves * kWave));
    switch (vecs) {
        case 1: hipLaunchKernelGGL((stream_probe_kernel<NR, NW, 1>), grid, block, 0, st, a); return true;
        case 2: hipLaunchKernelGGL((stream_probe_kernel<NR, NW, 2>), grid, block, 0, st, a); return true;
        case 4: hipLaunchKernelGGL((stream_probe_kernel<NR, NW, 4>), grid, block, 0, st, a); return true;
        case 8: hipLaunchKernelGGL((stream_probe_kernel<NR, NW, 8>), grid, block, 0, st, a); return true;
        default: return false;
    }
}

}  // namespace

bool probe_mixture_supported(int reads, int writes) {
    const int key = reads * 10 + writes;
    return key == 10 || key == 1 || key == 11 || key == 21 || key == 22 || key == 31 || key == 33 || key == 42;
}

hipError_t launch_stream_probe(const void* const* in, int reads, void* const* out, int writes, size_t bytes,
                               int blocks, int waves, int vecs, hipStream_t st) {
    ProbeArgs a{};
    a.nvec = static_cast<int64_t>(bytes / 16);
    if (a.nvec == 0) return hipSuccess;
    for (int i = 0; i < reads; ++i) a.in[i] = static_cast<const u32x4*>(in[i]);
    for (int j = 0; j < (writes > 0 ? writes : 1); ++j) a.out[j] = static_cast<u32x4*>(out[j]);
    const int key = reads * 10 + writes;
    if (blocks <= 0 || waves <= 0 || vecs <= 0) {
        if (key == 10) { blocks = 2 * kNumCU; waves = 4; vecs = 4; }
        else if (key == 1) { blocks = kNumCU / 2; waves = 1; vecs = 8; }
        else if (key == 22) { blocks = kNumCU; waves = 2; vecs = 4; }
        else { blocks = kNumCU; waves = 4; vecs = 4; }
    }
    if (waves > 8 || blocks > 65536) return hipErrorInvalidConfiguration;
    bool ok = false;
    switch (key) {
        case 10: ok = go_probe<1, 0>(a, blocks, waves, vecs, st); break;
        case 1: ok = go_probe<0, 1>(a, blocks, waves, vecs, st); break;
        case 11: ok = go_probe<1, 1>(a, blocks, waves, vecs, st); break;
        case 21: ok = go_probe<2, 1>(a, blocks, waves, vecs, st); break;
        case 22: ok = go_probe<2, 2>(a, blocks, waves, vecs, st); break;
        case 31: ok = go_probe<3, 1>(a, blocks, waves, vecs, st); break;
        case 33: ok = go_probe<3, 3>(a, blocks, waves, vecs, st); break;
        case 42: ok = go_probe<4, 2>(a, blocks, waves, vecs, st); break;
        default: break;
    }
    return ok ? hipGetLastError() : hipErrorInvalidConfiguration;
}

}  // namespace lnmod
