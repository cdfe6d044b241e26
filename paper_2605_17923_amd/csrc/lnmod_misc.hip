// lnmod_misc.hip -- measurement comparators: the unfused LayerNorm -> modulate chain and a
// plain device copy.  Neither is on the fused path.
#include "lnmod_kernels.hpp"
#include "lnmod_launch.hpp"

namespace lnmod {
namespace {

constexpr int kWaves = 4;

template <typename Tag, int VPL>
void go_unfused(FwdArgs ln, FwdArgs mod, hipStream_t st) {
    int64_t blocks = (ln.T + kWaves - 1) / kWaves;
    const int64_t cap = static_cast<int64_t>(kNumCU) * (ln.nchunks >= 512 ? 2 : 4);
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    const dim3 grid(static_cast<unsigned>(blocks)), block(kWaves * kWave);
    hipLaunchKernelGGL((unfused_ln_kernel<Tag, VPL, kWaves, false>), grid, block, 0, st, ln);
    hipLaunchKernelGGL((unfused_mod_kernel<Tag, VPL, kWaves, false>), grid, block, 0, st, mod);
}

template <typename Tag>
void dispatch_unfused(int need, const FwdArgs& ln, const FwdArgs& mod, hipStream_t st) {
    if (need <= 1) go_unfused<Tag, 1>(ln, mod, st);
    else if (need <= 2) go_unfused<Tag, 2>(ln, mod, st);
    else if (need <= 3) go_unfused<Tag, 3>(ln, mod, st);
    else if (need <= 4) go_unfused<Tag, 4>(ln, mod, st);
    else if (need <= 6) go_unfused<Tag, 6>(ln, mod, st);
    else if (need <= 8) go_unfused<Tag, 8>(ln, mod, st);
    else if (need <= 10) go_unfused<Tag, 10>(ln, mod, st);
    else if (need <= 12) go_unfused<Tag, 12>(ln, mod, st);
    else if (need <= 16) go_unfused<Tag, 16>(ln, mod, st);
    else if (need <= 20) go_unfused<Tag, 20>(ln, mod, st);
    else if (need <= 24) go_unfused<Tag, 24>(ln, mod, st);
    else go_unfused<Tag, 32>(ln, mod, st);
}

}  // namespace

hipError_t launch_unfused(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* xhat, void* y, float* mean, float* rstd, hipStream_t st) {
    const int E = p.dtype == 0 ? 8 : 4;
    FwdArgs ln;
    ln.x = x;
    ln.shift = nullptr;
    ln.scale = nullptr;
    ln.y = xhat;
    ln.mean = mean;
    ln.rstd = rstd;
    ln.seg = Segments{p.cu, p.S, p.nseg};
    ln.T = p.T;
    ln.rows_per_cluster = 0;
    ln.nb = 1;
    ln.D = static_cast<int32_t>(p.D);
    ln.nchunks = static_cast<int32_t>(p.D / E);
    ln.eps = p.eps;
    ln.inv_D = 1.0f / static_cast<float>(p.D);
    FwdArgs mod = ln;
    mod.x = xhat;
    mod.shift = shift;
    mod.scale = scale;
    mod.y = y;
    const int need = (ln.nchunks + kWave - 1) / kWave;
    if (p.dtype == 0) dispatch_unfused<bf16_io>(need, ln, mod, st);
    else dispatch_unfused<f32_io>(need, ln, mod, st);
    return hipGetLastError();
}

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
