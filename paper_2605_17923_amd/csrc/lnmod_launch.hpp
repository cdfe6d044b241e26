// lnmod_launch.hpp -- host-side launch interface between the C ABI (lnmod_api.cpp) and the
// translation units that instantiate the gfx950 kernels.  Plain data in, hipError_t out.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

namespace lnmod {

constexpr int kNumCU = 256;            // MI355X: 8 XCDs x 32 CUs
constexpr int64_t kMaxD = 8192;
constexpr int kMaxBwdBlocks = 2048;    // upper bound of the backward grid (sizes the workspace)

struct Problem {
    int dtype;                 // LNMOD_BF16 / LNMOD_F32
    const int32_t* cu;         // device segment offsets or nullptr (fixed length)
    int64_t nseg;              // samples or segments
    int64_t S;                 // tokens per sample when cu == nullptr
    int64_t T;                 // total tokens
    int64_t D;
    float eps;
};

// Rows every backward block owns for this problem; the same function sizes the workspace,
// drives the main kernel's grid and tells the second pass which slots belong to a segment.
int64_t bwd_rows_per_block(int64_t T, int64_t D, int dtype);
int64_t bwd_num_blocks(int64_t T, int64_t D, int dtype);

hipError_t launch_fwd_seg(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st);
hipError_t launch_fwd_tok(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* y, float* mean, float* rstd, hipStream_t st);
hipError_t launch_bwd_seg(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, float* dshift,
                          float* dscale, float* ws, hipStream_t st);
hipError_t launch_bwd_tok(const Problem& p, const void* dy, const void* x, const void* scale,
                          const float* mean, const float* rstd, void* dx, void* dshift,
                          void* dscale, hipStream_t st);
hipError_t launch_unfused(const Problem& p, const void* x, const void* shift, const void* scale,
                          void* xhat, void* y, float* mean, float* rstd, hipStream_t st);
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
hipError_t launch_zero_f32(float* p, int64_t n, hipStream_t st);

}  // namespace lnmod
