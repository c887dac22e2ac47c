// The parameter server's model update (Sec. 2, "Distributed Training": mini-batch SGD,
// w_k = w_{k-1} - (gamma/|S_k|) * sum of the batch's gradients) applied to the decoded sum.
#include "device_util.hpp"

namespace draco {

// w <- w - scale * u, one 16-byte read of u and one read-modify-write of w per lane
// (12 bytes of HBM traffic per parameter: the minimum).  The sum is read once and never
// again (non-temporal); the parameters are written with ordinary stores, they are the
// next step's input.
template <bool FULL>
__device__ __forceinline__ void apply_update_body(float* __restrict__ w, const float* __restrict__ u, float scale,
                                                  int64_t d) {
    const int64_t c0 = lane_column<kSpreadUpdate>();
    if (!FULL && c0 >= d) return;
    const int n = FULL ? 4 : clamp4(d - c0);
    const float4 g = ldx<FULL>(u + c0, n);
    if constexpr (FULL) {
        float4 p = *reinterpret_cast<const float4*>(w + c0);
        p.x = fmaf(-scale, g.x, p.x);
        p.y = fmaf(-scale, g.y, p.y);
        p.z = fmaf(-scale, g.z, p.z);
        p.w = fmaf(-scale, g.w, p.w);
        *reinterpret_cast<float4*>(w + c0) = p;
    } else {
        const float gv[4] = {g.x, g.y, g.z, g.w};
        for (int i = 0; i < n; ++i) w[c0 + i] = fmaf(-scale, gv[i], w[c0 + i]);
    }
}

__global__ __launch_bounds__(kBlock) void apply_update_kernel(float* __restrict__ w, const float* __restrict__ u,
                                                              float scale, int64_t d) {
    if (block_is_full<kSpreadUpdate>(d)) apply_update_body<true>(w, u, scale, d);
    else apply_update_body<false>(w, u, scale, d);
}

hipError_t launch_apply_update(float* params, const float* sum, float scale, int64_t d, hipStream_t stream) {
    hipLaunchKernelGGL(apply_update_kernel, dim3(grid_cols<kSpreadUpdate>(d)), dim3(kBlock), 0, stream, params, sum, scale,
                       d);
    return hipGetLastError();
}

}  // namespace draco
