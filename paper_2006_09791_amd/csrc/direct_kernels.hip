// Direct (sliding-window) grouped convolution kernels: the convolution stage of
// Algorithm 1 of arXiv 2006.09791 with the input and output reshapes fused
// away.  These cover every shape; the matrix-core kernels take over where the
// per-group contraction is wide.
#include "gspc_internal.h"

namespace gspc {

__device__ __forceinline__ float load_in(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_in(const uint16_t *p, size_t i) {
    return __uint_as_float((uint32_t)p[i] << 16);
}

__device__ __forceinline__ float epilogue(float v, const float *res, size_t idx, int relu) {
    if (res) v += res[idx];
    return relu ? fmaxf(v, 0.f) : v;
}

// One thread = one output pixel x OCT consecutive filters of one group.
// Weights come from the direct section [g][Kred][KPGd]; the OCT values of a
// tap are adjacent and their address is uniform over the block.
template <int OCT, typename TIN>
__global__ __launch_bounds__(256) void conv_direct_generic(ConvParams p) {
    const int HWo = p.Hout * p.Wout;
    const int pix = blockIdx.x * blockDim.x + threadIdx.x;
    const int tiles = p.KPGd / OCT;
    const int j = blockIdx.y / tiles;
    const int oc0 = (blockIdx.y % tiles) * OCT;
    const int n = blockIdx.z;
    if (pix >= HWo) return;
    const int oh = pix / p.Wout, ow = pix % p.Wout;
    const int ih0 = oh * p.stride - p.pad, iw0 = ow * p.stride - p.pad;
    const size_t plane = (size_t)p.H * p.W;
    const TIN *xg = static_cast<const TIN *>(p.x) + ((size_t)n * p.Cin + (size_t)j * p.CPG) * plane;
    const float *wg = p.wd + (size_t)j * p.CPG * p.KH * p.KW * p.KPGd + oc0;

    float acc[OCT];
#pragma unroll
    for (int o = 0; o < OCT; ++o) acc[o] = 0.f;

    for (int c = 0; c < p.CPG; ++c) {
        for (int kh = 0; kh < p.KH; ++kh) {
            const int ih = ih0 + kh;
            const bool row_ok = ih >= 0 && ih < p.H;
            for (int kw = 0; kw < p.KW; ++kw) {
                const int iw = iw0 + kw;
                float xv = 0.f;
                if (row_ok && iw >= 0 && iw < p.W) xv = load_in(xg, c * plane + (size_t)ih * p.W + iw);
                const float *wk = wg + (size_t)((c * p.KH + kh) * p.KW + kw) * p.KPGd;
#pragma unroll
                for (int o = 0; o < OCT; ++o) acc[o] = fmaf(xv, wk[o], acc[o]);
            }
        }
    }
#pragma unroll
    for (int o = 0; o < OCT; ++o) {
        if (oc0 + o < p.KPG) {
            const size_t idx = (((size_t)n * p.Cout + (size_t)j * p.KPG + oc0 + o) * p.Hout + oh) * p.Wout + ow;
            p.y[idx] = epilogue(acc[o], p.res, idx, p.relu);
        }
    }
}

template <int OCT, typename TIN>
static hipError_t launch_generic(const ConvParams &p, hipStream_t s) {
    const int HWo = p.Hout * p.Wout;
    dim3 grid((HWo + 255) / 256, p.groups * (p.KPGd / OCT), p.N);
    if (grid.y > 65535u || grid.z > 65535u) return hipErrorNotSupported;
    hipLaunchKernelGGL((conv_direct_generic<OCT, TIN>), grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_direct(const ConvParams &p, hipStream_t s, const char **name) {
    const bool oct8 = p.KPGd % 8 == 0;
    if (p.in_bf16) {
        *name = oct8 ? "conv_direct_generic<8,bf16>" : "conv_direct_generic<4,bf16>";
        return oct8 ? launch_generic<8, uint16_t>(p, s) : launch_generic<4, uint16_t>(p, s);
    }
    *name = oct8 ? "conv_direct_generic<8,f32>" : "conv_direct_generic<4,f32>";
    return oct8 ? launch_generic<8, float>(p, s) : launch_generic<4, float>(p, s);
}

}  // namespace gspc
