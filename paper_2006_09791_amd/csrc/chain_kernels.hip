// Non-convolution steps of the residual stacks of Section IV-A of
// arXiv 2006.09791: ReLU, element-wise add, max pooling.  All fp32.
#include "gspc_internal.h"

namespace gspc {

__global__ void relu_kernel(const float *__restrict__ x, float *__restrict__ y, size_t count) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += step) y[i] = fmaxf(x[i], 0.f);
}

__global__ void add_kernel(const float *__restrict__ a, const float *__restrict__ b,
                           float *__restrict__ y, size_t count, int relu) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (; i < count; i += step) {
        float v = a[i] + b[i];
        y[i] = relu ? fmaxf(v, 0.f) : v;
    }
}

__global__ void maxpool_kernel(const float *__restrict__ x, float *__restrict__ y, int C, int H,
                               int W, int K, int stride, int pad, int Hout, int Wout,
                               size_t total) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    const int ow = (int)(i % Wout);
    size_t r = i / Wout;
    const int oh = (int)(r % Hout);
    const size_t plane = r / Hout;  // n * C + c
    const float *xp = x + plane * (size_t)H * W;
    float m = -INFINITY;
    for (int kh = 0; kh < K; ++kh) {
        const int ih = oh * stride - pad + kh;
        if (ih < 0 || ih >= H) continue;
        for (int kw = 0; kw < K; ++kw) {
            const int iw = ow * stride - pad + kw;
            if (iw < 0 || iw >= W) continue;
            m = fmaxf(m, xp[(size_t)ih * W + iw]);
        }
    }
    y[i] = m;
}

static unsigned grid_for(size_t count) {
    size_t b = (count + 255) / 256;
    if (b > 262144) b = 262144;
    if (b == 0) b = 1;
    return (unsigned)b;
}

hipError_t launch_relu(const float *x, float *y, size_t count, hipStream_t s) {
    hipLaunchKernelGGL(relu_kernel, dim3(grid_for(count)), dim3(256), 0, s, x, y, count);
    return hipGetLastError();
}

hipError_t launch_add(const float *a, const float *b, float *y, size_t count, int relu,
                      hipStream_t s) {
    hipLaunchKernelGGL(add_kernel, dim3(grid_for(count)), dim3(256), 0, s, a, b, y, count, relu);
    return hipGetLastError();
}

hipError_t launch_maxpool(const float *x, float *y, int N, int C, int H, int W, int K, int stride,
                          int pad, int Hout, int Wout, hipStream_t s) {
    const size_t total = (size_t)N * C * Hout * Wout;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    hipLaunchKernelGGL(maxpool_kernel, dim3(blocks), dim3(256), 0, s, x, y, C, H, W, K, stride, pad,
                       Hout, Wout, total);
    return hipGetLastError();
}

}  // namespace gspc
