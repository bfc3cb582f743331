// Unfolding of a convolution's input into the matrix the matmuls take, for the layers whose
// geometry the activation-source kernels do not read directly (strides, windows that leave K
// off a multiple of 64, tiny images): X[(b, yo, xo), c*kh*kw + ty*kw + tx] =
// act[b, c, yo*stride + ty - ph, xo*stride + tx - pw], zero outside the image.  Pure data
// movement, one launch per layer (a framework's per-sample unfold costs a launch per image).
#include "common.hpp"

namespace hdqt {

namespace {

constexpr int kRowsPerBlock = 4;

// A workgroup writes kRowsPerBlock rows of X; its threads run along a row, so the stores are
// contiguous and neighbouring threads read neighbouring taps of one input row.
__global__ __launch_bounds__(256) void im2col_kernel(Im2colArgs a)
{
    const int64_t K = (int64_t)a.C * a.kh * a.kw;
    const int khw = a.kh * a.kw;
    for (int r = 0; r < kRowsPerBlock; ++r) {
        const int64_t m = (int64_t)blockIdx.x * kRowsPerBlock + r;
        if (m >= a.M) return;
        // (the same in every thread)
        const int64_t b = m / ((int64_t)a.Ho * a.Wo);
        const int rem = (int)(m - b * (int64_t)a.Ho * a.Wo);
        const int yo = rem / a.Wo, xo = rem - yo * a.Wo;
        const int y0 = yo * a.stride - a.ph, x0 = xo * a.stride - a.pw;
        const float* img = a.act + b * (int64_t)a.C * a.H * a.W;
        float* dst = a.X + m * K;
        for (int k = threadIdx.x; k < K; k += blockDim.x) {
            const int c = k / khw, tap = k - c * khw;
            const int ty = tap / a.kw, tx = tap - ty * a.kw;
            const int y = y0 + ty, x = x0 + tx;
            float v = 0.0f;
            if (y >= 0 && y < a.H && x >= 0 && x < a.W) v = img[((int64_t)c * a.H + y) * a.W + x];
            dst[k] = v;
        }
    }
}

} // namespace

hipError_t launch_im2col(const Im2colArgs& a, hipStream_t stream)
{
    const int64_t blocks = (a.M + kRowsPerBlock - 1) / kRowsPerBlock;
    ProfileScope ps(K_IM2COL, stream);
    hipLaunchKernelGGL(im2col_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

} // namespace hdqt
