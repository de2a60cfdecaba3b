// Second pass of a split-K product: D = act(alpha * sum_s W_s + beta * c_act(C) + bias), where W_s
// are the raw partial products the first pass left in the workspace (column-major, leading
// dimension ldw, `stride` elements apart).  The paper names this use of the epilogue (a reduction
// across all workgroups) in Section 4.2.5.  The partials are added in ascending s, so the result
// does not depend on how the launch was scheduled.
#include "kernel_table.hpp"

namespace fg {
namespace {

// One thread per 4 consecutive rows of one column: 16-byte accesses, lanes along M.
__global__ __launch_bounds__(256) void splitk_reduce(const float *W, int64_t stride, int splits, int M, int N, int ldw,
                                                     float alpha, float beta, const float *C, int64_t ldc, float *D,
                                                     int64_t ldd, const float *bias, int bias_dim, int act, int c_act) {
    const int m4 = (M + 3) / 4;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)m4 * N) return;
    const int n = (int)(idx / m4);
    const int m = (int)(idx - (int64_t)n * m4) * 4;
    const int valid = M - m < 4 ? M - m : 4;
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
    const float *w = W + m + (int64_t)n * ldw;
    if (valid == 4) {
        // ldw is a multiple of 4 and the workspace is 256-byte aligned: one 16-byte read per partial
        for (int s = 0; s < splits; ++s) {
            const float4 v = *(const float4 *)(w + s * stride);
            sum[0] += v.x; sum[1] += v.y; sum[2] += v.z; sum[3] += v.w;
        }
    } else {
        for (int s = 0; s < splits; ++s)
            for (int t = 0; t < valid; ++t) sum[t] += w[s * stride + t];
    }
    const float floor_v = act == 1 ? 0.f : -__builtin_inff();
    const float floor_c = c_act == 1 ? 0.f : -__builtin_inff();
    for (int t = 0; t < valid; ++t) {
        float y = alpha * sum[t];
        if (C) {
            const float c = C[m + t + (int64_t)n * ldc];
            y += beta * (c > floor_c ? c : floor_c);
        }
        if (bias) y += bias[bias_dim == 0 ? m + t : n];
        y = y > floor_v ? y : floor_v;
        D[m + t + (int64_t)n * ldd] = y;
    }
}

}  // namespace

hipError_t launch_splitk_reduce(const float *W, int64_t stride, int splits, int M, int N, int ldw, float alpha, float beta,
                                const float *C, int64_t ldc, float *D, int64_t ldd, const float *bias, int bias_dim,
                                int act, int c_act, hipStream_t stream) {
    const int64_t work = (int64_t)((M + 3) / 4) * N;
    const unsigned blocks = (unsigned)((work + 255) / 256);
    hipLaunchKernelGGL(splitk_reduce, dim3(blocks), dim3(256), 0, stream, W, stride, splits, M, N, ldw, alpha, beta, C, ldc, D,
                       ldd, bias, bias_dim, act, c_act);
    return hipGetLastError();
}

}  // namespace fg
