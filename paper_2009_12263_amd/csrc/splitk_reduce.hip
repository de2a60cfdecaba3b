// Second pass of a split-K product: D = act(alpha * sum_s W_s + beta * c_act(C) + bias) on the
// tiles tile_begin .. tile_begin + tile_count - 1, where slot s * tile_count + t of the workspace
// holds the raw BM x BN partial product (column-major, leading dimension BM) that K range s
// contributed to tile tile_begin + t.  The paper names this use of the epilogue (a reduction
// across workgroups) in Section 4.2.5.  The partials are added in ascending s, so the result does
// not depend on how the first pass was scheduled.
#include "kernel_table.hpp"

namespace fg {
namespace {

// One thread per 4 consecutive rows of one column of one tile: 16-byte reads of the partials,
// lanes along M.
__global__ __launch_bounds__(256) void splitk_reduce(const float *W, int splits, int tile_begin, int tile_count, int bm, int bn,
                                                     int tiles_m, int tiles_n, int M, int N, float alpha, float beta,
                                                     const float *C, int64_t ldc, float *D, int64_t ldd, const float *bias,
                                                     int bias_dim, int act, int c_act) {
    const int per_tile = (bm / 4) * bn;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)per_tile * tile_count) return;
    const int t = (int)(idx / per_tile);
    const int e = (int)(idx - (int64_t)t * per_tile);
    const int col = e / (bm / 4), row = (e - col * (bm / 4)) * 4;
    int tm, tn;
    block_to_tile(tile_begin + t, tiles_m, tiles_n, tm, tn);
    const int m = tm * bm + row, n = tn * bn + col;
    if (m >= M || n >= N) return;
    const int valid = M - m < 4 ? M - m : 4;
    const int64_t slot_elems = (int64_t)bm * bn;
    const float *w = W + (int64_t)t * slot_elems + row + (int64_t)col * bm;
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < splits; ++s) {
        const float4 v = *(const float4 *)(w + (int64_t)s * tile_count * slot_elems);   // 16-byte aligned: bm % 4 == 0
        sum[0] += v.x; sum[1] += v.y; sum[2] += v.z; sum[3] += v.w;
    }
    const float floor_v = act == 1 ? 0.f : -__builtin_inff();
    const float floor_c = c_act == 1 ? 0.f : -__builtin_inff();
    const bool act_none = act != 1, c_act_none = c_act != 1;
    for (int q = 0; q < valid; ++q) {
        float y = alpha * sum[q];
        if (C) {
            const float c = C[m + q + (int64_t)n * ldc];
            y += beta * act_clamp(c, floor_c, c_act_none);
        }
        if (bias) y += bias[bias_dim == 0 ? m + q : n];
        y = act_clamp(y, floor_v, act_none);
        D[m + q + (int64_t)n * ldd] = y;
    }
}

}  // namespace

hipError_t launch_splitk_reduce(const float *W, int splits, int tile_begin, int tile_count, int bm, int bn, int tiles_m,
                                int tiles_n, int M, int N, float alpha, float beta, const float *C, int64_t ldc, float *D,
                                int64_t ldd, const float *bias, int bias_dim, int act, int c_act, hipStream_t stream) {
    const int64_t work = (int64_t)(bm / 4) * bn * tile_count;
    const unsigned blocks = (unsigned)((work + 255) / 256);
    hipLaunchKernelGGL(splitk_reduce, dim3(blocks), dim3(256), 0, stream, W, splits, tile_begin, tile_count, bm, bn, tiles_m,
                       tiles_n, M, N, alpha, beta, C, ldc, D, ldd, bias, bias_dim, act, c_act);
    return hipGetLastError();
}

}  // namespace fg
