// General kernel for real products whose operands do not meet the alignment the tiled MFMA
// kernels need (16-byte aligned bases, leading dimensions in whole 16-byte chunks, K a multiple of
// 8): any leading dimension, bases aligned to an element only, any K.  It reads A and B element
// by element into LDS (converted to FP32; a product of two 16-bit values is exact in FP32), and
// each thread accumulates a 4 x 4 block of a 64 x 64 tile with FP32 FMAs.  Same operation as the
// fast kernels (Sections 2.2, 4.3.2, 5.1, 5.3 and the transforms of Section 4.3), far from their
// speed: a safety net, not a tuned path.
#include "kernel_table.hpp"

namespace fg {
namespace {

constexpr int FT = 64, FK = 32;     // tile 64 x 64, K step 32

__device__ __forceinline__ float widen(uint16_t bits, bool bf16, uint16_t add_bits, bool add) {
    if (bf16) return __builtin_bit_cast(float, (uint32_t)bits << 16);
    _Float16 h = __builtin_bit_cast(_Float16, bits);
    if (add) h = h + __builtin_bit_cast(_Float16, add_bits);      // FP16 addition, round to nearest even
    return (float)h;
}

__global__ __launch_bounds__(256) void gemm_fallback(FallbackParams p) {
    __shared__ float As[FK][FT + 1];
    __shared__ float Bs[FK][FT + 1];
    const int tid = threadIdx.x;
    const int tiles_m = (p.M + FT - 1) / FT;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
    const int m0 = tm * FT, n0 = tn * FT;
    const int tx = tid & 15, ty = tid >> 4;                         // rows 4 tx .. + 3, columns 4 ty .. + 3
    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += FK) {
        // 64 x 32 elements of each operand, 8 per thread; consecutive threads along the operand's
        // contiguous direction
        for (int e = tid; e < FT * FK; e += 256) {
            int r, k;
            if (p.a_rs == 1) { r = e % FT; k = e / FT; } else { k = e % FK; r = e / FK; }
            const int m = m0 + r, kk = k0 + k;
            As[k][r] = (m < p.M && kk < p.K) ? widen(p.A[(int64_t)m * p.a_rs + (int64_t)kk * p.a_ks], p.bf16, p.a_add, p.ab_add) : 0.f;
            if (p.b_rs == 1) { r = e % FT; k = e / FT; } else { k = e % FK; r = e / FK; }
            const int n = n0 + r; const int kb = k0 + k;
            Bs[k][r] = (n < p.N && kb < p.K) ? widen(p.B[(int64_t)n * p.b_rs + (int64_t)kb * p.b_ks], p.bf16, p.b_add, p.ab_add) : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < FK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][4 * tx + i]; b[i] = Bs[k][4 * ty + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    const float floor_v = p.act == 1 ? 0.f : -__builtin_inff();
    const float floor_c = p.c_act == 1 ? 0.f : -__builtin_inff();
    const bool act_none = p.act != 1, c_act_none = p.c_act != 1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = n0 + 4 * ty + j;
        if (n >= p.N) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + 4 * tx + i;
            if (m >= p.M) continue;
            float y = p.alpha * acc[i][j];
            if (p.C) {
                const float c = p.C[m + (int64_t)n * p.ldc];
                y += p.beta * act_clamp(c, floor_c, c_act_none);
            }
            if (p.bias) y += p.bias[p.bias_dim == 0 ? m : n];
            y = act_clamp(y, floor_v, act_none);
            p.D[m + (int64_t)n * p.ldd] = y;
        }
    }
}

}  // namespace

hipError_t launch_gemm_fallback(const FallbackParams &p, hipStream_t stream) {
    const int64_t tiles = (int64_t)((p.M + FT - 1) / FT) * ((p.N + FT - 1) / FT);
    hipLaunchKernelGGL(gemm_fallback, dim3((unsigned)tiles), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace fg
