// General kernel for tensor contractions (Section 5.5) that the tiled MFMA kernels cannot take:
// no mode of A or B with stride 1 and an extent that is a multiple of 8, strides or base pointers
// that do not keep every 16-byte piece aligned, A and B contiguous along different summed modes,
// tensors of 2 GiB and more (element offsets are 64-bit here), and contractions without a summed
// mode (outer products).  The same mode-to-tile mapping as the fast kernels --
// element (m, k) of A sits at group_offset(rows, m) + group_offset(summed, k) + group_offset(batch, t),
// nothing is transposed in memory -- with element-wise loads and FP32 FMAs (a product of two
// binary16 values is exact in FP32): a safety net far from the tiled kernels' speed.
#include "kernel_table.hpp"

namespace fg {
namespace {

constexpr int CT = 64, CK = 32;     // tile 64 x 64, K step 32

__global__ __launch_bounds__(256) void contract_fallback(const ContractFallbackParams p) {
    __shared__ float As[CK][CT + 1];
    __shared__ float Bs[CK][CT + 1];
    const int tid = threadIdx.x;
    const int64_t tiles_m = (p.M + CT - 1) / CT, tiles_n = (p.N + CT - 1) / CT;
    int64_t id = blockIdx.x;
    const int64_t batch = id / (tiles_m * tiles_n);
    id -= batch * tiles_m * tiles_n;
    const int m0 = (int)(id % tiles_m) * CT, n0 = (int)(id / tiles_m) * CT;
    const _Float16 *A = p.A + group_offset(p.a_b, (int)batch);
    const _Float16 *B = p.B + group_offset(p.b_b, (int)batch);
    const int64_t c_base = group_offset(p.c_b, (int)batch);
    const int tx = tid & 15, ty = tid >> 4;                         // rows 4 tx .. + 3, columns 4 ty .. + 3

    // Each thread loads 8 elements of each operand per K step.  With `kfast` (the operand's leading
    // summed mode has stride 1) consecutive threads run along k, else along the row index; either
    // way a thread's row (or its k inside the step) is the same in every K step.
    float acc[4][4] = {};
    for (int k0 = 0; k0 < p.K; k0 += CK) {
#pragma unroll 1
        for (int e = tid; e < CT * CK; e += 256) {
            int r, k;
            if (p.a_kfast) { k = e % CK; r = e / CK; } else { r = e % CT; k = e / CT; }
            float v = 0.f;
            if (m0 + r < p.M && k0 + k < p.K) v = (float)A[group_offset(p.a_m, m0 + r) + group_offset(p.a_k, k0 + k)];
            As[k][r] = v;
            if (p.b_kfast) { k = e % CK; r = e / CK; } else { r = e % CT; k = e / CT; }
            v = 0.f;
            if (n0 + r < p.N && k0 + k < p.K) v = (float)B[group_offset(p.b_n, n0 + r) + group_offset(p.b_k, k0 + k)];
            Bs[k][r] = v;
        }
        __syncthreads();
#pragma unroll 8
        for (int k = 0; k < CK; ++k) {
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
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int n = n0 + 4 * ty + j;
        if (n >= p.N) continue;
        const int64_t col = c_base + group_offset(p.c_n, n);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int m = m0 + 4 * tx + i;
            if (m >= p.M) continue;
            const int64_t at = col + group_offset(p.c_m, m);
            float y = p.alpha * acc[i][j];
            if (p.C) y += p.beta * p.C[at];
            p.D[at] = y;
        }
    }
}

}  // namespace

hipError_t launch_contract_fallback(const ContractFallbackParams &p, hipStream_t stream) {
    const int64_t tiles = ((int64_t)(p.M + CT - 1) / CT) * ((p.N + CT - 1) / CT) * p.batches;
    hipLaunchKernelGGL(contract_fallback, dim3((unsigned)tiles), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace fg
