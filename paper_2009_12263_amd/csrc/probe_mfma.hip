// Measurement aid: the rate at which the matrix units of the chip retire
// v_mfma_f32_32x32x16_f16 (fg_probe_mfma) or v_mfma_f32_16x16x32_f16 (fg_probe_mfma_k32) when
// nothing else runs, for operands taken from a caller's buffer.
// The engine clock of this GPU is power-managed, and dense MFMA power depends on how many operand
// bits toggle: the same instruction stream measured 2.3-2.45 PFLOP/s on zeros or smooth values and
// 1.7 PFLOP/s on uniform random FP16 operands, and the 16x16x32 shape 2.0 PFLOP/s on those.  The
// benchmark reports these figures next to the GEMM so that the fraction of the *sustainable* MFMA
// rate for the workload's data can be read off.
#include "../../include/flexgemm.h"

#include <hip/hip_runtime.h>

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// Each wave holds 4 + 2 operand fragments and 8 accumulators (the register picture of the GEMM's
// wave tile) and issues iters * 32 MFMAs back to back.
__global__ __launch_bounds__(512) void mfma_only(const half8 *src, float *sink, int iters) {
    half8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = src[threadIdx.x + 512 * i];
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = src[threadIdx.x + 512 * (4 + j)];
    floatx16 c[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) c[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) c[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[j], a[i], c[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) s += c[i][j][r];
    if (s == 12345.678f && sink) sink[0] = s;   // keeps the accumulators live; never true in practice
}

// The same operand registers as 16-row fragments of 32 k: 8 + 4 fragments (the second half repeats
// the first) and 32 accumulators of 16x16; iters * 64 MFMAs per wave, the same flops per iteration.
typedef float floatx4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512) void mfma_only_k32(const half8 *src, float *sink, int iters) {
    half8 a[8], b[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = src[threadIdx.x + 512 * (i % 4)];
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = src[threadIdx.x + 512 * (4 + j % 2)];
    floatx4 c[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) c[i][j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) c[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b[j], a[i], c[i][j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += c[i][j][r];
    if (s == 12345.678f && sink) sink[0] = s;
}

// The instruction mix of the 256x256x64 kernel's K loop without its dependences: per K tile a
// wave issues 64 matrix instructions (16x16x32), 24 fragment reads of 1 KB from LDS and 8
// direct-to-LDS loads of 1 KB from global memory (a window of the caller's buffer that stays in
// the L2).  The matrix instructions use fixed operand registers, nothing waits for the data that
// is loaded, and there is no barrier: what remains is what the compute unit's issue logic, LDS
// and vector-memory path (and the power they draw) leave of the matrix-instruction rate.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(512) void kloop_mix(const half8 *src, uint32_t window_bytes, float *sink, int iters) {
    __shared__ half8 lds[8192];     // 128 KB, the size of the GEMM's tile ring
    for (int i = threadIdx.x; i < 8192; i += 512) lds[i] = src[i];
    __syncthreads();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    u32x4 rsrc;
    {
        const uint64_t a = (uint64_t)src;
        rsrc[0] = (uint32_t)a; rsrc[1] = (uint32_t)(a >> 32) & 0xffffu; rsrc[2] = window_bytes; rsrc[3] = 0x00020000u;
    }
    const uint32_t slabs = window_bytes / 1024u;        // a power of two (checked by the host)
    half8 a[8], b[4];
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = src[threadIdx.x + 512 * (i % 4)];
#pragma unroll
    for (int j = 0; j < 4; ++j) b[j] = src[threadIdx.x + 512 * (4 + j % 2)];
    floatx4 c[8][4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) c[i][j][r] = 0.f;
    const uint32_t lane_lds = (uint32_t)(uintptr_t)(lds + threadIdx.x);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < 64; ++r) {
            // written as assembly so that the order below is the order issued
            asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(c[(r >> 2) & 7][r & 3]) : "v"(b[r & 3]), "v"(a[(r >> 2) & 7]));
            if ((r * 24) / 64 != ((r + 1) * 24) / 64) {
                half8 frag;
                asm volatile("ds_read_b128 %0, %1" : "=v"(frag) : "v"(lane_lds + 8192u * (r & 7)));
            }
            if ((r * 8) / 64 != ((r + 1) * 8) / 64) {
                const uint32_t dst = (uint32_t)(uintptr_t)lds + wave * 1024u + (r & 7) * 8192u;
                const uint32_t voff = ((((uint32_t)it * 64u + r) * 8u + wave) & (slabs - 1)) * 1024u + (threadIdx.x & 63) * 16u;
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" : : "s"(dst), "v"(voff), "s"(rsrc) : "memory", "m0");
            }
        }
        asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) s += c[i][j][r];
    if (s == 12345.678f && sink) sink[0] = s;
}

fg_status probe(bool k32, const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream) {
    if (!fp16_operands || !flops_out) return FG_ERR_NULL;
    if (iters < 1 || iters > (1 << 20)) return FG_ERR_SHAPE;
    if (operand_bytes < 48 * 1024) return FG_ERR_SHAPE;      // the kernels read the first 48 KiB
    if (reinterpret_cast<uintptr_t>(fp16_operands) & 15u) return FG_ERR_ALIGN;
    const int blocks = 256;   // one workgroup of 8 waves per compute unit: 2 waves per SIMD
    hipLaunchKernelGGL(k32 ? mfma_only_k32 : mfma_only, dim3(blocks), dim3(512), 0, (hipStream_t)hip_stream,
                       (const half8 *)fp16_operands, (float *)nullptr, iters);
    if (hipGetLastError() != hipSuccess) return FG_ERR_LAUNCH;
    *flops_out = (int64_t)blocks * 8 * iters * 32 * 32768;      // 32 x 32768 = 64 x 16384 flop per wave and iteration
    return FG_OK;
}

}  // namespace

extern "C" fg_status fg_probe_kloop_mix(const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream) {
    if (!fp16_operands || !flops_out) return FG_ERR_NULL;
    if (iters < 1 || iters > (1 << 20)) return FG_ERR_SHAPE;
    if (operand_bytes < 128 * 1024) return FG_ERR_SHAPE;      // the LDS fill reads the first 128 KiB
    if (reinterpret_cast<uintptr_t>(fp16_operands) & 15u) return FG_ERR_ALIGN;
    // the direct loads walk the largest power-of-two window of the buffer, at most 4 MiB (one L2)
    uint32_t window = 128 * 1024;
    while (window < (4u << 20) && (int64_t)window * 2 <= operand_bytes) window *= 2;
    const int blocks = 256;
    hipLaunchKernelGGL(kloop_mix, dim3(blocks), dim3(512), 0, (hipStream_t)hip_stream, (const half8 *)fp16_operands, window, (float *)nullptr, iters);
    if (hipGetLastError() != hipSuccess) return FG_ERR_LAUNCH;
    *flops_out = (int64_t)blocks * 8 * iters * 64 * 16384;
    return FG_OK;
}

extern "C" fg_status fg_probe_mfma_k32(const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream) {
    return probe(true, fp16_operands, operand_bytes, iters, flops_out, hip_stream);
}

extern "C" fg_status fg_probe_mfma(const void *fp16_operands, int64_t operand_bytes, int32_t iters, int64_t *flops_out, void *hip_stream) {
    return probe(false, fp16_operands, operand_bytes, iters, flops_out, hip_stream);
}
