// Registry of the compiled kernel variants.  A variant is chosen by
// (tile shape, A K-contiguous?, B K-contiguous?, strided tensor addressing?, operator).
#pragma once
#include "gemm_kernel.hpp"

namespace fg {

// TILE_128x128_DEEP: the 128x128 tile with a ring of four buffers (128 KB of LDS, one workgroup per
// compute unit) and eight waves of 32x64 (two per SIMD, so that one wave's LDS and barrier latencies
// are covered by the other's matrix instructions), for outputs of at most one such tile per unit: a
// lone workgroup turns a K tile over too fast for a two-buffer ring to cover the memory latency.
// (2048^3: 26.5 us against 28.8 us with four waves of 64x64 and the same ring.)  Matrix and
// contraction kernels; no 16x16x32 form.
// TILE_256x256_K32: the 256x256 tile computed with 16x16x32 matrix instructions (TileCfg::M16), for
// products that fill (most of) the GPU: there the chip runs at its power limit and that instruction shape
// sustains a higher rate on the same data; on a partly filled GPU the 32x32x16 kernels are faster.
// Plain, BF16 and binary16-result matrix kernels, and the A/B-addition kernels of two layout pairs
// (other tables leave the entry empty).
enum TileId { TILE_256x256 = 0, TILE_256x128 = 1, TILE_128x128 = 2, TILE_64x64 = 3, TILE_128x128_DEEP = 4,
              TILE_256x256_K32 = 5, TILE_COUNT = 6, DIAG_TILE_COUNT = 4 };

struct KernelEntry {
    void (*fn)(const GemmParams);
    const char *name;
    int bm, bn, threads, lds_bytes;
};

// Defined by the instantiation files (one per layout pair).
const KernelEntry *kernel_table_nn();   // A M-contiguous, B K-contiguous  (A 'N', B 'N')
const KernelEntry *kernel_table_nt();   // A M-contiguous, B N-contiguous  (A 'N', B 'T')
const KernelEntry *kernel_table_tn();   // A K-contiguous, B K-contiguous  (A 'T', B 'N')
const KernelEntry *kernel_table_tt();   // A K-contiguous, B N-contiguous  (A 'T', B 'T')

// The same four layout pairs with bfloat16 A and B (plain matrices only): index = tile.
const KernelEntry *kernel_table_nn_bf16();
const KernelEntry *kernel_table_nt_bf16();
const KernelEntry *kernel_table_tn_bf16();
const KernelEntry *kernel_table_tt_bf16();

// The four layout pairs with a constant added to every loaded element of A and B: index = tile.
const KernelEntry *kernel_table_nn_xf();
const KernelEntry *kernel_table_nt_xf();
const KernelEntry *kernel_table_tn_xf();
const KernelEntry *kernel_table_tt_xf();

// The four layout pairs with C and D stored as binary16 (TileCfg::CD16): index = tile.
const KernelEntry *kernel_table_nn_h16();
const KernelEntry *kernel_table_nt_h16();
const KernelEntry *kernel_table_tn_h16();
const KernelEntry *kernel_table_tt_h16();

// Diagonal operands: index tile * 4 + {0: A diag, B K-contiguous; 1: A diag, B N-contiguous;
//                                       2: B diag, A K-contiguous; 3: B diag, A M-contiguous}.
const KernelEntry *kernel_table_diag();
// Planar complex: index ctile * 4 + {nn, nt, tn, tt}; ctile 0: 256x128, 1: 128x128, 2: 64x64.
const KernelEntry *kernel_table_cplx();
// Interleaved complex (real and imaginary part adjacent in A, B, C and D): same indexing.
const KernelEntry *kernel_table_cplx_il();
// Planar dual numbers (eps^2 = 0): same indexing as the complex table.
const KernelEntry *kernel_table_dual();
enum { CTILE_COUNT = 3 };

// Second pass of a split-K product (splitk_reduce.hip).
hipError_t launch_splitk_reduce(const float *W, int splits, int tile_begin, int tile_count, int bm, int bn, int tiles_m,
                                int tiles_n, int M, int N, float alpha, float beta, const float *C, int64_t ldc, float *D,
                                int64_t ldd, const float *bias, int bias_dim, int act, int c_act, hipStream_t stream);

// General kernel for real products with unaligned operands or a K that is not a multiple of 8
// (gemm_fallback.hip).  D is column-major; A is addressed as A[m * a_rs + k * a_ks], B as
// B[n * b_rs + k * b_ks] (element strides).
struct FallbackParams {
    int32_t M, N, K;
    const uint16_t *A, *B;
    int64_t a_rs, a_ks, b_rs, b_ks;
    const float *C;
    float *D;
    int64_t ldc, ldd;
    const float *bias;
    int32_t bias_dim, act, c_act;
    float alpha, beta;
    uint16_t a_add, b_add;       // FP16 bit patterns added to loaded A and B elements when ab_add
    bool ab_add, bf16;
};
hipError_t launch_gemm_fallback(const FallbackParams &p, hipStream_t stream);

// General kernel for contractions the tiled kernels cannot take (contract_fallback.hip): same
// mode groups as GemmParams, 64-bit element offsets.
struct ContractFallbackParams {
    int32_t M, N, K, batches;
    const _Float16 *A, *B;
    const float *C;
    float *D;
    ModeGroup a_m, a_k, b_n, b_k, c_m, c_n, a_b, b_b, c_b;
    float alpha, beta;
    int32_t a_kfast, b_kfast;    // the operand's leading summed mode has stride 1: load with lanes along k
};
hipError_t launch_contract_fallback(const ContractFallbackParams &p, hipStream_t stream);

// Entry index inside one table of real kernels: three variants per tile.
enum Variant { VARIANT_MATRIX = 0, VARIANT_CONTRACT = 1, VARIANT_CONTRACT_STREAM = 2, VARIANT_COUNT = 3 };
inline int entry_index(int tile, int variant) { return tile * VARIANT_COUNT + variant; }

// real kernels with BK = 64: ring refills are spread between the MFMAs (TileCfg::SPREAD)
#define FG_CFG(BM, BN, BK, ST, WGM, WGN, AKC, BKC, STR) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, STR, 0, 0, true>
#define FG_EMPTY_ENTRY { nullptr, nullptr, 0, 0, 0, 0 }
// the same with 16x16x32 matrix instructions (TileCfg::M16); BF: bfloat16 inputs, H: binary16 C and D
#define FG_CFG_K32(BM, BN, BK, ST, WGM, WGN, AKC, BKC, BF, H) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, 0, 0, true, BF, false, false, false, H, true>
#define FG_ENTRY_K32(BM, BN, BK, ST, WGM, WGN, AKC, BKC, BF, H, NAME)                              \
    { gemm_kernel<FG_CFG_K32(BM, BN, BK, ST, WGM, WGN, AKC, BKC, BF, H)>, NAME, BM, BN,            \
      FG_CFG_K32(BM, BN, BK, ST, WGM, WGN, AKC, BKC, BF, H)::NTHREADS,                             \
      FG_CFG_K32(BM, BN, BK, ST, WGM, WGN, AKC, BKC, BF, H)::LDS_BYTES }
#define FG_ENTRY(BM, BN, BK, ST, WGM, WGN, AKC, BKC, STR, NAME)                                    \
    { gemm_kernel<FG_CFG(BM, BN, BK, ST, WGM, WGN, AKC, BKC, STR)>, NAME, BM, BN,                  \
      FG_CFG(BM, BN, BK, ST, WGM, WGN, AKC, BKC, STR)::NTHREADS,                                   \
      FG_CFG(BM, BN, BK, ST, WGM, WGN, AKC, BKC, STR)::LDS_BYTES }

// contraction kernels whose result streams past the L2 (TileCfg::CSTREAM)
#define FG_CFG_GS(BM, BN, BK, ST, WGM, WGN, AKC, BKC) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, true, 0, 0, true, false, false, false, true>
#define FG_ENTRY_GS(BM, BN, BK, ST, WGM, WGN, AKC, BKC, NAME)                                      \
    { gemm_kernel<FG_CFG_GS(BM, BN, BK, ST, WGM, WGN, AKC, BKC)>, NAME, BM, BN,                    \
      FG_CFG_GS(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::NTHREADS,                                     \
      FG_CFG_GS(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::LDS_BYTES }

#define FG_CFG_BF16(BM, BN, BK, ST, WGM, WGN, AKC, BKC) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, 0, 0, true, true>
#define FG_ENTRY_BF16(BM, BN, BK, ST, WGM, WGN, AKC, BKC, NAME)                                    \
    { gemm_kernel<FG_CFG_BF16(BM, BN, BK, ST, WGM, WGN, AKC, BKC)>, NAME, BM, BN,                  \
      FG_CFG_BF16(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::NTHREADS,                                   \
      FG_CFG_BF16(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::LDS_BYTES }

#define FG_DEFINE_TABLE_BF16(FUNC, AKC, BKC, TAG)                                                  \
    const KernelEntry *FUNC() {                                                                    \
        static const KernelEntry t[TILE_COUNT] = {                                                 \
            FG_ENTRY_BF16(256, 256, 64, 2, 2, 4, AKC, BKC, "gemm_bf16_" TAG "_256x256x64"),        \
            FG_ENTRY_BF16(256, 128, 64, 2, 4, 2, AKC, BKC, "gemm_bf16_" TAG "_256x128x64"),        \
            FG_ENTRY_BF16(128, 128, 64, 2, 2, 2, AKC, BKC, "gemm_bf16_" TAG "_128x128x64"),        \
            FG_ENTRY_BF16(64, 64, 64, 2, 2, 2, AKC, BKC, "gemm_bf16_" TAG "_64x64x64"),            \
            FG_ENTRY_BF16(128, 128, 64, 4, 4, 2, AKC, BKC, "gemm_bf16_" TAG "_128x128x64_deep"),   \
            FG_ENTRY_K32(256, 256, 64, 2, 2, 4, AKC, BKC, true, false, "gemm_bf16_" TAG "_256x256x64_k32"), \
        };                                                                                         \
        return t;                                                                                  \
    }

#define FG_CFG_H16(BM, BN, BK, ST, WGM, WGN, AKC, BKC) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, 0, 0, true, false, false, false, false, true>
#define FG_ENTRY_H16(BM, BN, BK, ST, WGM, WGN, AKC, BKC, NAME)                                     \
    { gemm_kernel<FG_CFG_H16(BM, BN, BK, ST, WGM, WGN, AKC, BKC)>, NAME, BM, BN,                   \
      FG_CFG_H16(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::NTHREADS,                                    \
      FG_CFG_H16(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::LDS_BYTES }

#define FG_DEFINE_TABLE_H16(FUNC, AKC, BKC, TAG)                                                   \
    const KernelEntry *FUNC() {                                                                    \
        static const KernelEntry t[TILE_COUNT] = {                                                 \
            FG_ENTRY_H16(256, 256, 64, 2, 2, 4, AKC, BKC, "gemm_h16_" TAG "_256x256x64"),          \
            FG_ENTRY_H16(256, 128, 64, 2, 4, 2, AKC, BKC, "gemm_h16_" TAG "_256x128x64"),          \
            FG_ENTRY_H16(128, 128, 64, 2, 2, 2, AKC, BKC, "gemm_h16_" TAG "_128x128x64"),          \
            FG_ENTRY_H16(64, 64, 64, 2, 2, 2, AKC, BKC, "gemm_h16_" TAG "_64x64x64"),              \
            FG_ENTRY_H16(128, 128, 64, 4, 4, 2, AKC, BKC, "gemm_h16_" TAG "_128x128x64_deep"),     \
            FG_ENTRY_K32(256, 256, 64, 2, 2, 4, AKC, BKC, false, true, "gemm_h16_" TAG "_256x256x64_k32"), \
        };                                                                                         \
        return t;                                                                                  \
    }

#define FG_CFG_XF(BM, BN, BK, ST, WGM, WGN, AKC, BKC) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, 0, 0, true, false, true>
#define FG_ENTRY_XF(BM, BN, BK, ST, WGM, WGN, AKC, BKC, NAME)                                      \
    { gemm_kernel<FG_CFG_XF(BM, BN, BK, ST, WGM, WGN, AKC, BKC)>, NAME, BM, BN,                    \
      FG_CFG_XF(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::NTHREADS,                                     \
      FG_CFG_XF(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::LDS_BYTES }

// The 256x256 tile of that family on 16x16x32 matrix instructions, for the two layout pairs on
// which it measured faster than the 32x32x16 kernel (A and B contiguous along different
// directions: -3.5 % and -1.5 % run time on 8192^3; the other two pairs 0 and +3 %).
template <bool AKC, bool BKC>
inline KernelEntry xf_k32_entry(const char *name) {
    if constexpr (AKC != BKC) {
        using Cfg = TileCfg<256, 256, 64, 2, 2, 4, AKC, BKC, false, 0, 0, true, false, true, false, false, false, true>;
        return { gemm_kernel<Cfg>, name, 256, 256, Cfg::NTHREADS, Cfg::LDS_BYTES };
    } else {
        return FG_EMPTY_ENTRY;
    }
}

#define FG_DEFINE_TABLE_XF(FUNC, AKC, BKC, TAG)                                                    \
    const KernelEntry *FUNC() {                                                                    \
        static const KernelEntry t[TILE_COUNT] = {                                                 \
            FG_ENTRY_XF(256, 256, 64, 2, 2, 4, AKC, BKC, "gemm_abadd_" TAG "_256x256x64"),         \
            FG_ENTRY_XF(256, 128, 64, 2, 4, 2, AKC, BKC, "gemm_abadd_" TAG "_256x128x64"),         \
            FG_ENTRY_XF(128, 128, 64, 2, 2, 2, AKC, BKC, "gemm_abadd_" TAG "_128x128x64"),         \
            FG_ENTRY_XF(64, 64, 64, 2, 2, 2, AKC, BKC, "gemm_abadd_" TAG "_64x64x64"),             \
            FG_ENTRY_XF(128, 128, 64, 4, 4, 2, AKC, BKC, "gemm_abadd_" TAG "_128x128x64_deep"),    \
            xf_k32_entry<AKC, BKC>("gemm_abadd_" TAG "_256x256x64_k32"),                           \
        };                                                                                         \
        return t;                                                                                  \
    }

#define FG_CFG_IL(BM, BN, BK, ST, WGM, WGN, AKC, BKC) TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, 0, 1, false, false, false, true>
#define FG_ENTRY_IL(BM, BN, BK, ST, WGM, WGN, AKC, BKC, NAME)                                      \
    { gemm_kernel<FG_CFG_IL(BM, BN, BK, ST, WGM, WGN, AKC, BKC)>, NAME, BM, BN,                    \
      FG_CFG_IL(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::NTHREADS,                                     \
      FG_CFG_IL(BM, BN, BK, ST, WGM, WGN, AKC, BKC)::LDS_BYTES }

#define FG_ENTRY_X(BM, BN, BK, ST, WGM, WGN, AKC, BKC, DG, CX, NAME)                                \
    { gemm_kernel<TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, DG, CX>>, NAME, BM, BN,       \
      TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, DG, CX>::NTHREADS,                        \
      TileCfg<BM, BN, BK, ST, WGM, WGN, AKC, BKC, false, DG, CX>::LDS_BYTES }

#define FG_DEFINE_TABLE(FUNC, AKC, BKC, TAG)                                                       \
    const KernelEntry *FUNC() {                                                                    \
        static const KernelEntry t[TILE_COUNT * VARIANT_COUNT] = {                                 \
            FG_ENTRY(256, 256, 64, 2, 2, 4, AKC, BKC, false, "gemm_" TAG "_256x256x64"),           \
            FG_ENTRY(256, 256, 64, 2, 2, 4, AKC, BKC, true, "gett_" TAG "_256x256x64"),            \
            FG_ENTRY_GS(256, 256, 64, 2, 2, 4, AKC, BKC, "gett_stream_" TAG "_256x256x64"),        \
            FG_ENTRY(256, 128, 64, 2, 4, 2, AKC, BKC, false, "gemm_" TAG "_256x128x64"),           \
            FG_ENTRY(256, 128, 64, 2, 4, 2, AKC, BKC, true, "gett_" TAG "_256x128x64"),            \
            FG_ENTRY_GS(256, 128, 64, 2, 4, 2, AKC, BKC, "gett_stream_" TAG "_256x128x64"),        \
            FG_ENTRY(128, 128, 64, 2, 2, 2, AKC, BKC, false, "gemm_" TAG "_128x128x64"),           \
            FG_ENTRY(128, 128, 64, 2, 2, 2, AKC, BKC, true, "gett_" TAG "_128x128x64"),            \
            FG_ENTRY_GS(128, 128, 64, 2, 2, 2, AKC, BKC, "gett_stream_" TAG "_128x128x64"),        \
            FG_ENTRY(64, 64, 64, 2, 2, 2, AKC, BKC, false, "gemm_" TAG "_64x64x64"),               \
            FG_ENTRY(64, 64, 64, 2, 2, 2, AKC, BKC, true, "gett_" TAG "_64x64x64"),                \
            FG_ENTRY_GS(64, 64, 64, 2, 2, 2, AKC, BKC, "gett_stream_" TAG "_64x64x64"),            \
            FG_ENTRY(128, 128, 64, 4, 4, 2, AKC, BKC, false, "gemm_" TAG "_128x128x64_deep"),      \
            FG_ENTRY(128, 128, 64, 4, 4, 2, AKC, BKC, true, "gett_" TAG "_128x128x64_deep"),       \
            FG_ENTRY_GS(128, 128, 64, 4, 4, 2, AKC, BKC, "gett_stream_" TAG "_128x128x64_deep"),   \
            FG_ENTRY_K32(256, 256, 64, 2, 2, 4, AKC, BKC, false, false, "gemm_" TAG "_256x256x64_k32"), \
        };                                                                                         \
        return t;                                                                                  \
    }

}  // namespace fg
