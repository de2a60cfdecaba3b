// Tiled mixed-precision GEMM kernel template for gfx950 (CDNA4, wave64).
//
// One workgroup computes a BM x BN tile of D.  The stages are those of Section 3.1 of the paper
// (tile of A and B from global to shared memory, fragments from shared memory to registers,
// matrix-unit product, result back to global memory), re-laid for this chip:
//   * global -> LDS uses the direct-to-LDS 128-bit buffer loads, double buffered over K, so the
//     tile of step k+1 streams in while step k is multiplied;
//   * LDS tiles are XOR-swizzled (the paper pads instead and names swizzling as the missing
//     optimisation, Section 5.1);
//   * fragments are read in the lane layout the matrix instruction wants (v_mfma_f32_32x32x16_f16,
//     or v_mfma_f32_16x16x32_f16 in the kernels of TileCfg::M16): a K-contiguous operand with
//     one ds_read_b128 per fragment, an M/N-contiguous operand with the transposing
//     ds_read_b64_tr_b16;
//   * C is read and D written straight from/to the accumulator registers with the epilogue
//     (alpha, beta, bias, activation; Sections 4.2.3, 4.2.5, 5.3) fused into that store, so
//     the paper's stages 1, 2, 4 and 5 (C and D through shared memory) do not exist here.
//
// The layout building block of Section 4.2.2 is the pair (row offset, k offset) of each
// operand: element (r, k) of a tile lives at base + rowoff(r) + koff(k).  For a plain matrix
// these are multiples of 1 and ld; for a tensor contraction (Section 5.5) they are mixed-radix
// sums over the tensor's modes.  The kernel needs one of the two directions to be contiguous
// (stride 1) so that 16-byte accesses are possible.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

namespace fg {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define FG_LDS __attribute__((address_space(3)))

constexpr int kMaxGroupModes = 4;

// A group of tensor modes merged into one GEMM coordinate (first mode fastest).
struct ModeGroup {
    int32_t n;
    int32_t extent[kMaxGroupModes];   // every extent is >= 2 (the host drops modes of extent 1)
    uint32_t magic[kMaxGroupModes];   // division by extent[t]: idx / e == mulhi(idx, magic) >> shift
    uint32_t shift[kMaxGroupModes];   //   for 0 <= idx < 2^31 (magic = floor(2^(32+shift)/e) + 1, 2^shift < e <= 2^(shift+1))
    int64_t stride[kMaxGroupModes];   // element stride of each mode inside the tensor
};

struct GemmParams {
    int32_t M, N, K;
    int32_t tiles_m, tiles_n;
    const _Float16 *A, *A_im;
    const _Float16 *B, *B_im;
    const float *C, *C_im;
    float *D, *D_im;
    const float *bias;
    // plain matrices: offsets of element (row, k) are row*a_rs + k*a_ks (one of them is 1)
    int64_t a_rs, a_ks, b_rs, b_ks;
    int64_t a_span, b_span;           // plain matrices: elements from the base to one past the last (rounded up to 8)
    int64_t ldc, ldd;                 // column-major C and D: (m, n) at m + n*ld
    float alpha, beta;
    int32_t bias_dim, act, has_c;
    int32_t diag_a;                   // A is diagonal: A points at the diagonal entries
    // transforms on loaded elements (Section 4.3): C_ij := act(C_ij); with TileCfg::XFORM also
    // A_ik := half(A_ik + a_add), B_kj := half(B_kj + b_add), the addend as two packed halves
    int32_t c_act;
    uint32_t a_add2, b_add2;
    // Plain real matrices: the launch covers the tile ids [tile_begin, tile_begin + tile_count).
    // splits > 1 (split-K): it covers `splits` copies of that range; work item w = s * tile_count
    // + t sums K tiles [s * split_kt, (s + 1) * split_kt) of tile tile_begin + t and writes the raw
    // BM x BN partial result (alpha = 1, no C, bias or activation) to slot w of the workspace D.
    int32_t tile_begin, tile_count;
    int32_t splits, split_kt;
    // tensor contraction: mode groups of each tensor
    ModeGroup a_m, a_k, b_n, b_k, c_m, c_n;
    // batch modes (present in A, B and C): the launch covers `batches` copies of the tile grid,
    // copy t works on the slices of A, B and C at batch index t
    ModeGroup a_b, b_b, c_b;
    int32_t batches;
    // Contractions with an M-contiguous A: order in which the matrix unit sees the rows of a block
    // tile (tile_row below).  1: the order in which they are loaded.
    int32_t perm_z;
    // Matrix kernels: C and D are accessed with the default cache policy instead of the streaming
    // one (set by the host when the whole problem fits the memory-side cache; see stream_policy).
    int32_t cd_cached;
};

// Row permutation inside a block tile of a contraction (A contiguous along its leading row mode).
// A's tiles are loaded in A's own order: with a leading row mode of extent 8 Y the tile holds, for
// each of Z = BM / (8 Y) values of the next row modes, Y chunks of 8 consecutive rows.  When the
// result is contiguous along the *second* row mode, lanes that hold 32 consecutive rows of that
// order store 32 values that are far apart in C.  The matrix unit is therefore fed the rows in
// the order (8 rows, Z, Y): position x + 8 (z + Z y) takes tile row x + 8 (y + Y z), so that the
// 32 rows of an accumulator are 8 rows x 4 consecutive values of the second mode and a store
// touches a quarter of the lines.  Only fragment reads and the epilogue know of it: both address
// rows per lane, so the permutation is free.  z_count = 1 is the identity.
__device__ __forceinline__ int tile_row(int pos, int rows, int z_count) {
    const int x = pos & 7, q = pos >> 3;
    const int z = q % z_count, y = q / z_count;
    return x + 8 * (y + (rows / 8 / z_count) * z);
}

// ---- tile configuration ---------------------------------------------------------------------
// BM x BN x BK block tile, WGM x WGN waves, each wave owns a (32*TI) x (32*TJ) sub-tile made of
// 32x32 MFMA accumulators (of four 16x16 ones each with M16, regrouped for the epilogue).  A_KC / B_KC: operand is K-contiguous in memory (A row-major,
// B column-major) rather than M/N-contiguous.  STAGES LDS buffers per operand form a ring over K.
template <int BM_, int BN_, int BK_, int STAGES_, int WGM_, int WGN_, bool A_KC_, bool B_KC_, bool STRIDED_,
          int DIAG_ = 0, int CPLX_ = 0, bool SPREAD_ = false, bool BF16_ = false, bool XFORM_ = false, bool ILV_ = false,
          bool CSTREAM_ = false, bool CD16_ = false, bool M16_ = false>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, STAGES = STAGES_;
    // M16: the product is made of v_mfma_f32_16x16x32 instructions (16x16 results, 32 k per
    // instruction) instead of v_mfma_f32_32x32x16.  Same flops per cycle; on operand data that
    // keeps the chip at its power limit the 16x16x32 stream sustains a markedly higher rate.
    static constexpr bool M16 = M16_;
    static constexpr int KSLICE = M16_ ? 32 : 16;                   // k per matrix instruction
    static constexpr int KSTEPS = BK / KSLICE;                      // MFMA k-slices per tile
    static constexpr int WGM = WGM_, WGN = WGN_;
    static constexpr int NWAVES = WGM * WGN, NTHREADS = 64 * NWAVES;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int TI = WTM / 32, TJ = WTN / 32;             // 32x32 blocks of results per wave (epilogue)
    static constexpr int FI = M16_ ? 2 * TI : TI, FJ = M16_ ? 2 * TJ : TJ;   // operand fragments per wave and k-slice
    // Epilogue view of the results: 32x32 blocks of 16 registers; register r of lane l holds row
    // l % 32 and column acc_col(r) + ACC_LH * (l / 32) of its block (see gather_blocks for M16).
    static constexpr int ACC_LH = M16_ ? 8 : 4;
    static constexpr int acc_col(int r) { return M16_ ? 16 * (r >> 3) + 4 * ((r >> 2) & 1) + (r & 3) : 8 * (r >> 2) + (r & 3); }
    static constexpr bool A_KC = A_KC_, B_KC = B_KC_, STRIDED = STRIDED_;
    // 0: real; 1: complex (i^2 = -1), 2: dual (eps^2 = 0) numbers in planar-split storage
    static constexpr int CPLX = CPLX_;
    static constexpr bool SPLITK = !STRIDED_ && DIAG_ == 0 && CPLX_ == 0 && !CD16_;   // kernel understands GemmParams::splits
    static constexpr bool BF16 = BF16_;                             // A, B are bfloat16 instead of binary16
    // XFORM: a constant is added to every element of A and of B after it is loaded (the fragment
    // registers are transformed just before the matrix instructions that consume them)
    static constexpr bool XFORM = XFORM_;
    // ILV: complex operands and results are interleaved in global memory (real and imaginary part
    // of an element adjacent); LDS and registers keep the planar form
    static constexpr bool ILV = ILV_;
    static constexpr int DIAG = DIAG_;                              // 0: none, 1: A diagonal, 2: B diagonal
    // CSTREAM (contractions): every run of 32 rows of the result is one whole, aligned 128-byte
    // line of C, so C and D stream past the L2 like a matrix's (see stream_policy)
    static constexpr bool CSTREAM = CSTREAM_;
    // CD16: C and D are stored as IEEE binary16 and converted on the way (the type-conversion use
    // of transforms, Section 4.2.3: lower precision in memory, FP32 in the computation): C is
    // widened exactly when loaded, the FP32 result is rounded to nearest even when stored
    static constexpr bool CD16 = CD16_;
    // SPREAD: the refill loads of a ring buffer are issued one at a time between the MFMAs of two
    // k-slices (A's part in the slice after the buffer is retired, B's part in the next one)
    // instead of as one burst: a burst from all waves queues up in the compute unit's single
    // vector-memory path and holds back the MFMAs behind it in each wave's in-order stream.
    static constexpr bool SPREAD = SPREAD_;
    static constexpr int PLANES = CPLX ? 2 : 1;                     // real / (real, imaginary)
    static constexpr int A_TILE_BYTES = BM * BK * 2, B_TILE_BYTES = BN * BK * 2;
    static constexpr int A_SLABS = A_TILE_BYTES / 1024 / NWAVES;   // 1 KB direct-to-LDS writes per wave
    static constexpr int B_SLABS = B_TILE_BYTES / 1024 / NWAVES;
    // direct loads per wave and K step (a diagonal operand is synthesised, not loaded)
    static constexpr int LOADS_PER_TILE = ((DIAG == 1 ? 0 : A_SLABS) + (DIAG == 2 ? 0 : B_SLABS)) * PLANES;
    // LDS map: [A plane 0: stage 0 .. S-1 | A plane 1 ... | B plane 0: stage 0 .. S-1 | B plane 1 ...]
    static constexpr int A_PLANE_BYTES = A_TILE_BYTES * STAGES, B_PLANE_BYTES = B_TILE_BYTES * STAGES;
    static constexpr int A_BYTES = A_PLANE_BYTES * PLANES;
    static constexpr int LDS_BYTES = A_BYTES + B_PLANE_BYTES * PLANES;
    static_assert(BK == 32 || BK == 64, "BK must be 32 or 64");
    static_assert((STAGES & (STAGES - 1)) == 0 && STAGES >= 2, "STAGES must be a power of two");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 accumulators");
    static_assert(A_SLABS >= 1 && B_SLABS >= 1, "tile too small for this many waves");
    static_assert(A_TILE_BYTES % (1024 * NWAVES) == 0 && B_TILE_BYTES % (1024 * NWAVES) == 0, "");
    static_assert((STAGES - 1) * LOADS_PER_TILE <= 63, "vmcnt is a 6-bit counter");
    static_assert(LDS_BYTES <= 160 * 1024, "tile ring exceeds the 160 KB LDS of a compute unit");
    static_assert(DIAG == 0 || !STRIDED, "diagonal operands are a matrix feature");
    static_assert(DIAG != 1 || A_KC, "a diagonal A is synthesised K-contiguous");
    static_assert(DIAG != 2 || B_KC, "a diagonal B is synthesised K-contiguous");
    static_assert(!(CPLX && (DIAG || STRIDED)), "complex products take plain matrices");
    static_assert(!SPREAD || STAGES >= 4 || BK >= 64, "spread refills need slack before the tile is needed");
    static_assert(!M16 || (CPLX == 0 && DIAG == 0 && !ILV && BK == 64), "16x16x32 products: real, non-diagonal operands, two k-slices per tile");
    static_assert(!M16 || !STRIDED, "16x16x32 products: matrix kernels (the contraction kernels measured slower with them and are not built)");
    static_assert(!XFORM || (DIAG == 0 && CPLX == 0 && !BF16 && !STRIDED), "element-wise addition on A and B: plain real FP16 matrices");
    static_assert(!CSTREAM || STRIDED, "the streaming variant is a contraction kernel");
    static_assert(!CD16 || (CPLX == 0 && DIAG == 0 && !STRIDED && !ILV), "binary16 C and D: plain real matrix kernels");
    static_assert(!ILV || (CPLX == 1 && STAGES == 2 && !SPREAD && !STRIDED && DIAG == 0), "interleaved storage: plain complex products");
};

// ---- swizzles -------------------------------------------------------------------------------
// The LDS has 64 banks of 4 bytes: addresses 256 bytes apart share a bank.
//
// K-contiguous tile: rows of BK halves (BK/8 chunks of 16 bytes).  Logical chunk c of row r is
// stored at chunk position c ^ swz(r), where swz counts 256-byte bank lines: sixteen consecutive
// rows reading the same logical chunk (one quarter of a ds_read_b128) then touch sixteen
// different 16-byte bank groups.
template <int BK>
__device__ __forceinline__ int kc_swz(int row) { return (row / (128 / BK)) & (BK / 8 - 1); }

// M/N-contiguous tile: k-rows of R halves.  The 64-byte chunk index of a k-row is XORed with
// (krow & 3) so that the four k-rows one transposing read touches fall into different banks.
// With 16-row fragments (TileCfg::M16) half a wave reads 16 rows of eight k-rows, krow = 0..3 and
// 8..11 (+4 for the second half of the fragment): k-rows whose bit 3 is set therefore also have
// the two 32-byte halves of every 64-byte chunk swapped, which puts the eight 32-byte pieces into
// eight different bank groups.
template <int R>
__device__ __forceinline__ int mc_swz(int krow) { return R == 64 ? (krow >> 1) & 1 : krow & ((R / 32 - 1) < 3 ? (R / 32 - 1) : 3); }
// Tiles read as 32-row fragments (every kernel but TileCfg::M16) also XOR the position of a
// 16-byte piece inside its 64-byte chunk with the k-row.  The LDS serves a transposing read 32
// lanes at a time: four k-rows times 32 rows, 8 bytes per lane, i.e. every bank once if the four
// k-rows' pieces are spread out.  In the tile's own row order the 32 rows of a k-row are one
// chunk and the XOR above suffices; when a contraction permutes the rows of a tile (tile_row) the
// 32 rows are 16-byte pieces of several chunks at the same position inside each, and the XOR
// above alone maps the four k-rows onto the same banks.  Tiles of 64 rows have two chunks per
// k-row and k-rows two apart share their banks, hence their own pattern.  (Found by enumerating
// the XOR patterns against a model of the bank use; SQ_LDS_BANK_CONFLICT confirms.)
template <int R>
__device__ __forceinline__ int mc_piece(int krow) { return R == 64 ? 3 * ((krow >> 1) & 1) : krow & 3; }

// ---- buffer resources and direct-to-LDS loads ------------------------------------------------
// Raw buffer descriptor over `bytes` bytes starting at p (p is workgroup-uniform, so the four
// words live in scalar registers).  A load whose byte offset reaches past `bytes` returns zeros
// and touches no memory: that is how tiles that hang over the edge of a matrix are predicated
// (the paper leaves this to future work, Section 7).
__device__ __forceinline__ u32x4 make_rsrc(const void *p, uint32_t bytes = 0x7fffffffu) {
    uint64_t a = (uint64_t)p;
    u32x4 r;
    r[0] = (uint32_t)a;
    r[1] = (uint32_t)(a >> 32) & 0xffffu;   // stride 0: offsets are plain byte offsets
    r[2] = bytes;                           // num_records (bytes)
    r[3] = 0x00020000u;                     // 32-bit data format, no swizzle
    return r;
}

constexpr uint32_t kOutOfRange = 0x80000000u;   // a byte offset no descriptor of ours reaches

// 64 lanes x 16 bytes from global memory straight into LDS: lane l's 16 bytes land at
// lds_addr + 16*l.  lds_addr is wave-uniform (it goes to M0).  The load is tracked by vmcnt only;
// the compiler does not see it, so the kernel waits explicitly (wait_tile) before the barrier that
// publishes a tile.  (Written as assembly because the compiler, not knowing which LDS bytes a
// direct load writes, otherwise drains every outstanding load before any LDS read, which would
// serialise the prefetch of later tiles with the product of the current one.)
__device__ __forceinline__ void load16_to_lds(u32x4 rsrc, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

// Wait until at most NEWER of this wave's direct loads are still in flight (loads complete in
// order) and until every LDS read this wave issued has returned.
template <int NEWER>
__device__ __forceinline__ void wait_tile() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(NEWER) : "memory");
}

// Element offset of merged index idx.  Branch-free: the host pads the unused modes of a group
// with magic 0 and stride 0, for which the quotient is 0 and the term vanishes.
__device__ __forceinline__ int64_t group_offset(const ModeGroup &g, int idx) {
    int64_t off = 0;
#pragma unroll
    for (int t = 0; t < kMaxGroupModes; ++t) {
        const int e = g.extent[t];
        const int q = (int)(__umulhi((uint32_t)idx, g.magic[t]) >> g.shift[t]);
        off += (int64_t)(idx - q * e) * g.stride[t];
        idx = q;
    }
    return off;
}

// ---- kernel parameters read at the point of use ------------------------------------------------
// Almost all parameters are needed only when an output tile starts and when it is stored.  Taken
// from the by-value kernel argument they would be loaded at kernel entry and stay in scalar
// registers across the K loop, where the spills cost v_readlane instructions between the MFMAs.
// Reading them from the kernel-argument segment (explicit arguments start at offset 0 of it)
// through a pointer the compiler cannot trace keeps the loads where they are written; words of
// the copy that are not used are never loaded.
#define FG_CONST __attribute__((address_space(4)))
template <class T>
__device__ __forceinline__ T load_param(unsigned offset) {
    static_assert(sizeof(T) % 4 == 0, "parameters are copied word by word");
    const FG_CONST char *base = (const FG_CONST char *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(base));
    const FG_CONST uint32_t *src = (const FG_CONST uint32_t *)(base + offset);
    T v;
    uint32_t *dst = (uint32_t *)&v;
#pragma unroll
    for (unsigned w = 0; w < sizeof(T) / 4; ++w) dst[w] = src[w];
    return v;
}

// ---- global -> LDS tile loader ----------------------------------------------------------------
// One operand tile: R rows (M or N index) x BK k.  Each wave issues SLABS direct-to-LDS loads per
// K step; a load writes 1024 consecutive LDS bytes (lane l writes bytes 16*l .. 16*l+15), so the
// swizzle is applied by choosing which global chunk each lane fetches.
// ES = 2: the operand is interleaved complex (two halves per element, Section 5.4's global
// layout).  Such a tile cannot be copied by direct loads, which cannot separate the parts: it is
// fetched into registers (fetch), split, and written into the two planes of the planar LDS
// layout (commit), the conversion the paper places in the global-to-shared copy.
// FLIP (M/N-contiguous tiles read as 16-row fragments, TileCfg::M16): see mc_swz.
template <int R, int BK, bool KC, int SLABS, bool STRIDED, int ES = 1, bool FLIP = false>
struct TileLoader {
    static_assert(ES == 1 || (ES == 2 && !STRIDED), "interleaved elements: plain matrices only");
    static_assert(!FLIP || ES == 1, "");
    uint32_t voff[SLABS];    // per-lane byte offset from the moving base (per slab)
    u32x4 stage[ES == 2 ? SLABS : 1][2];   // ES == 2: the 32 fetched bytes of each slab's chunk
    const char *base;        // uniform: start of this block's panel at the current K step
    int64_t kstep_bytes;     // uniform: plain matrices, bytes to advance per K step
    int kn, kext[kMaxGroupModes];     // contraction: summed modes (count, extents, element strides)
    int64_t kstr[kMaxGroupModes];
    int kdigit[kMaxGroupModes];   // contraction: mixed-radix digits of the current K step's first k
    int64_t koff;            // contraction: element offset of those digits (kept incrementally)
    int ktile;
    // plain matrices: one byte past the last stored element, the extent of K, and (K-contiguous
    // operands) the k offset inside the tile of the chunk this lane fetches in each slab
    int64_t rem;             // bytes from `base` to the end of the stored span (negative once past it)
    int kdim, klim;          // extent of K; k's left from the current K step on
    int kchunk[SLABS];

    __device__ __forceinline__ void init(const _Float16 *ptr, int row0, int wave, int lane,
                                         int64_t rs, int64_t ks, const ModeGroup &rg, const ModeGroup &kgrp,
                                         int64_t span = 0, int kdim_ = 0, int rdim = 0) {
        ktile = 0;
        klim = BK;
        if constexpr (!STRIDED) {
            base = (const char *)(ptr + (int64_t)row0 * rs * ES);
            kstep_bytes = BK * ks * 2 * ES;
            rem = (span - (int64_t)row0 * rs) * 2 * ES;
            kdim = kdim_;
        } else {
            base = (const char *)ptr;
            kn = kgrp.n;
#pragma unroll
            for (int t = 0; t < kMaxGroupModes; ++t) { kext[t] = kgrp.extent[t]; kstr[t] = kgrp.stride[t]; }
            kstep_bytes = 0;
            koff = 0;
#pragma unroll
            for (int t = 0; t < kMaxGroupModes; ++t) kdigit[t] = 0;
        }
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            int slab = wave * SLABS + s;
            int64_t off;
            if constexpr (KC) {
                // slab = (512/BK) rows x BK/8 chunks; lane -> physical (row, chunk); fetch the
                // logical chunk that the swizzle stores there
                constexpr int CPR = BK / 8;
                int r = slab * (64 / CPR) + lane / CPR;
                int c = (lane % CPR) ^ kc_swz<BK>(r);
                kchunk[s] = c * 8;
                if constexpr (!STRIDED) off = (int64_t)r * rs + c * 8;
                else off = group_offset(rg, row0 + r) + c * 8;     // leading K mode has stride 1
                if constexpr (STRIDED) {
                    // a row past the merged row extent: the load is dropped and LDS gets zeros
                    if (row0 + r >= rdim) off = kOutOfRange / 2;
                }
            } else {
                // slab = (512/R) k-rows x R/8 chunks of 16 bytes
                constexpr int CH = R / 8;                          // 16-byte chunks per k-row
                int kr = slab * (64 / CH) + lane / CH;
                if constexpr (STRIDED) kchunk[s] = kr;             // k offset of this lane's k-row inside the tile
                int p = lane % CH;                                  // physical chunk
                int c = p ^ (mc_swz<R>(kr) << 2);                   // 64-byte granular XOR
                if constexpr (FLIP) c ^= ((kr >> 3) & 1) << 1;      // and the 32-byte halves of k-rows 8..15 mod 16 swapped
                else c ^= mc_piece<R>(kr);                          // 32-row fragments: see mc_piece
                if constexpr (!STRIDED) off = (int64_t)kr * ks + c * 8;
                else off = group_offset(rg, row0 + c * 8) + (int64_t)kr * kgrp.stride[0];
                if constexpr (STRIDED) {
                    // chunks of 8 rows never straddle the extent (the leading row mode's extent is
                    // a multiple of 8)
                    if (row0 + c * 8 >= rdim) off = kOutOfRange / 2;
                }
            }
            voff[s] = (uint32_t)(off * 2 * ES);
        }
    }

    // start at K tile kt0 instead of 0 (plain matrices only)
    __device__ __forceinline__ void skip(int kt0) {
        if constexpr (!STRIDED) {
            base += kstep_bytes * kt0;
            rem -= kstep_bytes * kt0;
        }
        ktile = kt0;
    }

    // The loads of one K step can be issued all at once (issue) or slab by slab between other
    // instructions (begin, issue_slab x SLABS, advance).
    u32x4 rsrc_cur;
    // Edges of a plain matrix: rows past the last one and (M/N-contiguous operands) k past K lie
    // beyond the stored span, so the descriptor returns zeros for them.  Rows that merely run into
    // the next column or row of the matrix read finite garbage that only reaches result rows or
    // columns nobody stores.  A K-contiguous operand's k >= K would read the neighbouring row, so
    // those chunks are sent out of range explicitly in the last K step.
    // Size of the descriptor window at `base`: what is left of the stored span, at most 2 GiB - 1
    // (the host keeps every offset a lane can form below that, so a longer rest is never needed).
    // Written on the two 32-bit halves: the scalar unit has no 64-bit ordered compare, and the
    // vector compares the compiler would use instead sit between the MFMAs of the K loop.
    __device__ __forceinline__ uint32_t window() const {
        int32_t hi = (int32_t)(rem >> 32);
        uint32_t lo = (uint32_t)rem;
        asm volatile("" : "+s"(hi), "+s"(lo));      // keeps the compiler from fusing the halves again
        const uint32_t w = (hi != 0 || lo > 0x7fffffffu) ? 0x7fffffffu : lo;
        return hi < 0 ? 0u : w;
    }
    __device__ __forceinline__ void begin() {
        const char *b = base;
        if constexpr (STRIDED) {
            b += koff * 2;
            rsrc_cur = make_rsrc(b);
        } else {
            rsrc_cur = make_rsrc(b, window());
            klim = kdim - ktile * BK;
        }
    }
    __device__ __forceinline__ void issue_slab(FG_LDS char *lds_tile, int wave, int s) {
        uint32_t dst = (uint32_t)(uintptr_t)lds_tile + (uint32_t)(wave * SLABS + s) * 1024u;
        uint32_t v = voff[s];
        if constexpr (KC && !STRIDED) {
            if (kchunk[s] >= klim) v = kOutOfRange;       // only ever true in the last K step
        }
        if constexpr (STRIDED) {
            // K steps walk the leading summed mode in strides of BK; when its extent is not a
            // multiple of BK the last step of each pass hangs over it: those k are zero-filled
            if (kdigit[0] + kchunk[s] >= kext[0]) v = kOutOfRange;
        }
        load16_to_lds(rsrc_cur, dst, v);
    }
    __device__ __forceinline__ void advance() {
        if constexpr (!STRIDED) {
            base += kstep_bytes;
            rem -= kstep_bytes;
        } else {
            // odometer step of BK along the leading summed mode (the steps of one pass cover its
            // extent rounded up to a multiple of BK); a carry moves one step along the next mode
            kdigit[0] += BK;
            koff += (int64_t)BK * kstr[0];
#pragma unroll
            for (int t = 0; t + 1 < kMaxGroupModes; ++t) {
                if (kdigit[t] >= kext[t] && t + 1 < kn) {
                    koff -= (int64_t)kdigit[t] * kstr[t];
                    kdigit[t] = 0;
                    kdigit[t + 1] += 1;
                    koff += kstr[t + 1];
                }
            }
        }
        ++ktile;
    }
    __device__ __forceinline__ void issue(FG_LDS char *lds_tile, int wave) {
        begin();
#pragma unroll
        for (int s = 0; s < SLABS; ++s) issue_slab(lds_tile, wave, s);
        advance();
    }

    // ES == 2: request the current K step's chunks (eight complex values, 32 bytes, per lane and
    // slab) into registers and move on to the next K step ...
    __device__ __forceinline__ void fetch() {
        klim = kdim - ktile * BK;
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(base), 0, (int)window(), 0x00020000);
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            uint32_t v = voff[s];
            if constexpr (KC) {
                if (kchunk[s] >= klim) v = kOutOfRange;
            }
            stage[s][0] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, v, 0, 0));
            stage[s][1] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, v, 16, 0));
        }
        advance();
    }
    // ... and, once they have arrived, split them into real and imaginary parts and write each
    // part where a direct load of a planar tile would have put it.
    __device__ __forceinline__ void commit(FG_LDS char *tile_re, FG_LDS char *tile_im, int wave) {
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            u32x4 re, im;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    // words 2w and 2w+1 of half h hold (re, im) of two consecutive elements
                    const uint32_t e0 = stage[s][h][2 * w], e1 = stage[s][h][2 * w + 1];
                    re[2 * h + w] = __builtin_amdgcn_perm(e1, e0, 0x05040100u);
                    im[2 * h + w] = __builtin_amdgcn_perm(e1, e0, 0x07060302u);
                }
            const uint32_t at = (uint32_t)(wave * SLABS + s) * 1024u + (threadIdx.x & 63) * 16u;
            *(FG_LDS u32x4 *)(tile_re + at) = re;
            *(FG_LDS u32x4 *)(tile_im + at) = im;
        }
    }
};

// ---- diagonal operand (Section 5.2) ---------------------------------------------------------------
// The operand is a vector d of diagonal entries: element (r, k) is d[r] if r == k and zero
// otherwise, and zeros are never read from memory.  The tile is synthesised straight into LDS in
// the K-contiguous swizzled layout, each lane writing the 16-byte chunk a direct load would have
// written for it.  (The second half of the paper's optimisation, skipping the inner-loop
// iterations that hold no diagonal entry, is the K range the kernel picks per tile row.)
template <int R, int BK, int SLABS>
struct DiagLoader {
    _Float16 dval[SLABS];    // d[row] of the chunk this lane writes in each slab
    int pos0[SLABS];         // row - 8*chunk: position of the diagonal inside the chunk when k0 == 0
    int ktile;

    __device__ __forceinline__ void init(const _Float16 *d, int row0, int ndiag, int wave, int lane) {
        ktile = 0;
        constexpr int CPR = BK / 8;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            int slab = wave * SLABS + s;
            int r = slab * (64 / CPR) + lane / CPR;
            int c = (lane % CPR) ^ kc_swz<BK>(r);
            dval[s] = (row0 + r < ndiag) ? d[row0 + r] : (_Float16)0.f;
            pos0[s] = row0 + r - 8 * c;
        }
    }
    __device__ __forceinline__ void skip(int kt0) { ktile = kt0; }
    __device__ __forceinline__ void begin() {}
    __device__ __forceinline__ void issue_slab(FG_LDS char *lds_tile, int wave, int s) {
        const int pos = pos0[s] - ktile * BK;      // the chunk holds k0+8c .. k0+8c+7
        half8 v;
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = (t == pos) ? dval[s] : (_Float16)0.f;
        *(FG_LDS half8 *)(lds_tile + (wave * SLABS + s) * 1024 + (threadIdx.x & 63) * 16) = v;
    }
    __device__ __forceinline__ void advance() { ++ktile; }
    __device__ __forceinline__ void issue(FG_LDS char *lds_tile, int wave) {
        begin();
#pragma unroll
        for (int s = 0; s < SLABS; ++s) issue_slab(lds_tile, wave, s);
        advance();
    }
};

// ---- LDS -> register fragment reads -----------------------------------------------------------
// Fragment of 32 rows x 16 k for v_mfma_f32_32x32x16_f16: lane l holds row l%32, k = 8*(l/32)+0..7;
// M16: 16 rows x 32 k for v_mfma_f32_16x16x32_f16: lane l holds row l%16, k = 8*(l/16)+0..7.
template <int R, int BK, bool KC, int NT, bool M16 = false>
struct FragReader {
    // KC: one address per k slice (the swizzle mixes the slice index into the chunk); sub-tiles
    //     are ROWS rows apart.
    // MC: one address per sub-tile; k slices are KW k-rows apart, the two halves of a fragment 4
    //     k-rows apart.
    static constexpr int KW = M16 ? 32 : 16, ROWS = M16 ? 16 : 32;
    static constexpr int KSTEPS = BK / KW;
    uint32_t addr[KC ? KSTEPS : NT];

    __device__ __forceinline__ void init(int row_base, int lane, int perm_z = 1) {
        if constexpr (KC) {
            int r = row_base + (lane & (ROWS - 1));
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                int c = ((KW / 8) * ks + lane / ROWS) ^ kc_swz<BK>(r);
                addr[ks] = r * (BK * 2) + c * 16;
            }
        } else if constexpr (M16) {
            // a group of 16 lanes transposes 4 k-rows x 16 rows; group g takes k-rows 8g .. 8g+3
            int g = lane >> 4, i16 = lane & 15;
            int kr = 8 * g + (i16 >> 2);                           // + 32*ks + 4*t
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                int m = tile_row(row_base + 16 * t + 4 * (i16 & 3), R, perm_z);   // 4 rows per address
                int c64 = (m >> 5) ^ mc_swz<R>(kr);
                addr[t] = kr * (R * 2) + c64 * 64 + ((m & 31) ^ (16 * (g & 1))) * 2;
            }
        } else {
            int g = lane >> 4, i16 = lane & 15;
            int kr = 8 * (g >> 1) + (i16 >> 2);                    // + 16*ks + 4*t
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                int m = tile_row(row_base + 32 * t + 16 * (g & 1) + 4 * (i16 & 3), R, perm_z);   // 4 rows per address
                int c64 = (m >> 5) ^ mc_swz<R>(kr);
                addr[t] = kr * (R * 2) + c64 * 64 + ((((m & 31) >> 3) ^ mc_piece<R>(kr)) << 4) + (m & 7) * 2;
            }
        }
    }

    __device__ __forceinline__ half8 read(FG_LDS const char *tile, int t, int ks) const {
        if constexpr (KC) {
            return *(FG_LDS const half8 *)(tile + addr[ks] + t * (ROWS * BK * 2));
        } else {
            FG_LDS const char *p = tile + addr[t] + ks * KW * (R * 2);
            short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS short4v *)(p));
            short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((FG_LDS short4v *)(p + 4 * (R * 2)));
            return __builtin_bit_cast(half8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    }
};

// ---- workgroup -> tile map ----------------------------------------------------------------------
// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Give every XCD a
// contiguous run of tiles, and walk tiles in groups of 4 tile rows so that the workgroups
// resident on one XCD at a time share A row panels and B column panels.
__device__ __forceinline__ void block_to_tile(int bid, int tiles_m, int tiles_n, int &tm, int &tn) {
    int nb = tiles_m * tiles_n;
    int id = bid;
    if ((nb & 7) == 0) id = (bid & 7) * (nb >> 3) + (bid >> 3);
    int gm = tiles_m >= 4 ? 4 : tiles_m;
    int per_group = gm * tiles_n;
    int group = id / per_group;
    int first_m = group * gm;
    int rows = (tiles_m - first_m) < gm ? (tiles_m - first_m) : gm;
    int within = id - group * per_group;
    tm = first_m + within % rows;
    tn = within / rows;
}

// ---- epilogue fused into the register -> global store -------------------------------------------
// D = act(alpha*acc + beta*C + bias) (Sections 4.2.3, 4.2.5, 5.3).  Accumulator (i, j), register r
// of lane l holds D[m][n] with m = 32 i + l % 32 and n = 32 j + 8 (r / 4) + 4 (l / 32) + r % 4: one
// store instruction writes two runs of 32 consecutive m, i.e. two full 128-byte lines of a
// column-major D.  The sixteen C values of an accumulator are fetched as one batch of independent
// loads before any of them is used.
// C is read once and D written once: in the matrix kernels both are marked non-temporal
// (streaming) so that they do not displace the A and B panels, which other workgroups of the same
// XCD re-read, from the L2 (measured: 4-5 % of the 8192^3 run time).  Not for a diagonal operand
// (no panel is re-read, and the hint only takes away what the caches would have kept of C and D);
// for contractions only in the variants the host picks when the stores are whole lines
// (TileCfg::CSTREAM): partial lines are merged by the L2, and streaming them past it measured
// three times slower.
// One element of C or D through a buffer descriptor: FP32, or binary16 widened / rounded (CD16).
template <bool HALF, int POLICY>
__device__ __forceinline__ float load_cd(__amdgpu_buffer_rsrc_t r, uint32_t voff, int soff) {
    if constexpr (HALF) {
        const unsigned short bits = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, POLICY);
        return (float)__builtin_bit_cast(_Float16, bits);
    } else {
        return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, POLICY));
    }
}
template <bool HALF, int POLICY>
__device__ __forceinline__ void store_cd(float y, __amdgpu_buffer_rsrc_t r, uint32_t voff, int soff) {
    if constexpr (HALF) {
        const _Float16 h = (_Float16)y;                                  // round to nearest even
        __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, h), r, voff, soff, POLICY);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, y), r, voff, soff, POLICY);
    }
}

// The activation as the comparison that defines it, relu(v) = v > 0 ? v : 0 (a NaN becomes 0); with
// no activation (`pass`, uniform) the value goes through untouched, so that NaN and infinities in
// the operands reach D as IEEE arithmetic produces them.  Written with a floor so that both cases
// are one compare and one select; the uniform flag is merged into the compare's lane mask.
__device__ __forceinline__ float act_clamp(float v, float floor_v, bool pass) { return ((v > floor_v) | pass) ? v : floor_v; }

template <class Cfg>
constexpr int stream_policy() { return (Cfg::DIAG == 0 && (!Cfg::STRIDED || Cfg::CSTREAM)) ? 2 : 0; }   // gfx950 cache policy: bit 1 = nt
// `block(i, j)` returns the 32x32 block (i, j) of the wave's results as sixteen registers.
template <class Cfg, bool HAS_C, class Blocks, bool CACHED = false>
__device__ __forceinline__ void epilogue(const GemmParams &p, const float *Cp, float *Dp, const Blocks &block,
                                         int m_base, int n_base, int lane) {
    constexpr int kStream = CACHED ? 0 : stream_policy<Cfg>();
    const int lm = lane & 31, lh = lane >> 5;
    const bool bias_m_on = p.bias && p.bias_dim == 0, bias_n_on = p.bias && p.bias_dim != 0;
    const float floor_v = p.act == 1 ? 0.f : -__builtin_inff();
    const float floor_c = p.c_act == 1 ? 0.f : -__builtin_inff();       // activation on loaded C
    const bool pass_v = p.act != 1, pass_c = p.c_act != 1;              // no activation: NaN and -inf pass through
    if constexpr (!Cfg::STRIDED) {
        // (m, n) at m + n*ld.  All accesses are buffer operations on a descriptor whose base is this
        // wave's corner of the tile: the per-lane part of the address is one register for all of
        // them, the rest is a scalar offset.
        constexpr bool H = Cfg::CD16;
        constexpr int ES = H ? 2 : 4;                                    // bytes per element of C and D
        const int voff_c = (lm + Cfg::ACC_LH * lh * (int)p.ldc) * ES;
        const int voff_d = (lm + Cfg::ACC_LH * lh * (int)p.ldd) * ES;
        const int ldc4 = (int)p.ldc * ES, ldd4 = (int)p.ldd * ES;
        const char *Cb = (const char *)Cp, *Db = (const char *)Dp;
        __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<char *>(HAS_C ? Cb + (m_base + (int64_t)n_base * p.ldc) * ES : Db), 0, 0x7fffffff, 0x00020000);
        __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(Db + (m_base + (int64_t)n_base * p.ldd) * ES), 0, 0x7fffffff, 0x00020000);
        const bool interior = m_base + Cfg::WTM <= p.M && n_base + Cfg::WTN <= p.N;
        constexpr bool PAIR = H && Cfg::TI % 2 == 0;
        if constexpr (PAIR) if (interior) {
            // Accumulators i and i+1 of a column block taken together.  In the accumulator layout a
            // store instruction covers 32 rows of column n (lower half-wave) and 32 rows of column
            // n + 4 (upper half-wave): for binary16 that is two half lines.  Exchanging the upper
            // half of accumulator i's register with the lower half of accumulator i+1's gives one
            // register with 64 consecutive rows of column n and one with those of column n + 4, so
            // that every instruction moves whole 128-byte lines; C arrives in that layout and the
            // same exchange brings it back to the accumulators'.  Batches of 16 values (8 registers
            // of each of the two accumulators), requested two batches ahead as below.
            constexpr int NB = Cfg::TI * Cfg::TJ;
            constexpr int AHEAD = 2;
            const int voff_p = lane * ES;
            float cv[AHEAD + 1][16];
            auto load_c = [&](int b, float (&dst)[16]) {
                const int ip = b / (2 * Cfg::TJ), j = (b >> 1) % Cfg::TJ, h = b & 1;
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) {
                    const int r = 8 * h + r8, col = 32 * j + Cfg::acc_col(r);
                    dst[2 * r8] = load_cd<H, kStream>(rc, voff_p, 64 * ES * ip + col * ldc4);
                    dst[2 * r8 + 1] = load_cd<H, kStream>(rc, voff_p, 64 * ES * ip + (col + Cfg::ACC_LH) * ldc4);
                }
            };
            auto exchange = [](float &x, float &y) {
                // upper half of x <-> lower half of y.  The two words are copied out of the result
                // before their bits are reinterpreted: a bit cast applied to an element of the
                // vector itself compiled to a read of element 0 both times.
                const auto s = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
                const unsigned s0 = s[0], s1 = s[1];
                x = __builtin_bit_cast(float, s0);
                y = __builtin_bit_cast(float, s1);
            };
            float bias_m[Cfg::TI];
#pragma unroll
            for (int i = 0; i < Cfg::TI; ++i) bias_m[i] = bias_m_on ? p.bias[m_base + 32 * i + lm] : 0.f;
            if constexpr (HAS_C) {
#pragma unroll
                for (int b = 0; b < AHEAD && b < NB; ++b) load_c(b, cv[b % (AHEAD + 1)]);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int ip = b / (2 * Cfg::TJ), j = (b >> 1) % Cfg::TJ, h = b & 1;
                if constexpr (HAS_C) {
                    if (b + AHEAD < NB) load_c(b + AHEAD, cv[(b + AHEAD) % (AHEAD + 1)]);
                }
                float b0[8], b1[8];
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) { b0[r8] = bias_m[2 * ip]; b1[r8] = bias_m[2 * ip + 1]; }
                if (bias_n_on) {
#pragma unroll
                    for (int r8 = 0; r8 < 8; ++r8) {
                        const int r = 8 * h + r8;
                        b0[r8] = b1[r8] = p.bias[n_base + 32 * j + Cfg::acc_col(r) + Cfg::ACC_LH * lh];
                    }
                }
                float y[16];
                const floatx16 acc0 = block(2 * ip, j), acc1 = block(2 * ip + 1, j);
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) {
                    const int r = 8 * h + r8;
                    float v0 = p.alpha * acc0[r] + b0[r8];
                    float v1 = p.alpha * acc1[r] + b1[r8];
                    if constexpr (HAS_C) {
                        float c0 = cv[b % (AHEAD + 1)][2 * r8], c1 = cv[b % (AHEAD + 1)][2 * r8 + 1];
                        exchange(c0, c1);
                        v0 += p.beta * act_clamp(c0, floor_c, pass_c);
                        v1 += p.beta * act_clamp(c1, floor_c, pass_c);
                    }
                    v0 = act_clamp(v0, floor_v, pass_v);
                    v1 = act_clamp(v1, floor_v, pass_v);
                    exchange(v0, v1);
                    y[2 * r8] = v0;
                    y[2 * r8 + 1] = v1;
                }
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) {
                    const int r = 8 * h + r8, col = 32 * j + Cfg::acc_col(r);
                    store_cd<H, kStream>(y[2 * r8], rd, voff_p, 64 * ES * ip + col * ldd4);
                    store_cd<H, kStream>(y[2 * r8 + 1], rd, voff_p, 64 * ES * ip + (col + Cfg::ACC_LH) * ldd4);
                }
            }
            return;
        }
        if (interior) {
            // Per accumulator (a batch of 16 values): the C values of the batch after next are
            // requested, the 16 results of this batch are computed, then their 16 stores go out
            // together.  Measured on 8192^3 against computing and storing value by value with one
            // batch of C requested ahead: +3 % (two batches ahead: +0.6 % of that).  Loads and
            // stores complete in issue order as far as the wave's counter can tell, so a batch of C
            // only counts as arrived once every store issued before its request is acknowledged;
            // two batches ahead, that is the stores of three batches ago.
            constexpr int NB = Cfg::TI * Cfg::TJ;
            constexpr int AHEAD = 2;                        // batches of C requested ahead of their use
            float cv[AHEAD + 1][16];
            auto load_c = [&](int b, float (&dst)[16]) {
                const int i = b / Cfg::TJ, j = b % Cfg::TJ;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    dst[r] = load_cd<H, kStream>(rc, voff_c, 32 * ES * i + (32 * j + Cfg::acc_col(r)) * ldc4);
            };
            float bias_m[Cfg::TI];
#pragma unroll
            for (int i = 0; i < Cfg::TI; ++i) bias_m[i] = bias_m_on ? p.bias[m_base + 32 * i + lm] : 0.f;
            if constexpr (HAS_C) {
#pragma unroll
                for (int b = 0; b < AHEAD && b < NB; ++b) load_c(b, cv[b % (AHEAD + 1)]);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int i = b / Cfg::TJ, j = b % Cfg::TJ;
                if constexpr (HAS_C) {
                    if (b + AHEAD < NB) load_c(b + AHEAD, cv[(b + AHEAD) % (AHEAD + 1)]);
                }
                float bv[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) bv[r] = bias_m[i];
                if (bias_n_on) {
#pragma unroll
                    for (int r = 0; r < 16; ++r) bv[r] = p.bias[n_base + 32 * j + Cfg::acc_col(r) + Cfg::ACC_LH * lh];
                }
                float y[16];
                const floatx16 acc_ij = block(i, j);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = p.alpha * acc_ij[r] + bv[r];
                    if constexpr (HAS_C) {
                        const float c = cv[b % (AHEAD + 1)][r];
                        v += p.beta * act_clamp(c, floor_c, pass_c);
                    }
                    y[r] = act_clamp(v, floor_v, pass_v);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    store_cd<H, kStream>(y[r], rd, voff_d, 32 * ES * i + (32 * j + Cfg::acc_col(r)) * ldd4);
            }
        } else {
            // a tile that hangs over the edge of D: rows m >= M are masked per lane (their offset is
            // sent out of the descriptor's range, which drops the access), columns n >= N per column.
            // Eight values at a time: their reads of C, then the arithmetic, then their stores.
            auto run_edge = [&](auto bias_n_tag) {
                constexpr bool BIAS_N = decltype(bias_n_tag)::value;
#pragma unroll
                for (int i = 0; i < Cfg::TI; ++i) {
                    const int m = m_base + 32 * i + lm;
                    const bool m_ok = m < p.M;
                    const uint32_t vc = m_ok ? (uint32_t)voff_c : kOutOfRange, vd = m_ok ? (uint32_t)voff_d : kOutOfRange;
                    const float bias_mi = (bias_m_on && m_ok) ? p.bias[m] : 0.f;
#pragma unroll
                    for (int j = 0; j < Cfg::TJ; ++j) {
                        const floatx16 acc_ij = block(i, j);
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            float cv[8], bv[8];
#pragma unroll
                            for (int r8 = 0; r8 < 8; ++r8) {
                                const int r = 8 * h + r8;
                                const int ncol = n_base + 32 * j + Cfg::acc_col(r) + Cfg::ACC_LH * lh;
                                const bool n_ok = ncol < p.N;
                                if constexpr (BIAS_N) bv[r8] = p.bias[n_ok ? ncol : p.N - 1];
                                else bv[r8] = bias_mi;
                                if constexpr (HAS_C)
                                    cv[r8] = load_cd<H, kStream>(rc, n_ok ? vc : kOutOfRange, 32 * ES * i + (32 * j + Cfg::acc_col(r)) * ldc4);
                            }
#pragma unroll
                            for (int r8 = 0; r8 < 8; ++r8) {
                                const int r = 8 * h + r8;
                                const bool n_ok = n_base + 32 * j + Cfg::acc_col(r) + Cfg::ACC_LH * lh < p.N;
                                float y = p.alpha * acc_ij[r] + bv[r8];
                                if constexpr (HAS_C) y += p.beta * act_clamp(cv[r8], floor_c, pass_c);
                                y = act_clamp(y, floor_v, pass_v);
                                store_cd<H, kStream>(y, rd, n_ok ? vd : kOutOfRange, 32 * ES * i + (32 * j + Cfg::acc_col(r)) * ldd4);
                            }
                        }
                    }
                }
            };
            if (bias_n_on) run_edge(std::true_type{});
            else run_edge(std::false_type{});
        }
    } else {
        // tensor contraction: element offsets are mixed-radix sums over C's row and column modes.
        // Row part: per lane, once per sub-tile row.  Column part: the 32 columns of a sub-tile are
        // decomposed in parallel, lane l taking column l % 32, and each register's column (the
        // upper half-wave sits 4 columns further) is then fetched from the lane that holds it;
        // decomposing them one after the other on the scalar unit cost several microseconds per tile.
        // C spans less than 2 GiB (checked by the host), so offsets are 32-bit buffer offsets.
        __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(HAS_C ? Cp : Dp), 0, 0x7fffffff, 0x00020000);
        __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(Dp, 0, 0x7fffffff, 0x00020000);
        const ModeGroup &c_m = p.c_m, &c_n = p.c_n;
        // rows past the merged row extent and columns past the merged column extent (edge tiles)
        // are dropped by sending their offset out of the descriptor's range
        // (a wave's rows can lie anywhere in the block tile when its rows are permuted, hence the
        // whole tile's row range)
        const int tile_m0 = m_base & ~(Cfg::BM - 1);
        const bool interior = tile_m0 + Cfg::BM <= p.M && n_base + Cfg::WTN <= p.N;
        uint32_t row4[Cfg::TI];
#pragma unroll
        for (int i = 0; i < Cfg::TI; ++i) {
            int m = m_base + 32 * i + lm;
            if constexpr (!Cfg::A_KC) m = tile_m0 + tile_row(m - tile_m0, Cfg::BM, p.perm_z);
            row4[i] = (interior || m < p.M) ? (uint32_t)group_offset(c_m, m) * 4u : kOutOfRange;
        }
#pragma unroll
        for (int j = 0; j < Cfg::TJ; ++j) {
            const int ncol = n_base + 32 * j + lm;
            const uint32_t col_of_lane = (interior || ncol < p.N) ? (uint32_t)group_offset(c_n, ncol) * 4u : kOutOfRange;
            uint32_t col4[16];
#pragma unroll
            for (int r = 0; r < 16; ++r)
                col4[r] = (uint32_t)__builtin_amdgcn_ds_bpermute((Cfg::acc_col(r) + Cfg::ACC_LH * lh) * 4, (int)col_of_lane);
            // both parts are below 2^31 when in range; if either is out of range the sum must not
            // wrap back into range (formed again for the store rather than kept: registers are short here)
            auto offset = [&](int i, int r) { return ((row4[i] | col4[r]) & kOutOfRange) ? kOutOfRange : row4[i] + col4[r]; };
            // As in the matrix epilogue: the 16 stores of an accumulator go out together, and, where
            // registers allow (the smaller tiles), the C values of the next accumulator of this
            // column block are requested before this one's results are computed.
            constexpr int AHEAD = (Cfg::TI * Cfg::TJ <= 4) ? 1 : 0;
            float cv[AHEAD + 1][16];
            auto load_c = [&](int i) {
                if constexpr (HAS_C) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        cv[i % (AHEAD + 1)][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rc, offset(i, r), 0, kStream));
                }
            };
            if constexpr (AHEAD == 1) load_c(0);
#pragma unroll
            for (int i = 0; i < Cfg::TI; ++i) {
                if constexpr (AHEAD == 1) {
                    if (i + 1 < Cfg::TI) load_c(i + 1);
                } else {
                    load_c(i);
                }
                float y[16];
                const floatx16 acc_ij = block(i, j);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v = p.alpha * acc_ij[r];
                    if constexpr (HAS_C) v += p.beta * cv[i % (AHEAD + 1)][r];
                    y[r] = act_clamp(v, floor_v, pass_v);
                }
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, y[r]), rd, offset(i, r), 0, kStream);
            }
        }
    }
}

// Interleaved complex C and D (plain complex products): element (m, n) is the pair of floats at
// 2 (m + n*ld), so a lane reads and writes 8 bytes per element and a half-wave covers 256
// consecutive bytes.  alpha and beta are real.  Rows and columns past the matrix are masked as in
// the edge path above; eight elements at a time.
template <class Cfg, bool HAS_C>
__device__ __forceinline__ void epilogue_interleaved(const GemmParams &p, floatx16 (&acc_re)[Cfg::TI][Cfg::TJ],
                                                     floatx16 (&acc_im)[Cfg::TI][Cfg::TJ], int m_base, int n_base, int lane) {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const int lm = lane & 31, lh = lane >> 5;
    const int voff_c = (lm + 4 * lh * (int)p.ldc) * 8, voff_d = (lm + 4 * lh * (int)p.ldd) * 8;
    const int ldc8 = (int)p.ldc * 8, ldd8 = (int)p.ldd * 8;
    __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<float *>(HAS_C ? p.C + 2 * (m_base + (int64_t)n_base * p.ldc) : p.D), 0, 0x7fffffff, 0x00020000);
    __amdgpu_buffer_rsrc_t rd = __builtin_amdgcn_make_buffer_rsrc(p.D + 2 * (m_base + (int64_t)n_base * p.ldd), 0, 0x7fffffff, 0x00020000);
#pragma unroll
    for (int i = 0; i < Cfg::TI; ++i) {
        const bool m_ok = m_base + 32 * i + lm < p.M;
        const uint32_t vc = m_ok ? (uint32_t)voff_c : kOutOfRange, vd = m_ok ? (uint32_t)voff_d : kOutOfRange;
#pragma unroll
        for (int j = 0; j < Cfg::TJ; ++j) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                u32x2 cv[8];
                if constexpr (HAS_C) {
#pragma unroll
                    for (int r8 = 0; r8 < 8; ++r8) {
                        const int r = 8 * h + r8;
                        const bool n_ok = n_base + 32 * j + 8 * (r >> 2) + (r & 3) + 4 * lh < p.N;
                        cv[r8] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(
                            rc, n_ok ? vc : kOutOfRange, 256 * i + (32 * j + 8 * (r >> 2) + (r & 3)) * ldc8, 2));
                    }
                }
#pragma unroll
                for (int r8 = 0; r8 < 8; ++r8) {
                    const int r = 8 * h + r8;
                    const bool n_ok = n_base + 32 * j + 8 * (r >> 2) + (r & 3) + 4 * lh < p.N;
                    float yr = p.alpha * acc_re[i][j][r], yi = p.alpha * acc_im[i][j][r];
                    if constexpr (HAS_C) {
                        yr += p.beta * __builtin_bit_cast(float, (uint32_t)cv[r8][0]);
                        yi += p.beta * __builtin_bit_cast(float, (uint32_t)cv[r8][1]);
                    }
                    u32x2 out = {__builtin_bit_cast(uint32_t, yr), __builtin_bit_cast(uint32_t, yi)};
                    __builtin_amdgcn_raw_buffer_store_b64(out, rd, n_ok ? vd : kOutOfRange,
                                                          256 * i + (32 * j + 8 * (r >> 2) + (r & 3)) * ldd8, 2);
                }
            }
        }
    }
}

// ---- the kernel -----------------------------------------------------------------------------------
// Workgroups are persistent: workgroup b computes tiles b, b + gridDim.x, ... so that the first
// loads of the next tile are in flight while the current tile is stored.
//
// C is not staged through the accumulators (stages 1-2 of Section 3.1): beta*C is added when D
// is stored, which measured faster here than starting the accumulators from C.
//
// K loop, software pipelined at two levels:
//   * tiles: STAGES LDS buffers; the direct loads of tile kt+STAGES are issued as soon as the
//     buffer of tile kt is free, so STAGES-1 tiles are in flight or ready ahead of the product;
//   * fragments: the registers of k-slice s+1 are read from LDS while the MFMAs of slice s run.
//     The barrier that publishes tile kt+1 (and retires tile kt) sits before the LAST slice of
//     tile kt, whose fragments are already in registers, so the first reads of tile kt+1 are
//     covered by that slice's MFMAs instead of stalling the matrix unit.
// Negate eight halves (flip the sign bits): exact.
__device__ __forceinline__ half8 neg8(half8 v) {
    u32x4 u = __builtin_bit_cast(u32x4, v);
    u ^= 0x80008000u;
    return __builtin_bit_cast(half8, u);
}

// Add the same two packed halves to each of the four register words of a fragment (FP16
// arithmetic, round to nearest even).
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ half8 add8(half8 v, uint32_t pair) {
    u32x4 u = __builtin_bit_cast(u32x4, v);
    const half2v w = __builtin_bit_cast(half2v, pair);
#pragma unroll
    for (int k = 0; k < 4; ++k) u[k] = __builtin_bit_cast(uint32_t, (half2v)(__builtin_bit_cast(half2v, (uint32_t)u[k]) + w));
    return __builtin_bit_cast(half8, u);
}

// One 32x32x16 matrix instruction on 16-bit fragments held as eight raw 16-bit lanes: the same
// registers are read as binary16 or as bfloat16.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
template <bool BF16>
__device__ __forceinline__ floatx16 mfma(half8 a, half8 b, floatx16 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

typedef float floatx4 __attribute__((ext_vector_type(4)));
template <bool BF16>
__device__ __forceinline__ floatx4 mfma(half8 a, half8 b, floatx4 c) {
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// M16: the 16x16 results of a wave, regrouped into the 32x32 blocks the epilogues work on.  In
// the 16x16 result (i, j) register r of lane l holds row 16 i + l % 16 and column 16 j +
// 4 (l / 16) + r.  Exchanging the odd 16-lane rows of (2i, j)'s register with the even ones of
// (2i+1, j)'s gives one register with rows 32 i + l % 32 at column 16 j + r + 8 (l / 32) and one
// with the same rows four columns further: the layout TileCfg::acc_col / ACC_LH describe, in
// which a store instruction again covers two whole 128-byte lines of a column-major result.
// One block (i, j) at a time, formed when the epilogue reaches it, so that the other results stay
// where they are until then.
template <class Cfg>
__device__ __forceinline__ floatx16 gather_block(const floatx4 (&a16)[Cfg::FI][Cfg::FJ], int i, int j) {
    floatx16 out;
#pragma unroll
    for (int nj = 0; nj < 2; ++nj)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float x = a16[2 * i][2 * j + nj][r], y = a16[2 * i + 1][2 * j + nj][r];
            const auto s = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, x), __builtin_bit_cast(unsigned, y), false, false);
            const unsigned s0 = s[0], s1 = s[1];
            out[8 * nj + r] = __builtin_bit_cast(float, s0);
            out[8 * nj + 4 + r] = __builtin_bit_cast(float, s1);
        }
    return out;
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::NTHREADS) void gemm_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    FG_LDS char *smem = (FG_LDS char *)smem_generic;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK;
    constexpr int TI = Cfg::FI, TJ = Cfg::FJ;           // operand fragments (and matrix-instruction results) per wave
    constexpr int S = Cfg::STAGES, KS = Cfg::KSTEPS, L = Cfg::LOADS_PER_TILE, P = Cfg::PLANES;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % Cfg::WGM, wn = wave / Cfg::WGM;
    const int ntiles = Cfg::SPLITK ? p.tile_count * p.splits : p.tiles_m * p.tiles_n * (Cfg::STRIDED ? p.batches : 1);
    [[maybe_unused]] const uint32_t xf_a = p.a_add2, xf_b = p.b_add2;   // used by TileCfg::XFORM only
    [[maybe_unused]] const int xf_k = p.K;

    FG_LDS char *lds_a = smem;
    FG_LDS char *lds_b = smem + Cfg::A_BYTES;

    using PlainA = TileLoader<BM, BK, Cfg::A_KC, Cfg::A_SLABS, Cfg::STRIDED, Cfg::ILV ? 2 : 1, Cfg::M16>;
    using PlainB = TileLoader<BN, BK, Cfg::B_KC, Cfg::B_SLABS, Cfg::STRIDED, Cfg::ILV ? 2 : 1, Cfg::M16>;
    constexpr int NLOADERS = Cfg::ILV ? 1 : P;      // an interleaved operand is one array, not one per plane
    using LoaderA = typename std::conditional<Cfg::DIAG == 1, DiagLoader<BM, BK, Cfg::A_SLABS>, PlainA>::type;
    using LoaderB = typename std::conditional<Cfg::DIAG == 2, DiagLoader<BN, BK, Cfg::B_SLABS>, PlainB>::type;
    LoaderA la[P];
    LoaderB lb[P];
    FragReader<BM, BK, Cfg::A_KC, TI, Cfg::M16> fa;
    FragReader<BN, BK, Cfg::B_KC, TJ, Cfg::M16> fb;
    if constexpr (Cfg::STRIDED && !Cfg::A_KC) fa.init(wm * Cfg::WTM, lane, p.perm_z);
    else fa.init(wm * Cfg::WTM, lane);
    fb.init(wn * Cfg::WTN, lane);

    // K tiles [kt0, kt0 + nkt) of the current output tile.  A diagonal operand has entries only
    // where its row index equals k, so a tile row m0 needs just the K tiles that meet
    // [m0, m0 + BM): the "skip iterations off the diagonal" predicate of Section 5.2.
    int kt0 = 0, nkt = 0;

    // start the loads of a tile: point the loaders at its panels and fill the ring
    auto start_tile = [&](int tile_id, int &m0, int &n0, int &split) {
        // parameters are re-read here rather than kept in registers across the K loop
        const GemmParams tp = load_param<GemmParams>(0);
        int tm, tn;
        split = 0;
        if constexpr (Cfg::SPLITK) {
            // which K range of a split product, and which tile of this launch's range
            split = tile_id / tp.tile_count;
            tile_id = tp.tile_begin + (tile_id - split * tp.tile_count);
        }
        if constexpr (Cfg::STRIDED) {
            // which batch index
            const int per_batch = tp.tiles_m * tp.tiles_n;
            split = tile_id / per_batch;
            tile_id -= split * per_batch;
        }
        block_to_tile(tile_id, tp.tiles_m, tp.tiles_n, tm, tn);
        m0 = tm * BM;
        n0 = tn * BN;
        const int nk = (tp.K + BK - 1) / BK;
        kt0 = 0;
        int kt1 = nk;
        if constexpr (Cfg::SPLITK) {
            if (tp.splits > 1) { kt0 = split * tp.split_kt; kt1 = kt0 + tp.split_kt; }
        }
        if constexpr (Cfg::DIAG == 1) { kt0 = m0 / BK; kt1 = (m0 + BM) / BK; }
        if constexpr (Cfg::DIAG == 2) { kt0 = n0 / BK; kt1 = (n0 + BN) / BK; }
        if (kt1 > nk) kt1 = nk;
        nkt = kt1 > kt0 ? kt1 - kt0 : 0;
        const _Float16 *ap[2] = {tp.A, tp.A_im};
        const _Float16 *bp[2] = {tp.B, tp.B_im};
        if constexpr (Cfg::STRIDED) {
            ap[0] += group_offset(tp.a_b, split);
            bp[0] += group_offset(tp.b_b, split);
        }
#pragma unroll
        for (int q = 0; q < NLOADERS; ++q) {
            if constexpr (Cfg::DIAG == 1) la[q].init(ap[q], m0, tp.M < tp.K ? tp.M : tp.K, wave, lane);
            else la[q].init(ap[q], m0, wave, lane, tp.a_rs, tp.a_ks, tp.a_m, tp.a_k, tp.a_span, tp.K, tp.M);
            if constexpr (Cfg::DIAG == 2) lb[q].init(bp[q], n0, tp.N < tp.K ? tp.N : tp.K, wave, lane);
            else lb[q].init(bp[q], n0, wave, lane, tp.b_rs, tp.b_ks, tp.b_n, tp.b_k, tp.b_span, tp.K, tp.N);
            if constexpr (Cfg::DIAG != 0 || Cfg::SPLITK) {
                if (kt0 > 0) { la[q].skip(kt0); lb[q].skip(kt0); }
            }
        }
#pragma unroll
        for (int st = 0; st < S; ++st)
            if (st < nkt) {
                if constexpr (Cfg::ILV) {
                    la[0].fetch();
                    lb[0].fetch();
                    la[0].commit(lds_a + st * Cfg::A_TILE_BYTES, lds_a + Cfg::A_PLANE_BYTES + st * Cfg::A_TILE_BYTES, wave);
                    lb[0].commit(lds_b + st * Cfg::B_TILE_BYTES, lds_b + Cfg::B_PLANE_BYTES + st * Cfg::B_TILE_BYTES, wave);
                } else {
#pragma unroll
                    for (int q = 0; q < P; ++q) {
                        la[q].issue(lds_a + q * Cfg::A_PLANE_BYTES + st * Cfg::A_TILE_BYTES, wave);
                        lb[q].issue(lds_b + q * Cfg::B_PLANE_BYTES + st * Cfg::B_TILE_BYTES, wave);
                    }
                }
            }
    };

    int tile = blockIdx.x;
    if (tile >= ntiles) return;
    int m0, n0, sp0;
    start_tile(tile, m0, n0, sp0);

    while (true) {
        const int m_base = m0 + wm * Cfg::WTM, n_base = n0 + wn * Cfg::WTN;
        using AccT = typename std::conditional<Cfg::M16, floatx4, floatx16>::type;
        AccT acc[P][TI][TJ];
#pragma unroll
        for (int q = 0; q < P; ++q)
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j)
#pragma unroll
                    for (int r = 0; r < (Cfg::M16 ? 4 : 16); ++r) acc[q][i][j][r] = 0.f;

        if (nkt > 0) {
            if (nkt >= S) wait_tile<(S - 1) * L>(); else wait_tile<0>();
            __builtin_amdgcn_s_barrier();

            // A fragments are reloaded in place (the registers of sub-tile i are free once its
            // MFMAs of this slice are issued); B fragments, used by every sub-tile row, are double
            // buffered.  Complex operands carry a second set for the imaginary planes.
            // M16 (a slice is 32 k: twice the fragment registers per row or column): A's fragments
            // pass through a window of AW registers, the one of row i being replaced by row i+AW's
            // as soon as row i's instructions are issued.
            constexpr int AW = Cfg::M16 ? (TI < 4 ? TI : 4) : TI;
            static_assert(TI % AW == 0, "row i of every slice must find its fragment in register i % AW");
            half8 af[P][AW], bf[P][2][TJ];
#pragma unroll
            for (int q = 0; q < P; ++q) {
#pragma unroll
                for (int i = 0; i < AW; ++i) af[q][i] = fa.read(lds_a + q * Cfg::A_PLANE_BYTES, i, 0);
#pragma unroll
                for (int j = 0; j < TJ; ++j) bf[q][0][j] = fb.read(lds_b + q * Cfg::B_PLANE_BYTES, j, 0);
            }

            [[maybe_unused]] bool fetched = false;      // ILV: a K step is waiting in registers
            // one K tile; MORE: another tile follows (publish it, refill the ring, prefetch its
            // first fragments)
            // RA: the ring buffer this tile retires is refilled (tile kt+S exists); RB (spread
            // refills): B's part of the previous tile's refill is still to be issued (tile kt-1+S
            // exists and kt >= 1).  Passed as compile-time constants by the peeled loop below, so
            // that the steady-state body is straight-line code (8192^3: +5 % over testing them per
            // tile, whose booleans lived in vector registers between the MFMAs); the interleaved
            // complex kernels, short of registers, test RA per tile as before.
            auto tile_body = [&](int kt, auto more_tag, auto ra_tag, auto rb_tag) {
                constexpr bool MORE = decltype(more_tag)::value;
                const bool RA = Cfg::ILV ? (kt + S < nkt) : decltype(ra_tag)::value;
                [[maybe_unused]] constexpr bool RB = decltype(rb_tag)::value;
                const int cur = kt & (S - 1);
                const int nxt = (kt + 1) & (S - 1);
                FG_LDS const char *ta = lds_a + cur * Cfg::A_TILE_BYTES;
                FG_LDS const char *tb = lds_b + cur * Cfg::B_TILE_BYTES;
                FG_LDS const char *na = lds_a + nxt * Cfg::A_TILE_BYTES;
                FG_LDS const char *nb = lds_b + nxt * Cfg::B_TILE_BYTES;
                if constexpr (Cfg::M16) {
                    // Two slices of 32 k, each TI rows of TJ matrix instructions.  The barrier that
                    // publishes tile kt+1 and retires tile kt sits in front of row BAR_I of the last
                    // slice, the first row after which a fragment of tile kt+1 is read (three
                    // quarters through the tile for the 128-row wave tile).
                    static_assert(KS == 2, "");
                    constexpr int BAR_I = TI - AW;
                    const int prev = (kt - 1) & (S - 1);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const int rb = ks & 1, wb = rb ^ 1;
                        const bool last = (ks + 1 == KS);
                        bool refill_a = false, refill_b = false;
                        if constexpr (Cfg::SPREAD) {
                            if (ks == 0 && RB) {
                                refill_b = true;
                                lb[0].begin();
                            }
                        }
                        if (!last) {
#pragma unroll
                            for (int j = 0; j < TJ; ++j) bf[0][wb][j] = fb.read(tb, j, ks + 1);
                        }
                        uint32_t add_a = 0, add_b = 0;          // two packed halves each
                        if constexpr (Cfg::XFORM) {
                            // only the last K tile can reach beyond K: before it the addends are
                            // the same in every lane and stay in scalar registers
                            const bool in_k = MORE || (kt0 + kt) * BK + ks * 32 + 8 * (lane >> 4) < xf_k;
                            add_a = in_k ? xf_a : 0u;
                            add_b = in_k ? xf_b : 0u;
#pragma unroll
                            for (int j = 0; j < TJ; ++j) bf[0][rb][j] = add8(bf[0][rb][j], add_b);
                        }
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int i = 0; i < TI; ++i) {
                            const int slot = i % AW;
                            if (last && MORE && i == BAR_I) {
                                if (RA) wait_tile<(S - 2) * L>(); else wait_tile<0>();
                                __builtin_amdgcn_s_barrier();
                                if (RA) {
                                    if constexpr (Cfg::SPREAD) {
                                        refill_a = true;
                                        la[0].begin();
                                    } else {
                                        la[0].issue(lds_a + cur * Cfg::A_TILE_BYTES, wave);
                                        lb[0].issue(lds_b + cur * Cfg::B_TILE_BYTES, wave);
                                    }
                                }
                            }
                            if constexpr (Cfg::XFORM) af[0][slot] = add8(af[0][slot], add_a);
#pragma unroll
                            for (int j = 0; j < TJ; ++j) acc[0][i][j] = mfma<Cfg::BF16>(bf[0][rb][j], af[0][slot], acc[0][i][j]);
                            // the window moves on
                            if (i + AW < TI) af[0][slot] = fa.read(ta, i + AW, ks);
                            else if (!last) af[0][slot] = fa.read(ta, i + AW - TI, ks + 1);
                            else if (MORE) af[0][slot] = fa.read(na, i + AW - TI, 0);
                            // B's first fragments of tile kt+1, over the rows after the barrier
                            // (measured against reading them all right after the barrier, and the
                            // second slice's over the rows of the first: 7 % faster on 8192^3)
                            if (last && MORE && i >= BAR_I) {
#pragma unroll
                                for (int j = 0; j < TJ; ++j)
                                    if (j * AW / TJ == i - BAR_I) bf[0][wb][j] = fb.read(nb, j, 0);
                            }
                            if constexpr (Cfg::SPREAD) {
                                // A's refill over the rows after the barrier, B's over the first slice
#pragma unroll
                                for (int n = 0; n < Cfg::A_SLABS; ++n)
                                    if (refill_a && i == BAR_I + n * AW / Cfg::A_SLABS) la[0].issue_slab(lds_a + cur * Cfg::A_TILE_BYTES, wave, n);
#pragma unroll
                                for (int n = 0; n < Cfg::B_SLABS; ++n)
                                    if (refill_b && i == n * TI / Cfg::B_SLABS) lb[0].issue_slab(lds_b + prev * Cfg::B_TILE_BYTES, wave, n);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if constexpr (Cfg::SPREAD) {
                            if (refill_a) la[0].advance();
                            if (refill_b) lb[0].advance();
                        }
                    }
                } else
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int rb = ks & 1, wb = rb ^ 1;     // KS is even: slice 0 always uses buffer 0
                    const bool last = (ks + 1 == KS);
                    // which refill loads ride along with this slice (SPREAD):
                    //   last slice (after the barrier): A's part of tile kt+S into the buffer of tile kt
                    //   slice 0: B's part of tile kt-1+S into the buffer of tile kt-1
                    bool refill_a = false, refill_b = false;
                    if (last && MORE) {
                        if constexpr (Cfg::ILV) {
                            // the K step fetched into registers one tile ago goes into the buffer
                            // that tile's barrier retired: it is published by the barrier below
                            if (fetched) {
                                la[0].commit(lds_a + nxt * Cfg::A_TILE_BYTES, lds_a + Cfg::A_PLANE_BYTES + nxt * Cfg::A_TILE_BYTES, wave);
                                lb[0].commit(lds_b + nxt * Cfg::B_TILE_BYTES, lds_b + Cfg::B_PLANE_BYTES + nxt * Cfg::B_TILE_BYTES, wave);
                            }
                        }
                        // tile kt+1 has landed (for this wave) and all of this wave's reads of tile
                        // kt have returned; after the barrier both hold for every wave
                        if (RA) wait_tile<(S - 2) * L>(); else wait_tile<0>();
                        __builtin_amdgcn_s_barrier();
                        if constexpr (Cfg::ILV) {
                            fetched = RA;
                            if (fetched) { la[0].fetch(); lb[0].fetch(); }
                        } else
                        if (RA) {
                            if constexpr (Cfg::SPREAD) {
                                refill_a = true;
#pragma unroll
                                for (int q = 0; q < P; ++q) la[q].begin();
                            } else {
#pragma unroll
                                for (int q = 0; q < P; ++q) {
                                    la[q].issue(lds_a + q * Cfg::A_PLANE_BYTES + cur * Cfg::A_TILE_BYTES, wave);
                                    lb[q].issue(lds_b + q * Cfg::B_PLANE_BYTES + cur * Cfg::B_TILE_BYTES, wave);
                                }
                            }
                        }
                    }
                    if constexpr (Cfg::SPREAD) {
                        if (ks == 0 && RB) {
                            refill_b = true;
#pragma unroll
                            for (int q = 0; q < P; ++q) lb[q].begin();
                        }
                    }
                    if (!last || MORE) {
#pragma unroll
                        for (int q = 0; q < P; ++q)
#pragma unroll
                            for (int j = 0; j < TJ; ++j)
                                bf[q][wb][j] = last ? fb.read(nb + q * Cfg::B_PLANE_BYTES, j, 0)
                                                    : fb.read(tb + q * Cfg::B_PLANE_BYTES, j, ks + 1);
                    }
                    // Scheduling fences keep the order written here: the compiler's scheduler would
                    // otherwise sink every fragment read down to its first use one slice later and
                    // expose the LDS latency in front of each MFMA pair.
                    __builtin_amdgcn_sched_barrier(0);
                    // Element-wise addition on the loaded A and B values of this slice.  Positions at
                    // or beyond K were filled with zeros by the loads and must stay zero, so their
                    // addend is zero (a lane's eight values share one k chunk, K is a multiple of 8).
                    uint32_t add_a = 0, add_b = 0;          // two packed halves each
                    if constexpr (Cfg::XFORM) {
                        const bool in_k = MORE || (kt0 + kt) * BK + ks * Cfg::KSLICE + 8 * (lane / (Cfg::M16 ? 16 : 32)) < xf_k;
                        add_a = in_k ? xf_a : 0u;
                        add_b = in_k ? xf_b : 0u;
#pragma unroll
                        for (int j = 0; j < TJ; ++j) bf[0][rb][j] = add8(bf[0][rb][j], add_b);
                        af[0][0] = add8(af[0][0], add_a);
                    }
#pragma unroll
                    for (int i = 0; i < TI; ++i) {
                        // MFMA rows <- our N index, MFMA columns <- our M index: lanes of the
                        // accumulator then run along M, the contiguous direction of D
                        if constexpr (Cfg::CPLX == 0) {
#pragma unroll
                            for (int j = 0; j < TJ; ++j)
                                acc[0][i][j] = mfma<Cfg::BF16>(bf[0][rb][j], af[0][i], acc[0][i][j]);
                        } else if constexpr (Cfg::CPLX == 1) {
                            // (Ar + i Ai)(Br + i Bi): the four real products of Section 5.4
                            const half8 nai = neg8(af[1][i]);
#pragma unroll
                            for (int j = 0; j < TJ; ++j) {
                                acc[0][i][j] = mfma<Cfg::BF16>(bf[0][rb][j], af[0][i], acc[0][i][j]);
                                acc[1][i][j] = mfma<Cfg::BF16>(bf[1][rb][j], af[0][i], acc[1][i][j]);
                                acc[0][i][j] = mfma<Cfg::BF16>(bf[1][rb][j], nai, acc[0][i][j]);
                                acc[1][i][j] = mfma<Cfg::BF16>(bf[0][rb][j], af[1][i], acc[1][i][j]);
                            }
                        } else {
                            // dual numbers (Ar + eps Ad)(Br + eps Bd), eps^2 = 0: three real products
#pragma unroll
                            for (int j = 0; j < TJ; ++j) {
                                acc[0][i][j] = mfma<Cfg::BF16>(bf[0][rb][j], af[0][i], acc[0][i][j]);
                                acc[1][i][j] = mfma<Cfg::BF16>(bf[1][rb][j], af[0][i], acc[1][i][j]);
                                acc[1][i][j] = mfma<Cfg::BF16>(bf[0][rb][j], af[1][i], acc[1][i][j]);
                            }
                        }
                        if constexpr (Cfg::XFORM) {
                            // the next sub-tile row's values, while this row's instructions run
                            if (i + 1 < TI) af[0][i + 1] = add8(af[0][i + 1], add_a);
                        }
                        if (!last || MORE) {
#pragma unroll
                            for (int q = 0; q < P; ++q)
                                af[q][i] = last ? fa.read(na + q * Cfg::A_PLANE_BYTES, i, 0)
                                                : fa.read(ta + q * Cfg::A_PLANE_BYTES, i, ks + 1);
                        }
                        if constexpr (Cfg::SPREAD) {
                            // one refill load after the MFMAs of sub-tile row i, evenly over the slice
                            const int prev = (kt - 1) & (S - 1);
#pragma unroll
                            for (int n = 0; n < Cfg::A_SLABS; ++n)
                                if (refill_a && i == n * TI / Cfg::A_SLABS) {
#pragma unroll
                                    for (int q = 0; q < P; ++q)
                                        la[q].issue_slab(lds_a + q * Cfg::A_PLANE_BYTES + cur * Cfg::A_TILE_BYTES, wave, n);
                                }
#pragma unroll
                            for (int n = 0; n < Cfg::B_SLABS; ++n)
                                if (refill_b && i == n * TI / Cfg::B_SLABS) {
#pragma unroll
                                    for (int q = 0; q < P; ++q)
                                        lb[q].issue_slab(lds_b + q * Cfg::B_PLANE_BYTES + prev * Cfg::B_TILE_BYTES, wave, n);
                                }
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (Cfg::SPREAD) {
                        if (refill_a) {
#pragma unroll
                            for (int q = 0; q < P; ++q) la[q].advance();
                        }
                        if (refill_b) {
#pragma unroll
                            for (int q = 0; q < P; ++q) lb[q].advance();
                        }
                    }
                }
            };
            constexpr std::true_type T{};
            constexpr std::false_type F{};
            if constexpr (Cfg::ILV) {
                for (int kt = 0; kt + 1 < nkt; ++kt) tile_body(kt, T, F, F);     // (RA is evaluated in the body)
            } else
            if (nkt > 1) {
                if (S < nkt) tile_body(0, T, T, F); else tile_body(0, T, F, F);
                int kt = 1;
                for (; kt + S < nkt; ++kt) tile_body(kt, T, T, T);
                for (; kt + 1 < nkt; ++kt) {            // at most S - 1 tiles: nothing left to refill with
                    if (kt - 1 + S < nkt) tile_body(kt, T, F, T); else tile_body(kt, T, F, F);
                }
            }
            tile_body(nkt - 1, F, F, F);
        }

        // next tile of this workgroup: once every wave has read its last fragments the LDS ring is
        // free, so its first loads go out before this tile's results are stored
        const int next = tile + (int)gridDim.x;
        const bool more_tiles = next < ntiles;
        int m1 = 0, n1 = 0, sp1 = 0;
        if (more_tiles) {
            wait_tile<0>();
            __builtin_amdgcn_s_barrier();
            start_tile(next, m1, n1, sp1);
        }

        {
            GemmParams ep = load_param<GemmParams>(0);
            [[maybe_unused]] int mb = m_base, nb = n_base;
            if constexpr (Cfg::SPLITK) {
                if (ep.splits > 1) {
                    // a whole BM x BN partial tile into workspace slot `tile`, tile-local coordinates
                    ep.D += (int64_t)tile * (BM * BN);
                    ep.ldd = BM; ep.M = BM; ep.N = BN;
                    mb = wm * Cfg::WTM; nb = wn * Cfg::WTN;
                }
            }
            if constexpr (Cfg::STRIDED) {
                const int64_t c_off = group_offset(ep.c_b, sp0);
                ep.D += c_off;
                if (ep.has_c) ep.C += c_off;
            }
            // the matrix kernels that stream C and D have a second copy of the epilogue without the hint
            constexpr bool TWO_POLICIES = !Cfg::STRIDED && Cfg::DIAG == 0 && Cfg::CPLX == 0 && !Cfg::ILV;
            if constexpr (Cfg::M16) {
                auto blocks = [&](int i, int j) { return gather_block<Cfg>(acc[0], i, j); };
                if (TWO_POLICIES && ep.cd_cached) {
                    if (ep.has_c) epilogue<Cfg, true, decltype(blocks), true>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                    else epilogue<Cfg, false, decltype(blocks), true>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                } else
                if (ep.has_c) epilogue<Cfg, true>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                else epilogue<Cfg, false>(ep, ep.C, ep.D, blocks, mb, nb, lane);
            } else {
                if constexpr (Cfg::ILV) {
                    if (ep.has_c) epilogue_interleaved<Cfg, true>(ep, acc[0], acc[1], m_base, n_base, lane);
                    else epilogue_interleaved<Cfg, false>(ep, acc[0], acc[1], m_base, n_base, lane);
                } else {
                    auto blocks = [&](int i, int j) -> floatx16 { return acc[0][i][j]; };
                    if (TWO_POLICIES && ep.cd_cached) {
                        if (ep.has_c) epilogue<Cfg, true, decltype(blocks), true>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                        else epilogue<Cfg, false, decltype(blocks), true>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                    } else
                    if (ep.has_c) epilogue<Cfg, true>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                    else epilogue<Cfg, false>(ep, ep.C, ep.D, blocks, mb, nb, lane);
                }
                if constexpr (Cfg::CPLX && !Cfg::ILV) {
                    auto blocks_im = [&](int i, int j) -> floatx16 { return acc[1][i][j]; };
                    if (ep.has_c) epilogue<Cfg, true>(ep, ep.C_im, ep.D_im, blocks_im, m_base, n_base, lane);
                    else epilogue<Cfg, false>(ep, ep.C_im, ep.D_im, blocks_im, m_base, n_base, lane);
                }
            }
        }

        if (!more_tiles) break;
        tile = next;
        m0 = m1;
        n0 = n1;
        sp0 = sp1;
    }
}

}  // namespace fg
