// Tiled mixed-precision GEMM kernel template for gfx950 (CDNA4, wave64).
//
// One workgroup computes a BM x BN tile of D.  The stages are those of Section 3.1 of the paper
// (tile of A and B from global to shared memory, fragments from shared memory to registers,
// matrix-unit product, result back to global memory), re-laid for this chip:
//   * global -> LDS uses the direct-to-LDS 128-bit buffer loads, double buffered over K, so the
//     tile of step k+1 streams in while step k is multiplied;
//   * LDS tiles are XOR-swizzled (the paper pads instead and names swizzling as the missing
//     optimisation, Section 5.1);
//   * fragments are read in the lane layout v_mfma_f32_32x32x16_f16 wants: a K-contiguous
//     operand with one ds_read_b128 per fragment, an M/N-contiguous operand with the
//     transposing ds_read_b64_tr_b16;
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
#include <stdint.h>

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
    int32_t extent[kMaxGroupModes];
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
    int64_t ldc, ldd;                 // column-major C and D: (m, n) at m + n*ld
    float alpha, beta;
    int32_t bias_dim, act, has_c;
    int32_t diag_a;                   // A is diagonal: A points at the diagonal entries
    // tensor contraction: mode groups of each tensor
    ModeGroup a_m, a_k, b_n, b_k, c_m, c_n;
};

// ---- tile configuration ---------------------------------------------------------------------
// BM x BN x BK block tile, WGM x WGN waves, each wave owns a (32*TI) x (32*TJ) sub-tile made of
// 32x32 MFMA accumulators.  A_KC / B_KC: operand is K-contiguous in memory (A row-major,
// B column-major) rather than M/N-contiguous.
template <int BM_, int BN_, int WGM_, int WGN_, bool A_KC_, bool B_KC_, bool STRIDED_, bool CPLX_ = false>
struct TileCfg {
    static constexpr int BM = BM_, BN = BN_, BK = 64;
    static constexpr int WGM = WGM_, WGN = WGN_;
    static constexpr int NWAVES = WGM * WGN, NTHREADS = 64 * NWAVES;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;
    static constexpr int TI = WTM / 32, TJ = WTN / 32;
    static constexpr bool A_KC = A_KC_, B_KC = B_KC_, STRIDED = STRIDED_, CPLX = CPLX_;
    static constexpr int PLANES = CPLX ? 2 : 1;
    static constexpr int A_TILE_BYTES = BM * BK * 2, B_TILE_BYTES = BN * BK * 2;
    static constexpr int A_SLABS = A_TILE_BYTES / 1024 / NWAVES;   // 1 KB direct-to-LDS writes per wave
    static constexpr int B_SLABS = B_TILE_BYTES / 1024 / NWAVES;
    static constexpr int STAGES = 2;
    // LDS map: [A plane0 stage0 | A plane0 stage1 | (A plane1 ...) | B ...]
    static constexpr int A_BYTES = A_TILE_BYTES * STAGES * PLANES;
    static constexpr int LDS_BYTES = A_BYTES + B_TILE_BYTES * STAGES * PLANES;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 accumulators");
    static_assert(A_SLABS >= 1 && B_SLABS >= 1, "tile too small for this many waves");
    static_assert(A_TILE_BYTES % (1024 * NWAVES) == 0 && B_TILE_BYTES % (1024 * NWAVES) == 0, "");
};

// ---- swizzles -------------------------------------------------------------------------------
// K-contiguous tile: rows of 128 bytes (64 halves) = 8 chunks of 16 bytes.  Logical chunk c of
// row r is stored at chunk position c ^ ((r >> 1) & 7): sixteen consecutive rows reading the
// same logical chunk then touch sixteen different 16-byte bank groups of the 64-bank LDS.
__device__ __forceinline__ int kc_swz(int row) { return (row >> 1) & 7; }

// M/N-contiguous tile: k-rows of R halves.  The 64-byte chunk index of a k-row is XORed with
// (krow & 3) so that the four k-rows one transposing read touches fall into different banks.
template <int R>
__device__ __forceinline__ int mc_swz(int krow) { return krow & ((R / 32 - 1) < 3 ? (R / 32 - 1) : 3); }

// ---- buffer resources and direct-to-LDS loads ------------------------------------------------
// Raw buffer descriptor over a 2 GiB window starting at p (p is workgroup-uniform, so the four
// words live in scalar registers).
__device__ __forceinline__ u32x4 make_rsrc(const void *p) {
    uint64_t a = (uint64_t)p;
    u32x4 r;
    r[0] = (uint32_t)a;
    r[1] = (uint32_t)(a >> 32) & 0xffffu;   // stride 0: offsets are plain byte offsets
    r[2] = 0x7fffffffu;                     // num_records (bytes)
    r[3] = 0x00020000u;                     // 32-bit data format, no swizzle
    return r;
}

// 64 lanes x 16 bytes from global memory straight into LDS: lane l's 16 bytes land at
// lds_addr + 16*l.  lds_addr is wave-uniform (it goes to M0).  The load is tracked by vmcnt only;
// the compiler does not see it, so the caller waits with s_waitcnt vmcnt(0) before the barrier
// that publishes the tile.  (Written as assembly because the compiler, not knowing which LDS
// bytes a direct load writes, otherwise drains every outstanding load before any LDS read, which
// would serialise the prefetch of the next tile with the product of the current one.)
__device__ __forceinline__ void load16_to_lds(u32x4 rsrc, uint32_t lds_addr, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

__device__ __forceinline__ int64_t group_offset(const ModeGroup &g, int idx) {
    int64_t off = 0;
#pragma unroll
    for (int t = 0; t < kMaxGroupModes; ++t) {
        if (t < g.n) {
            int e = g.extent[t];
            int q = idx / e;
            off += (int64_t)(idx - q * e) * g.stride[t];
            idx = q;
        }
    }
    return off;
}

// ---- global -> LDS tile loader ----------------------------------------------------------------
// One operand tile: R rows (M or N index) x 64 k.  Each wave issues SLABS direct-to-LDS loads per
// K step; a load writes 1024 consecutive LDS bytes (lane l writes bytes 16*l .. 16*l+15), so the
// swizzle is applied by choosing which global chunk each lane fetches.
template <int R, bool KC, int SLABS, int NWAVES, bool STRIDED>
struct TileLoader {
    uint32_t voff[SLABS];    // per-lane byte offset from the moving base (per slab)
    const char *base;        // uniform: start of this block's panel at the current K step
    int64_t kstep_bytes;     // uniform: plain matrices, bytes to advance per K step
    ModeGroup kg;            // contraction: K mode group (for the per-step offset)
    int ktile;

    __device__ __forceinline__ void init(const _Float16 *ptr, int row0, int wave, int lane,
                                         int64_t rs, int64_t ks, const ModeGroup &rg, const ModeGroup &kgrp) {
        ktile = 0;
        if constexpr (!STRIDED) {
            base = (const char *)(ptr + (int64_t)row0 * rs);
            kstep_bytes = 64 * ks * 2;
        } else {
            base = (const char *)ptr;
            kg = kgrp;
            kstep_bytes = 0;
        }
#pragma unroll
        for (int s = 0; s < SLABS; ++s) {
            int slab = wave * SLABS + s;
            int64_t off;
            if constexpr (KC) {
                // slab = 8 rows x 8 chunks; lane -> physical (row, chunk); fetch the logical chunk
                int r = slab * 8 + (lane >> 3);
                int c = (lane & 7) ^ kc_swz(r);
                if constexpr (!STRIDED) off = (int64_t)r * rs + c * 8;
                else off = group_offset(rg, row0 + r) + c * 8;     // leading K mode has stride 1
            } else {
                // slab = (512/R) k-rows x R/8 chunks of 16 bytes
                constexpr int CH = R / 8;                          // 16-byte chunks per k-row
                int kr = slab * (64 / CH) + lane / CH;
                int p = lane % CH;                                  // physical chunk
                int c = p ^ (mc_swz<R>(kr) << 2);                   // 64-byte granular XOR
                if constexpr (!STRIDED) off = (int64_t)kr * ks + c * 8;
                else off = group_offset(rg, row0 + c * 8) + (int64_t)kr * kgrp.stride[0];
            }
            voff[s] = (uint32_t)(off * 2);
        }
    }

    // issue the loads of the current K step into the LDS tile at `lds_tile`, then advance
    __device__ __forceinline__ void issue(FG_LDS char *lds_tile, int wave) {
        const char *b = base;
        if constexpr (STRIDED) b += group_offset(kg, ktile * 64) * 2;
        u32x4 rsrc = make_rsrc(b);
        uint32_t dst = (uint32_t)(uintptr_t)lds_tile + (uint32_t)(wave * SLABS) * 1024u;
#pragma unroll
        for (int s = 0; s < SLABS; ++s) load16_to_lds(rsrc, dst + s * 1024u, voff[s]);
        if constexpr (!STRIDED) base += kstep_bytes;
        ++ktile;
    }
};

// Wait until every direct-to-LDS load this wave issued has written its bytes.
__device__ __forceinline__ void wait_direct_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// ---- LDS -> register fragment reads -----------------------------------------------------------
// Fragment of 32 rows x 16 k for v_mfma_f32_32x32x16_f16: lane l holds row l%32, k = 8*(l/32)+0..7.
template <int R, bool KC, int NT>
struct FragReader {
    // KC: one address per 16-wide k slice (the swizzle mixes the slice index into the chunk);
    //     sub-tiles are 32 rows = 4096 bytes apart.
    // MC: one address per 32-row sub-tile; k slices are 16 k-rows apart, the two halves of a
    //     fragment 4 k-rows apart.
    uint32_t addr[KC ? 4 : NT];

    __device__ __forceinline__ void init(int row_base, int lane) {
        if constexpr (KC) {
            int r = row_base + (lane & 31);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                int c = (2 * ks + (lane >> 5)) ^ kc_swz(r);
                addr[ks] = r * 128 + c * 16;
            }
        } else {
            int g = lane >> 4, i16 = lane & 15;
            int kr = 8 * (g >> 1) + (i16 >> 2);                    // + 16*ks + 4*t
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                int m = row_base + 32 * t + 16 * (g & 1) + 4 * (i16 & 3);
                int c64 = (m >> 5) ^ mc_swz<R>(kr);
                addr[t] = kr * (R * 2) + c64 * 64 + (m & 31) * 2;
            }
        }
    }

    __device__ __forceinline__ half8 read(FG_LDS const char *tile, int t, int ks) const {
        if constexpr (KC) {
            return *(FG_LDS const half8 *)(tile + addr[ks] + t * 4096);
        } else {
            FG_LDS const char *p = tile + addr[t] + ks * 16 * (R * 2);
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

// ---- the kernel -----------------------------------------------------------------------------------
template <class Cfg>
__global__ __launch_bounds__(Cfg::NTHREADS) void gemm_kernel(const GemmParams p) {
    extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
    FG_LDS char *smem = (FG_LDS char *)smem_generic;
    constexpr int BM = Cfg::BM, BN = Cfg::BN, TI = Cfg::TI, TJ = Cfg::TJ;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave % Cfg::WGM, wn = wave / Cfg::WGM;

    int tm, tn;
    block_to_tile(blockIdx.x, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    TileLoader<BM, Cfg::A_KC, Cfg::A_SLABS, Cfg::NWAVES, Cfg::STRIDED> la;
    TileLoader<BN, Cfg::B_KC, Cfg::B_SLABS, Cfg::NWAVES, Cfg::STRIDED> lb;
    la.init(p.A, m0, wave, lane, p.a_rs, p.a_ks, p.a_m, p.a_k);
    lb.init(p.B, n0, wave, lane, p.b_rs, p.b_ks, p.b_n, p.b_k);

    FragReader<BM, Cfg::A_KC, TI> fa;
    FragReader<BN, Cfg::B_KC, TJ> fb;
    fa.init(wm * Cfg::WTM, lane);
    fb.init(wn * Cfg::WTN, lane);

    floatx16 acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    FG_LDS char *lds_a = smem;
    FG_LDS char *lds_b = smem + Cfg::A_BYTES;
    const int nk = p.K / 64;

    if (nk > 0) {
        la.issue(lds_a, wave);
        lb.issue(lds_b, wave);
    }
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        // the loads of step kt (issued one step ago) have landed, for every wave, and every wave
        // is done reading the other buffer
        wait_direct_loads();
        __builtin_amdgcn_s_barrier();
        if (kt + 1 < nk) {
            la.issue(lds_a + (cur ^ 1) * Cfg::A_TILE_BYTES, wave);
            lb.issue(lds_b + (cur ^ 1) * Cfg::B_TILE_BYTES, wave);
        }
        FG_LDS const char *ta = lds_a + cur * Cfg::A_TILE_BYTES;
        FG_LDS const char *tb = lds_b + cur * Cfg::B_TILE_BYTES;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            half8 af[TI], bf[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i) af[i] = fa.read(ta, i, ks);
#pragma unroll
            for (int j = 0; j < TJ; ++j) bf[j] = fb.read(tb, j, ks);
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j)
                    // MFMA rows <- our N index, MFMA columns <- our M index: lanes of the
                    // accumulator then run along M, the contiguous direction of D
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[j], af[i], acc[i][j], 0, 0, 0);
        }
    }

    // ---- epilogue fused into the register -> global store ----
    // Accumulator (i, j), register r of lane l holds D[m][n] with m = 32 i + l % 32 and
    // n = 32 j + 8 (r / 4) + 4 (l / 32) + r % 4: a store instruction writes two runs of 32
    // consecutive m, i.e. two full 128-byte lines of a column-major D.
    const int lm = lane & 31, lh = lane >> 5;
#pragma unroll
    for (int i = 0; i < TI; ++i) {
        const int m = m0 + wm * Cfg::WTM + 32 * i + lm;
        float bias_m = 0.f;
        if (p.bias && p.bias_dim == 0) bias_m = p.bias[m];
        int64_t c_row, d_row;
        if constexpr (Cfg::STRIDED) c_row = d_row = group_offset(p.c_m, m);
        else { c_row = m; d_row = m; }
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int n = n0 + wn * Cfg::WTN + 32 * j + 8 * (r >> 2) + 4 * lh + (r & 3);
                int64_t c_off, d_off;
                if constexpr (Cfg::STRIDED) c_off = d_off = c_row + group_offset(p.c_n, n);
                else { c_off = c_row + (int64_t)n * p.ldc; d_off = d_row + (int64_t)n * p.ldd; }
                float y = p.alpha * acc[i][j][r];
                if (p.has_c) y += p.beta * p.C[c_off];
                if (p.bias) y += (p.bias_dim == 0) ? bias_m : p.bias[n];
                if (p.act == 1) y = y > 0.f ? y : 0.f;
                p.D[d_off] = y;
            }
        }
    }
}

}  // namespace fg
