// Grouped MFMA GEMM kernels: the time-batched GEMMs of the LSTM gradient
// (input projections, output layers, weight gradients, input gradients).
//
// Five tile configurations are built; 11-13 bring their operands in by direct global->LDS loads (no staging
// registers, no LDS store instructions), transpose an operand that is not K-contiguous (dW = dA' X, dX = dA W)
// on the LDS read, and run a main loop that is software-pipelined by hand (GemmDma::run_deep); they need bf16,
// 16-byte aligned rows and K a multiple of 64:
//   12  256x256 tile on 4 waves (128x128 each, one wave per SIMD, accumulators in AGPRs), three 64-byte K
//       stages.  Problems with a rows-contiguous operand (dW, dX).
//   11  the same with two 128-byte stages: when both operands are K-contiguous (input projections) their rows
//       are fetched in whole 128-byte lines, which 64-byte stages split in two requests (measured inside the
//       training step: 1.40 against 1.48 ms per input projection, and the reverse, 1.32 against 1.25 ms, for dX).
//   13  128x256 tile on 4 waves (64x128 each), three 64-byte stages, two workgroups per CU: K-contiguous
//       operands with K < 512 or a narrow output (output layer, layer-0 input projection), whose tiles spend
//       as long storing as computing; the second workgroup's loop runs during the first one's epilogue.
//   5   256x256 tile on 8 waves (128x64 each) staged through registers, the transposition done between
//       the registers and LDS.  Large bf16 problems that miss the conditions of 11-13 (ragged K, 8-byte rows).
//   0   128x128 tile, 4 waves (64x64 each), 64-byte stages, staged through registers.  Small
//       problems and fp32 operands.
// A 256x256 tile needs half the operand bytes per flop of a 128x128 one.
#include <type_traits>
#include "gemm_core.hpp"
#include "gemm_dma.hpp"
#include "kernels.hpp"

namespace adpsgd {

// Workgroup ids are handed to the 8 XCDs round-robin; this maps them back so that each
// XCD (its own L2) works on a contiguous range of tiles.
__device__ inline int xcd_contiguous_id(int bid, int nb) {
    const int q = nb >> 3, r = nb & 7;
    const int xcd = bid & 7, local = bid >> 3;
    const int start = xcd < r ? xcd * (q + 1) : r * (q + 1) + (xcd - r) * q;
    return start + local;
}

// Workgroup -> (group, tile row, tile column).  The grid is one-dimensional over all tiles of all
// groups.  Each XCD (own L2, 32 CUs) owns a contiguous range of the ordered tile list, so it works on
// whole groups when there are enough of them instead of on a slice of every group; inside a group
// the tiles are ordered in bands of gm <= 8 tile rows walked column by column, so that the 32 tiles an
// XCD runs at one time form a gm x 32/gm patch that shares gm + 32/gm operand panels (an m-fastest
// walk of the whole group needs tiles_m + 32/tiles_m and re-reads every A panel in every round).
__device__ inline void map_tile(int bid, int total, int tiles_m, int tiles_n, int& grp, int& tm, int& tn) {
    const int id = xcd_contiguous_id(bid, total);
    const int per = tiles_m * tiles_n;
    grp = id / per;
    const int t = id - grp * per;
    const int nband = (tiles_m + 7) >> 3;
    const int gm = (tiles_m + nband - 1) / nband;
    const int band = t / (gm * tiles_n);
    const int first = band * gm;
    const int rows = tiles_m - first < gm ? tiles_m - first : gm;
    const int r = t - band * gm * tiles_n;
    tn = r / rows;
    tm = first + r - tn * rows;
}

// Epilogue shared by the GEMM kernels: C tile = acc (+ bias), fp32 or operand type.
// Every store reads its data from a register of its own (the bias is added in place, the
// bf16 values are converted into a separate array first): with one temporary register
// reused for all stores the compiler has to wait for each store before the next one.
// Bias of this lane's FN accumulator columns (0 without a bias or past the last column).  Loaded before the
// main loop: in the epilogue the load's latency would stand in front of the stores of every tile.
template <class Core, int FN>
__device__ inline void load_bias(float (&bv)[FN], const GemmDesc& p, int n0, int gi, int gd) {
    const float* bias = p.bias ? p.bias + gi * p.sBiasI + gd * p.sBiasD : nullptr;
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
        const int col = n0 + Core::acc_col(fn);
        bv[fn] = (bias && col < p.N) ? bias[col] : 0.f;
    }
}

template <typename T, class Core, int FM, int FN>
__device__ inline void store_tile(f32x16_t (&acc)[FM][FN], const float (&bias)[FN], const GemmDesc& p, int m0, int n0, int gi, int gd) {
    const int64_t coff = gi * p.sCi + gd * p.sCd;
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
        const int col = n0 + Core::acc_col(fn);
        if (col >= p.N) continue;
        const float bv = bias[fn];
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            const int row0 = m0 + Core::acc_row(fm, 0);          // rows of this lane: row0 + 8*(i/4) + i%4
            const int64_t o = coff + (int64_t)row0 * p.ldc + col;
            if (p.c_elem) {
                T* c = (T*)p.C + o;
                if constexpr (sizeof(T) == 2) {
                    uint32_t hb[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) hb[i] = f32_to_bf16(acc[fm][fn][i] + bv);
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int r = 8 * (i >> 2) + (i & 3);
                        if (row0 + r < p.M) c[(int64_t)r * p.ldc] = (bf16_t)hb[i];
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[fm][fn][i] += bv;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int r = 8 * (i >> 2) + (i & 3);
                        if (row0 + r < p.M) c[(int64_t)r * p.ldc] = acc[fm][fn][i];
                    }
                }
            } else {
                float* c = (float*)p.C + o;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[fm][fn][i] += bv;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int r = 8 * (i >> 2) + (i & 3);
                    // written once, read by a later kernel: keep it from displacing the operand panels in L2
                    if (row0 + r < p.M) __builtin_nontemporal_store(acc[fm][fn][i], c + (int64_t)r * p.ldc);
                }
            }
        }
    }
}

// Stores whose address is a wave-uniform 64-bit pointer (SGPR pair) plus a per-lane 32-bit byte offset.
// Written as inline asm because the compiler otherwise folds the uniform part into a 64-bit vector
// address and recomputes it with vector multiply-adds for every store.
__device__ inline void store_u_f32_(uint32_t off, float v, const void* base_uniform) {
    asm volatile("global_store_dword %0, %1, %2" :: "v"(off), "v"(v), "s"(base_uniform) : "memory");
}
__device__ inline void store_u_f32_nt_(uint32_t off, float v, const void* base_uniform) {
    asm volatile("global_store_dword %0, %1, %2 nt" :: "v"(off), "v"(v), "s"(base_uniform) : "memory");
}
__device__ inline void store_u_b16_(uint32_t off, uint32_t v, const void* base_uniform) {
    asm volatile("global_store_short %0, %1, %2" :: "v"(off), "v"(v), "s"(base_uniform) : "memory");
}

// The same for a tile that lies wholly inside C (no row or column guard): every store is one
// instruction whose address is a wave-uniform row pointer plus a per-lane byte offset that is the
// same for all stores of the lane, so the epilogue costs no vector address arithmetic and no branches.
// Needs (4 * ldc + 32) * 4 bytes to fit the 32-bit offset (checked by the caller).
template <typename T, class Core, int FM, int FN>
__device__ inline void store_tile_interior(f32x16_t (&acc)[FM][FN], const float (&bias)[FN], const GemmDesc& p, int m0, int n0, int gi, int gd) {
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wave_m = wave / Core::kWN, wave_n = wave % Core::kWN;
    const uint32_t lane_elem = (uint32_t)(4 * (lane >> 5)) * (uint32_t)p.ldc + (uint32_t)(lane & 31);
    const int64_t tile_off = gi * p.sCi + gd * p.sCd + (int64_t)(m0 + wave_m * FM * 32) * p.ldc + n0 + wave_n * FN * 32;
    const bool narrow = p.c_elem && sizeof(T) == 2;
    const int esz = narrow ? 2 : 4;
    const char* cbase = (const char*)p.C + tile_off * esz;
    const uint32_t lane_off = lane_elem * (uint32_t)esz;
    const int64_t row_bytes = (int64_t)p.ldc * esz;
#pragma unroll
    for (int fn = 0; fn < FN; ++fn) {
        const float bv = bias[fn];
#pragma unroll
        for (int fm = 0; fm < FM; ++fm) {
            const char* fbase = cbase + (int64_t)(fm * 32) * row_bytes + fn * 32 * esz;
            if (narrow) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    store_u_b16_(lane_off, f32_to_bf16(acc[fm][fn][i] + bv), fbase + (8 * (i >> 2) + (i & 3)) * row_bytes);
            } else if (p.c_elem) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    store_u_f32_(lane_off, acc[fm][fn][i] + bv, fbase + (8 * (i >> 2) + (i & 3)) * row_bytes);
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i)   // written once, read by a later kernel: keep it out of L2
                    store_u_f32_nt_(lane_off, acc[fm][fn][i] + bv, fbase + (8 * (i >> 2) + (i & 3)) * row_bytes);
            }
        }
    }
}

template <int FM, int FN> __device__ inline void zero_tile(f32x16_t (&acc)[FM][FN]) {
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
}

template <typename T, bool AKC, bool BKC, int WM, int WN, int FM, int FN, int VB, int SB>
__global__ __launch_bounds__(64 * WM * WN) void gemm_kernel(GemmDesc p) {
    typedef typename std::conditional<AKC, KcSrc<T>, McSrc<T>>::type ASrc;
    typedef typename std::conditional<BKC, KcSrc<T>, McSrc<T>>::type BSrc;
    typedef GemmCore<T, ASrc, BSrc, WM, WN, FM, FN, VB, SB> Core;
    __shared__ __attribute__((aligned(16))) char lds[Core::LDS_BYTES];

    const int tiles_m = (p.M + Core::BM - 1) / Core::BM, tiles_n = (p.N + Core::BN - 1) / Core::BN;
    int grp, tm, tn;
    map_tile(blockIdx.x, gridDim.x, tiles_m, tiles_n, grp, tm, tn);
    const int gi = p.lmap.idx[grp / p.groupsD], gd = grp % p.groupsD;
    const int m0 = tm * Core::BM, n0 = tn * Core::BN;
    const T* A = (const T*)p.A + gi * p.sAi + gd * p.sAd;
    const T* B = (const T*)p.B + gi * p.sBi + gd * p.sBd;

    ASrc a; BSrc b;
    if constexpr (AKC) { a.base = A + (int64_t)m0 * p.lda; } else { a.base = A + m0; }
    a.ld = p.lda; a.R = p.M - m0;
    if constexpr (BKC) { b.base = B + (int64_t)n0 * p.ldb; } else { b.base = B + n0; }
    b.ld = p.ldb; b.R = p.N - n0;

    f32x16_t acc[FM][FN];
    zero_tile<FM, FN>(acc);
    Core::run(acc, a, b, p.K, lds);
    float bias[FN];          // (this register-staged loop has no registers to spare for an early load)
    load_bias<Core, FN>(bias, p, n0, gi, gd);
    store_tile<T, Core, FM, FN>(acc, bias, p, m0, n0, gi, gd);
}

// Same tile bookkeeping with the direct-to-LDS main loop (16-byte aligned operands, K a multiple of
// the stage length).
template <typename T, bool AKC, bool BKC, int WM, int WN, int FM, int FN, int SB, int NS>
__global__ __launch_bounds__(64 * WM * WN, (WM * WN == 4 && FM * FN == 8) ? 2 : 1) void gemm_dma_kernel(GemmDesc p) {
    typedef typename std::conditional<AKC, KcSrc<T>, McSrc<T>>::type ASrc;
    typedef typename std::conditional<BKC, KcSrc<T>, McSrc<T>>::type BSrc;
    typedef GemmDma<T, ASrc, BSrc, WM, WN, FM, FN, SB, NS> Core;
    __shared__ __attribute__((aligned(1024))) char lds[Core::LDS_BYTES];

    const int tiles_m = (p.M + Core::BM - 1) / Core::BM, tiles_n = (p.N + Core::BN - 1) / Core::BN;
    int grp, tm, tn;
    map_tile(blockIdx.x, gridDim.x, tiles_m, tiles_n, grp, tm, tn);
    const int gi = p.lmap.idx[grp / p.groupsD], gd = grp % p.groupsD;
    const int m0 = tm * Core::BM, n0 = tn * Core::BN;
    const T* A = (const T*)p.A + gi * p.sAi + gd * p.sAd;
    const T* B = (const T*)p.B + gi * p.sBi + gd * p.sBd;
    ASrc a; BSrc b;
    // A rows-contiguous operand is loaded in chunks of 8 rows: its row count is rounded up (its k-rows
    // are ld >= that many elements long, so the extra rows are readable; their products are never stored).
    if constexpr (AKC) { a.base = A + (int64_t)m0 * p.lda; a.R = p.M - m0; } else { a.base = A + m0; a.R = (p.M - m0 + 7) & ~7; }
    a.ld = p.lda;
    if constexpr (BKC) { b.base = B + (int64_t)n0 * p.ldb; b.R = p.N - n0; } else { b.base = B + n0; b.R = (p.N - n0 + 7) & ~7; }
    b.ld = p.ldb;

    float bias[FN];
    load_bias<Core, FN>(bias, p, n0, gi, gd);
    f32x16_t acc[FM][FN];
    zero_tile<FM, FN>(acc);
    if constexpr (WM * WN == 4 && (FM * FN == 16 || FM * FN == 8)) Core::run_deep(acc, a, b, p.K, lds);
    else Core::run(acc, a, b, p.K, lds);
    if (m0 + Core::BM <= p.M && n0 + Core::BN <= p.N && p.ldc < (1 << 26)) store_tile_interior<T, Core, FM, FN>(acc, bias, p, m0, n0, gi, gd);
    else store_tile<T, Core, FM, FN>(acc, bias, p, m0, n0, gi, gd);
}

template <typename T, bool AKC, bool BKC, int WM, int WN, int FM, int FN, int VB, int SB>
static hipError_t launch_t(const GemmDesc& d, hipStream_t s) {
    constexpr int BM = 32 * FM * WM, BN = 32 * FN * WN;
    const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
    dim3 grid((unsigned)(tiles_m * tiles_n * d.groupsI * d.groupsD));
    hipLaunchKernelGGL((gemm_kernel<T, AKC, BKC, WM, WN, FM, FN, VB, SB>), grid, dim3(64 * WM * WN), 0, s, d);
    return hipGetLastError();
}

template <typename T, int WM, int WN, int FM, int FN, int VB, int SB>
static hipError_t launch_layout(const GemmDesc& d, hipStream_t s) {
    const int key = (d.a_kc ? 2 : 0) | (d.b_kc ? 1 : 0);
    switch (key) {
        case 0: return launch_t<T, false, false, WM, WN, FM, FN, VB, SB>(d, s);
        case 1: return launch_t<T, false, true, WM, WN, FM, FN, VB, SB>(d, s);
        case 2: return launch_t<T, true, false, WM, WN, FM, FN, VB, SB>(d, s);
        default: return launch_t<T, true, true, WM, WN, FM, FN, VB, SB>(d, s);
    }
}

template <typename T, bool AKC, bool BKC, int WM, int WN, int FM, int FN, int SB, int NS>
static hipError_t launch_dma_t(const GemmDesc& d, hipStream_t s) {
    constexpr int BM = 32 * FM * WM, BN = 32 * FN * WN;
    const int tiles_m = (d.M + BM - 1) / BM, tiles_n = (d.N + BN - 1) / BN;
    dim3 grid((unsigned)(tiles_m * tiles_n * d.groupsI * d.groupsD));
    hipLaunchKernelGGL((gemm_dma_kernel<T, AKC, BKC, WM, WN, FM, FN, SB, NS>), grid, dim3(64 * WM * WN), 0, s, d);
    return hipGetLastError();
}

template <typename T, int WM, int WN, int FM, int FN, int SB, int NS>
static hipError_t launch_dma(const GemmDesc& d, hipStream_t s) {
    const int key = (d.a_kc ? 2 : 0) | (d.b_kc ? 1 : 0);
    switch (key) {
        case 0: return launch_dma_t<T, false, false, WM, WN, FM, FN, SB, NS>(d, s);
        case 1: return launch_dma_t<T, false, true, WM, WN, FM, FN, SB, NS>(d, s);
        case 2: return launch_dma_t<T, true, false, WM, WN, FM, FN, SB, NS>(d, s);
        default: return launch_dma_t<T, true, true, WM, WN, FM, FN, SB, NS>(d, s);
    }
}

static bool aligned_to(const void* p, int64_t ld, int64_t s1, int64_t s2, int esz, int bytes) {
    return ((uintptr_t)p % bytes == 0) && ((ld * esz) % bytes == 0) && ((s1 * esz) % bytes == 0) &&
           ((s2 * esz) % bytes == 0);
}

hipError_t launch_gemm(const GemmDesc& d, hipStream_t s) {
    if (d.M < 1 || d.N < 1 || d.K < 1 || d.groupsI < 1 || d.groupsI > 128 || d.groupsD < 1) return hipErrorInvalidValue;
    if (d.tile != -1 && d.tile != 0 && d.tile != 5 && (d.tile < 11 || d.tile > 13)) return hipErrorInvalidValue;
    // one-dimensional grid over all tiles of all groups (smallest tile 128 x 128)
    if ((int64_t)((d.M + 127) / 128) * ((d.N + 127) / 128) * d.groupsI * d.groupsD > 0x7fffffff) return hipErrorInvalidValue;
    const int esz = d.precision ? 2 : 4;
    const int quad = 4 * esz;    // every operand must allow loads of 4 elements
    if (!aligned_to(d.A, d.lda, d.sAi, d.sAd, esz, quad) || !aligned_to(d.B, d.ldb, d.sBi, d.sBd, esz, quad))
        return hipErrorInvalidValue;
    if (d.precision == 0) return launch_layout<float, 2, 2, 2, 2, 16, 64>(d, s);
    bool wide = true;
    if (d.a_kc && !aligned_to(d.A, d.lda, d.sAi, d.sAd, esz, 16)) wide = false;
    if (d.b_kc && !aligned_to(d.B, d.ldb, d.sBi, d.sBd, esz, 16)) wide = false;
    if (!wide) return launch_layout<bf16_t, 2, 2, 2, 2, 8, 64>(d, s);
    int v = d.tile;
    if (v < 0) {
        // 256x256 tiles once there are enough of them to fill the 256 CUs
        const int64_t big_tiles = (int64_t)((d.M + 255) / 256) * ((d.N + 255) / 256) * d.groupsI * d.groupsD;
        // Short contractions (a tile's first loads, stores and hand-over weigh as much as its loop) and row counts that
        // leave the last 256-row band mostly empty take the 128x256 tiles, two workgroups per CU, whatever the storage
        // order (16 x 1344-row problems with K <= 1344: 4.31 -> 4.07 ms over the 18 GEMMs of an iteration; only the
        // 2048 x 512 x 1344 weight-gradient problem is 5 % slower that way); long contractions keep the 256x256 tiles,
        // which move half the operand bytes per flop.
        const bool short_k = d.K <= 1536;
        const bool ragged_m = (int64_t)(((d.M + 255) / 256) * 256 - d.M) * 10 >= d.M;
        v = big_tiles < 128 ? 0 : (short_k || ragged_m) ? 13 : !(d.a_kc && d.b_kc) ? 12 : (d.M >= 512 && d.N >= 512) ? 11 : 13;
    }
    // direct-to-LDS loads need whole stages and, for a rows-contiguous operand, whole 16-byte chunks of rows
    // (16-byte aligned k-rows of a rows-contiguous operand must be at least round_up(rows, 8) long)
    // (the per-lane load offsets inside a tile are 32-bit: row strides below 2^22 elements)
    const bool dma = d.K % 64 == 0 && d.lda < (1 << 22) && d.ldb < (1 << 22) && aligned_to(d.A, d.lda, d.sAi, d.sAd, esz, 16) &&
                     aligned_to(d.B, d.ldb, d.sBi, d.sBd, esz, 16) &&
                     (d.a_kc || d.lda >= ((d.M + 7) & ~7)) && (d.b_kc || d.ldb >= ((d.N + 7) & ~7));
    if (v == 13 && dma) return launch_dma<bf16_t, 2, 2, 2, 4, 64, 3>(d, s);
    if (v == 12 && dma) return launch_dma<bf16_t, 2, 2, 4, 4, 64, 3>(d, s);
    if (v == 11 && dma) return launch_dma<bf16_t, 2, 2, 4, 4, 128, 2>(d, s);
    if (v >= 5) return launch_layout<bf16_t, 2, 4, 4, 2, 16, 128>(d, s);
    return launch_layout<bf16_t, 2, 2, 2, 2, 16, 64>(d, s);
}

}  // namespace adpsgd
