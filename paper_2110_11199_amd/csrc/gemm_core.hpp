// LDS-tiled MFMA GEMM main loop for gfx950 (64-wide wavefronts).
//
// C[m][n] = sum_k A(m,k) * B(n,k).  A workgroup of WM x WN waves owns a
// (32*FM*WM) x (32*FN*WN) tile of C; each wave owns FM x FN MFMA 32x32 tiles.
// K is consumed in stages of SB = 64 or 128 bytes per operand row,
// double-buffered in LDS with a register prefetch of the next stage.
//
// An operand comes from global memory in one of two storage orders:
//   "kc"  K contiguous:  element (r,k) at row(r)[k]         (rows may be gathered)
//   "mc"  rows contiguous: element (r,k) at base[k*ld + r]  (transposed on the way
//         into LDS, so that C = A'*B and C = A*B need no transposed copies)
// LDS layouts: kc tiles are row-major with a row stride of SB+16 bytes (16-byte
// fragment reads hit distinct banks); mc tiles are stored as planes of
// 4-element k-granules, plane q holding k = 4q..4q+3 of every row, so that the
// transposing store is contiguous per lane and fragment reads are contiguous
// across lanes.
//
// MFMA operand mapping: lane (r = lane%32, g = lane/32) supplies, per 32-byte
// chunk pair c of a stage, the 16 bytes of row r at chunk 2c+g, for both A and
// B alike, so the contraction pairs equal k whatever order the instruction
// walks them in.  bf16: one v_mfma_f32_32x32x16_bf16 per chunk pair; fp32:
// four v_mfma_f32_32x32x2_f32.  Accumulator element i of a lane is
// C[8*(i/4) + 4*g + i%4][lane%32] of the 32x32 tile.
#pragma once
#include "common.hpp"

namespace adpsgd {

// SB (template parameter below) = bytes of K per operand row per LDS stage: 64 or 128.
// LDS row stride of a kc tile = SB + 16.

template <typename T> struct KcSrc {  // K-contiguous rows base + r*ld, r < R
    static constexpr bool kc = true;
    const T* base; int64_t ld; int R;
    __device__ const T* row(int r) const { return r < R ? base + (int64_t)r * ld : nullptr; }
    __device__ const T* row_nocheck(int r) const { return base + (int64_t)r * ld; }
    __device__ const T* row_clamped(int r) const { return base + (int64_t)(r < R ? r : R - 1) * ld; }
    __device__ int64_t row_offset_clamped(int r) const { return (int64_t)(r < R ? r : R - 1) * ld; }   // elements from base
    __device__ bool full(int rows) const { return R >= rows; }
};

// Rows of a [4][H] gate-blocked matrix gathered so that tile row n holds gate
// (n % 128) / 32 of hidden unit u0 + 32*(n / 128) + n % 32.
template <typename T> struct GateSrc {
    static constexpr bool kc = true;
    const T* base; int64_t ld; int H; int u0;
    __device__ const T* row(int n) const {
        int u = u0 + 32 * (n >> 7) + (n & 31);
        int gate = (n & 127) >> 5;
        return u < H ? base + ((int64_t)gate * H + u) * ld : nullptr;
    }
    __device__ const T* row_nocheck(int n) const {
        return base + ((int64_t)((n & 127) >> 5) * H + u0 + 32 * (n >> 7) + (n & 31)) * ld;
    }
    __device__ const T* row_clamped(int n) const {
        int u = u0 + 32 * (n >> 7) + (n & 31);
        u = u < H ? u : H - 1;
        return base + ((int64_t)((n & 127) >> 5) * H + u) * ld;
    }
    __device__ int64_t row_offset_clamped(int n) const { return row_clamped(n) - base; }
    __device__ bool full(int rows) const { return u0 + rows / 4 <= H; }
};

template <typename T> struct McSrc {  // element (r,k) at base[k*ld + r], r < R
    static constexpr bool kc = false;
    const T* base; int64_t ld; int R;
    __device__ bool full(int rows) const { return R >= rows; }
    // 8 consecutive rows r = 8*chunk.. of k-row k (R a multiple of 8); chunks past the end repeat the last one
    __device__ int64_t chunk_offset_clamped(int k, int chunk) const {      // elements from base
        const int last = (R >> 3) - 1;
        return (int64_t)k * ld + 8 * (chunk < last ? chunk : last);
    }
};

template <typename T, int ROWS, int SB, bool KC> struct LdsTile;

template <typename T, int ROWS, int SB> struct LdsTile<T, ROWS, SB, true> {
    static constexpr int STRIDE = SB + 16;
    static constexpr int BYTES = ROWS * STRIDE;
    __device__ static uint4 frag(const char* lds, int row, int ch) {
        return *(const uint4*)(lds + row * STRIDE + ch * 16);
    }
};
template <int ROWS, int SB> struct LdsTile<bf16_t, ROWS, SB, false> {
    static constexpr int BYTES = ROWS * SB;
    __device__ static uint4 frag(const char* lds, int row, int ch) {
        uint2 lo = *(const uint2*)(lds + (2 * ch) * (ROWS * 8) + row * 8);
        uint2 hi = *(const uint2*)(lds + (2 * ch + 1) * (ROWS * 8) + row * 8);
        return make_uint4(lo.x, lo.y, hi.x, hi.y);
    }
};
template <int ROWS, int SB> struct LdsTile<float, ROWS, SB, false> {
    static constexpr int BYTES = ROWS * SB;
    __device__ static uint4 frag(const char* lds, int row, int ch) {
        return *(const uint4*)(lds + ch * (ROWS * 16) + row * 16);
    }
};

// ---- global -> register -> LDS loaders -------------------------------------

template <typename T, int ROWS, int VB, int NT, int SB> struct KcLoader {
    static constexpr int STRIDE = SB + 16;
    static constexpr int EPV = VB / (int)sizeof(T);          // elements per vector load
    static constexpr int CPR = SB / VB;                      // vectors per tile row
    static constexpr int CHUNKS = ROWS * CPR;
    static constexpr int PER = (CHUNKS + NT - 1) / NT;
    static constexpr int WORDS = VB / 4;
    uint32_t regs[PER][WORDS];

    // Whole stage inside the matrix (all tile rows valid, k0 + stage <= K): no guards, no branches.
    template <class Src> __device__ void load_full(const Src& src, int k0, int tid) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int c = tid + j * NT;
            if (CHUNKS % NT != 0 && c >= CHUNKS) continue;
            const int row = c / CPR, kc = c % CPR;
            const T* p = src.row_nocheck(row) + k0 + kc * EPV;
            if constexpr (VB == 16) {
                const uint4 v = *(const uint4*)p;
                regs[j][0] = v.x; regs[j][1] = v.y; regs[j][2] = v.z; regs[j][3] = v.w;
            } else {
                const uint2 v = *(const uint2*)p;
                regs[j][0] = v.x; regs[j][1] = v.y;
            }
        }
    }
    template <class Src> __device__ void load(const Src& src, int k0, int K, int tid) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            int c = tid + j * NT;
#pragma unroll
            for (int w = 0; w < WORDS; ++w) regs[j][w] = 0u;
            if (CHUNKS % NT != 0 && c >= CHUNKS) continue;
            int row = c / CPR, kc = c % CPR;
            int k = k0 + kc * EPV;
            const T* p = src.row(row);
            if (p == nullptr || k >= K) continue;
            if (k + EPV <= K) {
                if constexpr (VB == 16) {
                    uint4 v = *(const uint4*)(p + k);
                    regs[j][0] = v.x; regs[j][1] = v.y; regs[j][2] = v.z; regs[j][3] = v.w;
                } else {
                    uint2 v = *(const uint2*)(p + k);
                    regs[j][0] = v.x; regs[j][1] = v.y;
                }
            } else {
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    if (k + e < K) {
                        if constexpr (sizeof(T) == 4) regs[j][e] = __builtin_bit_cast(uint32_t, *(const float*)(p + k + e));
                        else regs[j][e >> 1] |= (uint32_t)(*(const uint16_t*)(p + k + e)) << (16 * (e & 1));
                    }
                }
            }
        }
    }
    __device__ void store(char* lds, int tid) const {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            int c = tid + j * NT;
            if (CHUNKS % NT != 0 && c >= CHUNKS) continue;
            int row = c / CPR, kc = c % CPR;
            char* dst = lds + row * STRIDE + kc * VB;
            if constexpr (VB == 16) *(uint4*)dst = make_uint4(regs[j][0], regs[j][1], regs[j][2], regs[j][3]);
            else *(uint2*)dst = make_uint2(regs[j][0], regs[j][1]);
        }
    }
};

template <typename T, int ROWS, int NT, int SB> struct McLoader {
    static constexpr int KT = SB / (int)sizeof(T);            // k per stage
    static constexpr int RQ = ROWS / 4;
    static constexpr int SUBS = (KT / 4) * RQ;                // 4(k) x 4(r) sub-blocks
    static constexpr int PER = (SUBS + NT - 1) / NT;
    static constexpr int WORDS = (int)sizeof(T);              // 32-bit words per 4 elements
    uint32_t regs[PER][4][WORDS];

    template <class Src> __device__ void load_full(const Src& src, int k0, int tid) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int s = tid + j * NT;
            if (SUBS % NT != 0 && s >= SUBS) continue;
            const int kq = s / RQ, r = (s % RQ) * 4;
            const T* p = src.base + (int64_t)(k0 + kq * 4) * src.ld + r;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                if constexpr (sizeof(T) == 4) {
                    const uint4 v = *(const uint4*)(p + jj * src.ld);
                    regs[j][jj][0] = v.x; regs[j][jj][1] = v.y; regs[j][jj][2] = v.z; regs[j][jj][3] = v.w;
                } else {
                    const uint2 v = *(const uint2*)(p + jj * src.ld);
                    regs[j][jj][0] = v.x; regs[j][jj][1] = v.y;
                }
            }
        }
    }
    template <class Src> __device__ void load(const Src& src, int k0, int K, int tid) {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            int s = tid + j * NT;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                for (int w = 0; w < WORDS; ++w) regs[j][jj][w] = 0u;
            if (SUBS % NT != 0 && s >= SUBS) continue;
            int kq = s / RQ, r = (s % RQ) * 4;
            if (r >= src.R) continue;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                int k = k0 + kq * 4 + jj;
                if (k >= K) continue;
                const T* p = src.base + (int64_t)k * src.ld + r;
                if (r + 4 <= src.R) {
                    if constexpr (sizeof(T) == 4) {
                        uint4 v = *(const uint4*)p;
                        regs[j][jj][0] = v.x; regs[j][jj][1] = v.y; regs[j][jj][2] = v.z; regs[j][jj][3] = v.w;
                    } else {
                        uint2 v = *(const uint2*)p;
                        regs[j][jj][0] = v.x; regs[j][jj][1] = v.y;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (r + e < src.R) {
                            if constexpr (sizeof(T) == 4) regs[j][jj][e] = __builtin_bit_cast(uint32_t, *(const float*)(p + e));
                            else regs[j][jj][e >> 1] |= (uint32_t)(*(const uint16_t*)(p + e)) << (16 * (e & 1));
                        }
                    }
                }
            }
        }
    }
    __device__ void store(char* lds, int tid) const {
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            int s = tid + j * NT;
            if (SUBS % NT != 0 && s >= SUBS) continue;
            int kq = s / RQ, rq = s % RQ;
            if constexpr (sizeof(T) == 4) {
                // granule = 4 floats (k..k+3) of one row; rows 4rq..4rq+3 are contiguous
                char* dst = lds + kq * (ROWS * 16) + rq * 64;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    *(uint4*)(dst + e * 16) = make_uint4(regs[j][0][e], regs[j][1][e], regs[j][2][e], regs[j][3][e]);
            } else {
                char* dst = lds + kq * (ROWS * 8) + rq * 32;
                uint32_t o[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
                    o[2 * e] = __builtin_amdgcn_perm(regs[j][1][e >> 1], regs[j][0][e >> 1], sel);
                    o[2 * e + 1] = __builtin_amdgcn_perm(regs[j][3][e >> 1], regs[j][2][e >> 1], sel);
                }
                *(uint4*)dst = make_uint4(o[0], o[1], o[2], o[3]);
                *(uint4*)(dst + 16) = make_uint4(o[4], o[5], o[6], o[7]);
            }
        }
    }
};

template <typename T, int ROWS, int VB, int NT, int SB, bool KC> struct LoaderSel;
template <typename T, int ROWS, int VB, int NT, int SB> struct LoaderSel<T, ROWS, VB, NT, SB, true> { typedef KcLoader<T, ROWS, VB, NT, SB> type; };
template <typename T, int ROWS, int VB, int NT, int SB> struct LoaderSel<T, ROWS, VB, NT, SB, false> { typedef McLoader<T, ROWS, NT, SB> type; };

template <typename T> __device__ inline void mma_chunk(f32x16_t& acc, const uint4& a, const uint4& b);
template <> __device__ inline void mma_chunk<bf16_t>(f32x16_t& acc, const uint4& a, const uint4& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc, 0, 0, 0);
}
template <> __device__ inline void mma_chunk<float>(f32x16_t& acc, const uint4& a, const uint4& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.x), __builtin_bit_cast(float, b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.y), __builtin_bit_cast(float, b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.z), __builtin_bit_cast(float, b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a.w), __builtin_bit_cast(float, b.w), acc, 0, 0, 0);
}

template <typename T, class ASrc, class BSrc, int WM, int WN, int FM, int FN, int VB, int SB = 64>
struct GemmCore {
    static constexpr int BM = 32 * FM * WM, BN = 32 * FN * WN, NT = 64 * WM * WN;
    static constexpr int kWM = WM, kWN = WN;
    static constexpr int KT = SB / (int)sizeof(T);
    typedef LdsTile<T, BM, SB, ASrc::kc> ATile;
    typedef LdsTile<T, BN, SB, BSrc::kc> BTile;
    static constexpr int STAGE_BYTES = ATile::BYTES + BTile::BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;

    // acc must be zero-initialised (or hold the value to accumulate onto).
    __device__ static void run(f32x16_t (&acc)[FM][FN], const ASrc& a, const BSrc& b, int K, char* lds) {
        const int tid = threadIdx.x;
        const int lane = tid & 63, wave = tid >> 6;
        const int wave_m = wave / WN, wave_n = wave % WN;
        const int r = lane & 31, g = lane >> 5;
        typename LoaderSel<T, BM, VB, NT, SB, ASrc::kc>::type la;
        typename LoaderSel<T, BN, VB, NT, SB, BSrc::kc>::type lb;
        const int nk = (K + KT - 1) / KT;
        if (nk <= 0) return;
        // stages that lie wholly inside both operands are loaded without guards
        const int nk_full = (a.full(BM) && b.full(BN)) ? K / KT : 0;
        if (nk_full > 0) { la.load_full(a, 0, tid); lb.load_full(b, 0, tid); }
        else { la.load(a, 0, K, tid); lb.load(b, 0, K, tid); }
        la.store(lds, tid);
        lb.store(lds + ATile::BYTES, tid);
        __syncthreads();
        for (int kt = 0; kt < nk; ++kt) {
            char* cur = lds + (kt & 1) * STAGE_BYTES;
            char* nxt = lds + ((kt + 1) & 1) * STAGE_BYTES;
            const bool more = kt + 1 < nk;
            if (kt + 1 < nk_full) {
                la.load_full(a, (kt + 1) * KT, tid);
                lb.load_full(b, (kt + 1) * KT, tid);
            } else if (more) {
                la.load(a, (kt + 1) * KT, K, tid);
                lb.load(b, (kt + 1) * KT, K, tid);
            }
#pragma unroll
            for (int c = 0; c < SB / 32; ++c) {
                const int ch = 2 * c + g;
                uint4 af[FM], bfr[FN];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) af[fm] = ATile::frag(cur, (wave_m * FM + fm) * 32 + r, ch);
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) bfr[fn] = BTile::frag(cur + ATile::BYTES, (wave_n * FN + fn) * 32 + r, ch);
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int fn = 0; fn < FN; ++fn) mma_chunk<T>(acc[fm][fn], af[fm], bfr[fn]);
            }
            if (more) {
                la.store(nxt, tid);
                lb.store(nxt + ATile::BYTES, tid);
            }
            __syncthreads();
        }
    }

    // Position of accumulator element i of tile (fm, fn) inside the workgroup tile.
    __device__ static int acc_row(int fm, int i) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return ((wave / WN) * FM + fm) * 32 + 8 * (i >> 2) + 4 * (lane >> 5) + (i & 3);
    }
    __device__ static int acc_col(int fn) {
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
        return ((wave % WN) * FN + fn) * 32 + (lane & 31);
    }
};

}  // namespace adpsgd
