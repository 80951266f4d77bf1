// MFMA GEMM main loop fed by direct global->LDS loads (gfx950 global_load_lds_dwordx4):
// no staging registers, no LDS store instructions, NS LDS stages in flight.
//
// Same contract as GemmCore (gemm_core.hpp): C[m][n] = sum_k A(m,k) B(n,k) for a
// (32*FM*WM) x (32*FN*WN) workgroup tile, K a multiple of the stage length, operand rows
// 16-byte aligned.  Rows past the end of an operand are clamped to its last row (their
// products land in accumulator rows/columns the caller discards), so no guard and no zero
// fill is needed.
//
// A wave-wide direct load writes lane l's 16 bytes to LDS at base + 16*l, i.e. 1 KB
// contiguous per instruction.  A tile is therefore stored row-major WITHOUT padding
// (row = SB bytes) and bank conflicts are avoided by a swizzle applied on the global
// side: the 16-byte slot s of row r holds chunk s ^ swz(r) of that row, with
// swz(r) = (r / (256/SB)) mod (SB/16), so that any 16 rows read at one chunk index hit 16
// different 16-byte bank groups.
//
// An operand stored rows-contiguous ("mc": element (r,k) at base[k*ld + r], bf16 only) is copied as
// it lies in memory, k-row by k-row (tile = [KT][ROWS], ROWS*2 bytes per k-row), and transposed
// on the LDS read: ds_read_b64_tr_b16 hands lane i of a 16-lane group the four 16-bit values that
// lanes 4c + i/4 (c = 0..3) of the group address at position i%4.  With lane 4c+q addressing
// (k0+c, r0+4q..r0+4q+3), lane i receives (k0..k0+3, r0+i): four consecutive k of its own row, so
// two such reads give the same 8-k fragment as one 16-byte read of a K-contiguous tile.  The 16-byte
// slot s of k-row k holds chunk s ^ 4*(k mod 4) of that row: the 32 lanes served in one LDS
// cycle (4 k-rows x 64 bytes, twice) then cover all 64 banks once.
#pragma once
#include <type_traits>
#include "gemm_core.hpp"

namespace adpsgd {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(1))) const void glb_void_t;

// One wave-wide direct load: lane l's 16 bytes at base + off (a wave-uniform 64-bit base in SGPRs plus
// a per-lane 32-bit byte offset) land in LDS at lds_addr + 16*l.  The per-lane offsets of a tile do not
// change from stage to stage, only the base does, so a stage costs no vector address arithmetic.
// Issued through inline asm so that the compiler's wait-count insertion does not see it
// (it would drain all loads before every LDS read); the main loop places its own waits.
__device__ inline void dma16_(uint32_t off, const void* base_uniform, uint32_t lds_addr_uniform) {
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base_uniform), "s"(lds_addr_uniform) : "memory", "m0");
}
__device__ inline uint32_t lds_addr_(const void* p) {
    return (uint32_t)(uintptr_t)(lds_void_t*)p;
}

template <int SB> __device__ inline int swz_(int r) { return (r / (256 / SB)) & (SB / 16 - 1); }

template <typename T, class ASrc, class BSrc, int WM, int WN, int FM, int FN, int SB, int NS>
struct GemmDma {
    static constexpr int BM = 32 * FM * WM, BN = 32 * FN * WN, NT = 64 * WM * WN;
    static constexpr int kWM = WM, kWN = WN;
    static constexpr int KT = SB / (int)sizeof(T);
    static constexpr int CPR = SB / 16;                       // 16-byte chunks per tile row
    static constexpr int A_BYTES = BM * SB, B_BYTES = BN * SB;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = NS * STAGE_BYTES;
    static constexpr int LA = BM * CPR / NT, LB = BN * CPR / NT;   // loads per thread per stage
    static_assert((BM * CPR) % NT == 0 && (BN * CPR) % NT == 0, "tile must divide over the workgroup");
    static_assert((ASrc::kc && BSrc::kc) || sizeof(T) == 2, "transposing LDS reads exist for 16-bit operands only");

    // Byte offsets, relative to the operand's stage base, of the L 16-byte chunks this lane loads per stage.
    template <int ROWS, int L, class Src>
    __device__ static void lane_offsets(const Src& src, int tid, uint32_t (&off)[L]) {
#pragma unroll
        for (int j = 0; j < L; ++j) {
            const int c = tid + j * NT;
            if constexpr (Src::kc) {
                const int row = c / CPR;
                const int slot = c % CPR;
                const int chunk = slot ^ swz_<SB>(row);
                off[j] = (uint32_t)(src.row_offset_clamped(row) * (int64_t)sizeof(T)) + (uint32_t)chunk * 16u;
            } else {
                constexpr int CPK = ROWS / 8;                 // 16-byte chunks per k-row
                static_assert(ROWS % 128 == 0, "the chunk swizzle needs k-rows of a multiple of 16 chunks");
                const int krow = c / CPK;
                const int slot = c % CPK;
                const int chunk = slot ^ (4 * (krow & 3));
                off[j] = (uint32_t)(src.chunk_offset_clamped(krow, chunk) * (int64_t)sizeof(T));
            }
        }
    }

    // Stage starting at k0 of one operand into lds_tile; wave = wave index of the caller (wave-uniform).
    template <int L, class Src>
    __device__ static void issue(const Src& src, const uint32_t (&off)[L], int k0, char* lds_tile, int wave) {
        const T* sbase = Src::kc ? src.base + k0 : src.base + (int64_t)k0 * src.ld;
        const uint32_t dst0 = lds_addr_(lds_tile) + (uint32_t)wave * 1024u;   // lane l lands at dst + 16*l
#pragma unroll
        for (int j = 0; j < L; ++j) dma16_(off[j], sbase, dst0 + (uint32_t)(j * NT) * 16u);
    }

    // 16-byte MFMA fragment of tile row `row0 + lane%32`, k-chunk `ch` (8 consecutive k) of the stage.
    template <int ROWS, bool KC>
    __device__ static uint4 frag(const char* tile, int row0, int ch, int lane) {
        if constexpr (KC) {
            const int row = row0 + (lane & 31);
            return *(const uint4*)(tile + row * SB + ((ch ^ swz_<SB>(row)) * 16));
        } else {
            const int j = lane & 15, c = j >> 2, q = j & 3;
            const int r = row0 + (lane & 16) + 4 * q;         // first of the 4 rows this lane addresses
            const char* p = tile + (ch * 8 + c) * (ROWS * 2) + (((r >> 3) ^ (4 * c)) * 16) + (r & 7) * 2;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)p);
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(p + 4 * (ROWS * 2)));
            const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
            return make_uint4(l2.x, l2.y, h2.x, h2.y);
        }
    }

    template <int N> __device__ static void wait_vm() {
        static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
        asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
    }

    // K must be a multiple of KT (checked by the host).  acc must be initialised.
    // rot (0 <= rot < K/KT) rotates the order in which the K stages are consumed: stage s reads
    // k-block (s + rot) mod nk.  Workgroups that would otherwise walk K in lockstep (same column
    // offset of every row at the same time, i.e. the same few memory channels) are given
    // different rotations by the caller; the sum is the same up to fp32 summation order.
    __device__ static void run(f32x16_t (&acc)[FM][FN], const ASrc& a, const BSrc& b, int K, char* lds, int rot = 0) {
        constexpr int LPT = LA + LB;
        const int tid = threadIdx.x;
        const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int wave_m = wave / WN, wave_n = wave % WN;
        const int g = lane >> 5;
        const int nk = K / KT;
        uint32_t aoff[LA], boff[LB];
        lane_offsets<BM, LA>(a, tid, aoff);
        lane_offsets<BN, LB>(b, tid, boff);
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) {
            if (s < nk) {
                int kb = s + rot; kb = kb >= nk ? kb - nk : kb;
                issue<LA>(a, aoff, kb * KT, lds + s * STAGE_BYTES, wave);
                issue<LB>(b, boff, kb * KT, lds + s * STAGE_BYTES + A_BYTES, wave);
            }
        }
        for (int kt = 0; kt < nk; ++kt) {
            // tiles issued after kt and still allowed in flight: min(NS-2, nk-1-kt)
            const int later = nk - 1 - kt;
            if (later >= NS - 2) wait_vm<(NS - 2) * LPT>();
            else if (NS > 3 && later == 1) wait_vm<LPT>();
            else wait_vm<0>();
            __builtin_amdgcn_s_barrier();      // every wave's share of tile kt has landed; stage (kt-1)%NS is free
            const int nt = kt + NS - 1;
            if (nt < nk) {
                char* st = lds + (nt % NS) * STAGE_BYTES;
                int kb = nt + rot; kb = kb >= nk ? kb - nk : kb;
                issue<LA>(a, aoff, kb * KT, st, wave);
                issue<LB>(b, boff, kb * KT, st + A_BYTES, wave);
            }
            const char* cur = lds + (kt % NS) * STAGE_BYTES;
#pragma unroll
            for (int c = 0; c < SB / 32; ++c) {
                const int ch = 2 * c + g;
                uint4 af[FM], bfr[FN];
#pragma unroll
                for (int fm = 0; fm < FM; ++fm) af[fm] = frag<BM, ASrc::kc>(cur, (wave_m * FM + fm) * 32, ch, lane);
#pragma unroll
                for (int fn = 0; fn < FN; ++fn) bfr[fn] = frag<BN, BSrc::kc>(cur + A_BYTES, (wave_n * FN + fn) * 32, ch, lane);
#pragma unroll
                for (int fm = 0; fm < FM; ++fm)
#pragma unroll
                    for (int fn = 0; fn < FN; ++fn) mma_chunk<T>(acc[fm][fn], af[fm], bfr[fn]);
            }
        }
    }

    // One fragment of k-chunk C for run_deep: fragment index F counts a0, b0, a1, b1, ... (A and B alternate
    // while both remain) so that the first MFMAs of a chunk can start before all of its fragments have arrived.
    template <int C, int F>
    __device__ static void load_one(const char* cur, int wave_m, int wave_n, int g, int lane, uint4 (&af)[FM], uint4 (&bfr)[FN]) {
        constexpr int kBoth = FM < FN ? FM : FN;
        constexpr bool is_a = F < 2 * kBoth ? (F % 2 == 0) : (FM > FN);
        constexpr int idx = F < 2 * kBoth ? F / 2 : F - kBoth;
        const int ch = 2 * C + g;
        if constexpr (is_a) af[idx] = frag<BM, ASrc::kc>(cur, (wave_m * FM + idx) * 32, ch, lane);
        else bfr[idx] = frag<BN, BSrc::kc>(cur + A_BYTES, (wave_n * FN + idx) * 32, ch, lane);
    }
    template <int C, int F = 0>
    __device__ static void load_all(const char* cur, int wave_m, int wave_n, int g, int lane, uint4 (&af)[FM], uint4 (&bfr)[FN]) {
        if constexpr (F < FM + FN) {
            load_one<C, F>(cur, wave_m, wave_n, g, lane, af, bfr);
            load_all<C, F + 1>(cur, wave_m, wave_n, g, lane, af, bfr);
        }
    }

    // MFMA number I of a chunk works on tile (fm, fn) = order(I): tiles whose fragments arrive first come first
    // (all tiles with max(fm, fn) = 0, then 1, ...).
    __device__ static constexpr int order_fm(int I) {
        int n = 0;
        for (int r = 0; r < (FM > FN ? FM : FN); ++r) {
            for (int j = 0; j <= r; ++j) {          // (r, j) for j < r, (j, r) for j <= r
                if (j < r && r < FM && j < FN) { if (n == I) return r; ++n; }
                if (j < FM && r < FN) { if (n == I) return j; ++n; }
            }
        }
        return 0;
    }
    __device__ static constexpr int order_fn(int I) {
        int n = 0;
        for (int r = 0; r < (FM > FN ? FM : FN); ++r) {
            for (int j = 0; j <= r; ++j) {
                if (j < r && r < FM && j < FN) { if (n == I) return j; ++n; }
                if (j < FM && r < FN) { if (n == I) return r; ++n; }
            }
        }
        return 0;
    }

    template <int LO, int HI, class Fn> __device__ static void static_for(Fn&& f) {
        if constexpr (LO < HI) { f(std::integral_constant<int, LO>{}); static_for<LO + 1, HI>(f); }
    }
    __device__ static constexpr int min_(int x, int y) { return x < y ? x : y; }

    // Direct load number D of a stage (the LA loads of the A tile, then the LB loads of the B tile).
    template <int D>
    __device__ static void issue_one(const ASrc& a, const BSrc& b, const uint32_t (&aoff)[LA], const uint32_t (&boff)[LB],
                                     int k0, char* stage, int wave) {
        if constexpr (D < LA) {
            const T* sbase = ASrc::kc ? a.base + k0 : a.base + (int64_t)k0 * a.ld;
            dma16_(aoff[D], sbase, lds_addr_(stage) + (uint32_t)wave * 1024u + (uint32_t)(D * NT) * 16u);
        } else {
            const T* sbase = BSrc::kc ? b.base + k0 : b.base + (int64_t)k0 * b.ld;
            dma16_(boff[D - LA], sbase, lds_addr_(stage + A_BYTES) + (uint32_t)wave * 1024u + (uint32_t)((D - LA) * NT) * 16u);
        }
    }

    // One K stage of run_deep.  Register set (C & 1) holds the fragments of chunk C; while the MFMAs of chunk C
    // run, the fragments of the next chunk are read into the other set: from this stage's buffer, or (last
    // chunk, NEXT) chunk 0 of the next stage's buffer.  The one barrier of the stage sits before the last chunk:
    // by then every wave has its last fragments of this stage in registers (their reads are issued in the first
    // half of the chunk before, and waited for), and its share of the next stage has landed, so that after it
    // the next stage may be read and this stage's buffer may be overwritten by the loads of the stage after next
    // (DMA), which are issued one per MFMA of the last chunk.  The scheduling barriers keep this order.
    template <bool NEXT, bool DMA, int OUT>
    __device__ static void deep_stage(f32x16_t (&acc)[FM][FN], const ASrc& a, const BSrc& b, const uint32_t (&aoff)[LA],
                                      const uint32_t (&boff)[LB], char* cur, const char* nxt, int dma_k0, int wave, int wave_m,
                                      int wave_n, int g, int lane, uint4 (&af)[2][FM], uint4 (&bfr)[2][FN]) {
        constexpr int NC = SB / 32, NM = FM * FN, NF = FM + FN, ND = LA + LB;
        static_assert(NC % 2 == 0 && NC >= 2, "the register sets alternate per chunk and must line up across stages");
        static_for<0, NC>([&](auto cc) {
            constexpr int C = decltype(cc)::value;
            constexpr bool last = C == NC - 1;
            if constexpr (last) {
                wait_vm<OUT * (LA + LB)>();          // the next stage has landed; OUT later stages may be in flight
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                __builtin_amdgcn_sched_barrier(0);
            }
            constexpr int R = (C >= NC - 2) ? 2 : 1;   // front-loaded before the barrier and before the loop's back edge
            static_for<0, NM>([&](auto ii) {
                constexpr int I = decltype(ii)::value;
                if constexpr (!last || NEXT) {
                    constexpr int f0 = min_(I * NF * R / NM, NF), f1 = min_((I + 1) * NF * R / NM, NF);
                    static_for<f0, f1>([&](auto ff) {
                        load_one<(C + 1) % NC, decltype(ff)::value>(last ? nxt : (const char*)cur, wave_m, wave_n, g, lane,
                                                                    af[(C + 1) & 1], bfr[(C + 1) & 1]);
                    });
                }
                if constexpr (last && DMA) {
                    constexpr int d0 = I * ND / NM, d1 = (I + 1) * ND / NM;
                    static_for<d0, d1>([&](auto dd) { issue_one<decltype(dd)::value>(a, b, aoff, boff, dma_k0, cur, wave); });
                }
                constexpr int fm = order_fm(I), fn = order_fn(I);
                mma_chunk<T>(acc[fm][fn], af[C & 1][fm], bfr[C & 1][fn]);
                __builtin_amdgcn_sched_barrier(0);
            });
        });
    }

    // The same main loop for one wave per SIMD (large wave tiles: fewer LDS bytes per flop, but no second
    // wave to hide latencies): software-pipelined by hand, NS LDS stages (the loads of stage kt + NS are issued
    // during the last chunk of stage kt, into the buffer that stage has just finished with).
    __device__ static void run_deep(f32x16_t (&acc)[FM][FN], const ASrc& a, const BSrc& b, int K, char* lds, int rot = 0) {
        static_assert(NS >= 2 && NS <= 4, "two to four stages");
        constexpr int LPT = LA + LB;
        const int tid = threadIdx.x;
        const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int wave_m = wave / WN, wave_n = wave % WN;
        const int g = lane >> 5;
        const int nk = K / KT;
        uint32_t aoff[LA], boff[LB];
        lane_offsets<BM, LA>(a, tid, aoff);
        lane_offsets<BN, LB>(b, tid, boff);
        auto kblock = [&](int s) { int kb = s + rot; return (kb >= nk ? kb - nk : kb) * KT; };
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s < nk) {
                issue<LA>(a, aoff, kblock(s), lds + s * STAGE_BYTES, wave);
                issue<LB>(b, boff, kblock(s), lds + s * STAGE_BYTES + A_BYTES, wave);
            }
        }
        const int later = (nk < NS ? nk : NS) - 1;          // stages issued after stage 0
        if (NS >= 4 && later >= 3) wait_vm<(NS >= 4 ? 3 : 0) * LPT>();
        else if (NS >= 3 && later == 2) wait_vm<(NS >= 3 ? 2 : 0) * LPT>();
        else if (later == 1) wait_vm<LPT>();
        else wait_vm<0>();
        __builtin_amdgcn_s_barrier();
        uint4 af[2][FM], bfr[2][FN];
        load_all<0>(lds, wave_m, wave_n, g, lane, af[0], bfr[0]);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0, buf = 0;
        auto next_buf = [](int x) { return x + 1 == NS ? 0 : x + 1; };
        for (; kt + NS < nk; ++kt) {
            deep_stage<true, true, NS - 2>(acc, a, b, aoff, boff, lds + buf * STAGE_BYTES, lds + next_buf(buf) * STAGE_BYTES,
                                           kblock(kt + NS), wave, wave_m, wave_n, g, lane, af, bfr);
            buf = next_buf(buf);
        }
        for (; kt + 1 < nk; ++kt) {
            char* cur = lds + buf * STAGE_BYTES;
            const char* nxt = lds + next_buf(buf) * STAGE_BYTES;
            // the last NS - 1 stages wait for everything in flight (issued at least a stage ago)
            deep_stage<true, false, 0>(acc, a, b, aoff, boff, cur, nxt, 0, wave, wave_m, wave_n, g, lane, af, bfr);
            buf = next_buf(buf);
        }
        deep_stage<false, false, 0>(acc, a, b, aoff, boff, lds + buf * STAGE_BYTES, lds, 0, wave, wave_m, wave_n, g, lane, af, bfr);
    }

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
