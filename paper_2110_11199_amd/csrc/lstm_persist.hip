// Persistent recurrent LSTM kernels: one launch runs ALL T frames of one layer for a set of
// (learner, direction) pairs, with the recurrent weights held on chip across the frames.
//
// The per-frame kernels of lstm.hip stream every learner's W_h from HBM once per frame (the weights
// are not shared between learners): T reads where the method needs one.  Here a workgroup owns 32
// hidden units of one (learner, direction) pair and keeps its slice of W_h in REGISTERS for the whole
// launch: the 4 x 32 gate rows of its units (forward, h W_h') or the 32 unit columns (backward,
// da W_h), 64 KB per wave, 256 KB per workgroup at 1024 units.  The H/32 workgroups of a pair
// exchange the per-frame operand (h_{t'} forward, da_{t''} backward; it goes through L2) and meet once
// per frame at a counter in the caller's workspace.
//
// Forward, frame by frame:  a = (W_x x_t + b) + h_{t'} W_h'; i,f,o = sigmoid(a), g = tanh(a);
//   c_t = f c_{t'} + i g;  h_t = o tanh(c_t).        Wave w of a workgroup owns gate w: its MFMA tile
//   is (batch rows) x (gate w of the 32 units), its accumulators start from the pre-activations
//   W_x x_t + b read from HBM, and the four waves swap gates through LDS so that every lane ends up
//   with the four gates of its (batch row, unit) positions.  c stays in registers across the frames.
// Backward, frame by frame:  dh_t = dY_t + da_{t''} W_h, then the cell backward of lstm.hip.  Wave w
//   contracts over the rows of gate w (a quarter of K = 4H), the four partial products are added
//   through LDS in a fixed order, dc stays in registers across the frames.
//
// Synchronisation.  The grid never exceeds one workgroup per compute unit, so all workgroups of a
// launch are resident together (checked on the host).  A workgroup that has stored its slice of the
// frame's operand makes it visible device-wide (release fence), then adds 1 to its pair's counter; a
// workgroup that needs the operand of frame s waits until the counter reaches (H/32) * s.  The wait is
// BOUNDED: one thread polls the counter and gives up after wait_ticks of the 100 MHz wall clock, or as
// soon as another workgroup has given up; the workgroup then raises kStatusWaitExpired in the handle's
// status word and returns.  Every workgroup therefore exits, whatever happens to the others.
#include "gemm_core.hpp"
#include "gemm_dma.hpp"
#include "kernels.hpp"

namespace adpsgd {

namespace {

template <int LO, int HI, class Fn> __device__ inline void unroll_(Fn&& f) {
    if constexpr (LO < HI) { f(std::integral_constant<int, LO>{}); unroll_<LO + 1, HI>(f); }
}

// ---- waiting for the other workgroups of a pair -------------------------------------------------
// Returns false when the wait ran out (or another workgroup's did): the caller returns at once.
__device__ inline bool wait_for_(const PersistDesc& p, uint32_t* cnt, uint32_t target, int* flag_lds) {
    if (threadIdx.x == 0) {
        int ok = 1;
        const uint64_t t0 = wall_clock64();
        while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            if ((__hip_atomic_load(p.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & kStatusWaitExpired) ||
                wall_clock64() - t0 > p.wait_ticks) {
                __hip_atomic_fetch_or(p.status, kStatusWaitExpired, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // device scope: what the other workgroups stored before they arrived
        *flag_lds = ok;
    }
    __syncthreads();
    const bool ok = *flag_lds != 0;
    __syncthreads();                                   // the flag may be rewritten by the next wait
    return ok;
}

// All threads have stored their part of the frame's operand: make it visible, then count this workgroup in.
// Every thread first waits until its own stores have been accepted by L2 (the vector L1 writes through), the
// workgroup meets, and ONE thread then releases at device scope (one L2 write-back per workgroup instead of one per
// wave: that write-back is what a release costs) and counts the workgroup in.
__device__ inline void arrive_(uint32_t* cnt) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace

// Global accesses of the elementwise phases are written as (wave-uniform 64-bit base) + (per-lane 32-bit byte
// offset): the row of a position splits into a uniform part (row tile, accumulator index) that goes into the
// base on the scalar unit and the lane's part (4 * (lane / 32) rows, unit lane % 32) that is ONE offset register
// per tensor.  The frame's base pointers pass through an empty asm so that the compiler recomputes the row
// pointers from them in every frame instead of keeping one induction variable per row alive across the frames
// (64 pointers: with the resident weights that spills).
template <class T> __device__ inline T* per_frame_(T* p) { asm volatile("" : "+s"(p)); return p; }
__device__ inline float ldg_(const float* sbase, uint32_t voff) {
    return __builtin_nontemporal_load((const float*)((const char*)sbase + voff));
}
__device__ inline void stg_(float v, float* sbase, uint32_t voff) {
    __builtin_nontemporal_store(v, (float*)((char*)sbase + voff));
}
// uniform part of the row of accumulator element i of row tile mt, and of position i of a wave's cells
__device__ constexpr int urow_(int mt, int i) { return 32 * mt + 8 * (i >> 2) + (i & 3); }
template <int MT> __device__ inline int ucell_(int wave, int i) {
    if constexpr (MT == 4) return urow_(wave, i);
    else return urow_(wave * MT / 4, (wave % (4 / MT)) * (4 * MT) + i);
}

// ---- forward ------------------------------------------------------------------------------------
template <int KSTEPS, int MT>
__global__ __launch_bounds__(256, 1) void rec_forward_persist_kernel(PersistDesc p) {
    constexpr int H = KSTEPS * 16, BM = 32 * MT;
    constexpr int SB = 256, KS = 128;                     // bytes and elements of K per stage row
    constexpr int NSTG = H / KS;                          // K stages per frame
    constexpr int NS = NSTG < 4 ? NSTG : 4;               // LDS stages
    typedef GemmDma<bf16_t, KcSrc<bf16_t>, KcSrc<bf16_t>, MT == 4 ? 4 : 2, MT == 4 ? 1 : 2, 1, 1, SB, (NS < 2 ? 2 : NS)> AL;
    static_assert(AL::BM == BM && AL::NT == 256, "loader geometry");
    constexpr int A_BYTES = BM * SB, LA = AL::LA;
    constexpr int EX_BYTES = 4 * BM * 32 * 4;             // gates swapped between the waves
    constexpr int LDS_BYTES = NS * A_BYTES > EX_BYTES ? NS * A_BYTES : EX_BYTES;
    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
    __shared__ int wait_flag;
    constexpr int PP = 4 * MT;                            // (batch row, unit) positions per lane

    const RecDesc& r = p.r;
    const int D = r.D, B = r.B, T = r.T;
    const int64_t DH = (int64_t)D * H, G4 = DH * 4;
    const int wg = blockIdx.x, gl = wg % p.ngl, slice = wg / p.ngl;
    const int li = __builtin_amdgcn_readfirstlane((int)p.gl_learner[gl]), d = __builtin_amdgcn_readfirstlane((int)p.gl_dir[gl]);
    const int u0 = slice * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, g = lane >> 5;
    uint32_t* cnt = p.counters + gl;
    constexpr uint32_t W = H / 32;                         // workgroups per pair

    // this wave's slice of W_h: gate `wave` of units u0 .. u0+31, all H columns, as MFMA B fragments
    uint4 wreg[KSTEPS];
    {
        const bf16_t* wrow = (const bf16_t*)r.wh + li * r.sWi + d * r.sWd + ((int64_t)wave * H + u0 + n) * H + 8 * g;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) wreg[kk] = *(const uint4*)(wrow + 16 * kk);
    }
    // wave-uniform tensor bases of this workgroup's 32 units, and the lane's offset into a row block of each
    float* const gates_u = r.gates + li * r.sGi + (int64_t)d * 4 * H + u0;              // + row * G4 + gate * H
    float* const cbuf_u = r.c + li * r.sCi + (int64_t)d * T * B * H + u0;               // + row * H
    bf16_t* const y_u = (bf16_t*)r.y + li * r.sYi + (int64_t)d * H + u0;                // + row * DH
    const uint32_t voff_g = (uint32_t)((4 * g * G4 + n) * 4);
    const uint32_t voff_c = (uint32_t)((4 * g * H + n) * 4);
    const uint32_t voff_y = (uint32_t)((4 * g * DH + n) * 2);

    KcSrc<bf16_t> a;
    a.ld = DH; a.R = B; a.base = (const bf16_t*)r.y;
    uint32_t aoff[LA];
    AL::template lane_offsets<BM, LA>(a, tid, aoff);

    f32x16_t acc[MT];
    // pre-activations W_x x_t + b of gate `wave`: the accumulators start from them
    auto load_preact = [&](int t) {
        const float* gp = per_frame_(gates_u + (int64_t)t * B * G4 + (int64_t)wave * H);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i)
                acc[mt][i] = urow_(mt, i) + 4 * g < B ? ldg_(gp + (int64_t)urow_(mt, i) * G4, voff_g) : 0.f;
    };
    float cst[PP];
#pragma unroll
    for (int i = 0; i < PP; ++i) cst[i] = 0.f;
    // The activated gates and the cell state of a frame (for the backward pass) are not stored right after they are
    // computed: their 5 * PP stores per lane would only queue behind HBM while the wave has nothing else to issue.
    // They stay in registers and go out one by one between the MFMAs of the next frame's K loop.
    float gi[PP], gf[PP], gg[PP], go[PP];
    float* pend_g = nullptr;             // base pointers of the frame whose results are pending (wave-uniform)
    float* pend_c = nullptr;
    auto store_pending = [&](auto j_) {  // pending store number j: gate j % 5 (4 = cell state) of position j / 5
        constexpr int j = decltype(j_)::value, i = j / 5, q = j % 5;
        const int ur = ucell_<MT>(wave, i);
        if (ur + 4 * g >= B) return;
        if constexpr (q == 4) stg_(cst[i], pend_c + (int64_t)ur * H, voff_c);
        else stg_(q == 0 ? gi[i] : q == 1 ? gf[i] : q == 2 ? gg[i] : go[i], pend_g + (int64_t)ur * G4 + q * H, voff_g);
    };

    load_preact(d == 0 ? 0 : T - 1);
    for (int s = 0; s < T; ++s) {
        const int t = d == 0 ? s : T - 1 - s;
        const int tp = d == 0 ? t - 1 : t + 1;
        if (s > 0) {
            if (!wait_for_(p, cnt, W * (uint32_t)s, &wait_flag)) return;
            a.base = per_frame_((const bf16_t*)r.y + li * r.sYi + (int64_t)tp * B * DH + (int64_t)d * H);
            unroll_<0, NS>([&](auto st) {
                constexpr int S0 = decltype(st)::value;
                if constexpr (S0 < NSTG) AL::template issue<LA>(a, aoff, S0 * KS, lds + S0 * A_BYTES, wave);
            });
            unroll_<0, NSTG>([&](auto kt_) {
                constexpr int kt = decltype(kt_)::value;
                // stages issued after stage kt and still allowed in flight
                constexpr int later = kt == 0 ? (NS - 1 < NSTG - 1 ? NS - 1 : NSTG - 1)
                                              : (NS - 2 < NSTG - 1 - kt ? (NS - 2 < 0 ? 0 : NS - 2) : NSTG - 1 - kt);
                AL::template wait_vm<later * LA>();
                __syncthreads();        // every wave's share of stage kt has landed; stage kt-1 is no longer read
                if constexpr (kt >= 1 && kt + NS - 1 < NSTG)
                    AL::template issue<LA>(a, aoff, (kt + NS - 1) * KS, lds + ((kt - 1) % NS) * A_BYTES, wave);
                const char* cur = lds + (kt % NS) * A_BYTES;
                // fragments of k-step c+1 are read while the MFMAs of k-step c run (two register sets, order pinned)
                uint4 af[2][MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) af[0][mt] = AL::template frag<BM, true>(cur, mt * 32, g, lane);
                __builtin_amdgcn_sched_barrier(0);
                unroll_<0, KS / 16>([&](auto c_) {
                    constexpr int c = decltype(c_)::value;
                    if constexpr (c + 1 < KS / 16) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) af[(c + 1) & 1][mt] = AL::template frag<BM, true>(cur, mt * 32, 2 * (c + 1) + g, lane);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) mma_chunk<bf16_t>(acc[mt], af[c & 1][mt], wreg[kt * (KS / 16) + c]);
                    // the previous frame's results: stores j0 .. j1-1 of the 5 * PP go out with this k-step
                    constexpr int kidx = kt * (KS / 16) + c;
                    constexpr int j0 = kidx * (5 * PP) / KSTEPS, j1 = (kidx + 1) * (5 * PP) / KSTEPS;
                    unroll_<j0, j1>(store_pending);
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
        }
        // swap gates between the waves: ex[gate][row][unit]
        float* ex = (float*)lds;
        __syncthreads();                 // the stage buffers are no longer read
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) ex[(wave * BM + urow_(mt, i) + 4 * g) * 32 + n] = acc[mt][i];
        __syncthreads();
        uint32_t hb[PP];
#pragma unroll
        for (int i = 0; i < PP; ++i) {
            const int row = ucell_<MT>(wave, i) + 4 * g;
            gi[i] = sigmoidf_(ex[(0 * BM + row) * 32 + n]);
            gf[i] = sigmoidf_(ex[(1 * BM + row) * 32 + n]);
            gg[i] = tanhf_(ex[(2 * BM + row) * 32 + n]);
            go[i] = sigmoidf_(ex[(3 * BM + row) * 32 + n]);
            cst[i] = gf[i] * cst[i] + gi[i] * gg[i];
            hb[i] = f32_to_bf16(go[i] * tanhf_(cst[i]));
        }
        // h_t first: the other workgroups of the pair wait for it
        {
            bf16_t* yp = per_frame_(y_u + (int64_t)t * B * DH);
#pragma unroll
            for (int i = 0; i < PP; ++i)
                if (ucell_<MT>(wave, i) + 4 * g < B) *(bf16_t*)((char*)(yp + (int64_t)ucell_<MT>(wave, i) * DH) + voff_y) = (bf16_t)hb[i];
        }
        if (s + 1 < T) arrive_(cnt);
        // activated gates and the cell state, for the backward pass: pending until the next frame's K loop; the
        // first frame is followed by no K loop of its own results' age (frame 0 runs none), the last by none at all
        pend_g = per_frame_(gates_u + (int64_t)t * B * G4);
        pend_c = per_frame_(cbuf_u + (int64_t)t * B * H);
        if (s + 1 == T) unroll_<0, 5 * PP>(store_pending);
        if (s + 1 < T) load_preact(d == 0 ? s + 1 : T - 2 - s);
    }
}

// ---- backward -----------------------------------------------------------------------------------
template <int KSTEPS, int MT>
__global__ __launch_bounds__(256, 1) void rec_backward_persist_kernel(PersistDesc p) {
    constexpr int H = KSTEPS * 16, BM = 32 * MT;
    constexpr int SB = 64, KS = 32;                       // per-wave stages: 32 gate rows of K, 64 bytes per batch row
    constexpr int NSTG = H / KS;                          // K stages per frame (of this wave's quarter of K)
    constexpr int NS = 4;
    typedef GemmDma<bf16_t, KcSrc<bf16_t>, KcSrc<bf16_t>, 1, 1, MT, 1, SB, NS> AL;      // one wave: NT = 64
    static_assert(AL::BM == BM && AL::NT == 64, "loader geometry");
    constexpr int A_BYTES = BM * SB, LA = AL::LA;
    constexpr int WAVE_BYTES = NS * A_BYTES;              // private to a wave
    constexpr int RED_BYTES = 4 * BM * 32 * 4;            // partial products of the four waves
    constexpr int LDS_BYTES = 4 * WAVE_BYTES > RED_BYTES ? 4 * WAVE_BYTES : RED_BYTES;
    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
    __shared__ float csum[4][32][4];                      // bias-gradient partial sums: [wave][unit][gate]
    __shared__ int wait_flag;
    constexpr int PP = 4 * MT;

    const RecDesc& r = p.r;
    const int D = r.D, B = r.B, T = r.T;
    const int64_t DH = (int64_t)D * H, G4 = DH * 4;
    const int wg = blockIdx.x, gl = wg % p.ngl, slice = wg / p.ngl;
    const int li = __builtin_amdgcn_readfirstlane((int)p.gl_learner[gl]), d = __builtin_amdgcn_readfirstlane((int)p.gl_dir[gl]);
    const int u0 = slice * 32;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, g = lane >> 5;
    uint32_t* cnt = p.counters + gl;
    constexpr uint32_t W = H / 32;

    // this wave's slice of W_h as MFMA B fragments of dh = da W_h: column = unit u0 + n, k = rows of gate `wave`;
    // the 8 values of a fragment are 8 consecutive rows of W_h (a column walk: gathered once per launch)
    uint4 wreg[KSTEPS];
    {
        const bf16_t* wcol = (const bf16_t*)r.wh + li * r.sWi + d * r.sWd + ((int64_t)wave * H + 8 * g) * H + u0 + n;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const bf16_t* q = wcol + (int64_t)16 * kk * H;
            uint32_t v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (uint32_t)q[(int64_t)(2 * e) * H] | ((uint32_t)q[(int64_t)(2 * e + 1) * H] << 16);
            wreg[kk] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    }
    const float* const gates_u = r.gates + li * r.sGi + (int64_t)d * 4 * H + u0;
    const float* const cbuf_u = r.c + li * r.sCi + (int64_t)d * T * B * H + u0;
    const float* const dy_u = r.dy + li * r.sDYi + (int64_t)d * H + u0;
    bf16_t* const da_u = (bf16_t*)r.da + li * r.sDAi + (int64_t)d * 4 * H + u0;
    const uint32_t voff_g = (uint32_t)((4 * g * G4 + n) * 4);
    const uint32_t voff_c = (uint32_t)((4 * g * H + n) * 4);
    const uint32_t voff_dy = (uint32_t)((4 * g * DH + n) * 4);
    const uint32_t voff_da = (uint32_t)((4 * g * G4 + n) * 2);
    char* mylds = lds + wave * WAVE_BYTES;

    KcSrc<bf16_t> a;
    a.ld = G4; a.R = B; a.base = (const bf16_t*)r.da;
    uint32_t aoff[LA];
    AL::template lane_offsets<BM, LA>(a, lane, aoff);

    float dcr[PP];
#pragma unroll
    for (int i = 0; i < PP; ++i) dcr[i] = 0.f;

    for (int s = 0; s < T; ++s) {
        const int t = d == 0 ? T - 1 - s : s;              // reverse of the forward processing order
        const int tn = d == 0 ? t + 1 : t - 1;             // frame handled in the previous step
        const int tp = d == 0 ? t - 1 : t + 1;             // frame the forward pass processed before t
        const bool has_prev = tp >= 0 && tp < T;
        float dh[PP];
#pragma unroll
        for (int i = 0; i < PP; ++i) dh[i] = 0.f;
        if (s > 0) {
            if (!wait_for_(p, cnt, W * (uint32_t)s, &wait_flag)) return;
            f32x16_t acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[mt][e] = 0.f;
            a.base = per_frame_((const bf16_t*)r.da + li * r.sDAi + (int64_t)tn * B * G4 + (int64_t)d * 4 * H + (int64_t)wave * H);
            unroll_<0, NS - 1>([&](auto st) {
                constexpr int S0 = decltype(st)::value;
                if constexpr (S0 < NSTG) AL::template issue<LA>(a, aoff, S0 * KS, mylds + S0 * A_BYTES, 0);
            });
            unroll_<0, NSTG>([&](auto kt_) {
                constexpr int kt = decltype(kt_)::value;
                // the fragments of stage kt-1 have been consumed (their MFMAs are issued): its buffer may be refilled
                if constexpr (kt + NS - 1 < NSTG) {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    AL::template issue<LA>(a, aoff, (kt + NS - 1) * KS, mylds + ((kt + NS - 1) % NS) * A_BYTES, 0);
                }
                constexpr int later = NS - 1 < NSTG - 1 - kt ? NS - 1 : NSTG - 1 - kt;
                AL::template wait_vm<later * LA>();
                const char* cur = mylds + (kt % NS) * A_BYTES;
                uint4 af[2][MT];
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) af[0][mt] = AL::template frag<BM, true>(cur, mt * 32, g, lane);
                __builtin_amdgcn_sched_barrier(0);
                unroll_<0, KS / 16>([&](auto c_) {
                    constexpr int c = decltype(c_)::value;
                    if constexpr (c + 1 < KS / 16) {
#pragma unroll
                        for (int mt = 0; mt < MT; ++mt) af[(c + 1) & 1][mt] = AL::template frag<BM, true>(cur, mt * 32, 2 * (c + 1) + g, lane);
                    }
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) mma_chunk<bf16_t>(acc[mt], af[c & 1][mt], wreg[kt * (KS / 16) + c]);
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
            // add the four waves' partial products in a fixed order
            float* red = (float*)lds;
            __syncthreads();             // every wave is done with its stage buffers
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int i = 0; i < 16; ++i) red[(wave * BM + urow_(mt, i) + 4 * g) * 32 + n] = acc[mt][i];
            __syncthreads();
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                const int row = ucell_<MT>(wave, i) + 4 * g;
                dh[i] = ((red[(0 * BM + row) * 32 + n] + red[(1 * BM + row) * 32 + n]) + red[(2 * BM + row) * 32 + n]) +
                        red[(3 * BM + row) * 32 + n];
            }
            __syncthreads();             // red overlaps the stage buffers of the next frame
        }
        // cell backward for this lane's positions
        float cs[4] = {0.f, 0.f, 0.f, 0.f};
        uint32_t pk0[PP], pk1[PP];
        {
            const float* gp = per_frame_(gates_u + (int64_t)t * B * G4);
            const float* cvp = per_frame_(cbuf_u + (int64_t)t * B * H);
            const float* cpp = per_frame_(cbuf_u + (int64_t)(has_prev ? tp : t) * B * H);
            const float* dyp = per_frame_(dy_u + (int64_t)t * B * DH);
            float dyv[PP], gi[PP], gf[PP], gg[PP], go[PP], cv[PP], cp[PP];
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                const int ur = ucell_<MT>(wave, i);
                const bool ok = ur + 4 * g < B;
                const float* rp = gp + (int64_t)ur * G4;
                dyv[i] = ok ? ldg_(dyp + (int64_t)ur * DH, voff_dy) : 0.f;
                gi[i] = ok ? ldg_(rp, voff_g) : 0.f; gf[i] = ok ? ldg_(rp + H, voff_g) : 0.f;
                gg[i] = ok ? ldg_(rp + 2 * H, voff_g) : 0.f; go[i] = ok ? ldg_(rp + 3 * H, voff_g) : 0.f;
                cv[i] = ok ? ldg_(cvp + (int64_t)ur * H, voff_c) : 0.f;
                cp[i] = (ok && has_prev) ? ldg_(cpp + (int64_t)ur * H, voff_c) : 0.f;
            }
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                // rows past the batch: all gates read as 0, so all four results are 0
                const float dhv = dyv[i] + dh[i];
                const float tc = tanhf_(cv[i]);
                const float dov = dhv * tc;
                const float dcv = dcr[i] + dhv * go[i] * (1.f - tc * tc);
                const float di = dcv * gg[i], dg = dcv * gi[i], df = dcv * cp[i];
                dcr[i] = dcv * gf[i];
                const float a0 = di * gi[i] * (1.f - gi[i]), a1 = df * gf[i] * (1.f - gf[i]);
                const float a2 = dg * (1.f - gg[i] * gg[i]), a3 = dov * go[i] * (1.f - go[i]);
                cs[0] += a0; cs[1] += a1; cs[2] += a2; cs[3] += a3;
                pk0[i] = pack_bf16(a0, a1);
                pk1[i] = pack_bf16(a2, a3);
            }
        }
        // da_t first: the other workgroups of the pair wait for it
        {
            bf16_t* dap = per_frame_(da_u + (int64_t)t * B * G4);
#pragma unroll
            for (int i = 0; i < PP; ++i) {
                const int ur = ucell_<MT>(wave, i);
                if (ur + 4 * g >= B) continue;
                char* rp = (char*)(dap + (int64_t)ur * G4) + voff_da;
                *(bf16_t*)rp = (bf16_t)(pk0[i] & 0xffffu); *(bf16_t*)(rp + 2 * H) = (bf16_t)(pk0[i] >> 16);
                *(bf16_t*)(rp + 4 * H) = (bf16_t)(pk1[i] & 0xffffu); *(bf16_t*)(rp + 6 * H) = (bf16_t)(pk1[i] >> 16);
            }
        }
        if (s + 1 < T) arrive_(cnt);
        // bias gradient: column sums of da over the rows of the tile, in a fixed order (lane pair, then the waves)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float v = cs[q] + __shfl_xor(cs[q], 32);
            if (lane < 32) csum[wave][n][q] = v;
        }
        __syncthreads();
        if (tid < 128) {
            const int col = tid & 31, q = tid >> 5;
            const float sum = ((csum[0][col][q] + csum[1][col][q]) + csum[2][col][q]) + csum[3][col][q];
            r.dbp[li * r.sDBi + (int64_t)t * G4 + (int64_t)d * 4 * H + (int64_t)q * H + u0 + col] = sum;
        }
        __syncthreads();                 // csum is rewritten in the next frame
    }
}

// ---- launchers -------------------------------------------------------------------------------------
bool rec_persist_supported(const RecDesc& d, int cu_count) {
    if (d.precision != 1 || d.D < 1 || d.D > 2 || d.T < 1 || d.B < 1 || d.B > 128) return false;
    if (d.H != 128 && d.H != 256 && d.H != 512 && d.H != 1024) return false;
    if (d.H / 32 > cu_count) return false;
    // 16-byte aligned rows of everything the direct loads and the 16-byte weight loads touch
    return (uintptr_t)d.wh % 16 == 0 && d.sWi % 8 == 0 && d.sWd % 8 == 0 && (uintptr_t)d.y % 16 == 0 && d.sYi % 8 == 0 &&
           (uintptr_t)d.da % 16 == 0 && d.sDAi % 8 == 0;
}

template <int KSTEPS>
static void launch_persist_t(const PersistDesc& p, bool backward, unsigned grid, hipStream_t s) {
    if (p.r.B > 64) {
        if (backward) hipLaunchKernelGGL((rec_backward_persist_kernel<KSTEPS, 4>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((rec_forward_persist_kernel<KSTEPS, 4>), dim3(grid), dim3(256), 0, s, p);
    } else {
        if (backward) hipLaunchKernelGGL((rec_backward_persist_kernel<KSTEPS, 2>), dim3(grid), dim3(256), 0, s, p);
        else hipLaunchKernelGGL((rec_forward_persist_kernel<KSTEPS, 2>), dim3(grid), dim3(256), 0, s, p);
    }
}

hipError_t launch_rec_persist(const PersistDesc& p, bool backward, int cu_count, hipStream_t s) {
    if (!rec_persist_supported(p.r, cu_count)) return hipErrorInvalidValue;
    if (p.ngl < 1 || p.ngl > 64 || !p.counters || !p.status) return hipErrorInvalidValue;
    const int W = p.r.H / 32;
    if ((int64_t)p.ngl * W > cu_count) return hipErrorInvalidValue;      // all workgroups must be resident together
    for (int j = 0; j < p.ngl; ++j)
        if (p.gl_dir[j] >= p.r.D) return hipErrorInvalidValue;
    const unsigned grid = (unsigned)(p.ngl * W);
    switch (p.r.H) {
        case 128: launch_persist_t<8>(p, backward, grid, s); break;
        case 256: launch_persist_t<16>(p, backward, grid, s); break;
        case 512: launch_persist_t<32>(p, backward, grid, s); break;
        default: launch_persist_t<64>(p, backward, grid, s); break;
    }
    return hipGetLastError();
}

}  // namespace adpsgd
