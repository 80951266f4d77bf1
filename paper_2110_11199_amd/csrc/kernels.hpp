// Host-side launch interface of the HIP kernels (internal to the library).
#pragma once
#include "common.hpp"

namespace adpsgd {

// Compacted list of the learners a launch works on: entry j of the launch is learner idx[j].
// Stragglers (Section IV-D: a learner that sits an iteration out) are left out of every launch
// of the gradient phase this way; without stragglers it is the identity.
struct LearnerMap {
    uint8_t idx[128];
    void identity() { for (int i = 0; i < 128; ++i) idx[i] = (uint8_t)i; }
};

// ---- grouped GEMM  C[z] = A[z] * B[z]' (+ bias) ------------------------------
// Group z = j*groupsD + d works on learner i = lmap.idx[j]; operand X of it starts at
// X + i*sXi + d*sXd (strides in elements).
struct GemmDesc {
    int precision;            // 0 fp32 operands, 1 bf16 operands
    int a_kc, b_kc;           // operand stored K-contiguous ([rows][K]) or not ([K][rows])
    int c_elem;               // C stored in the operand type instead of fp32
    int M, N, K;
    const void* A; int64_t lda, sAi, sAd;
    const void* B; int64_t ldb, sBi, sBd;
    void* C; int64_t ldc, sCi, sCd;
    const float* bias; int64_t sBiasI, sBiasD;
    int groupsI, groupsD;
    int tile;                 // tile configuration (see gemm.hip): -1 automatic, or 0, 5, 11, 12, 13
    LearnerMap lmap;
};
// Returns hipSuccess, or hipErrorInvalidValue when the operands do not meet the
// alignment rules (rows and strides multiples of 4 elements).
hipError_t launch_gemm(const GemmDesc& d, hipStream_t s);

// ---- fused mixing + SGD update ------------------------------------------------
struct UpdateDesc {
    int L;
    int mix;                   // 0 pair, 1 ring neighbours (thirds), 2 all, 3 / 4 hybrid: mean inside super-learners of
                               // group_size consecutive learners, pair / ring-neighbour operator across them (partner and
                               // order are then over the L / group_size super-learners)
    int group_size;
    int64_t P;                 // elements per learner
    const float* src;          // x^k, learner i at src + i*stride
    float* dst;                // x^{k+1}, learner i at dst + i*stride (may equal src)
    int64_t stride;
    const float* g[128];       // gradient of learner i
    int16_t partner[128];
    int16_t order[128];        // ring order (mix 1): order[p] = learner at ring position p
    int16_t active[128];
    float lr;
    bf16_t* shadow;            // optional [L][stride] bf16 copy of the next gradient point, or NULL
    int emit_input;            // shadow = bf16(x^k) (tau = 1) instead of bf16(x^{k+1})
    int update_first;          // mix 2 only: average the updated models x_j - lr*g_j (synchronous baseline)
    int pair_split;            // mix 0: 64 / 128 = one member of a pair per thread in workgroups of that many positions (models
                               // exchanged through LDS), 0 = both members per thread, -1 = default
    int sync_segment;          // synchronous baseline: learners per thread (2, 4 or 8), 0: one thread owns all learners of a position, -1: default
    int tri_segment;           // mix 1: ring positions per thread (2, 4 or 8), 0: one thread walks the whole ring, -1: default
    float* mean_buf;           // mix 2: optional buffer of mean_elems floats; when given the global mean runs chunk by
    int64_t mean_elems;        //   chunk of that many elements in two kernels (fewer streams per thread); NULL: one kernel
};
hipError_t launch_update(const UpdateDesc& d, hipStream_t s);
hipError_t launch_average(const float* x, int64_t stride, int L, int64_t P, float* out, hipStream_t s);
// out[0] = sum_i sum_e (x_i[e] - mean_i x_i[e])^2 in fp64; partial: kConsensusBlocks doubles of scratch
constexpr int kConsensusBlocks = 2048;
hipError_t launch_consensus(const float* x, int64_t stride, int L, int64_t P, double* partial, double* out, hipStream_t s);
// the same with the partial sums in a device array owned by the library (one per GPU, shared by all calls on it)
constexpr int kMaxDevices = 64;
hipError_t launch_consensus_static(const float* x, int64_t stride, int L, int64_t P, double* out, hipStream_t s);

// ---- LSTM gradient pieces -------------------------------------------------------
struct StageDesc {             // copy / cast the minibatches into the workspace
    int L, precision;          // L: learners of this launch (entries of lmap)
    LearnerMap lmap;
    int64_t rows;              // T*B
    int I, ldx;                // feature dim and padded row stride of the staged copy
    const float* feats[128];
    const int32_t* labels[128];
    void* x0; int64_t sX0;     // [L][rows][ldx] operand type
    int32_t* y; int64_t sY;    // [L][rows]
};
hipError_t launch_stage(const StageDesc& d, hipStream_t s);
hipError_t launch_cast_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t s);
// dst[z][r][0..ld) = bf16(src[z][r][0..cols)), zero padded; z < L, strides sS / sD in elements
hipError_t launch_pad_rows_bf16(const float* src, int64_t sS, bf16_t* dst, int64_t sD, int64_t rows, int cols, int ld,
                                int L, hipStream_t s);

struct RecDesc {               // one time step of one layer, all learners and directions
    int precision;
    int L, D, B, H, T;         // L: learners of this launch (entries of lmap)
    LearnerMap lmap;
    int direct;                // 0: never use the direct-to-LDS or the small-batch kernels (tuning)
    int step;                  // processing step 0..T-1 (frame = step, or T-1-step for d = 1)
    // forward: gates buffer holds W_x x + b on entry, the activated gates on exit
    float* gates; int64_t sGi;           // [L][T*B][D*4H] fp32
    float* c; int64_t sCi;               // [L][D][T*B][H] fp32
    void* y; int64_t sYi;                // [L][T*B][D*H] operand type (layer output)
    const void* wh; int64_t sWi, sWd;    // W_h [D][4H][H] operand type, learner stride
    // backward only
    const float* dy; int64_t sDYi;       // [L][T*B][D*H] fp32, gradient w.r.t. the layer output
    void* da; int64_t sDAi;              // [L][T*B][D*4H] operand type, gate pre-activation grads
    float* dc; int64_t sDCi;             // [L][D][B][H] fp32 running dL/dc
    // column sums of da over the batch rows of every tile (partial bias gradients), summed over the
    // frames and batch tiles afterwards: [L][T * batch tiles][D*4H] fp32
    float* dbp; int64_t sDBi;
};
// Batch tiles of the backward step kernels for a batch of B rows (rows of dbp per frame).
int rec_backward_batch_tiles(int B);
hipError_t launch_rec_forward(const RecDesc& d, hipStream_t s);
hipError_t launch_rec_backward(const RecDesc& d, hipStream_t s);
// The same step for batches of at most 32 rows (lstm_small.hip): contraction split over the waves of a workgroup,
// operands read straight into registers.  launch_rec_forward / launch_rec_backward use it when it applies.
bool rec_small_supported(const RecDesc& d);
hipError_t launch_rec_small(const RecDesc& d, bool backward, hipStream_t s);

// Bits of the device-side status word of a handle (0 = fine).
constexpr uint32_t kStatusBadLabel = 1u;       // a label outside [0, classes) was met (and clamped)
constexpr uint32_t kStatusWaitExpired = 2u;    // a bounded wait between workgroups ran out

// All T frames of one layer for ngl (learner, direction) pairs in one launch, W_h held in registers
// (lstm_persist.hip).  r: the tensors of the layer (r.L, r.lmap, r.step and r.direct are not used);
// pair j of the launch is learner gl_learner[j], direction gl_dir[j].
struct PersistDesc {
    RecDesc r;
    int ngl;                             // pairs of this launch, 1..64; ngl * H/32 workgroups, at most one per compute unit
    uint8_t gl_learner[64], gl_dir[64];
    uint32_t* counters;                  // [ngl] device words, zero before the launch: workgroups that have finished a frame
    uint32_t* status;                    // the handle's status word (kStatusWaitExpired is or-ed in)
    unsigned long long wait_ticks;       // bound of one wait between workgroups, in ticks of the 100 MHz wall clock
};
bool rec_persist_supported(const RecDesc& d, int cu_count);
hipError_t launch_rec_persist(const PersistDesc& p, bool backward, int cu_count, hipStream_t s);

// one wave that idles for `ticks` of the 100 MHz wall clock (the wall-clock model of the slow-learner experiment)
hipError_t launch_delay(unsigned long long ticks, hipStream_t s);

// ---- measurement probes (probe.hip) ----------------------------------------------------------------
hipError_t launch_mfma_peak(float* out, int blocks, int iters, hipStream_t s);       // out: [blocks * 256] floats
// reads : writes_f32 : writes_bf16 one of 1:0:0, 1:1:0, 2:1:0, 2:1:1, 4:2:0, 4:2:2, 8:4:4, 16:8:8, 32:16:16; the streams
// are `pitch` bytes apart in buf
hipError_t launch_stream_probe(int reads, int writes_f32, int writes_bf16, void* buf, int64_t pitch, int64_t elems, hipStream_t s);

struct SoftmaxDesc {
    int precision, L;          // L: learners of this launch (entries of lmap)
    LearnerMap lmap;
    int L_all;                 // all learners of the handle (loss[] has this many entries)
    uint32_t active_bits[4];   // bit i: learner i takes part; the loss of the others is reported as 0
    uint32_t* status;          // device status word: kStatusBadLabel is or-ed in
    int64_t rows; int C;
    const float* logits; int64_t sLi;    // [L][rows][C]
    const int32_t* y; int64_t sYi;
    void* dlogits; int64_t sDi;          // [L][rows][C] operand type: (softmax - onehot)/rows
    float* row_loss;                     // [L][rows]
    float* loss;                         // [L]
};
hipError_t launch_softmax_ce(const SoftmaxDesc& d, hipStream_t s);

// out[z][n] = sum_m in[z][m][n]   (bias gradients), z = lmap.idx[0..L)
hipError_t launch_colsum(int precision, const void* in, int64_t ld, int64_t sIi, int64_t rows, int N,
                         float* out, int64_t sOi, int L, const LearnerMap& lmap, hipStream_t s);
// dst[z][0..n) = 0 for z = lmap.idx[0..L)  (a fill kernel, not a memset node: safe under stream capture)
hipError_t launch_zero(float* dst, int64_t sDi, int64_t n, int L, const LearnerMap& lmap, hipStream_t s);

}  // namespace adpsgd
