/*
 * adpsgd.h -- C ABI of the MI355X (gfx950) ADPSGD hot-path library.
 *
 * One ADPSGD iteration over L learners held as replicas on ONE GPU, following
 * the paper's model (Section II, Eq. 2)
 *
 *        W_{k+1} = W_k T_k - a_k g(Phi_k, xi_k),       Phi_k = W_{k-tau}
 *
 *   (a) every learner's minibatch gradient of the mean cross-entropy of a
 *       stacked (bi)directional LSTM acoustic model (Section IV: LSTM layers,
 *       optional linear bottleneck, softmax over context-dependent states,
 *       segments of T frames with zero initial state);
 *   (b) the mixing term W_k T_k for the fixed ring (Section III-B), the
 *       randomly permuted ring (Section III-C, Fisher-Yates) or the
 *       delay-by-one scheme (Section III-D: T = 11'/L, gradient one iterate behind);
 *       on the rings either pairwise (weights 1/2) or with both ring neighbours
 *       (weights 1/3, the operator T^f of Eq. 9);
 *   (c) the fused mixing + SGD update  w <- (mixed model) - lr * g  (Algorithm 1).
 * The synchronous baseline of Section III-A (Algorithm 2: update, then the mean
 * of all learners) runs on the same engine as a fourth pattern.
 *
 * Conventions
 *   - Every function returns ADPSGD_OK (0) or a negative ADPSGD_E* code; the
 *     text of the last error of the calling thread is adpsgd_last_error().
 *     No C++ exception crosses this boundary.
 *   - "dev" pointers are HIP device pointers on the device that was current at
 *     adpsgd_create; "host" pointers are ordinary host memory.
 *   - The library allocates NO device memory.  The caller allocates one
 *     workspace of adpsgd_workspace_bytes() bytes (256-byte aligned), hands it
 *     to adpsgd_create and keeps it alive until adpsgd_destroy.  All state
 *     (models, gradients, activations) lives inside it.
 *   - All work is enqueued on the HIP stream given at create; calls return
 *     without waiting unless stated.  Calls on one handle must not overlap.
 *   - Flat parameter layout of one learner (fp32, row-major, rows = output
 *     units, gate blocks ordered i,f,g,o), I_0 = input_dim, I_l = D*hidden:
 *         for l in layers:  W_x[l] [D][4H][I_l], W_h[l] [D][4H][H], b[l] [D][4H]
 *         (bottleneck > 0)  W_p [Bn][D*H], b_p [Bn]
 *         W_o [C][F], b_o [C]                         F = Bn or D*H
 *     input_dim, hidden, bottleneck and classes must be multiples of 4.
 *   - Batch layout: features [T][B][I] fp32 (time-major), labels [T][B] int32
 *     in [0, classes).  Labels are device data, so they are checked on the device: a
 *     label outside the range is clamped (it is never used as an index) and raises a
 *     sticky error flag of the handle; the first adpsgd_losses / adpsgd_status call
 *     after that step, and every adpsgd_step issued once that step has completed,
 *     return ADPSGD_EINVAL.
 */
#ifndef ADPSGD_H
#define ADPSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADPSGD_OK        0
#define ADPSGD_EINVAL   (-1)   /* bad argument or unsupported combination        */
#define ADPSGD_ENOMEM   (-2)   /* workspace too small or misaligned              */
#define ADPSGD_EHIP     (-3)   /* a HIP call failed (text in adpsgd_last_error)  */

#define ADPSGD_MAX_LEARNERS 128

typedef struct adpsgd_handle* adpsgd_t;   /* opaque; owned by the library (host memory) */
typedef struct adpsgd_graph* adpsgd_graph_t;   /* opaque: a recorded sequence of iterations (host memory) */

/* Communication pattern (Section III-B / III-C / III-D), or the synchronous baseline
 * SDPSGD of Section III-A (Algorithm 2): every learner updates its own model,
 * u_j = x_j - lr * g_j, then all models are replaced by their mean
 * (((u_0 + u_1) + ...) * fl(1/L)), W_{k+1} = (W_k - a_k g(W_k)) 11'/L.  SDPSGD fixes
 * mix = ALL and tau = 0 and takes no stragglers.                                */
typedef enum { ADPSGD_FIXED_RING = 0, ADPSGD_RANDOM_RING = 1, ADPSGD_D1D = 2, ADPSGD_SDPSGD = 3 } adpsgd_pattern;
/* Mixing operator applied along that pattern.
 *   PAIR  (x_i + x_j)/2 with the partner j of a perfect matching on the ring order
 *   TRI   (x_left + x_i + x_right)/3 with the two neighbours on the ring order: the
 *         circulant operator T^f of Eq. 9 (Section III-B) on the fixed ring and its
 *         permuted form T^r = P' T^f P on the random ring (Section III-C); summed as
 *         (x_left + x_i) + x_right in that order, then times fl(1/3); needs L >= 3
 *         (with fewer learners the three ring positions are not distinct)
 *   ALL   the global mean, T = 11'/L (allreduce, Section III-A / III-D)
 *   HYBRID_PAIR, HYBRID_TRI   the hybrid strategy of Section V (its hierarchical ring
 *         figure): consecutive blocks of group_size learners form super-learners that
 *         average synchronously, m_a = (((x_{aS} + x_{aS+1}) + ...)) * fl(1/S), and the
 *         G = L / group_size super-learners form the asynchronous ring, on whose means
 *         the PAIR or TRI operator acts; every learner of super-learner a then takes
 *         x_i <- m - lr * g_i.  The ring patterns only, no stragglers (a super-learner
 *         waits for its members); L a multiple of group_size; TRI needs G >= 3 or G == 1.
 *         The schedule (ring order, matching) is that of G ring positions.
 *   DEFAULT = PAIR for the rings, ALL for delay-by-one and the synchronous baseline. */
typedef enum { ADPSGD_MIX_DEFAULT = -1, ADPSGD_MIX_PAIR = 0, ADPSGD_MIX_TRI = 1, ADPSGD_MIX_ALL = 2,
               ADPSGD_MIX_HYBRID_PAIR = 3, ADPSGD_MIX_HYBRID_TRI = 4 } adpsgd_mix;
/* Arithmetic of the GEMMs: fp32 operands, or bf16 operands (rounded to nearest
 * even from the fp32 master) with fp32 accumulation.  State, gates, softmax
 * and the update are fp32 in both.                                              */
typedef enum { ADPSGD_FP32 = 0, ADPSGD_BF16_GEMM = 1 } adpsgd_precision;

typedef struct {
    int32_t input_dim;      /* I: feature dimension (260 in the paper)           */
    int32_t hidden;         /* H: LSTM cells per direction                       */
    int32_t layers;         /* stacked LSTM layers (>= 1)                        */
    int32_t bidirectional;  /* 0: one direction, 1: two, outputs concatenated    */
    int32_t bottleneck;     /* Bn: width of the linear projection, 0 = none      */
    int32_t classes;        /* C: softmax outputs                                */
    int32_t batch;          /* B: segments per learner minibatch                 */
    int32_t frames;         /* T: frames per segment (21 in the paper)           */
    int64_t flat_params;    /* > 0: model-free mode, a learner is a flat vector
                               of this many floats and adpsgd_step is handed
                               gradients instead of minibatches                  */
} adpsgd_model_shape;

typedef struct {
    int32_t            L;            /* learners, 1..ADPSGD_MAX_LEARNERS          */
    adpsgd_model_shape shape;
    int32_t            pattern;      /* adpsgd_pattern                            */
    int32_t            mix;          /* adpsgd_mix                                */
    int32_t            tau;          /* staleness of the gradient's model: 0, 1,
                                        or -1 = default (1 for D1D, else 0)       */
    int32_t            precision;    /* adpsgd_precision                          */
    uint64_t           seed;         /* seed of the schedule (and of init_scale)  */
    float              straggler_p;  /* probability that a learner sits an
                                        iteration out (0 = never); pairwise mixing
                                        on the rings with tau = 0 only            */
    float              init_scale;   /* > 0: all learners start from the same
                                        w_0 ~ U(-a, a) (Algorithm 1, input);
                                        0: models start as zeros, set them with
                                        adpsgd_set_params                         */
    int32_t            group_size;   /* learners per super-learner (hybrid mixes);
                                        0 or 1 with every other mix                */
} adpsgd_config;

/* Bytes of device workspace a handle with this configuration needs.
 * cfg, out: host.  EINVAL if the configuration is not supported.               */
int adpsgd_workspace_bytes(const adpsgd_config* cfg, size_t* out);

/* Build a handle inside the caller's workspace (Algorithm 1, "Input": every
 * learner starts from the same w_0).  dev_workspace: device, 256-byte aligned,
 * at least adpsgd_workspace_bytes; hip_stream: a hipStream_t (NULL = the null
 * stream).  Synchronises the stream once.  *out is valid only on ADPSGD_OK.    */
int adpsgd_create(const adpsgd_config* cfg, void* dev_workspace, size_t bytes,
                  void* hip_stream, adpsgd_t* out);

/* One iteration k -> k+1 (Algorithm 3 / Algorithm 4, or Algorithm 2 for the
 * synchronous baseline, on every learner at once): schedule, gradients at
 * x^{k-tau}, mixing, update.  Asynchronous.
 * batch_ptrs: host array of device pointers.
 *   model mode: [2L], batch_ptrs[2i] = features of learner i ([T][B][I] fp32),
 *               batch_ptrs[2i+1] = labels of learner i ([T][B] int32);
 *   flat mode:  [L],  batch_ptrs[i] = gradient of learner i ([flat_params] fp32).
 * The buffers are read during the call's stream work and never written.
 * A straggler (Section IV-D: a learner that sits the iteration out) computes nothing:
 * its model is left bit-unchanged, its pointers are not read and may be NULL, its loss
 * is reported as 0 and its slot of adpsgd_grads keeps the gradient it computed last.
 * Returns the sticky error of an earlier step (see the conventions above) instead of
 * enqueuing work once that error has reached the host.                          */
int adpsgd_step(adpsgd_t h, const void* const* batch_ptrs, float lr);

/* The same iteration with the stragglers GIVEN by the caller instead of drawn from the seed: active: host
 * int32 [L], 0 = learner i sits this iteration out (Section IV-D: a learner that is observed to be late; the
 * others do not wait for it).  The ring order and the matching are those of iteration k as always; a learner
 * matched with a straggler mixes with nobody.  A mask with a zero needs a ring pattern with pairwise mixing
 * and tau = 0 (what straggler_p needs), otherwise ADPSGD_EINVAL.  Used by the wall-clock model of the
 * paper's slow-learner experiment (paper_2110_11199_amd/straggler_model.py).                             */
int adpsgd_step_masked(adpsgd_t h, const void* const* batch_ptrs, float lr, const int32_t* active);

/* HIP-graph replay of iterations, for models small enough that an iteration is a few hundred launches of
 * microseconds each (HIP streams and graphs take the place a tracing compiler has elsewhere).
 * adpsgd_step enqueues kernels and one 4-byte copy to pinned host memory and nothing else, so its stream work can
 * be recorded once and replayed.
 *   adpsgd_capture_begin(h)      puts the handle's stream into capture mode.  Until adpsgd_capture_end, calls of
 *                                adpsgd_step / adpsgd_step_masked on h are RECORDED, not run; every other entry
 *                                point that takes h returns ADPSGD_EINVAL.  Needs: a stream of the handle's own (not
 *                                the null stream), a schedule that does not change with the iteration (not
 *                                ADPSGD_RANDOM_RING, straggler_p = 0), phase profiling off, and in bf16 mode one
 *                                iteration run before; else ADPSGD_EINVAL.
 *   adpsgd_capture_end(h, &g)    ends the recording and puts the handle back to the iteration it stood at (nothing
 *                                has run).  At least one iteration must have been recorded, an even number on
 *                                ADPSGD_FIXED_RING and with tau = 1 (the matching phase and the two model buffers
 *                                alternate): else ADPSGD_EINVAL and *g = NULL.
 *   adpsgd_graph_replay(g)       runs the recorded iterations on the handle's stream, asynchronously, and advances
 *                                adpsgd_iteration by their number.  A replay repeats what was recorded: the SAME
 *                                batch pointers (refill those buffers, in stream order, before the call), the same
 *                                learning rate, the same masks.  On the alternating patterns the handle must stand
 *                                at an iteration of the same parity as the recording's first one (ADPSGD_EINVAL).
 *                                Sticky errors of the handle are reported as by adpsgd_step.
 *   adpsgd_graph_steps(g)        iterations recorded (-1 for NULL).
 *   adpsgd_graph_destroy(g)      waits for the stream, frees the recording (host memory owned by the library).
 * Results are those of the same adpsgd_step calls made directly, bit for bit (the same kernels in the same order).
 * A recording belongs to its handle; after adpsgd_destroy(h) it can only be destroyed.                             */
int adpsgd_capture_begin(adpsgd_t h);
int adpsgd_capture_end(adpsgd_t h, adpsgd_graph_t* out);
int adpsgd_graph_replay(adpsgd_graph_t g);
int64_t adpsgd_graph_steps(adpsgd_graph_t g);
void adpsgd_graph_destroy(adpsgd_graph_t g);

/* A kernel of one wave that does nothing for `microseconds` of wall-clock time (at most 10 000 000) and
 * returns: stands for a learner's gradient computation on its own device in the wall-clock model of the
 * slow-learner experiment (Section IV-D, where the slow learner is put to sleep for a set time).
 * Asynchronous on hip_stream.                                                                            */
int adpsgd_delay(uint64_t microseconds, void* hip_stream);

/* Device pointer to learner i's current model x_i^k ([P] fp32), borrowed.  With
 * tau = 1 the two model buffers swap every iteration: query again after each
 * step.  NULL on a bad argument.                                               */
float* adpsgd_params(adpsgd_t h, int i);

/* Overwrite learner i's model (i = -1: every learner) with [P] floats read from
 * dev_src; also resets the one-iteration-old copy used when tau = 1
 * (x^{-1} := x^0).  Asynchronous device-to-device copy.                        */
int adpsgd_set_params(adpsgd_t h, int i, const float* dev_src);

/* Device pointer to the gradient learner i used in the last step ([P] fp32;
 * model mode only), borrowed.  NULL on a bad argument.                         */
float* adpsgd_grads(adpsgd_t h, int i);

/* Mean cross-entropy of every learner's last minibatch (0 for a straggler), host_out [L].
 * Waits for the stream; returns the handle's sticky error if a kernel has raised one.  */
int adpsgd_losses(adpsgd_t h, float* host_out);

/* Waits for the stream and returns ADPSGD_OK or the handle's sticky error: ADPSGD_EINVAL
 * after a label outside [0, classes), ADPSGD_EHIP after a bounded wait between the
 * workgroups of a kernel has run out.                                            */
int adpsgd_status(adpsgd_t h);

/* Number of parameters P of one learner.                                       */
int64_t adpsgd_param_count(adpsgd_t h);

/* Number of tensors in the flat layout (model mode), and tensor idx's place in
 * it: offset (floats), rows, cols.  EINVAL when idx is out of range.           */
int adpsgd_layout_count(adpsgd_t h);
int adpsgd_layout(adpsgd_t h, int idx, int64_t* offset, int64_t* rows, int64_t* cols);

/* The schedule of iteration k, a pure function of (config, k): ring order,
 * matching partner (partner[i] == i: none) and active flag of each learner.
 * order, partner, active: host int32 [L] (any may be NULL).  With a hybrid mix the
 * ring is that of the G = L / group_size super-learners: entries 0..G-1 describe it
 * and entries G..L-1 are set to -1.                                              */
int adpsgd_schedule(adpsgd_t h, int64_t k, int32_t* order, int32_t* partner, int32_t* active);

/* Same without a handle.  mix is not needed: the matching does not depend on it. */
int adpsgd_schedule_of(int32_t pattern, uint64_t seed, float straggler_p, int32_t L, int64_t k,
                       int32_t* order, int32_t* partner, int32_t* active);

/* Learning rate of the 1-based epoch under the schedules of the paper's experiments
 * (Section IV): constant peak_lr up to and including epoch hold_until_epoch, multiplied
 * by 1/sqrt(2) for every epoch after it; when warmup_epochs >= 2, the epochs 1 ..
 * warmup_epochs rise linearly from start_lr (epoch 1) to peak_lr (epoch warmup_epochs).
 * The single-learner baseline is (peak 0.1, no warm-up, hold 10); the 8192-segment
 * batches use (peak 3.2, start 0.32, warm-up 10, hold 10).  Computed in double, rounded
 * once to float.  out: host.  EINVAL for epoch < 1, warmup_epochs < 0 or a NULL out.   */
int adpsgd_lr_at_epoch(int32_t epoch, float peak_lr, float start_lr, int32_t warmup_epochs,
                       int32_t hold_until_epoch, float* out);

/* Iterations done so far.                                                      */
int64_t adpsgd_iteration(adpsgd_t h);

/* Output model of Algorithm 1: dev_out[P] = (1/L) sum_i x_i (fp32 sum in
 * learner order).  Asynchronous.                                               */
int adpsgd_average(adpsgd_t h, float* dev_out);

/* Consensus distance of the current models, sum_i ||x_i - xbar||^2 with xbar the
 * learner average: the quantity the mixing operators contract by their second
 * largest eigenvalue magnitude (Section II, Eq. 5-7).  Means, differences and sums
 * in fp64, fixed summation order.  Waits for the stream; host_out[0] receives the
 * value.                                                                        */
int adpsgd_consensus(adpsgd_t h, double* host_out);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the consensus distance of adpsgd_consensus without a
 * handle and without a workspace.  dev_x: device, L models of P floats each, model i at
 * dev_x + i * stride (stride >= P, in floats); dev_out: device, one double (8-byte aligned),
 * written on the stream; the call does not wait and copies nothing to the host.  Same
 * kernels, same summation order and so the same value, bit for bit, as adpsgd_consensus.
 * The per-workgroup partial sums (2048 doubles, 16 KB) live in a device array inside the
 * library, one copy per GPU, held until the process ends; the call allocates nothing
 * (no hipMalloc, no hipFree, no workspace).  Limits: 1 <= L <= 128 and L * P <=
 * ADPSGD_STATIC_MAX_ELEMENTS, otherwise ADPSGD_EINVAL.  Every call on a GPU shares that
 * GPU's array: calls that overlap in time on one GPU (different streams or threads) race
 * and must be serialised by the caller.  Runs on the current device.              */
#define ADPSGD_STATIC_MAX_ELEMENTS (((int64_t)1) << 34)
int adpsgd_consensus_static(const float* dev_x, int64_t stride, int32_t L, int64_t P, double* dev_out, void* hip_stream);

/* Per-phase GPU time of a step, taken with HIP events recorded on the handle's
 * stream at every change of phase (no host synchronisation inside the step).
 * Phases: 0 minibatch staging + bf16 weight copy, 1 time-batched GEMMs,
 * 2 recurrent forward steps, 3 recurrent backward steps, 4 softmax
 * cross-entropy, 5 bias-gradient column sums, 6 mixing + update.
 * adpsgd_profile waits for the stream, reports the totals over all steps since
 * profiling was switched on or last read, and starts a new total:
 * host_ms[7] GPU milliseconds, host_launches[7] kernel launches, host_work[7]
 * algorithmic work (flops 2*M*N*K summed for phases 1-3; bytes, 12 per active
 * learner and element (14 when the bf16 copy of the model is written along), for
 * phase 6; 0 elsewhere), host_bytes[7] algorithmic HBM bytes of phases 1-3 and 6
 * (every operand and result counted once per launch).  Any pointer may be NULL.
 * Each change of phase costs one HIP event; they are kept until destroy.        */
#define ADPSGD_PHASES 7
int adpsgd_set_profiling(adpsgd_t h, int enable);
int adpsgd_profile(adpsgd_t h, float* host_ms, int32_t* host_launches, double* host_work, double* host_bytes);

/* Release the handle (host memory only; the workspace stays the caller's).     */
void adpsgd_destroy(adpsgd_t h);

/* Text of the calling thread's last error ("" if none).                        */
const char* adpsgd_last_error(void);

/* ---- single kernels exposed for unit tests and micro-benchmarks ------------ */

/* C[g] = A[g] * B[g]' (+ bias) on MFMA for g = 0..groups-1 (the GEMMs of the
 * LSTM gradient).  Element type: fp32 (precision 0) or bf16 (precision 1) for A
 * and B; C is fp32, or the element type when c_is_elem != 0.
 *   a_kmajor != 0: A is [M][K] (row stride lda); else A is stored [K][M].
 *   b_kmajor != 0: B is [N][K] (row stride ldb); else B is stored [K][N].
 * bias (fp32 [N], or NULL) is added to every row.  Strides are in elements.
 * All pointers: device.  M, N, K >= 1; groups in 1..128; lda, ldb and the group
 * strides must be multiples of 4.  tile_config: -1 = automatic choice, or one of the
 * tile configurations 0, 5, 11, 12, 13 of csrc/gemm.hip (a configuration whose
 * alignment rules the operands do not meet falls back to one that fits).        */
int adpsgd_gemm(int precision, int a_kmajor, int b_kmajor, int c_is_elem,
                int M, int N, int K,
                const void* A, int64_t lda, int64_t strideA,
                const void* B, int64_t ldb, int64_t strideB,
                void* C, int64_t ldc, int64_t strideC,
                const float* bias, int64_t strideBias,
                int groups, int tile_config, void* hip_stream);

/* Measurement probes: what the device attains on the two resources the kernels are bound by, for the
 * benchmark to set kernel rates against an attained peak besides the published one.
 * adpsgd_probe_mfma: a register-only loop of the bf16 MFMA instruction of the GEMM kernels; blocks workgroups
 *   of 4 waves, iters x 8 instructions (32x32x16: 32768 flops each) per wave; dev_out: device, blocks * 256
 *   floats (written once at the end).
 * adpsgd_probe_stream: one streaming pass over elems positions with reads fp32 read streams, writes_f32 fp32
 *   and writes_bf16 bf16 write streams per position (1:0:0 read only, 1:1:0 copy, 2:1:0 the pairwise update's
 *   mix, 2:1:1 the update that also writes the bf16 model copy; 4:2:0, 4:2:2, 8:4:4, 16:8:8, 32:16:16 the same
 *   mixes with the streams of 2 .. 16 learners owned by one thread, as in the update kernels, whose rate
 *   falls with the number of streams a thread walks at once); the streams are consecutive slices of
 *   dev_buf, pitch_bytes apart (dev_buf: device, 16-byte aligned, (reads + writes) * pitch_bytes long; its
 *   contents are overwritten).  Both are asynchronous on hip_stream; EINVAL for anything else.             */
int adpsgd_probe_mfma(float* dev_out, int blocks, int iters, void* hip_stream);
int adpsgd_probe_stream(int reads, int writes_f32, int writes_bf16, void* dev_buf, int64_t pitch_bytes,
                        int64_t elems, void* hip_stream);

/* Tuning of ONE handle (benchmarks and tests; the defaults are the measured best):
 *   ADPSGD_TUNE_GEMM_TILE        tile configuration of the time-batched GEMMs, as tile_config above
 *   ADPSGD_TUNE_REC_DIRECT       1 (default) / 0: specialised recurrent step kernels (direct-to-LDS loads for bf16 and
 *                                batches over 32; contraction split over the waves for batches up to 32) allowed, or
 *                                the general register-staged kernels everywhere
 *   ADPSGD_TUNE_REC_FWD_GROUPS   learner groups the forward recurrence is run in, 0 = automatic
 *   ADPSGD_TUNE_REC_PERSISTENT   persistent recurrent kernels (all frames of a layer in one launch, W_h held in
 *                                registers; bf16 operands, hidden 128/256/512/1024, batch <= 128): 1 on where the
 *                                shape allows, 0 off, -1 (default) automatic
 *   ADPSGD_TUNE_REC_WAIT_US      bound, in microseconds, of one wait between the workgroups of a persistent
 *                                kernel (default 2 000 000); when it runs out every workgroup returns and the
 *                                handle's sticky error becomes ADPSGD_EHIP
 * Takes effect from the next adpsgd_step of that handle; other handles are not touched. */
#define ADPSGD_TUNE_GEMM_TILE       0
#define ADPSGD_TUNE_REC_DIRECT      1
#define ADPSGD_TUNE_REC_FWD_GROUPS  2
#define ADPSGD_TUNE_REC_PERSISTENT  3
#define ADPSGD_TUNE_REC_WAIT_US     4
#define ADPSGD_TUNE_MEAN_CHUNK      5   /* global-mean update: elements per chunk of its two-kernel form (a multiple of
                                           1024, at most 16777216), 0 = the single-kernel form, -1 (default) = automatic
                                           (two kernels from 4M parameters on); same results bit for bit */
#define ADPSGD_TUNE_TRI_SEGMENT     6   /* ring-neighbour update (ADPSGD_MIX_TRI): ring positions one thread owns, 1, 2, 4 or 8
                                           (a workgroup then covers the ring of its element positions and the update stays
                                           safe in place), 0 = one thread walks the whole ring, -1 = default; same results
                                           bit for bit */
#define ADPSGD_TUNE_PAIR_SPLIT      7   /* pairwise update: 64 or 128 = one member of a pair per thread, in workgroups of that
                                           many element positions x 2 members (the partner's model comes through LDS), 0 =
                                           both members per thread, -1 = default (64 from 1M parameters on); same results
                                           bit for bit */
#define ADPSGD_TUNE_SYNC_SEGMENT    8   /* update of the synchronous baseline (ADPSGD_SDPSGD): learners one thread owns, 2, 4 or
                                           8 (the sum then runs through the segments of a workgroup in learner order), 0 =
                                           all learners of a position in one thread, -1 = default; same results bit for bit */
int adpsgd_set_tuning(adpsgd_t h, int key, int value);

#ifdef __cplusplus
}
#endif
#endif /* ADPSGD_H */
