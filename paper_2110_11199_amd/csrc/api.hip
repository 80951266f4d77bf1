// C ABI of the ADPSGD library: configuration checks, workspace carving, the
// host-side integer schedule and the orchestration of one iteration.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <stdexcept>
#include <string>
#include <vector>
#include "../../include/adpsgd.h"
#include "kernels.hpp"

using namespace adpsgd;

namespace {

thread_local std::string g_err;

int fail(int code, const std::string& msg) { g_err = msg; return code; }
int hipfail(hipError_t e, const char* what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return ADPSGD_EHIP;
}
#define HIPCHK(call, what) do { hipError_t e_ = (call); if (e_ != hipSuccess) return hipfail(e_, what); } while (0)

// ---- counter-based generator of the schedule -----------------------------------
// u64(seed, stream, k, idx) = mix(mix(mix(seed + GOLDEN*(stream+1)) + k) + idx), mix = the
// SplitMix64 output function.  Streams: 1 ring permutation, 2 straggler mask, 3 initial model.
const uint64_t kGolden = 0x9E3779B97F4A7C15ull;
enum { kStreamPerm = 1, kStreamMask = 2, kStreamInit = 3 };

inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
inline uint64_t draw(uint64_t seed, uint64_t stream, uint64_t k, uint64_t idx) {
    return mix64(mix64(mix64(seed + kGolden * (stream + 1)) + k) + idx);
}
inline double draw01(uint64_t seed, uint64_t stream, uint64_t k, uint64_t idx) {
    return (double)(draw(seed, stream, k, idx) >> 11) * (1.0 / 9007199254740992.0);
}

// Ring order (identity, or a Fisher-Yates shuffle per iteration for the random
// ring, Section III-C), straggler mask, and the matching along the ring order
// whose phase alternates with k on a fixed order.
void make_schedule(int pattern, uint64_t seed, float straggler_p, int L, int64_t k,
                   int32_t* order, int32_t* partner, int32_t* active) {
    for (int i = 0; i < L; ++i) order[i] = i;
    if (pattern == ADPSGD_RANDOM_RING) {
        for (int p = L - 1; p >= 1; --p) {
            const int q = (int)(draw(seed, kStreamPerm, (uint64_t)k, (uint64_t)p) % (uint64_t)(p + 1));
            const int32_t tmp = order[p]; order[p] = order[q]; order[q] = tmp;
        }
    }
    for (int i = 0; i < L; ++i) {
        active[i] = 1;
        if (straggler_p > 0.f && draw01(seed, kStreamMask, (uint64_t)k, (uint64_t)i) < (double)straggler_p) active[i] = 0;
        partner[i] = i;
    }
    const int phase = pattern == ADPSGD_RANDOM_RING ? 0 : (int)(k & 1);
    for (int m = 0; m < L / 2; ++m) {
        const int a = order[(2 * m + phase) % L], b = order[(2 * m + 1 + phase) % L];
        if (a != b) { partner[a] = b; partner[b] = a; }
    }
    for (int i = 0; i < L; ++i) {
        if (!active[i]) { const int j = partner[i]; partner[j] = j; partner[i] = i; }
    }
}

struct Tensor { int64_t off, rows, cols; };

struct Carver {
    char* base; size_t used;
    explicit Carver(void* b) : base((char*)b), used(0) {}
    void* take(size_t bytes) {
        void* p = base ? base + used : nullptr;
        used += (size_t)round_up((int64_t)bytes, 256);
        return p;
    }
};

}  // namespace

// Chunk of the parameter index the two-kernel global mean works on at a time (elements; the buffer holds the maximum)
constexpr int64_t kMeanChunkMax = 16 << 20, kMeanChunkDefault = 4 << 20;   // measured best on 16 x 145M: 2M .. 6M within 3 %

struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;        // ev[j] opens segment j; ev[j+1] closes it
    std::vector<int> seg_phase;
    int cur = -1;
    int launches[ADPSGD_PHASES];
    double work[ADPSGD_PHASES];
    double bytes[ADPSGD_PHASES];      // algorithmic HBM bytes (each operand and result once)
};

struct adpsgd_graph;

struct adpsgd_handle {
    Profiler prof;
    adpsgd_config cfg;
    hipStream_t stream;
    // tuning (adpsgd_set_tuning): per handle, so that two handles of a process cannot interfere
    int tune_gemm_tile = -1;               // forced GEMM tile configuration, -1 = automatic
    int tune_rec_direct = 1;               // direct-to-LDS recurrent kernels allowed
    int tune_rec_fwd_groups = 0;           // learner groups of the forward recurrence, 0 = automatic
    int tune_rec_persist = -1;             // persistent recurrent kernels: 0 off, 1 on where the shape allows, -1 automatic
    int64_t tune_wait_us = 2000000;        // bound of one wait between the workgroups of a persistent kernel
    int cu_count = 0;                      // compute units of the device (a persistent grid must not exceed it)
    uint32_t* rec_counters = nullptr;      // [layers][2 passes][L * D] frame counters of the persistent kernels
    float* mean_buf = nullptr;             // chunk buffer of the two-kernel global mean (mix ALL)
    int64_t mean_cap = 0;                  // its size in elements: min(kMeanChunkMax, P rounded up to 1024)
    int64_t tune_mean_chunk = -1;          // elements per chunk; 0: the single-kernel global mean; -1: automatic
    int tune_pair_split = -1;              // pairwise update: one member of a pair per thread (positions per workgroup), 0 off, -1 default
    int tune_sync_segment = -1;            // synchronous baseline: learners per thread of the update (0: all of them), -1: default
    int tune_tri_segment = -1;             // ring-neighbour update: ring positions per thread (0: the whole ring), -1: default
    // device status word (kStatus* bits, sticky) and its pinned host mirror, refreshed by an asynchronous
    // copy at the end of every step
    uint32_t* status = nullptr;
    volatile uint32_t* status_host = nullptr;
    int L, D, H, T, B, I, C, Bn, layers, F, ldx;
    int mix, tau, prec, esz;
    bool flat;
    int64_t P, Ppad, M;
    int64_t k;
    int cur;                               // index of the buffer holding x^k
    bool shadow_valid;                     // the bf16 copy already holds the next gradient point
    // iterations being recorded into a HIP graph (adpsgd_capture_begin .. adpsgd_capture_end): nothing runs, and the
    // host-side state of the handle is put back to these values when the recording ends
    std::vector<struct adpsgd_graph*> graphs;   // recordings made on this handle that are still alive
    bool capturing = false;
    int64_t capture_k0 = 0;
    int capture_cur0 = 0;
    std::vector<Tensor> tensors;           // flat layout
    std::vector<int> ix_wx, ix_wh, ix_b;   // tensor index per layer
    int ix_wp, ix_bp, ix_wo, ix_bo;
    // workspace regions
    float* params[2];
    double* consensus;  // scratch of adpsgd_consensus
    float* grads;
    float* dbp;        // [L][T * batch tiles][D*4H]: per-frame column sums of da (partial bias gradients)
    bf16_t* wx0p;      // [L][D*4H][ldx] bf16: W_x of layer 0 with zero-padded rows, or NULL
    bf16_t* shadow;
    void* x0; int32_t* labels;
    void* ybuf;        // [layers][L][M][D*H]
    float* gates;      // [layers][L][M][D*4H]
    float* cbuf;       // [layers][L][D][M][H]
    void* z; void* dz; float* logits; void* dlogits; float* dy; void* da; float* dc;
    float* row_loss; float* loss;
};

// A recorded sequence of iterations of one handle (adpsgd_capture_end), replayed by adpsgd_graph_replay.
struct adpsgd_graph {
    adpsgd_t owner;
    hipGraph_t graph;
    hipGraphExec_t exec;
    int64_t steps;                         // iterations recorded
    int64_t k0;                            // iteration number of the first one (its parity must match at replay)
};

namespace {

// Number of learner groups the forward recurrence of n learners is run in (see compute_gradients).
int rec_forward_parts(const adpsgd_handle* h, int n) {
    if (h->tune_rec_fwd_groups > 0) return h->tune_rec_fwd_groups < n ? h->tune_rec_fwd_groups : n;
    const double per_step = (double)n * h->D * (4.0 * h->H * h->H * h->esz + (double)h->B * h->H * (2 * h->esz + 8 * 4 + 2 * 4));
    const double cache = 256e6;
    // workgroups of one launch: (learner, direction) x 32-unit slices x 128-row batch tiles
    const int64_t wgs = (int64_t)n * h->D * ((h->H + 31) / 32) * ((h->B + 127) / 128);
    if (per_step <= cache) return 1;
    // the fewest groups whose step fits the cache, as long as a group's launch still fills the chip twice over
    for (int parts = 2; parts <= n && wgs / parts >= 512; ++parts)
        if (per_step / parts <= cache) return parts;
    return 1;
}

// Pairs (learner, direction) one persistent launch takes: one workgroup of 32 units per compute unit at most.
int persist_cap(const adpsgd_handle* h) {
    int cap = h->cu_count / (h->H / 32);
    if (cap > 64) cap = 64;
    if (cap >= 8) cap -= cap % 8;
    return cap < 1 ? 1 : cap;
}

// Whether the recurrences of this handle run on the persistent kernels (all frames of a layer in one launch,
// W_h resident in registers) instead of one launch per frame.
bool use_persistent(const adpsgd_handle* h) {
    if (h->flat || h->tune_rec_persist == 0 || h->cu_count < 1) return false;
    RecDesc r{};
    r.precision = h->prec; r.D = h->D; r.B = h->B; r.H = h->H; r.T = h->T;
    // the alignment of the tensors follows from the layout: 256-byte aligned regions, strides that are multiples of 64
    if (!rec_persist_supported(r, h->cu_count)) return false;
    if (h->tune_rec_persist == 1) return true;
    return false;       // automatic: off
}

// Turns the status bits a kernel has raised (as last copied to the host) into an error.
int status_error(const adpsgd_handle* h) {
    const uint32_t st = h->status_host ? *h->status_host : 0u;
    if (st & kStatusWaitExpired)
        return fail(ADPSGD_EHIP, "a bounded wait between the workgroups of a persistent recurrent kernel ran out in an earlier "
                                 "step; the results of this handle are not valid");
    if (st & kStatusBadLabel)
        return fail(ADPSGD_EINVAL, "a label outside [0, classes) was met in an earlier step (it was clamped); the models of "
                                   "this handle have taken an update from it");
    return ADPSGD_OK;
}

bool all_by_default(int pattern) { return pattern == ADPSGD_D1D || pattern == ADPSGD_SDPSGD; }
bool is_hybrid(int mix) { return mix == ADPSGD_MIX_HYBRID_PAIR || mix == ADPSGD_MIX_HYBRID_TRI; }

int check_config(const adpsgd_config* c, std::string& why) {
    if (!c) { why = "config is NULL"; return ADPSGD_EINVAL; }
    if (c->L < 1 || c->L > ADPSGD_MAX_LEARNERS) { why = "L must be in 1..128"; return ADPSGD_EINVAL; }
    if (c->pattern < 0 || c->pattern > 3) { why = "unknown pattern"; return ADPSGD_EINVAL; }
    if (c->mix < ADPSGD_MIX_DEFAULT || c->mix > ADPSGD_MIX_HYBRID_TRI) { why = "unknown mix"; return ADPSGD_EINVAL; }
    if (c->tau < -1 || c->tau > 1) { why = "tau must be 0, 1 or -1"; return ADPSGD_EINVAL; }
    if (c->precision != ADPSGD_FP32 && c->precision != ADPSGD_BF16_GEMM) { why = "unknown precision"; return ADPSGD_EINVAL; }
    if (!(c->straggler_p >= 0.f && c->straggler_p < 1.f)) { why = "straggler_p must be in [0,1)"; return ADPSGD_EINVAL; }
    const int tau = c->tau >= 0 ? c->tau : (c->pattern == ADPSGD_D1D ? 1 : 0);
    const int mix = c->mix != ADPSGD_MIX_DEFAULT ? c->mix : (all_by_default(c->pattern) ? ADPSGD_MIX_ALL : ADPSGD_MIX_PAIR);
    if (is_hybrid(mix)) {
        const int S = c->group_size;
        if (S < 1 || c->L % S != 0) { why = "hybrid mixing: L must be a multiple of group_size >= 1"; return ADPSGD_EINVAL; }
        if (c->pattern != ADPSGD_FIXED_RING && c->pattern != ADPSGD_RANDOM_RING) {
            why = "hybrid mixing joins the super-learners by a ring: fixed or random ring pattern only"; return ADPSGD_EINVAL;
        }
        if (c->straggler_p > 0.f) { why = "hybrid mixing takes no stragglers (a super-learner waits for its members)"; return ADPSGD_EINVAL; }
        const int G = c->L / S;
        if (mix == ADPSGD_MIX_HYBRID_TRI && G == 2) {
            why = "ring-neighbour mixing across super-learners needs at least 3 of them (or a single one)"; return ADPSGD_EINVAL;
        }
    } else if (c->group_size != 0 && c->group_size != 1) {
        why = "group_size is for the hybrid mixes only"; return ADPSGD_EINVAL;
    }
    if (mix == ADPSGD_MIX_TRI && c->L < 3) {
        why = "ring-neighbour mixing (weights 1/3, Eq. 9) needs at least 3 learners"; return ADPSGD_EINVAL;
    }
    if (c->pattern == ADPSGD_SDPSGD && (mix != ADPSGD_MIX_ALL || tau != 0 || c->straggler_p > 0.f)) {
        why = "the synchronous baseline averages all learners (mix ALL), with tau = 0 and no stragglers";
        return ADPSGD_EINVAL;
    }
    if (c->straggler_p > 0.f && (c->pattern == ADPSGD_D1D || tau != 0 || mix != ADPSGD_MIX_PAIR)) {
        why = "stragglers need a ring pattern with pairwise mixing and tau = 0 (delay-by-one waits for every learner)";
        return ADPSGD_EINVAL;
    }
    if (!(c->init_scale >= 0.f)) { why = "init_scale must be >= 0"; return ADPSGD_EINVAL; }
    const adpsgd_model_shape& s = c->shape;
    if (s.flat_params > 0) return ADPSGD_OK;
    if (s.flat_params < 0) { why = "flat_params < 0"; return ADPSGD_EINVAL; }
    if (s.input_dim < 4 || s.hidden < 4 || s.classes < 4 || s.layers < 1 || s.batch < 1 || s.frames < 1 || s.bottleneck < 0) {
        why = "model shape out of range"; return ADPSGD_EINVAL;
    }
    if (s.input_dim % 4 || s.hidden % 4 || s.classes % 4 || s.bottleneck % 4) {
        why = "input_dim, hidden, bottleneck and classes must be multiples of 4"; return ADPSGD_EINVAL;
    }
    if (s.bidirectional != 0 && s.bidirectional != 1) { why = "bidirectional must be 0 or 1"; return ADPSGD_EINVAL; }
    return ADPSGD_OK;
}

// Fills the derived fields and the layout; carves the workspace when base != NULL.
size_t plan(adpsgd_handle* h, void* base) {
    const adpsgd_config& c = h->cfg;
    const adpsgd_model_shape& s = c.shape;
    h->L = c.L;
    h->tau = c.tau >= 0 ? c.tau : (c.pattern == ADPSGD_D1D ? 1 : 0);
    h->mix = c.mix != ADPSGD_MIX_DEFAULT ? c.mix : (all_by_default(c.pattern) ? ADPSGD_MIX_ALL : ADPSGD_MIX_PAIR);
    h->prec = c.precision; h->esz = c.precision ? 2 : 4;
    h->flat = s.flat_params > 0;
    h->tensors.clear(); h->ix_wx.clear(); h->ix_wh.clear(); h->ix_b.clear();
    h->ix_wp = h->ix_bp = h->ix_wo = h->ix_bo = -1;
    if (h->flat) {
        h->P = s.flat_params;
        h->D = h->H = h->T = h->B = h->I = h->C = h->Bn = h->layers = h->F = h->ldx = 0; h->M = 0;
    } else {
        h->D = s.bidirectional ? 2 : 1; h->H = s.hidden; h->T = s.frames; h->B = s.batch; h->I = s.input_dim;
        h->C = s.classes; h->Bn = s.bottleneck; h->layers = s.layers; h->M = (int64_t)h->T * h->B;
        // staged input rows: whole 16-byte chunks; whole 64-element K stages for the direct-to-LDS GEMM (bf16)
        h->ldx = (int)round_up(h->I, c.precision ? 64 : 8);
        int64_t off = 0;
        const int64_t G4 = (int64_t)h->D * 4 * h->H;
        for (int l = 0; l < h->layers; ++l) {
            const int64_t Il = l == 0 ? h->I : (int64_t)h->D * h->H;
            h->ix_wx.push_back((int)h->tensors.size()); h->tensors.push_back({off, G4, Il}); off += G4 * Il;
            h->ix_wh.push_back((int)h->tensors.size()); h->tensors.push_back({off, G4, h->H}); off += G4 * h->H;
            h->ix_b.push_back((int)h->tensors.size()); h->tensors.push_back({off, 1, G4}); off += G4;
        }
        int64_t F = (int64_t)h->D * h->H;
        if (h->Bn > 0) {
            h->ix_wp = (int)h->tensors.size(); h->tensors.push_back({off, h->Bn, F}); off += h->Bn * F;
            h->ix_bp = (int)h->tensors.size(); h->tensors.push_back({off, 1, h->Bn}); off += h->Bn;
            F = h->Bn;
        }
        h->F = (int)F;
        h->ix_wo = (int)h->tensors.size(); h->tensors.push_back({off, h->C, F}); off += h->C * F;
        h->ix_bo = (int)h->tensors.size(); h->tensors.push_back({off, 1, h->C}); off += h->C;
        h->P = off;
    }
    h->Ppad = round_up(h->P, 64);
    Carver w(base);
    const size_t L = (size_t)h->L;
    h->params[0] = (float*)w.take(L * h->Ppad * 4);
    h->params[1] = h->tau == 1 ? (float*)w.take(L * h->Ppad * 4) : h->params[0];
    h->consensus = (double*)w.take((size_t)(kConsensusBlocks + 1) * 8);     // partial sums + the result
    h->status = (uint32_t*)w.take(256);
    h->mean_cap = round_up(h->P, 1024) < kMeanChunkMax ? round_up(h->P, 1024) : kMeanChunkMax;
    h->mean_buf = h->mix == ADPSGD_MIX_ALL ? (float*)w.take((size_t)h->mean_cap * 4) : nullptr;
    if (s.flat_params == 0) h->rec_counters = (uint32_t*)w.take((size_t)s.layers * 2 * c.L * 2 * 4);
    if (!h->flat) {
        const size_t M = (size_t)h->M, DH = (size_t)h->D * h->H, G4 = DH * 4, e = (size_t)h->esz;
        h->grads = (float*)w.take(L * h->Ppad * 4);
        h->shadow = h->prec ? (bf16_t*)w.take(L * h->Ppad * 2) : nullptr;
        h->x0 = w.take(L * M * h->ldx * e);
        // bf16 W_x of layer 0 with its rows zero-padded to ldx (when the input width is not a multiple of 64)
        h->wx0p = (h->prec && h->ldx != h->I) ? (bf16_t*)w.take(L * G4 * h->ldx * 2) : nullptr;
        h->labels = (int32_t*)w.take(L * M * 4);
        h->ybuf = w.take((size_t)h->layers * L * M * DH * e);
        h->gates = (float*)w.take((size_t)h->layers * L * M * G4 * 4);
        h->cbuf = (float*)w.take((size_t)h->layers * L * M * DH * 4);
        h->z = h->Bn ? w.take(L * M * h->Bn * e) : nullptr;
        h->dz = h->Bn ? w.take(L * M * h->Bn * e) : nullptr;
        h->logits = (float*)w.take(L * M * h->C * 4);
        h->dlogits = w.take(L * M * h->C * e);
        h->dy = (float*)w.take(L * M * DH * 4);
        h->da = w.take(L * M * G4 * e);
        h->dc = (float*)w.take(L * (size_t)h->B * DH * 4);
        h->dbp = (float*)w.take(L * (size_t)h->T * rec_backward_batch_tiles(h->B) * G4 * 4);
        h->row_loss = (float*)w.take(L * M * 4);
        h->loss = (float*)w.take(L * 4);
    }
    return w.used;
}

// Marks the start of work belonging to `phase` (-1: end of the step).
int mark(adpsgd_handle* h, int phase, int launches = 0, double work = 0.0, double bytes = 0.0) {
    Profiler& p = h->prof;
    if (!p.on) return ADPSGD_OK;
    if (phase >= 0) { p.launches[phase] += launches; p.work[phase] += work; p.bytes[phase] += bytes; }
    if (phase == p.cur) return ADPSGD_OK;
    const size_t need = p.seg_phase.size() + 1;     // events recorded so far + this one
    while (p.ev.size() < need) {
        hipEvent_t e;
        HIPCHK(hipEventCreate(&e), "event create");
        p.ev.push_back(e);
    }
    HIPCHK(hipEventRecord(p.ev[need - 1], h->stream), "event record");
    p.seg_phase.push_back(phase);                    // phase of the segment this event opens
    p.cur = phase;
    return ADPSGD_OK;
}

void prof_reset(adpsgd_handle* h) {
    Profiler& p = h->prof;
    p.seg_phase.clear(); p.cur = -1;
    for (int i = 0; i < ADPSGD_PHASES; ++i) { p.launches[i] = 0; p.work[i] = 0.0; p.bytes[i] = 0.0; }
}

// k_alg: the contraction length the flop and byte counts are taken for (0: d.K; smaller than d.K when
// the operands carry zero padding along K)
int gemm(adpsgd_handle* h, const GemmDesc& d, const char* what, int k_alg = 0) {
    const double esz = d.precision ? 2.0 : 4.0, g = (double)d.groupsI * d.groupsD;
    const double K = k_alg > 0 ? k_alg : d.K;
    if (int rc = mark(h, 1, 1, 2.0 * d.M * d.N * K * g,
                      g * (((double)d.M + d.N) * K * esz + (double)d.M * d.N * (d.c_elem ? esz : 4.0)))) return rc;
    GemmDesc q = d;
    q.tile = h->tune_gemm_tile;
    HIPCHK(launch_gemm(q, h->stream), what);
    return ADPSGD_OK;
}

// Gradient of every active learner's minibatch loss at the models in `at` (A1-A8).  A straggler
// (active[i] == 0) computes nothing: it is left out of every launch, its loss is reported as 0 and its
// slot of the gradient buffer keeps whatever it held.
int compute_gradients(adpsgd_handle* h, const float* at, const void* const* batch_ptrs, const int32_t* active) {
    const int L = h->L, D = h->D, H = h->H, T = h->T, B = h->B, prec = h->prec;
    const int64_t M = h->M, DH = (int64_t)D * H, G4 = DH * 4, Pp = h->Ppad;
    const int esz = h->esz;
    hipStream_t s = h->stream;
    LearnerMap act, ident;
    ident.identity(); act.identity();
    int n = 0;
    uint32_t bits[4] = {0, 0, 0, 0};
    for (int i = 0; i < L; ++i)
        if (active[i]) { act.idx[n++] = (uint8_t)i; bits[i >> 5] |= 1u << (i & 31); }
    if (n == 0) {
        if (int rc = mark(h, 4, 1)) return rc;
        HIPCHK(launch_zero(h->loss, 0, L, 1, ident, s), "zero losses");
        return ADPSGD_OK;
    }
    // weights as GEMM operands: the fp32 models themselves, or their bf16 copy
    const char* wbase = (const char*)at;
    const bool persist = use_persistent(h);
    if (int rc = mark(h, 0, (prec ? (h->wx0p ? 3 : 2) : 1) + (persist ? 1 : 0))) return rc;
    if (persist)     // frame counters of the persistent kernels start from zero (a fill kernel, not a memset node)
        HIPCHK(launch_zero((float*)h->rec_counters, 0, (int64_t)h->layers * 2 * L * 2, 1, ident, s), "zero frame counters");
    // the (learner, direction) pairs of the active learners, in the order the persistent launches take them
    uint8_t pair_l[256], pair_d[256];
    int npairs = 0;
    for (int j = 0; j < n; ++j)
        for (int dd = 0; dd < D; ++dd) { pair_l[npairs] = act.idx[j]; pair_d[npairs] = (uint8_t)dd; ++npairs; }
    // all T frames of layer l for every pair: as many pairs per launch as fit one workgroup per compute unit
    auto run_persistent = [&](const RecDesc& r, int l, bool backward) -> int {
        const int per_pair = H / 32;
        int cap = h->cu_count / per_pair;
        if (cap > 64) cap = 64;
        if (cap >= 8) cap -= cap % 8;            // whole pairs per XCD (workgroup ids go round-robin over the 8 XCDs)
        for (int p0 = 0; p0 < npairs; p0 += cap) {
            PersistDesc pd;
            pd.r = r;
            pd.ngl = npairs - p0 < cap ? npairs - p0 : cap;
            for (int j = 0; j < 64; ++j) { pd.gl_learner[j] = j < pd.ngl ? pair_l[p0 + j] : 0; pd.gl_dir[j] = j < pd.ngl ? pair_d[p0 + j] : 0; }
            pd.counters = h->rec_counters + ((size_t)(l * 2 + (backward ? 1 : 0)) * L * 2 + p0);
            pd.status = h->status;
            pd.wait_ticks = (unsigned long long)h->tune_wait_us * 100ull;
            HIPCHK(launch_rec_persist(pd, backward, h->cu_count, s), backward ? "persistent recurrent backward" : "persistent recurrent forward");
        }
        return ADPSGD_OK;
    };
    const int persist_launches = persist ? (npairs + persist_cap(h) - 1) / persist_cap(h) : 0;
    if (prec) {
        // the update of the previous iteration has normally written this copy already
        if (!h->shadow_valid) HIPCHK(launch_cast_bf16(at, h->shadow, (int64_t)L * Pp, s), "cast weights to bf16");
        wbase = (const char*)h->shadow;
        if (h->wx0p)
            HIPCHK(launch_pad_rows_bf16(at + h->tensors[h->ix_wx[0]].off, Pp, h->wx0p, (int64_t)G4 * h->ldx, G4, h->I, h->ldx,
                                        L, s), "pad W_x of layer 0");
    }
    auto W = [&](int ix) { return (const void*)(wbase + h->tensors[ix].off * esz); };
    auto Bias = [&](int ix) { return at + h->tensors[ix].off; };
    auto Gr = [&](int ix) { return h->grads + h->tensors[ix].off; };

    StageDesc st;
    st.L = n; st.lmap = act; st.precision = prec; st.rows = M; st.I = h->I; st.ldx = h->ldx;
    st.x0 = h->x0; st.sX0 = M * h->ldx; st.y = h->labels; st.sY = M;
    for (int i = 0; i < 128; ++i) {
        st.feats[i] = i < L ? (const float*)batch_ptrs[2 * i] : nullptr;
        st.labels[i] = i < L ? (const int32_t*)batch_ptrs[2 * i + 1] : nullptr;
    }
    HIPCHK(launch_stage(st, s), "stage minibatches");

    auto Y = [&](int l) { return (void*)((char*)h->ybuf + (size_t)l * L * M * DH * esz); };
    auto Gates = [&](int l) { return h->gates + (size_t)l * L * M * G4; };
    auto Cb = [&](int l) { return h->cbuf + (size_t)l * L * M * DH; };
    // a GEMM over the active learners, one group per learner (and direction)
    auto G = [&]() { GemmDesc g{}; g.precision = prec; g.groupsI = n; g.groupsD = 1; g.lmap = act; return g; };

    GemmDesc g;
    // ---- forward ----
    for (int l = 0; l < h->layers; ++l) {
        const int64_t Il = l == 0 ? h->I : DH;
        g = G();
        g.a_kc = 1; g.b_kc = 1; g.c_elem = 0;
        g.M = (int)M; g.N = (int)G4; g.K = (int)Il;
        g.A = l == 0 ? h->x0 : Y(l - 1); g.lda = l == 0 ? h->ldx : DH; g.sAi = M * g.lda;
        g.B = W(h->ix_wx[l]); g.ldb = Il; g.sBi = Pp;
        if (l == 0 && h->wx0p) {     // zero-padded K: the staged input and this copy of W_x share the row length ldx
            g.K = h->ldx; g.B = h->wx0p; g.ldb = h->ldx; g.sBi = G4 * h->ldx;
        }
        g.C = Gates(l); g.ldc = G4; g.sCi = M * G4;
        g.bias = Bias(h->ix_b[l]); g.sBiasI = Pp;
        if (int rc = gemm(h, g, "input projection GEMM", (int)Il)) return rc;
        RecDesc r{};
        r.precision = prec; r.L = n; r.lmap = act; r.direct = h->tune_rec_direct; r.D = D; r.B = B; r.H = H; r.T = T;
        r.gates = Gates(l); r.sGi = M * G4;
        r.c = Cb(l); r.sCi = M * DH;
        r.y = Y(l); r.sYi = M * DH;
        r.wh = W(h->ix_wh[l]); r.sWi = Pp; r.sWd = (int64_t)4 * H * H;
        // Learners in groups, all T steps of a group before the next group: a step re-reads W_h of its learners,
        // and a group whose per-step traffic fits the 256 MB memory-side cache finds it there (measured on the
        // 16 x 1024-unit workload: 10.7 -> 8.9 ms per iteration in two groups; three or four groups leave too
        // few workgroups per launch and are slower than one).
        const int parts = rec_forward_parts(h, n);
        if (persist) {
            // per (learner, direction): W_h once; per frame: pre-activations in, gates, c and h out, h in
            if (int rc = mark(h, 2, persist_launches, 2.0 * B * H * 4 * H * (T - 1) * n * D,
                              (double)n * D * (4.0 * H * H * esz + (double)T * B * H * (2 * esz + 16 + 16 + 4)))) return rc;
            if (int rc = run_persistent(r, l, false)) return rc;
            continue;
        }
        // per frame and (learner, direction): W_h once, h in and out, 4 gates in and out (fp32), c in and out
        if (int rc = mark(h, 2, T * parts, 2.0 * B * H * 4 * H * (T - 1) * n * D,
                          (double)T * n * D * (4.0 * H * H * esz + (double)B * H * (2 * esz + 8 * 4 + 2 * 4)))) return rc;
        for (int part = 0; part < parts; ++part) {
            const int per = n / parts, l0 = part * per;
            RecDesc q = r;
            q.L = part == parts - 1 ? n - l0 : per;
            for (int j = 0; j < q.L; ++j) q.lmap.idx[j] = act.idx[l0 + j];
            for (int t = 0; t < T; ++t) {
                q.step = t;
                HIPCHK(launch_rec_forward(q, s), "recurrent forward step");
            }
        }
    }
    const void* top = Y(h->layers - 1);
    const void* zin = top; int64_t ldz = DH;
    if (h->Bn) {
        g = G();
        g.a_kc = 1; g.b_kc = 1; g.c_elem = 1;
        g.M = (int)M; g.N = h->Bn; g.K = (int)DH;
        g.A = top; g.lda = DH; g.sAi = M * DH;
        g.B = W(h->ix_wp); g.ldb = DH; g.sBi = Pp;
        g.C = h->z; g.ldc = h->Bn; g.sCi = M * h->Bn;
        g.bias = Bias(h->ix_bp); g.sBiasI = Pp;
        if (int rc = gemm(h, g, "bottleneck GEMM")) return rc;
        zin = h->z; ldz = h->Bn;
    }
    const int F = h->F, C = h->C;
    g = G();
    g.a_kc = 1; g.b_kc = 1; g.c_elem = 0;
    g.M = (int)M; g.N = C; g.K = F;
    g.A = zin; g.lda = ldz; g.sAi = M * ldz;
    g.B = W(h->ix_wo); g.ldb = F; g.sBi = Pp;
    g.C = h->logits; g.ldc = C; g.sCi = M * C;
    g.bias = Bias(h->ix_bo); g.sBiasI = Pp;
    if (int rc = gemm(h, g, "output GEMM")) return rc;

    SoftmaxDesc sm{};
    sm.precision = prec; sm.L = n; sm.lmap = act; sm.L_all = L; sm.rows = M; sm.C = C;
    for (int i = 0; i < 4; ++i) sm.active_bits[i] = bits[i];
    sm.status = h->status;
    sm.logits = h->logits; sm.sLi = M * C; sm.y = h->labels; sm.sYi = M;
    sm.dlogits = h->dlogits; sm.sDi = M * C; sm.row_loss = h->row_loss; sm.loss = h->loss;
    if (int rc = mark(h, 4, 2)) return rc;
    HIPCHK(launch_softmax_ce(sm, s), "softmax cross-entropy");

    // ---- backward: output layer(s) ----
    // dW_o = dlogits' z
    g = G();
    g.a_kc = 0; g.b_kc = 0; g.c_elem = 0;
    g.M = C; g.N = F; g.K = (int)M;
    g.A = h->dlogits; g.lda = C; g.sAi = M * C;
    g.B = zin; g.ldb = ldz; g.sBi = M * ldz;
    g.C = Gr(h->ix_wo); g.ldc = F; g.sCi = Pp;
    if (int rc = gemm(h, g, "dW_o GEMM")) return rc;
    if (int rc = mark(h, 5, 1)) return rc;
    HIPCHK(launch_colsum(prec, h->dlogits, C, M * C, M, C, Gr(h->ix_bo), Pp, n, act, s), "db_o");
    // d(z) = dlogits W_o
    g = G();
    g.a_kc = 1; g.b_kc = 0; g.c_elem = h->Bn ? 1 : 0;
    g.M = (int)M; g.N = F; g.K = C;
    g.A = h->dlogits; g.lda = C; g.sAi = M * C;
    g.B = W(h->ix_wo); g.ldb = F; g.sBi = Pp;
    g.C = h->Bn ? h->dz : (void*)h->dy; g.ldc = F; g.sCi = M * F;
    if (int rc = gemm(h, g, "dz GEMM")) return rc;
    if (h->Bn) {
        g = G();
        g.a_kc = 0; g.b_kc = 0; g.c_elem = 0;
        g.M = h->Bn; g.N = (int)DH; g.K = (int)M;
        g.A = h->dz; g.lda = h->Bn; g.sAi = M * h->Bn;
        g.B = top; g.ldb = DH; g.sBi = M * DH;
        g.C = Gr(h->ix_wp); g.ldc = DH; g.sCi = Pp;
        if (int rc = gemm(h, g, "dW_p GEMM")) return rc;
        if (int rc = mark(h, 5, 1)) return rc;
        HIPCHK(launch_colsum(prec, h->dz, h->Bn, M * h->Bn, M, h->Bn, Gr(h->ix_bp), Pp, n, act, s), "db_p");
        g = G();
        g.a_kc = 1; g.b_kc = 0; g.c_elem = 0;
        g.M = (int)M; g.N = (int)DH; g.K = h->Bn;
        g.A = h->dz; g.lda = h->Bn; g.sAi = M * h->Bn;
        g.B = W(h->ix_wp); g.ldb = DH; g.sBi = Pp;
        g.C = h->dy; g.ldc = DH; g.sCi = M * DH;
        if (int rc = gemm(h, g, "dY GEMM")) return rc;
    }
    // ---- backward through the LSTM layers ----
    for (int l = h->layers - 1; l >= 0; --l) {
        const int64_t Il = l == 0 ? h->I : DH;
        const void* in = l == 0 ? h->x0 : Y(l - 1);
        const int64_t ldin = l == 0 ? h->ldx : DH;
        RecDesc r{};
        r.precision = prec; r.L = n; r.lmap = act; r.direct = h->tune_rec_direct; r.D = D; r.B = B; r.H = H; r.T = T;
        r.gates = Gates(l); r.sGi = M * G4;
        r.c = Cb(l); r.sCi = M * DH;
        r.y = Y(l); r.sYi = M * DH;
        r.wh = W(h->ix_wh[l]); r.sWi = Pp; r.sWd = (int64_t)4 * H * H;
        r.dy = h->dy; r.sDYi = M * DH;
        r.da = h->da; r.sDAi = M * G4;
        r.dc = h->dc; r.sDCi = (int64_t)B * DH;
        // rows of partial bias sums per learner: one per frame and batch tile (the persistent kernel writes one per frame)
        const int64_t dbrows = persist ? (int64_t)T : (int64_t)T * rec_backward_batch_tiles(B);
        r.dbp = h->dbp; r.sDBi = dbrows * G4;
        if (persist) {
            // per (learner, direction): W_h once; per frame: da in (4 gates) and out, dY, 4 gates, c, c'
            if (int rc = mark(h, 3, persist_launches, 2.0 * B * H * 4 * H * (T - 1) * n * D,
                              (double)n * D * (4.0 * H * H * esz + (double)T * B * H * (8 * esz + 4 + 16 + 8)))) return rc;
            if (int rc = run_persistent(r, l, true)) return rc;
        } else {
            // per frame and (learner, direction): W_h once, da in (4 gates) and out, dY, 4 gates, c, c', dc in and out
            if (int rc = mark(h, 3, T, 2.0 * B * H * 4 * H * (T - 1) * n * D,
                              (double)T * n * D * (4.0 * H * H * esz + (double)B * H * (8 * esz + 4 + 16 + 8 + 8)))) return rc;
            for (int t = 0; t < T; ++t) {
                r.step = t;
                HIPCHK(launch_rec_backward(r, s), "recurrent backward step");
            }
        }
        // dW_x = da' x  (both directions at once: rows of W_x are [D][4H])
        g = G();
        g.a_kc = 0; g.b_kc = 0; g.c_elem = 0;
        g.M = (int)G4; g.N = (int)Il; g.K = (int)M;
        g.A = h->da; g.lda = G4; g.sAi = M * G4;
        g.B = in; g.ldb = ldin; g.sBi = M * ldin;
        g.C = Gr(h->ix_wx[l]); g.ldc = Il; g.sCi = Pp;
        if (int rc = gemm(h, g, "dW_x GEMM")) return rc;
        // dW_h[d] = da_d' h_{t'}: frames with a predecessor only (T-1 of them)
        if (T > 1) {
            g = G();
            g.a_kc = 0; g.b_kc = 0; g.c_elem = 0;
            g.M = 4 * H; g.N = H; g.K = (int)((int64_t)(T - 1) * B);
            // d = 0: da rows of frames 1..T-1 against h of frames 0..T-2
            // d = 1: da rows of frames 0..T-2 (columns 4H..) against h of frames 1..T-1 (columns H..)
            g.A = (const char*)h->da + (size_t)B * G4 * esz; g.lda = G4; g.sAi = M * G4;
            g.sAd = (int64_t)4 * H - (int64_t)B * G4;
            g.B = Y(l); g.ldb = DH; g.sBi = M * DH; g.sBd = (int64_t)B * DH + H;
            g.C = Gr(h->ix_wh[l]); g.ldc = H; g.sCi = Pp; g.sCd = (int64_t)4 * H * H;
            g.groupsD = D;
            if (int rc = gemm(h, g, "dW_h GEMM")) return rc;
        } else {
            // a single frame has no predecessor: dW_h = 0 (a fill kernel, so that the step holds no memset node)
            if (int rc = mark(h, 5, 1)) return rc;
            HIPCHK(launch_zero(Gr(h->ix_wh[l]), Pp, G4 * H, n, act, s), "zero dW_h");
        }
        // db = sum over the frames (and batch tiles) of the column sums the backward steps left behind
        if (int rc = mark(h, 5, 1)) return rc;
        HIPCHK(launch_colsum(0, h->dbp, G4, dbrows * G4, dbrows, (int)G4, Gr(h->ix_b[l]), Pp, n, act, s), "db");
        if (l > 0) {
            // dY_{l-1} = da W_x  (sum over both directions: K = D*4H)
            g = G();
            g.a_kc = 1; g.b_kc = 0; g.c_elem = 0;
            g.M = (int)M; g.N = (int)DH; g.K = (int)G4;
            g.A = h->da; g.lda = G4; g.sAi = M * G4;
            g.B = W(h->ix_wx[l]); g.ldb = DH; g.sBi = Pp;
            g.C = h->dy; g.ldc = DH; g.sCi = M * DH;
            if (int rc = gemm(h, g, "dX GEMM")) return rc;
        }
    }
    return ADPSGD_OK;
}

}  // namespace

extern "C" {

int adpsgd_workspace_bytes(const adpsgd_config* cfg, size_t* out) {
    std::string why;
    if (int rc = check_config(cfg, why)) return fail(rc, why);
    if (!out) return fail(ADPSGD_EINVAL, "out is NULL");
    adpsgd_handle tmp{};
    tmp.cfg = *cfg;
    *out = plan(&tmp, nullptr);
    return ADPSGD_OK;
}

static int create_impl(const adpsgd_config* cfg, void* dev_workspace, size_t bytes, void* hip_stream, adpsgd_t* out) {
    std::string why;
    if (int rc = check_config(cfg, why)) return fail(rc, why);
    if (!out) return fail(ADPSGD_EINVAL, "out is NULL");
    if (!dev_workspace || ((uintptr_t)dev_workspace % 256) != 0) return fail(ADPSGD_ENOMEM, "workspace is NULL or not 256-byte aligned");
    adpsgd_handle* h = new adpsgd_handle{};
    h->cfg = *cfg;
    h->stream = (hipStream_t)hip_stream;
    const size_t need = plan(h, dev_workspace);
    if (bytes < need) {
        delete h;
        return fail(ADPSGD_ENOMEM, "workspace too small: need " + std::to_string(need) + " bytes");
    }
    h->k = 0; h->cur = 0; h->shadow_valid = false;
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
            h->cu_count = cus;
    }
    hipStream_t s = h->stream;
    const size_t slab = (size_t)h->L * h->Ppad * 4;
    void* mirror = nullptr;                       // pinned host word the status is copied to after every step
    hipError_t e = hipHostMalloc(&mirror, 64, hipHostMallocDefault);
    if (e != hipSuccess) { delete h; return hipfail(e, "pinned status word"); }
    h->status_host = (volatile uint32_t*)mirror;
    *h->status_host = 0u;
    e = hipMemsetAsync(h->status, 0, 256, s);
    if (e == hipSuccess) e = hipMemsetAsync(h->params[0], 0, slab, s);
    if (e == hipSuccess && h->tau == 1) e = hipMemsetAsync(h->params[1], 0, slab, s);
    if (e == hipSuccess && !h->flat) e = hipMemsetAsync(h->grads, 0, slab, s);
    if (e != hipSuccess) { (void)hipHostFree(mirror); delete h; return hipfail(e, "clear models"); }
    if (cfg->init_scale > 0.f) {
        // same w_0 on every learner (Algorithm 1, input)
        std::vector<float> w0((size_t)h->P);
        const double a = (double)cfg->init_scale;
        for (int64_t i = 0; i < h->P; ++i)
            w0[(size_t)i] = (float)((2.0 * draw01(cfg->seed, kStreamInit, 0, (uint64_t)i) - 1.0) * a);
        for (int b = 0; b <= h->tau && e == hipSuccess; ++b)
            for (int i = 0; i < h->L && e == hipSuccess; ++i)
                e = hipMemcpyAsync(h->params[b] + (size_t)i * h->Ppad, w0.data(), (size_t)h->P * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipStreamSynchronize(s);
        if (e != hipSuccess) { (void)hipHostFree(mirror); delete h; return hipfail(e, "initial model upload"); }
    } else {
        e = hipStreamSynchronize(s);
        if (e != hipSuccess) { (void)hipHostFree(mirror); delete h; return hipfail(e, "stream sync"); }
    }
    *out = h;
    return ADPSGD_OK;
}

int adpsgd_create(const adpsgd_config* cfg, void* dev_workspace, size_t bytes, void* hip_stream, adpsgd_t* out) {
    try {
        return create_impl(cfg, dev_workspace, bytes, hip_stream, out);
    } catch (const std::bad_alloc&) {
        return fail(ADPSGD_ENOMEM, "out of host memory");
    } catch (const std::exception& ex) {
        return fail(ADPSGD_EINVAL, std::string("unexpected failure: ") + ex.what());
    } catch (...) {
        return fail(ADPSGD_EINVAL, "unexpected failure");
    }
}

static int step_impl(adpsgd_t h, const void* const* batch_ptrs, float lr, const int32_t* given_active) {
    if (!h || !batch_ptrs) return fail(ADPSGD_EINVAL, "NULL argument");
    if (int rc = status_error(h)) return rc;
    const int L = h->L;
    int32_t order[ADPSGD_MAX_LEARNERS], partner[ADPSGD_MAX_LEARNERS], active[ADPSGD_MAX_LEARNERS];
    if (given_active) {
        bool all = true;
        for (int i = 0; i < L; ++i) all = all && given_active[i] != 0;
        const bool rings = h->cfg.pattern == ADPSGD_FIXED_RING || h->cfg.pattern == ADPSGD_RANDOM_RING;
        if (!all && (!rings || h->tau != 0 || h->mix != ADPSGD_MIX_PAIR))
            return fail(ADPSGD_EINVAL, "a learner can sit out only on a ring pattern with pairwise mixing and tau = 0");
        if (!is_hybrid(h->mix)) {
            make_schedule(h->cfg.pattern, h->cfg.seed, 0.f, L, h->k, order, partner, active);
            for (int i = 0; i < L; ++i) active[i] = given_active[i] != 0;
            for (int i = 0; i < L; ++i)
                if (!active[i]) { const int j = partner[i]; partner[j] = j; partner[i] = i; }
        }
    }
    if (given_active && !is_hybrid(h->mix)) {
        // schedule taken above
    } else if (is_hybrid(h->mix)) {
        // the ring is that of the super-learners; every learner takes part
        make_schedule(h->cfg.pattern, h->cfg.seed, 0.f, L / h->cfg.group_size, h->k, order, partner, active);
        for (int i = 0; i < L; ++i) active[i] = 1;
    } else {
        make_schedule(h->cfg.pattern, h->cfg.seed, h->cfg.straggler_p, L, h->k, order, partner, active);
    }
    const int nptr = h->flat ? L : 2 * L;
    for (int i = 0; i < nptr; ++i) {
        const int li = h->flat ? i : i / 2;
        if (!batch_ptrs[i] && active[li]) return fail(ADPSGD_EINVAL, "batch_ptrs[" + std::to_string(i) + "] is NULL");
    }
    float* xk = h->params[h->cur];
    float* xnext = h->tau == 1 ? h->params[1 - h->cur] : xk;
    UpdateDesc u{};
    u.L = L; u.mix = h->mix; u.P = h->P; u.src = xk; u.dst = xnext; u.stride = h->Ppad; u.lr = lr;
    u.update_first = h->cfg.pattern == ADPSGD_SDPSGD;
    u.group_size = is_hybrid(h->mix) ? h->cfg.group_size : 1;
    u.tri_segment = h->tune_tri_segment;
    u.sync_segment = h->tune_sync_segment;
    u.pair_split = h->tune_pair_split;
    {   // two-kernel global mean: by default on models large enough for the extra launches not to matter
        int64_t chunk = h->tune_mean_chunk >= 0 ? h->tune_mean_chunk : (h->P >= (4 << 20) ? kMeanChunkDefault : 0);
        if (chunk > h->mean_cap) chunk = h->mean_cap;
        u.mean_buf = chunk > 0 ? h->mean_buf : nullptr;
        u.mean_elems = chunk;
    }
    if (h->flat) {
        for (int i = 0; i < L; ++i) u.g[i] = (const float*)batch_ptrs[i];
    } else {
        // the gradient is evaluated at x^{k-tau}: the other buffer holds x^{k-1}
        const float* at = h->tau == 1 ? h->params[1 - h->cur] : xk;
        if (int rc = compute_gradients(h, at, batch_ptrs, active)) return rc;
        for (int i = 0; i < L; ++i) u.g[i] = h->grads + (size_t)i * h->Ppad;
    }
    for (int i = 0; i < L; ++i) { u.partner[i] = (int16_t)partner[i]; u.active[i] = (int16_t)active[i]; u.order[i] = (int16_t)order[i]; }
    // bf16 GEMM operands of the next iteration: its gradient point is x^k when tau = 1, x^{k+1} otherwise
    u.shadow = (!h->flat && h->prec) ? h->shadow : nullptr;
    u.emit_input = h->tau == 1;
    {
        int nact = 0;
        for (int i = 0; i < L; ++i) nact += active[i];
        const double ub = (u.shadow ? 14.0 : 12.0) * (double)h->P * nact;
        if (int rc = mark(h, 6, 1, ub, ub)) return rc;
    }
    HIPCHK(launch_update(u, h->stream), "mix + update");
    if (int rc = mark(h, -1)) return rc;
    if (!h->flat)    // what the kernels of this step have reported reaches the host with the stream, without a wait
        HIPCHK(hipMemcpyAsync((void*)h->status_host, h->status, 4, hipMemcpyDeviceToHost, h->stream), "status copy");
    if (h->tau == 1) h->cur = 1 - h->cur;
    if (u.shadow) h->shadow_valid = true;
    h->k += 1;
    return ADPSGD_OK;
}

static int step_guarded(adpsgd_t h, const void* const* batch_ptrs, float lr, const int32_t* active) {
    try {
        return step_impl(h, batch_ptrs, lr, active);
    } catch (const std::bad_alloc&) {
        return fail(ADPSGD_ENOMEM, "out of host memory");
    } catch (const std::exception& ex) {
        return fail(ADPSGD_EINVAL, std::string("unexpected failure: ") + ex.what());
    } catch (...) {
        return fail(ADPSGD_EINVAL, "unexpected failure");
    }
}

float* adpsgd_params(adpsgd_t h, int i) {
    if (!h || i < 0 || i >= h->L) { g_err = "bad learner index"; return nullptr; }
    return h->params[h->cur] + (size_t)i * h->Ppad;
}

int adpsgd_set_params(adpsgd_t h, int i, const float* dev_src) {
    if (!h || !dev_src || i < -1 || i >= h->L) return fail(ADPSGD_EINVAL, "bad argument");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    const int lo = i < 0 ? 0 : i, hi = i < 0 ? h->L : i + 1;
    h->shadow_valid = false;
    for (int b = 0; b <= h->tau; ++b)
        for (int j = lo; j < hi; ++j)
            HIPCHK(hipMemcpyAsync(h->params[b] + (size_t)j * h->Ppad, dev_src, (size_t)h->P * 4, hipMemcpyDeviceToDevice, h->stream), "set_params copy");
    return ADPSGD_OK;
}

float* adpsgd_grads(adpsgd_t h, int i) {
    if (!h || h->flat || i < 0 || i >= h->L) { g_err = "bad argument"; return nullptr; }
    return h->grads + (size_t)i * h->Ppad;
}

int adpsgd_losses(adpsgd_t h, float* host_out) {
    if (!h || !host_out || h->flat) return fail(ADPSGD_EINVAL, "bad argument");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    HIPCHK(hipMemcpyAsync(host_out, h->loss, (size_t)h->L * 4, hipMemcpyDeviceToHost, h->stream), "loss copy");
    HIPCHK(hipStreamSynchronize(h->stream), "stream sync");
    return status_error(h);
}

int adpsgd_step(adpsgd_t h, const void* const* batch_ptrs, float lr) { return step_guarded(h, batch_ptrs, lr, nullptr); }

int adpsgd_step_masked(adpsgd_t h, const void* const* batch_ptrs, float lr, const int32_t* active) {
    if (!active) return fail(ADPSGD_EINVAL, "active is NULL");
    return step_guarded(h, batch_ptrs, lr, active);
}

// ---- HIP-graph replay of iterations ----------------------------------------------------------------
// adpsgd_step enqueues kernels and one 4-byte copy to pinned memory, nothing else (no host wait, no allocation, no
// memset node), so its stream work can be recorded once and replayed.  What a recording fixes: the batch pointers, the
// learning rate, and the schedule of the recorded iterations; it therefore needs a schedule that repeats (not the
// random ring, no drawn stragglers), and on the patterns whose schedule or buffers alternate (fixed ring: the matching
// phase; delay-by-one: the two model buffers) a whole number of periods, i.e. an even number of iterations.
int adpsgd_capture_begin(adpsgd_t h) {
    if (!h) return fail(ADPSGD_EINVAL, "NULL handle");
    if (h->capturing) return fail(ADPSGD_EINVAL, "already recording");
    if (int rc = status_error(h)) return rc;
    if (!h->stream) return fail(ADPSGD_EINVAL, "the null stream cannot be recorded: create the handle on a stream of its own");
    if (h->cfg.pattern == ADPSGD_RANDOM_RING || h->cfg.straggler_p > 0.f)
        return fail(ADPSGD_EINVAL, "a recording replays the schedule of its iterations: the random ring and drawn stragglers change it every iteration");
    if (h->prof.on) return fail(ADPSGD_EINVAL, "switch phase profiling off before recording");
    if (!h->flat && h->prec && !h->shadow_valid)
        return fail(ADPSGD_EINVAL, "run one iteration before recording (the bf16 copy of the models is made by the first one)");
    HIPCHK(hipStreamBeginCapture(h->stream, hipStreamCaptureModeThreadLocal), "begin stream capture");
    h->capturing = true;
    h->capture_k0 = h->k;
    h->capture_cur0 = h->cur;
    return ADPSGD_OK;
}

int adpsgd_capture_end(adpsgd_t h, adpsgd_graph_t* out) {
    if (!h || !out) return fail(ADPSGD_EINVAL, "NULL argument");
    if (!h->capturing) return fail(ADPSGD_EINVAL, "not recording");
    *out = nullptr;
    hipGraph_t graph = nullptr;
    const hipError_t e = hipStreamEndCapture(h->stream, &graph);
    // nothing has run: the handle goes back to where the recording began
    const int64_t steps = h->k - h->capture_k0;
    h->capturing = false;
    h->k = h->capture_k0;
    h->cur = h->capture_cur0;
    if (e != hipSuccess || !graph) {
        if (graph) (void)hipGraphDestroy(graph);
        return hipfail(e != hipSuccess ? e : hipErrorUnknown, "end stream capture");
    }
    const bool alternates = h->tau == 1 || h->cfg.pattern == ADPSGD_FIXED_RING;
    if (steps < 1 || (alternates && steps % 2 != 0)) {
        (void)hipGraphDestroy(graph);
        return fail(ADPSGD_EINVAL, steps < 1 ? "no iteration was recorded"
                                             : "record an even number of iterations: the fixed ring's matching and the two model "
                                               "buffers of delay-by-one alternate from one iteration to the next");
    }
    hipGraphExec_t exec = nullptr;
    const hipError_t ei = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (ei != hipSuccess) {
        (void)hipGraphDestroy(graph);
        return hipfail(ei, "graph instantiate");
    }
    adpsgd_graph* g = new (std::nothrow) adpsgd_graph{h, graph, exec, steps, h->capture_k0};
    if (!g) {
        (void)hipGraphExecDestroy(exec);
        (void)hipGraphDestroy(graph);
        return fail(ADPSGD_ENOMEM, "out of host memory");
    }
    try { h->graphs.push_back(g); } catch (...) {
        (void)hipGraphExecDestroy(exec); (void)hipGraphDestroy(graph); delete g;
        return fail(ADPSGD_ENOMEM, "out of host memory");
    }
    *out = g;
    return ADPSGD_OK;
}

int adpsgd_graph_replay(adpsgd_graph_t g) {
    if (!g) return fail(ADPSGD_EINVAL, "NULL graph");
    if (!g->owner) return fail(ADPSGD_EINVAL, "the handle of this recording has been destroyed");
    adpsgd_t h = g->owner;
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    if (int rc = status_error(h)) return rc;
    const bool alternates = h->tau == 1 || h->cfg.pattern == ADPSGD_FIXED_RING;
    if (alternates && ((h->k - g->k0) % 2 != 0))
        return fail(ADPSGD_EINVAL, "the handle stands at an iteration of the other parity than the recording's first one");
    if (h->prof.on) return fail(ADPSGD_EINVAL, "switch phase profiling off before replaying");
    HIPCHK(hipGraphLaunch(g->exec, h->stream), "graph launch");
    h->k += g->steps;
    return ADPSGD_OK;
}

int64_t adpsgd_graph_steps(adpsgd_graph_t g) { return g ? g->steps : -1; }

void adpsgd_graph_destroy(adpsgd_graph_t g) {
    if (!g) return;
    if (g->owner) {
        (void)hipStreamSynchronize(g->owner->stream);               // a replay may still be running
        std::vector<adpsgd_graph*>& v = g->owner->graphs;
        for (size_t i = 0; i < v.size(); ++i)
            if (v[i] == g) { v.erase(v.begin() + (long)i); break; }
    }
    (void)hipGraphExecDestroy(g->exec);
    (void)hipGraphDestroy(g->graph);
    delete g;
}

int adpsgd_delay(uint64_t microseconds, void* hip_stream) {
    if (microseconds > 10000000ull) return fail(ADPSGD_EINVAL, "at most 10 000 000 microseconds");
    HIPCHK(launch_delay(microseconds * 100ull, (hipStream_t)hip_stream), "delay kernel");
    return ADPSGD_OK;
}

int adpsgd_status(adpsgd_t h) {
    if (!h) return fail(ADPSGD_EINVAL, "NULL handle");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    if (!h->flat) HIPCHK(hipMemcpyAsync((void*)h->status_host, h->status, 4, hipMemcpyDeviceToHost, h->stream), "status copy");
    HIPCHK(hipStreamSynchronize(h->stream), "stream sync");
    return status_error(h);
}

int64_t adpsgd_param_count(adpsgd_t h) { return h ? h->P : -1; }

int adpsgd_layout_count(adpsgd_t h) { return h ? (int)h->tensors.size() : -1; }

int adpsgd_layout(adpsgd_t h, int idx, int64_t* offset, int64_t* rows, int64_t* cols) {
    if (!h || idx < 0 || idx >= (int)h->tensors.size()) return fail(ADPSGD_EINVAL, "tensor index out of range");
    if (offset) *offset = h->tensors[idx].off;
    if (rows) *rows = h->tensors[idx].rows;
    if (cols) *cols = h->tensors[idx].cols;
    return ADPSGD_OK;
}

int adpsgd_schedule_of(int32_t pattern, uint64_t seed, float straggler_p, int32_t L, int64_t k,
                       int32_t* order, int32_t* partner, int32_t* active) {
    if (L < 1 || L > ADPSGD_MAX_LEARNERS || pattern < 0 || pattern > 3 || k < 0) return fail(ADPSGD_EINVAL, "bad argument");
    int32_t o[ADPSGD_MAX_LEARNERS], p[ADPSGD_MAX_LEARNERS], a[ADPSGD_MAX_LEARNERS];
    make_schedule(pattern, seed, straggler_p, L, k, o, p, a);
    if (order) memcpy(order, o, (size_t)L * 4);
    if (partner) memcpy(partner, p, (size_t)L * 4);
    if (active) memcpy(active, a, (size_t)L * 4);
    return ADPSGD_OK;
}

int adpsgd_schedule(adpsgd_t h, int64_t k, int32_t* order, int32_t* partner, int32_t* active) {
    if (!h) return fail(ADPSGD_EINVAL, "NULL handle");
    if (is_hybrid(h->mix)) {
        const int G = h->L / h->cfg.group_size;
        if (int rc = adpsgd_schedule_of(h->cfg.pattern, h->cfg.seed, 0.f, G, k, order, partner, active)) return rc;
        for (int i = G; i < h->L; ++i) {
            if (order) order[i] = -1;
            if (partner) partner[i] = -1;
            if (active) active[i] = -1;
        }
        return ADPSGD_OK;
    }
    return adpsgd_schedule_of(h->cfg.pattern, h->cfg.seed, h->cfg.straggler_p, h->L, k, order, partner, active);
}

int adpsgd_lr_at_epoch(int32_t epoch, float peak_lr, float start_lr, int32_t warmup_epochs, int32_t hold_until_epoch, float* out) {
    if (!out || epoch < 1 || warmup_epochs < 0) return fail(ADPSGD_EINVAL, "epoch >= 1, warmup_epochs >= 0 and a result pointer are needed");
    double lr;
    if (warmup_epochs >= 2 && epoch <= warmup_epochs) {
        lr = (double)start_lr + ((double)peak_lr - (double)start_lr) * (double)(epoch - 1) / (double)(warmup_epochs - 1);
    } else if (epoch <= hold_until_epoch) {
        lr = (double)peak_lr;
    } else {
        lr = (double)peak_lr * std::pow(std::sqrt(0.5), (double)(epoch - hold_until_epoch));
    }
    *out = (float)lr;
    return ADPSGD_OK;
}

int64_t adpsgd_iteration(adpsgd_t h) { return h ? h->k : -1; }

int adpsgd_average(adpsgd_t h, float* dev_out) {
    if (!h || !dev_out) return fail(ADPSGD_EINVAL, "NULL argument");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    HIPCHK(launch_average(h->params[h->cur], h->Ppad, h->L, h->P, dev_out, h->stream), "average");
    return ADPSGD_OK;
}

int adpsgd_consensus(adpsgd_t h, double* host_out) {
    if (!h || !host_out) return fail(ADPSGD_EINVAL, "NULL argument");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    HIPCHK(launch_consensus(h->params[h->cur], h->Ppad, h->L, h->P, h->consensus, h->consensus + kConsensusBlocks, h->stream),
           "consensus distance");
    HIPCHK(hipMemcpyAsync(host_out, h->consensus + kConsensusBlocks, 8, hipMemcpyDeviceToHost, h->stream), "consensus copy");
    HIPCHK(hipStreamSynchronize(h->stream), "stream sync");
    return ADPSGD_OK;
}

int adpsgd_consensus_static(const float* dev_x, int64_t stride, int32_t L, int64_t P, double* dev_out, void* hip_stream) {
    if (!dev_x || !dev_out) return fail(ADPSGD_EINVAL, "NULL argument");
    if (L < 1 || L > ADPSGD_MAX_LEARNERS) return fail(ADPSGD_EINVAL, "L must be in 1..128");
    if (P < 1 || stride < P) return fail(ADPSGD_EINVAL, "P must be >= 1 and stride >= P");
    if ((uintptr_t)dev_out % 8 != 0 || (uintptr_t)dev_x % 4 != 0) return fail(ADPSGD_EINVAL, "misaligned pointer");
    if (P > ADPSGD_STATIC_MAX_ELEMENTS / L)
        return fail(ADPSGD_EINVAL, "input beyond the maximum of the allocation-free entry point: L * P must not exceed 2^34 elements");
    HIPCHK(launch_consensus_static(dev_x, stride, L, P, dev_out, (hipStream_t)hip_stream), "consensus distance (static scratch)");
    return ADPSGD_OK;
}

int adpsgd_set_profiling(adpsgd_t h, int enable) {
    if (!h) return fail(ADPSGD_EINVAL, "NULL handle");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    h->prof.on = enable != 0;
    prof_reset(h);
    return ADPSGD_OK;
}

int adpsgd_profile(adpsgd_t h, float* host_ms, int32_t* host_launches, double* host_work, double* host_bytes) {
    if (!h) return fail(ADPSGD_EINVAL, "NULL handle");
    if (h->capturing) return fail(ADPSGD_EINVAL, "not while iterations are being recorded (adpsgd_capture_begin)");
    Profiler& p = h->prof;
    HIPCHK(hipStreamSynchronize(h->stream), "stream sync");
    float ms[ADPSGD_PHASES] = {0};
    for (size_t j = 0; j + 1 < p.seg_phase.size(); ++j) {
        const int ph = p.seg_phase[j];
        if (ph < 0) continue;
        float t = 0.f;
        HIPCHK(hipEventElapsedTime(&t, p.ev[j], p.ev[j + 1]), "event elapsed");
        ms[ph] += t;
    }
    for (int i = 0; i < ADPSGD_PHASES; ++i) {
        if (host_ms) host_ms[i] = ms[i];
        if (host_launches) host_launches[i] = p.launches[i];
        if (host_work) host_work[i] = p.work[i];
        if (host_bytes) host_bytes[i] = p.bytes[i];
    }
    prof_reset(h);
    return ADPSGD_OK;
}

void adpsgd_destroy(adpsgd_t h) {
    if (!h) return;
    if (h->capturing) {                              // a recording left open: close it and drop what it holds
        hipGraph_t graph = nullptr;
        (void)hipStreamEndCapture(h->stream, &graph);
        if (graph) (void)hipGraphDestroy(graph);
        h->capturing = false;
    }
    for (hipEvent_t e : h->prof.ev) (void)hipEventDestroy(e);
    for (adpsgd_graph* g : h->graphs) g->owner = nullptr;   // they can still be destroyed, no longer replayed
    if (h->status_host) {
        (void)hipStreamSynchronize(h->stream);       // the last status copy may still be in flight
        (void)hipHostFree((void*)h->status_host);
    }
    delete h;
}

const char* adpsgd_last_error(void) { return g_err.c_str(); }

int adpsgd_gemm(int precision, int a_kmajor, int b_kmajor, int c_is_elem, int M, int N, int K,
                const void* A, int64_t lda, int64_t strideA, const void* B, int64_t ldb, int64_t strideB,
                void* C, int64_t ldc, int64_t strideC, const float* bias, int64_t strideBias,
                int groups, int tile_config, void* hip_stream) {
    if (!A || !B || !C || (precision != 0 && precision != 1)) return fail(ADPSGD_EINVAL, "bad argument");
    if (groups < 1 || groups > ADPSGD_MAX_LEARNERS) return fail(ADPSGD_EINVAL, "groups must be in 1..128");
    GemmDesc g{};
    g.tile = tile_config; g.lmap.identity();
    g.precision = precision; g.a_kc = a_kmajor != 0; g.b_kc = b_kmajor != 0; g.c_elem = c_is_elem != 0;
    g.M = M; g.N = N; g.K = K;
    g.A = A; g.lda = lda; g.sAi = strideA;
    g.B = B; g.ldb = ldb; g.sBi = strideB;
    g.C = C; g.ldc = ldc; g.sCi = strideC;
    g.bias = bias; g.sBiasI = strideBias;
    g.groupsI = groups; g.groupsD = 1;
    hipError_t e = launch_gemm(g, (hipStream_t)hip_stream);
    if (e == hipErrorInvalidValue) return fail(ADPSGD_EINVAL, "GEMM operands violate the size/alignment rules");
    if (e != hipSuccess) return hipfail(e, "gemm launch");
    return ADPSGD_OK;
}

int adpsgd_probe_mfma(float* dev_out, int blocks, int iters, void* hip_stream) {
    hipError_t e = launch_mfma_peak(dev_out, blocks, iters, (hipStream_t)hip_stream);
    if (e == hipErrorInvalidValue) return fail(ADPSGD_EINVAL, "dev_out, blocks >= 1 and iters >= 1 are needed");
    if (e != hipSuccess) return hipfail(e, "mfma probe");
    return ADPSGD_OK;
}

int adpsgd_probe_stream(int reads, int writes_f32, int writes_bf16, void* dev_buf, int64_t pitch_bytes, int64_t elems, void* hip_stream) {
    hipError_t e = launch_stream_probe(reads, writes_f32, writes_bf16, dev_buf, pitch_bytes, elems, (hipStream_t)hip_stream);
    if (e == hipErrorInvalidValue)
        return fail(ADPSGD_EINVAL, "mix must be 1:0:0, 1:1:0, 2:1:0, 2:1:1, 4:2:0, 4:2:2, 8:4:4, 16:8:8 or 32:16:16; elems a multiple of 4; pitch >= 4 * elems, a multiple of 16");
    if (e != hipSuccess) return hipfail(e, "stream probe");
    return ADPSGD_OK;
}

int adpsgd_set_tuning(adpsgd_t h, int key, int value) {
    if (!h) return fail(ADPSGD_EINVAL, "NULL handle");
    switch (key) {
        case ADPSGD_TUNE_GEMM_TILE:
            if (value != -1 && value != 0 && value != 5 && (value < 11 || value > 13))
                return fail(ADPSGD_EINVAL, "GEMM tile configuration must be -1, 0, 5, 11, 12 or 13");
            h->tune_gemm_tile = value; return ADPSGD_OK;
        case ADPSGD_TUNE_REC_DIRECT:
            if (value != 0 && value != 1) return fail(ADPSGD_EINVAL, "0 or 1");
            h->tune_rec_direct = value; return ADPSGD_OK;
        case ADPSGD_TUNE_REC_FWD_GROUPS:
            if (value < 0 || value > ADPSGD_MAX_LEARNERS) return fail(ADPSGD_EINVAL, "0 (automatic) or 1..128 groups");
            h->tune_rec_fwd_groups = value; return ADPSGD_OK;
        case ADPSGD_TUNE_REC_PERSISTENT:
            if (value < -1 || value > 1) return fail(ADPSGD_EINVAL, "-1 (automatic), 0 or 1");
            h->tune_rec_persist = value; return ADPSGD_OK;
        case ADPSGD_TUNE_MEAN_CHUNK:
            if (value != 0 && value != -1 && (value < 1024 || value > kMeanChunkMax || value % 1024))
                return fail(ADPSGD_EINVAL, "-1 (automatic), 0 (single kernel) or a multiple of 1024 elements up to 16777216");
            h->tune_mean_chunk = value; return ADPSGD_OK;
        case ADPSGD_TUNE_PAIR_SPLIT:
            if (value != -1 && value != 0 && value != 64 && value != 128) return fail(ADPSGD_EINVAL, "-1 (default), 0, 64 or 128");
            h->tune_pair_split = value; return ADPSGD_OK;
        case ADPSGD_TUNE_SYNC_SEGMENT:
            if (value != -1 && value != 0 && value != 2 && value != 4 && value != 8)
                return fail(ADPSGD_EINVAL, "-1 (default), 0 (one thread owns all learners of a position), 2, 4 or 8 learners per thread");
            h->tune_sync_segment = value; return ADPSGD_OK;
        case ADPSGD_TUNE_TRI_SEGMENT:
            if (value != -1 && value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
                return fail(ADPSGD_EINVAL, "-1 (default), 0 (one thread walks the whole ring), 1, 2, 4 or 8 ring positions per thread");
            h->tune_tri_segment = value; return ADPSGD_OK;
        case ADPSGD_TUNE_REC_WAIT_US:
            if (value < 0) return fail(ADPSGD_EINVAL, "microseconds >= 0");
            h->tune_wait_us = value; return ADPSGD_OK;
        default: return fail(ADPSGD_EINVAL, "unknown tuning key");
    }
}

}  // extern "C"
