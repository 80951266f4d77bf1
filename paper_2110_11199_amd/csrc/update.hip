// Fused mixing + SGD update over the learners' flat fp32 vectors (Algorithm 1:
// model averaging followed by the local update; Eq. 2 in matrix form).
//
// One streaming pass: every element of every active learner is read once (model
// and gradient) and written once, 12 bytes per (active learner, element).
// Pairwise mixing handles both members of a matched pair in the same thread, so
// the update is safe in place.  Arithmetic order (each operation rounded once,
// no fused multiply-add):
//     pair: m = (x_i + x_j) * 0.5      all: m = (((x_0 + x_1) + ...) ) * (1/L)
//     ring neighbours: m = ((x_left + x_i) + x_right) * (1/3)
//     x_i <- m - (lr * g_i)
// Synchronous baseline (Section III-A, Algorithm 2), the same operations in the other order:
//     u_j = x_j - (lr * g_j);   x_i <- (((u_0 + u_1) + ...)) * (1/L) for every i
#include <mutex>
#include "kernels.hpp"

namespace adpsgd {

struct PairArgs {
    const float* src; float* dst; int64_t stride; int64_t P; float lr;
    bf16_t* shadow; int emit_input;   // bf16 copy of the next gradient point: the inputs (tau = 1) or the outputs
    int nwork;
    const float* g[128];
    int16_t a[128], b[128];     // work item w mixes learners a[w], b[w] (a == b: no partner)
};

__device__ inline float sgd_(float m, float lr, float g) { return __fsub_rn(m, __fmul_rn(lr, g)); }

__device__ inline float4 pair_new_(const float4& m, float lr, const float4& g) {
    return make_float4(sgd_(m.x, lr, g.x), sgd_(m.y, lr, g.y), sgd_(m.z, lr, g.z), sgd_(m.w, lr, g.w));
}
__device__ inline float4 half_sum_(const float4& p, const float4& q) {
    return make_float4(__fmul_rn(__fadd_rn(p.x, q.x), 0.5f), __fmul_rn(__fadd_rn(p.y, q.y), 0.5f),
                       __fmul_rn(__fadd_rn(p.z, q.z), 0.5f), __fmul_rn(__fadd_rn(p.w, q.w), 0.5f));
}

// float4 positions per thread and stream.  One is best: on the 64-learner random-ring workload 5.88 TB/s
// against 5.63 (2), 5.60 (4) and 5.47 (8): smaller workgroups spread more evenly over the CUs.
constexpr int kUnroll = 1;

// one element of one work item (scalar path and tails)
__device__ inline void pair_scalar_(const float* xa, const float* xb, const float* ga, const float* gb, float* oa, float* ob,
                                    bf16_t* sha, bf16_t* shb, bool solo, int emit_input, float lr, int64_t e) {
    const float x = xa[e], y = xb[e];
    if (solo) {
        const float r = sgd_(x, lr, ga[e]);
        oa[e] = r;
        if (sha) sha[e] = f32_to_bf16(emit_input ? x : r);
    } else {
        const float m = __fmul_rn(__fadd_rn(x, y), 0.5f);
        const float va = sgd_(m, lr, ga[e]), vb = sgd_(m, lr, gb[e]);
        oa[e] = va; ob[e] = vb;
        if (sha) { sha[e] = f32_to_bf16(emit_input ? x : va); shb[e] = f32_to_bf16(emit_input ? y : vb); }
    }
}

// The models and gradients are streamed once per iteration: non-temporal loads and stores keep them
// from displacing each other in L2 (measured +11% on the 2-reads-1-write pattern).
typedef float vf4_t __attribute__((ext_vector_type(4)));
__device__ inline float4 ldnt_(const float* p, int64_t e4) {
    const vf4_t v = __builtin_nontemporal_load((const vf4_t*)p + e4);
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ inline void emit4_(bf16_t* sh, int64_t e4, const float4& v) {
    uint2 o;
    o.x = pack_bf16(v.x, v.y);
    o.y = pack_bf16(v.z, v.w);
    ((uint2*)sh)[e4] = o;
}
__device__ inline void stnt_(float* p, int64_t e4, const float4& v) {
    vf4_t w; w.x = v.x; w.y = v.y; w.z = v.z; w.w = v.w;
    __builtin_nontemporal_store(w, (vf4_t*)p + e4);
}

template <bool VEC>
__global__ __launch_bounds__(256) void pair_update_kernel(PairArgs p) {
    const int w = blockIdx.y;
    const int a = p.a[w], b = p.b[w];
    const float* xa = p.src + a * p.stride;
    const float* xb = p.src + b * p.stride;
    float* oa = p.dst + a * p.stride;
    float* ob = p.dst + b * p.stride;
    const float* ga = p.g[a];
    const float* gb = p.g[b];
    const float lr = p.lr;
    bf16_t* sha = p.shadow ? p.shadow + a * p.stride : nullptr;
    bf16_t* shb = p.shadow ? p.shadow + b * p.stride : nullptr;
    if constexpr (VEC) {
        const int64_t n4 = p.P >> 2;
        const int64_t base = (int64_t)blockIdx.x * (blockDim.x * kUnroll) + threadIdx.x;
        if (a == b) {
            float4 x[kUnroll], g[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t e = base + u * blockDim.x;
                if (e < n4) { x[u] = ldnt_(xa, e); g[u] = ldnt_(ga, e); }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t e = base + u * blockDim.x;
                if (e < n4) {
                    const float4 r = pair_new_(x[u], lr, g[u]);
                    stnt_(oa, e, r);
                    if (sha) emit4_(sha, e, p.emit_input ? x[u] : r);
                }
            }
        } else {
            float4 x[kUnroll], y[kUnroll], g[kUnroll], h[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t e = base + u * blockDim.x;
                if (e < n4) {
                    x[u] = ldnt_(xa, e); y[u] = ldnt_(xb, e);
                    g[u] = ldnt_(ga, e); h[u] = ldnt_(gb, e);
                }
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t e = base + u * blockDim.x;
                if (e < n4) {
                    const float4 m = half_sum_(x[u], y[u]);
                    const float4 ra = pair_new_(m, lr, g[u]), rb = pair_new_(m, lr, h[u]);
                    stnt_(oa, e, ra);
                    stnt_(ob, e, rb);
                    if (sha) { emit4_(sha, e, p.emit_input ? x[u] : ra); emit4_(shb, e, p.emit_input ? y[u] : rb); }
                }
            }
        }
        // tail (P % 4 elements), handled by the first block
        if (blockIdx.x == 0 && threadIdx.x < (p.P & 3)) {
            const int64_t e = (n4 << 2) + threadIdx.x;
            pair_scalar_(xa, xb, ga, gb, oa, ob, sha, shb, a == b, p.emit_input, lr, e);
        }
    } else {
        const int64_t base = (int64_t)blockIdx.x * (blockDim.x * kUnroll) + threadIdx.x;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int64_t e = base + u * blockDim.x;
            if (e >= p.P) continue;
            pair_scalar_(xa, xb, ga, gb, oa, ob, sha, shb, a == b, p.emit_input, lr, e);
        }
    }
}

// The same pairwise update with ONE member of a pair per thread: a workgroup of NX positions x 2 members; a thread
// reads its member's model and gradient (two streams, 1 KB contiguous per wave and stream), hands the model to its
// partner thread through LDS, and writes its member's result after the workgroup's barrier, i.e. after both models
// of these positions have been read: safe in place like the two-member form, same operations (the pair sum is
// commutative), bit-identical results.  For a work item without a partner (a == b) the two halves of the workgroup
// take adjacent positions of the one learner (and the workgroups past its end have nothing to do).
template <int NX>
__global__ __launch_bounds__(2 * NX) void pair_split_update_kernel(PairArgs p) {
    __shared__ float4 other[2 * NX];
    const int w = blockIdx.y, member = threadIdx.y, tx = threadIdx.x;
    const int a = p.a[w], b = p.b[w];
    const bool solo = a == b;
    const int i = member ? b : a;
    const int64_t n4 = p.P >> 2;
    // a pair: both halves of the workgroup at the same NX positions; no partner: the halves at adjacent ones
    const int64_t e = solo ? (int64_t)blockIdx.x * (2 * NX) + member * NX + tx : (int64_t)blockIdx.x * NX + tx;
    const bool ok = e < n4;
    float4 x = make_float4(0.f, 0.f, 0.f, 0.f), g = x;
    if (ok) { x = ldnt_(p.src + i * p.stride, e); g = ldnt_(p.g[i], e); }
    other[member * NX + tx] = x;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (ok) {
        const float4 m = solo ? x : half_sum_(x, other[(1 - member) * NX + tx]);
        const float4 r = pair_new_(m, p.lr, g);
        stnt_(p.dst + i * p.stride, e, r);
        if (p.shadow) emit4_(p.shadow + i * p.stride, e, p.emit_input ? x : r);
    }
    // tail (P % 4 elements): one thread handles both members of an element
    if (blockIdx.x == 0 && member == 0 && tx < (p.P & 3))
        pair_scalar_(p.src + a * p.stride, p.src + b * p.stride, p.g[a], p.g[b], p.dst + a * p.stride, p.dst + b * p.stride,
                     p.shadow ? p.shadow + a * p.stride : nullptr, p.shadow ? p.shadow + b * p.stride : nullptr, solo,
                     p.emit_input, p.lr, (n4 << 2) + tx);
}

struct AllArgs {
    const float* src; float* dst; int64_t stride; int64_t P; float lr; float inv_L; int L;
    bf16_t* shadow; int emit_input;
    const float* g[128];
};

// synchronous baseline: one element of all learners
__device__ inline void sync_scalar_(const AllArgs& p, int64_t t) {
    float s = sgd_(p.src[t], p.lr, p.g[0][t]);
    for (int j = 1; j < p.L; ++j) s = __fadd_rn(s, sgd_(p.src[j * p.stride + t], p.lr, p.g[j][t]));
    const float m = __fmul_rn(s, p.inv_L);
    for (int i = 0; i < p.L; ++i) {
        p.dst[i * p.stride + t] = m;
        if (p.shadow) p.shadow[i * p.stride + t] = f32_to_bf16(m);
    }
}

// Synchronous baseline: one thread owns an element index of all learners, reads L models and L
// gradients, and writes the mean of the updated models to all L learners (12 bytes per learner and
// element, as the other updates).  The bf16 copy, if any, is of the output (tau = 0).
template <bool VEC>
__global__ __launch_bounds__(256) void sync_update_kernel(AllArgs p) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if constexpr (VEC) {
        const int64_t n4 = p.P >> 2;
        if (e < n4) {
            float4 s = pair_new_(ldnt_(p.src, e), p.lr, ldnt_(p.g[0], e));
#pragma unroll 8
            for (int j = 1; j < p.L; ++j) {
                const float4 u = pair_new_(ldnt_(p.src + j * p.stride, e), p.lr, ldnt_(p.g[j], e));
                s.x = __fadd_rn(s.x, u.x); s.y = __fadd_rn(s.y, u.y); s.z = __fadd_rn(s.z, u.z); s.w = __fadd_rn(s.w, u.w);
            }
            const float4 m = make_float4(__fmul_rn(s.x, p.inv_L), __fmul_rn(s.y, p.inv_L), __fmul_rn(s.z, p.inv_L), __fmul_rn(s.w, p.inv_L));
#pragma unroll 8
            for (int i = 0; i < p.L; ++i) {
                stnt_(p.dst + i * p.stride, e, m);
                if (p.shadow) emit4_(p.shadow + i * p.stride, e, m);
            }
        }
        if (blockIdx.x == 0 && threadIdx.x < (p.P & 3)) sync_scalar_(p, (n4 << 2) + threadIdx.x);
    } else {
        if (e < p.P) sync_scalar_(p, e);
    }
}

// The same update with the learners cut into segments of SEG: a workgroup of blockDim.x positions x blockDim.y segments;
// a thread reads the SEG models and gradients of its segment (2 SEG streams instead of 2 L), and the sum of the updated
// models runs through the segments in learner order, one segment per barrier, through LDS: the same additions in the
// same order as the single walk, bit-identical results.  Every model of the workgroup's positions has been read before
// the first result is written (the writes follow the last barrier), so it stays safe in place.
template <int SEG>
__global__ __launch_bounds__(1024) void sync_seg_update_kernel(AllArgs p) {
    __shared__ float4 chain[64];
    const int tx = threadIdx.x, sy = threadIdx.y, nx = blockDim.x, ns = blockDim.y;
    const int64_t e = (int64_t)blockIdx.x * nx + tx;
    const bool ok = e < (p.P >> 2);
    const int j0 = sy * SEG;
    float4 u[SEG];
#pragma unroll
    for (int j = 0; j < SEG; ++j)
        if (ok && j0 + j < p.L) u[j] = pair_new_(ldnt_(p.src + (j0 + j) * p.stride, e), p.lr, ldnt_(p.g[j0 + j], e));
    for (int step = 0; step < ns; ++step) {
        if (sy == step && ok) {
            float4 s = u[0];
            if (step > 0) { const float4 c = chain[tx]; s = make_float4(__fadd_rn(c.x, s.x), __fadd_rn(c.y, s.y), __fadd_rn(c.z, s.z), __fadd_rn(c.w, s.w)); }
#pragma unroll
            for (int j = 1; j < SEG; ++j)
                if (j0 + j < p.L) { s.x = __fadd_rn(s.x, u[j].x); s.y = __fadd_rn(s.y, u[j].y); s.z = __fadd_rn(s.z, u[j].z); s.w = __fadd_rn(s.w, u[j].w); }
            chain[tx] = s;
        }
        __syncthreads();
    }
    if (!ok) return;
    const float4 t = chain[tx];
    const float4 m = make_float4(__fmul_rn(t.x, p.inv_L), __fmul_rn(t.y, p.inv_L), __fmul_rn(t.z, p.inv_L), __fmul_rn(t.w, p.inv_L));
#pragma unroll
    for (int j = 0; j < SEG; ++j) {
        if (j0 + j >= p.L) break;
        stnt_(p.dst + (j0 + j) * p.stride, e, m);
        if (p.shadow) emit4_(p.shadow + (j0 + j) * p.stride, e, m);
    }
}

// the P % 4 last elements of every learner of the synchronous baseline (one thread each)
__global__ void sync_tail_kernel(AllArgs p) {
    if (threadIdx.x < (p.P & 3)) sync_scalar_(p, ((p.P >> 2) << 2) + threadIdx.x);
}

template <int SEG>
static void launch_sync_seg(const AllArgs& a, hipStream_t s) {
    const int ns = (a.L + SEG - 1) / SEG;
    int nx = 64;
    while (nx * ns > 512 && nx > 8) nx >>= 1;
    const int64_t n4 = a.P >> 2;
    hipLaunchKernelGGL(sync_seg_update_kernel<SEG>, dim3((unsigned)((n4 + nx - 1) / nx)), dim3((unsigned)nx, (unsigned)ns), 0, s, a);
    if (a.P & 3) hipLaunchKernelGGL(sync_tail_kernel, dim3(1), dim3(64), 0, s, a);
}

__device__ inline void all_scalar_(const AllArgs& p, int64_t t) {
    float s = p.src[t];
    if (p.shadow && p.emit_input) p.shadow[t] = f32_to_bf16(s);
    for (int j = 1; j < p.L; ++j) {
        const float v = p.src[j * p.stride + t];
        if (p.shadow && p.emit_input) p.shadow[j * p.stride + t] = f32_to_bf16(v);
        s = __fadd_rn(s, v);
    }
    const float m = __fmul_rn(s, p.inv_L);
    for (int i = 0; i < p.L; ++i) {
        const float r = sgd_(m, p.lr, p.g[i][t]);
        p.dst[i * p.stride + t] = r;
        if (p.shadow && !p.emit_input) p.shadow[i * p.stride + t] = f32_to_bf16(r);
    }
}

// One thread owns an element index of all learners: reads L models, forms the
// mean once, reads L gradients, writes L models.
template <bool VEC>
__global__ __launch_bounds__(256) void all_update_kernel(AllArgs p) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if constexpr (VEC) {
        const int64_t n4 = p.P >> 2;
        if (e < n4) {
            float4 s = ldnt_(p.src, e);
            const bool emit_in = p.shadow && p.emit_input, emit_out = p.shadow && !p.emit_input;
            if (emit_in) emit4_(p.shadow, e, s);
#pragma unroll 8
            for (int j = 1; j < p.L; ++j) {
                const float4 v = ldnt_(p.src + j * p.stride, e);
                if (emit_in) emit4_(p.shadow + j * p.stride, e, v);
                s.x = __fadd_rn(s.x, v.x); s.y = __fadd_rn(s.y, v.y); s.z = __fadd_rn(s.z, v.z); s.w = __fadd_rn(s.w, v.w);
            }
            const float4 m = make_float4(__fmul_rn(s.x, p.inv_L), __fmul_rn(s.y, p.inv_L), __fmul_rn(s.z, p.inv_L), __fmul_rn(s.w, p.inv_L));
#pragma unroll 8
            for (int i = 0; i < p.L; ++i) {
                const float4 g = ldnt_(p.g[i], e);
                const float4 r = pair_new_(m, p.lr, g);
                stnt_(p.dst + i * p.stride, e, r);
                if (emit_out) emit4_(p.shadow + i * p.stride, e, r);
            }
        }
        if (blockIdx.x == 0 && threadIdx.x < (p.P & 3)) {
            const int64_t t = (n4 << 2) + threadIdx.x;
            all_scalar_(p, t);
        }
    } else {
        if (e < p.P) all_scalar_(p, e);
    }
}

// ---- global mean in two kernels per chunk of the parameter index --------------------------------------
// The rate of a streaming kernel on this device falls with the number of streams one thread walks at once (measured
// with the stream probe: 6.5 TB/s with 3 streams per thread, 5.3 with 64).  The single-kernel global mean owns
// 4 streams per learner and thread.  Split: `all_mean_kernel` reads the L models of a chunk of the index and
// writes their mean to a small buffer (and the bf16 copies of the models read, when asked for); `all_apply_kernel`
// then runs once per learner (grid y) with three streams per thread: the mean (from the buffer, which a chunk
// at a time stays in the caches), the learner's gradient, the learner's new model.  Same operations in the same
// order per element as all_update_kernel, so the results are bit-identical.
struct AllSplitArgs {
    AllArgs a;
    float* mean;            // [chunk] fp32
    int64_t e0, n4c;        // chunk start and length in float4 positions
};

__global__ __launch_bounds__(256) void all_mean_kernel(AllSplitArgs q) {
    const AllArgs& p = q.a;
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= q.n4c) return;
    const int64_t e = q.e0 + c;
    float4 s = ldnt_(p.src, e);
    const bool emit_in = p.shadow && p.emit_input;
    if (emit_in) emit4_(p.shadow, e, s);
#pragma unroll 8
    for (int j = 1; j < p.L; ++j) {
        const float4 v = ldnt_(p.src + j * p.stride, e);
        if (emit_in) emit4_(p.shadow + j * p.stride, e, v);
        s.x = __fadd_rn(s.x, v.x); s.y = __fadd_rn(s.y, v.y); s.z = __fadd_rn(s.z, v.z); s.w = __fadd_rn(s.w, v.w);
    }
    ((float4*)q.mean)[c] = make_float4(__fmul_rn(s.x, p.inv_L), __fmul_rn(s.y, p.inv_L), __fmul_rn(s.z, p.inv_L), __fmul_rn(s.w, p.inv_L));
}

__global__ __launch_bounds__(256) void all_apply_kernel(AllSplitArgs q) {
    const AllArgs& p = q.a;
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= q.n4c) return;
    const int64_t e = q.e0 + c;
    const int i = blockIdx.y;
    const float4 m = ((const float4*)q.mean)[c];
    const float4 r = pair_new_(m, p.lr, ldnt_(p.g[i], e));
    stnt_(p.dst + i * p.stride, e, r);
    if (p.shadow && !p.emit_input) emit4_(p.shadow + i * p.stride, e, r);
}

// the P % 4 last elements of every learner (one thread each)
__global__ void all_tail_kernel(AllArgs p) {
    if (threadIdx.x < (p.P & 3)) all_scalar_(p, ((p.P >> 2) << 2) + threadIdx.x);
}

// ---- ring-neighbour mixing with weights 1/3 (the circulant operator T^f of Eq. 9, and T^r = P' T^f P) -------
// One thread owns an element index of all learners and walks the ring order with the previous, current and
// next model value in registers: every model is read once (the last one of the order twice), so the update
// is safe in place and moves the same 12 bytes per learner and element as the pairwise one.
struct TriArgs {
    const float* src; float* dst; int64_t stride; int64_t P; float lr; float third; int L;
    bf16_t* shadow; int emit_input;
    const float* g[128];
    int16_t order[128];
};

__device__ inline float tri_mean_(float l, float c, float r, float third) { return __fmul_rn(__fadd_rn(__fadd_rn(l, c), r), third); }

__device__ inline void tri_scalar_(const TriArgs& p, int64_t t) {
    const float first = p.src[p.order[0] * p.stride + t];
    float prev = p.src[p.order[p.L - 1] * p.stride + t], cur = first;
    for (int q = 0; q < p.L; ++q) {
        const int i = p.order[q];
        const float next = q + 1 < p.L ? p.src[p.order[q + 1] * p.stride + t] : first;
        const float r = sgd_(tri_mean_(prev, cur, next, p.third), p.lr, p.g[i][t]);
        p.dst[i * p.stride + t] = r;
        if (p.shadow) p.shadow[i * p.stride + t] = f32_to_bf16(p.emit_input ? cur : r);
        prev = cur; cur = next;
    }
}

template <bool VEC>
__global__ __launch_bounds__(256) void tri_update_kernel(TriArgs p) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if constexpr (VEC) {
        const int64_t n4 = p.P >> 2;
        if (e < n4) {
            const float4 first = ldnt_(p.src + p.order[0] * p.stride, e);
            float4 prev = ldnt_(p.src + p.order[p.L - 1] * p.stride, e), cur = first;
            for (int q = 0; q < p.L; ++q) {
                const int i = p.order[q];
                float4 next = first;
                if (q + 1 < p.L) next = ldnt_(p.src + p.order[q + 1] * p.stride, e);
                const float4 g = ldnt_(p.g[i], e);
                const float4 m = make_float4(tri_mean_(prev.x, cur.x, next.x, p.third), tri_mean_(prev.y, cur.y, next.y, p.third),
                                             tri_mean_(prev.z, cur.z, next.z, p.third), tri_mean_(prev.w, cur.w, next.w, p.third));
                const float4 r = pair_new_(m, p.lr, g);
                stnt_(p.dst + i * p.stride, e, r);
                if (p.shadow) emit4_(p.shadow + i * p.stride, e, p.emit_input ? cur : r);
                prev = cur; cur = next;
            }
        }
        if (blockIdx.x == 0 && threadIdx.x < (p.P & 3)) tri_scalar_(p, (n4 << 2) + threadIdx.x);
    } else {
        if (e < p.P) tri_scalar_(p, e);
    }
}

// The same operator with the ring cut into segments of SEG positions.  A workgroup of blockDim.x element positions
// x blockDim.y segments covers all L learners of its element positions; a thread owns one segment at one position:
// it reads its SEG models and gradients (2 SEG streams instead of 2 L: the rate of a streaming kernel on this
// device falls with the number of streams a thread walks at once), hands the first and last model of its segment to
// the neighbouring segments through LDS, and writes its SEG results after the workgroup's barrier, i.e. after every
// model of these positions has been read: safe in place like the single walk, the same 12 bytes per learner and
// element (no model is read twice), the same operations per element, bit-identical results.
template <int SEG>
__global__ __launch_bounds__(1024) void tri_seg_update_kernel(TriArgs p) {
    __shared__ float4 edge[2 * 1024];                            // [first | last][segment][position]
    const int tx = threadIdx.x, sy = threadIdx.y, nx = blockDim.x, ns = blockDim.y;
    const int64_t e = (int64_t)blockIdx.x * nx + tx;
    const bool ok = e < (p.P >> 2);
    const int q0 = sy * SEG;
    float4 x[SEG], g[SEG];
    float4 lastv = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < SEG; ++j) {
        if (ok && q0 + j < p.L) {
            const int i = p.order[q0 + j];
            x[j] = ldnt_(p.src + i * p.stride, e);
            g[j] = ldnt_(p.g[i], e);
            lastv = x[j];
        }
    }
    if (ok) { edge[sy * nx + tx] = x[0]; edge[(ns + sy) * nx + tx] = lastv; }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // every model of this thread is in registers ...
    __syncthreads();                                             // ... and so is every other thread's: writing may begin
    if (!ok) return;
    float4 prev = edge[(ns + (sy + ns - 1) % ns) * nx + tx];
    const float4 after = edge[((sy + 1) % ns) * nx + tx];
#pragma unroll
    for (int j = 0; j < SEG; ++j) {
        if (q0 + j >= p.L) break;
        const int i = p.order[q0 + j];
        float4 next = after;
        if (j + 1 < SEG && q0 + j + 1 < p.L) next = x[j + 1 < SEG ? j + 1 : j];
        const float4 m = make_float4(tri_mean_(prev.x, x[j].x, next.x, p.third), tri_mean_(prev.y, x[j].y, next.y, p.third),
                                     tri_mean_(prev.z, x[j].z, next.z, p.third), tri_mean_(prev.w, x[j].w, next.w, p.third));
        const float4 r = pair_new_(m, p.lr, g[j]);
        stnt_(p.dst + i * p.stride, e, r);
        if (p.shadow) emit4_(p.shadow + i * p.stride, e, p.emit_input ? x[j] : r);
        prev = x[j];
    }
}

// the P % 4 last elements of every learner (one thread each walks the whole ring)
__global__ void tri_tail_kernel(TriArgs p) {
    if (threadIdx.x < (p.P & 3)) tri_scalar_(p, ((p.P >> 2) << 2) + threadIdx.x);
}

template <int SEG>
static void launch_tri_seg(const TriArgs& a, hipStream_t s) {
    const int ns = (a.L + SEG - 1) / SEG;                        // at most 128 segments (L <= 128)
    int nx = 64;
    while (nx * ns > 512 && nx > 8) nx >>= 1;
    const int64_t n4 = a.P >> 2;
    hipLaunchKernelGGL(tri_seg_update_kernel<SEG>, dim3((unsigned)((n4 + nx - 1) / nx)), dim3((unsigned)nx, (unsigned)ns), 0, s, a);
    if (a.P & 3) hipLaunchKernelGGL(tri_tail_kernel, dim3(1), dim3(64), 0, s, a);
}

// ---- hybrid mixing (Section V: synchronous super-learners joined by the asynchronous ring) -----------
// Consecutive blocks of S learners form super-learners.  The mean of every super-learner first,
//     m_a = (((x_{aS} + x_{aS+1}) + ...) + x_{aS+S-1}) * (1/S),
// then the ring operator on the means (pair: (m_a + m_b) * 0.5; neighbours: ((m_left + m_a) + m_right) * (1/3)),
// then x_i <- m - (lr * g_i) for every learner i of super-learner a.  One thread owns an element index (a float4,
// or one float on the unaligned path and the tail) of all the learners it touches and reads every model once
// before it writes any of them, so the update is safe in place at 12 bytes per learner and element.
struct HybridArgs {
    const float* src; float* dst; int64_t stride; int64_t P; float lr;
    bf16_t* shadow; int emit_input;
    int S, G; float inv_S, third;
    const float* g[128];
    int16_t order[128];            // neighbours: ring order of the super-learners
    int16_t a[64], b[64];          // pair: work item w mixes super-learners a[w], b[w] (a == b: unmatched)
};

// the same code for a float4 position and for a single float
struct V4 { typedef float4 type; };
struct V1 { typedef float type; };
__device__ inline float4 hy_ld_(V4, const float* p, int64_t e) { return ldnt_(p, e); }
__device__ inline float hy_ld_(V1, const float* p, int64_t e) { return p[e]; }
__device__ inline void hy_st_(float* p, int64_t e, const float4& v) { stnt_(p, e, v); }
__device__ inline void hy_st_(float* p, int64_t e, float v) { p[e] = v; }
__device__ inline void hy_emit_(bf16_t* sh, int64_t e, const float4& v) { emit4_(sh, e, v); }
__device__ inline void hy_emit_(bf16_t* sh, int64_t e, float v) { sh[e] = f32_to_bf16(v); }
__device__ inline float4 hy_add_(const float4& p, const float4& q) {
    return make_float4(__fadd_rn(p.x, q.x), __fadd_rn(p.y, q.y), __fadd_rn(p.z, q.z), __fadd_rn(p.w, q.w));
}
__device__ inline float hy_add_(float p, float q) { return __fadd_rn(p, q); }
__device__ inline float4 hy_mul_(const float4& p, float c) {
    return make_float4(__fmul_rn(p.x, c), __fmul_rn(p.y, c), __fmul_rn(p.z, c), __fmul_rn(p.w, c));
}
__device__ inline float hy_mul_(float p, float c) { return __fmul_rn(p, c); }
__device__ inline float4 hy_sgd_(const float4& m, float lr, const float4& g) { return pair_new_(m, lr, g); }
__device__ inline float hy_sgd_(float m, float lr, float g) { return sgd_(m, lr, g); }

// mean of super-learner a at position e; emit: also write the bf16 copy of the models read (tau = 1)
template <class V>
__device__ inline typename V::type hy_mean_(const HybridArgs& p, int a, int64_t e, bool emit) {
    const int i0 = a * p.S;
    typename V::type s = hy_ld_(V(), p.src + i0 * p.stride, e);
    if (emit) hy_emit_(p.shadow + i0 * p.stride, e, s);
    for (int j = 1; j < p.S; ++j) {
        const typename V::type v = hy_ld_(V(), p.src + (i0 + j) * p.stride, e);
        if (emit) hy_emit_(p.shadow + (i0 + j) * p.stride, e, v);
        s = hy_add_(s, v);
    }
    return hy_mul_(s, p.inv_S);
}
template <class V>
__device__ inline void hy_write_(const HybridArgs& p, int a, int64_t e, const typename V::type& m, bool emit_out) {
    for (int i = a * p.S; i < (a + 1) * p.S; ++i) {
        const typename V::type r = hy_sgd_(m, p.lr, hy_ld_(V(), p.g[i], e));
        hy_st_(p.dst + i * p.stride, e, r);
        if (emit_out) hy_emit_(p.shadow + i * p.stride, e, r);
    }
}

template <class V>
__device__ inline void hy_pair_one_(const HybridArgs& p, int a, int b, int64_t e) {
    const bool emit_in = p.shadow && p.emit_input, emit_out = p.shadow && !p.emit_input;
    const typename V::type ma = hy_mean_<V>(p, a, e, emit_in);
    if (a == b) { hy_write_<V>(p, a, e, ma, emit_out); return; }
    const typename V::type mb = hy_mean_<V>(p, b, e, emit_in);
    const typename V::type m = hy_mul_(hy_add_(ma, mb), 0.5f);
    hy_write_<V>(p, a, e, m, emit_out);
    hy_write_<V>(p, b, e, m, emit_out);
}

template <class V>
__device__ inline void hy_tri_one_(const HybridArgs& p, int64_t e) {
    const bool emit_in = p.shadow && p.emit_input, emit_out = p.shadow && !p.emit_input;
    const typename V::type first = hy_mean_<V>(p, p.order[0], e, emit_in);
    if (p.G == 1) { hy_write_<V>(p, p.order[0], e, first, emit_out); return; }
    typename V::type prev = hy_mean_<V>(p, p.order[p.G - 1], e, false), cur = first;     // read again (and copied) as "next" below
    for (int q = 0; q < p.G; ++q) {
        const typename V::type next = q + 1 < p.G ? hy_mean_<V>(p, p.order[q + 1], e, emit_in) : first;
        const typename V::type m = hy_mul_(hy_add_(hy_add_(prev, cur), next), p.third);
        hy_write_<V>(p, p.order[q], e, m, emit_out);
        prev = cur; cur = next;
    }
}

template <bool VEC, bool TRI>
__global__ __launch_bounds__(256) void hybrid_update_kernel(HybridArgs p) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int a = TRI ? 0 : p.a[blockIdx.y], b = TRI ? 0 : p.b[blockIdx.y];
    if constexpr (VEC) {
        const int64_t n4 = p.P >> 2;
        if (e < n4) { if constexpr (TRI) hy_tri_one_<V4>(p, e); else hy_pair_one_<V4>(p, a, b, e); }
        if (blockIdx.x == 0 && threadIdx.x < (p.P & 3)) {
            const int64_t t = (n4 << 2) + threadIdx.x;
            if constexpr (TRI) hy_tri_one_<V1>(p, t); else hy_pair_one_<V1>(p, a, b, t);
        }
    } else {
        if (e < p.P) { if constexpr (TRI) hy_tri_one_<V1>(p, e); else hy_pair_one_<V1>(p, a, b, e); }
    }
}

static hipError_t launch_hybrid(const UpdateDesc& d, bool vec, hipStream_t s) {
    const int S = d.group_size, L = d.L;
    if (S < 1 || L % S != 0) return hipErrorInvalidValue;
    const int G = L / S;
    const bool tri = d.mix == 4;
    if (tri && G == 2) return hipErrorInvalidValue;
    for (int i = 0; i < L; ++i)
        if (!d.active[i]) return hipErrorInvalidValue;          // super-learners average synchronously: everybody takes part
    HybridArgs a;
    a.src = d.src; a.dst = d.dst; a.stride = d.stride; a.P = d.P; a.lr = d.lr;
    a.shadow = d.shadow; a.emit_input = d.emit_input;
    a.S = S; a.G = G; a.inv_S = 1.0f / (float)S; a.third = 1.0f / 3.0f;
    for (int i = 0; i < 128; ++i) { a.g[i] = i < L ? d.g[i] : nullptr; a.order[i] = 0; }
    for (int i = 0; i < 64; ++i) a.a[i] = a.b[i] = 0;
    bool seen[128] = {false};
    for (int q = 0; q < G; ++q) {      // the ring order must be a permutation of the super-learners, the matching an involution
        const int o = d.order[q], pq = d.partner[q];
        if (o < 0 || o >= G || seen[o] || pq < 0 || pq >= G || d.partner[pq] != q) return hipErrorInvalidValue;
        seen[o] = true; a.order[q] = (int16_t)o;
    }
    const int64_t n = vec ? ((d.P >> 2) > 0 ? (d.P >> 2) : 1) : d.P;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (tri) {
        if (vec) hipLaunchKernelGGL((hybrid_update_kernel<true, true>), dim3(blocks), dim3(256), 0, s, a);
        else hipLaunchKernelGGL((hybrid_update_kernel<false, true>), dim3(blocks), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    int nw = 0;
    for (int q = 0; q < G; ++q) {
        const int j = d.partner[q];
        if (j == q || q < j) {
            if (nw >= 64) return hipErrorInvalidValue;
            a.a[nw] = (int16_t)q; a.b[nw] = (int16_t)j; ++nw;
        }
    }
    if (vec) hipLaunchKernelGGL((hybrid_update_kernel<true, false>), dim3(blocks, (unsigned)nw), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((hybrid_update_kernel<false, false>), dim3(blocks, (unsigned)nw), dim3(256), 0, s, a);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void average_kernel(const float* x, int64_t stride, int L, int64_t P,
                                                      float inv_L, float* out) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= P) return;
    float s = x[e];
    for (int j = 1; j < L; ++j) s = __fadd_rn(s, x[j * stride + e]);
    out[e] = __fmul_rn(s, inv_L);
}

hipError_t launch_update(const UpdateDesc& d, hipStream_t s) {
    if (d.L < 1 || d.L > 128 || d.P < 1) return hipErrorInvalidValue;
    bool vec = ((uintptr_t)d.src % 16 == 0) && ((uintptr_t)d.dst % 16 == 0) && (d.stride % 4 == 0);
    for (int i = 0; i < d.L; ++i)
        if ((uintptr_t)d.g[i] % 16 != 0) vec = false;
    if (d.update_first && d.mix != 2) return hipErrorInvalidValue;
    if (d.mix == 3 || d.mix == 4) return launch_hybrid(d, vec, s);
    if (d.mix == 2) {
        AllArgs a;
        a.src = d.src; a.dst = d.dst; a.stride = d.stride; a.P = d.P; a.lr = d.lr; a.L = d.L;
        a.inv_L = 1.0f / (float)d.L;
        a.shadow = d.shadow; a.emit_input = d.emit_input;
        for (int i = 0; i < 128; ++i) a.g[i] = i < d.L ? d.g[i] : nullptr;
        if (d.update_first) {
            for (int i = 0; i < d.L; ++i)
                if (!d.active[i]) return hipErrorInvalidValue;     // the baseline waits for every learner
            if (d.emit_input) return hipErrorInvalidValue;         // and has no staleness
        }
        if (vec && !d.update_first && d.mean_buf && d.mean_elems >= 1024 && d.L >= 4 && (d.P >> 2) > 0 &&
            (uintptr_t)d.mean_buf % 16 == 0) {
            const int64_t n4 = d.P >> 2, chunk4 = d.mean_elems >> 2;
            AllSplitArgs q;
            q.a = a; q.mean = d.mean_buf;
            for (int64_t e0 = 0; e0 < n4; e0 += chunk4) {
                q.e0 = e0; q.n4c = n4 - e0 < chunk4 ? n4 - e0 : chunk4;
                // (workgroups of 64 or 128 threads instead of 256 change nothing here: 5.8 - 6.0 TB/s in all nine combinations;
                // a mean kernel with one (position, learner) per thread and the sum through LDS is slower: 5.1 - 5.8)
                const unsigned blocks = (unsigned)((q.n4c + 255) / 256);
                hipLaunchKernelGGL(all_mean_kernel, dim3(blocks), dim3(256), 0, s, q);
                hipLaunchKernelGGL(all_apply_kernel, dim3(blocks, (unsigned)d.L), dim3(256), 0, s, q);
            }
            if (d.P & 3) hipLaunchKernelGGL(all_tail_kernel, dim3(1), dim3(64), 0, s, a);
        } else if (vec) {
            const int64_t n4 = d.P >> 2;
            const unsigned blocks = (unsigned)((n4 > 0 ? n4 : 1) + 255) / 256;
            // two learners per thread are the measured best on large models (64 x 135M: 5.16 -> 5.48 TB/s, 16 x 145M:
            // 5.49 -> 5.99; four 5.40 / 5.75, eight 5.34 / 5.67)
            const int seg = d.sync_segment < 0 ? ((d.P >= (4 << 20) && d.L >= 4) ? 2 : 0) : d.sync_segment;
            if (d.update_first && n4 > 0 && seg >= 2 && d.L > seg) {
                if (seg >= 8) launch_sync_seg<8>(a, s);
                else if (seg >= 4) launch_sync_seg<4>(a, s);
                else launch_sync_seg<2>(a, s);
            } else if (d.update_first) hipLaunchKernelGGL(sync_update_kernel<true>, dim3(blocks), dim3(256), 0, s, a);
            else hipLaunchKernelGGL(all_update_kernel<true>, dim3(blocks), dim3(256), 0, s, a);
        } else {
            const unsigned blocks = (unsigned)((d.P + 255) / 256);
            if (d.update_first) hipLaunchKernelGGL(sync_update_kernel<false>, dim3(blocks), dim3(256), 0, s, a);
            else hipLaunchKernelGGL(all_update_kernel<false>, dim3(blocks), dim3(256), 0, s, a);
        }
        return hipGetLastError();
    }
    if (d.mix == 1) {
        TriArgs a;
        a.src = d.src; a.dst = d.dst; a.stride = d.stride; a.P = d.P; a.lr = d.lr; a.L = d.L;
        a.third = 1.0f / 3.0f;
        a.shadow = d.shadow; a.emit_input = d.emit_input;
        for (int i = 0; i < 128; ++i) { a.g[i] = i < d.L ? d.g[i] : nullptr; a.order[i] = i < d.L ? d.order[i] : 0; }
        // the order must be a permutation of 0..L-1 (an index out of range would address another learner's memory)
        bool seen[128] = {false};
        for (int i = 0; i < d.L; ++i) {
            if (d.order[i] < 0 || d.order[i] >= d.L || seen[d.order[i]]) return hipErrorInvalidValue;
            seen[d.order[i]] = true;
        }
        // Two ring positions per thread are the measured best on large models (64 x 135M: 5.0 -> 5.4-5.5 TB/s, 16 x 145M:
        // 5.5 -> 6.1; one position 5.2 / 5.8, four 5.4 / 5.0, eight 4.9 / 3.3); on small ones the single walk's fewer,
        // larger workgroups are as fast or faster.
        const int seg = d.tri_segment < 0 ? ((d.P >= (4 << 20) && d.L >= 4) ? 2 : 0) : d.tri_segment;
        if (vec && (d.P >> 2) > 0 && seg >= 1 && d.L > seg) {
            if (seg == 1) launch_tri_seg<1>(a, s);
            else if (seg >= 8) launch_tri_seg<8>(a, s);
            else if (seg >= 4) launch_tri_seg<4>(a, s);
            else launch_tri_seg<2>(a, s);
        } else if (vec) {
            const int64_t n4 = d.P >> 2;
            hipLaunchKernelGGL(tri_update_kernel<true>, dim3((unsigned)(((n4 > 0 ? n4 : 1) + 255) / 256)), dim3(256), 0, s, a);
        } else {
            hipLaunchKernelGGL(tri_update_kernel<false>, dim3((unsigned)((d.P + 255) / 256)), dim3(256), 0, s, a);
        }
        return hipGetLastError();
    }
    PairArgs a;
    a.src = d.src; a.dst = d.dst; a.stride = d.stride; a.P = d.P; a.lr = d.lr;
    a.shadow = d.shadow; a.emit_input = d.emit_input;
    for (int i = 0; i < 128; ++i) { a.g[i] = i < d.L ? d.g[i] : nullptr; a.a[i] = a.b[i] = 0; }
    int n = 0;
    for (int i = 0; i < d.L; ++i) {
        if (!d.active[i]) continue;
        const int j = d.partner[i];
        if (j == i) { a.a[n] = a.b[n] = (int16_t)i; ++n; }
        else if (i < j) { a.a[n] = (int16_t)i; a.b[n] = (int16_t)j; ++n; }
    }
    a.nwork = n;
    if (n == 0) return hipSuccess;
    // One member per thread in workgroups of 64 positions x 2 members is the measured best on large models (64 x 135M,
    // random ring, 10 % stragglers: 5.9 -> 6.3 TB/s; 16 x 145M: 5.9 -> 6.6; 128 positions 6.15 / 6.3, 32: 6.1 / 6.45,
    // 256: 6.0 / 6.25; the two-member kernel in workgroups of 64 threads 6.1 / 6.3).
    const int split = d.pair_split < 0 ? (d.P >= (1 << 20) ? 64 : 0) : d.pair_split;
    if (vec && split > 0 && (d.P >> 2) > 0) {
        const int64_t n4 = d.P >> 2;
        if (split == 128)
            hipLaunchKernelGGL(pair_split_update_kernel<128>, dim3((unsigned)((n4 + 127) / 128), (unsigned)n), dim3(128, 2), 0, s, a);
        else
            hipLaunchKernelGGL(pair_split_update_kernel<64>, dim3((unsigned)((n4 + 63) / 64), (unsigned)n), dim3(64, 2), 0, s, a);
        return hipGetLastError();
    }
    if (vec) {
        const int64_t n4 = d.P >> 2;
        const int64_t per = 256 * kUnroll;
        const unsigned blocks = (unsigned)(((n4 > 0 ? n4 : 1) + per - 1) / per);
        hipLaunchKernelGGL(pair_update_kernel<true>, dim3(blocks, (unsigned)n), dim3(256), 0, s, a);
    } else {
        const int64_t per = 256 * kUnroll;
        hipLaunchKernelGGL(pair_update_kernel<false>, dim3((unsigned)((d.P + per - 1) / per), (unsigned)n), dim3(256), 0, s, a);
    }
    return hipGetLastError();
}

// Consensus distance: every thread walks element indices with the grid stride and accumulates, in fp64,
// the squared deviations of the L models from their mean at that index; block sums through LDS, then one
// block adds the per-block partial sums in index order (a fixed order: the result is reproducible).
__global__ __launch_bounds__(256) void consensus_partial_kernel(const float* x, int64_t stride, int L, int64_t P, double* partial) {
    double acc = 0.0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < P; e += (int64_t)gridDim.x * 256) {
        double s = 0.0;
        for (int j = 0; j < L; ++j) s += (double)x[j * stride + e];
        const double mean = s / (double)L;
        for (int j = 0; j < L; ++j) { const double d = (double)x[j * stride + e] - mean; acc += d * d; }
    }
    __shared__ double sh[256];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = sh[0];
}
__global__ __launch_bounds__(256) void consensus_final_kernel(const double* partial, int n, double* out) {
    __shared__ double sh[256];
    double acc = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) acc += partial[i];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sh[0];
}

hipError_t launch_consensus(const float* x, int64_t stride, int L, int64_t P, double* partial, double* out, hipStream_t s) {
    if (L < 1 || P < 1) return hipErrorInvalidValue;
    int64_t blocks = (P + 255) / 256;
    if (blocks > kConsensusBlocks) blocks = kConsensusBlocks;
    hipLaunchKernelGGL(consensus_partial_kernel, dim3((unsigned)blocks), dim3(256), 0, s, x, stride, L, P, partial);
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(256), 0, s, partial, (int)blocks, out);
    return hipGetLastError();
}

// ---- the same reduction for callers that cannot allocate ----------------------------------------
// The per-workgroup partial sums live in a file-scope device array instead of caller-provided memory.
// Every GPU holds its own copy of the array at its own address: the address is looked up once per device,
// with that device current, and only that address (never the array's name, which is a host-side stand-in
// in host code) is handed to kernels.  All calls on one GPU share the array: calls that overlap on one GPU
// race.  Nothing in it has to start at zero (a call writes every partial sum it later reads).
static __device__ __align__(256) double scratch[kConsensusBlocks];

static std::mutex g_scratch_mutex;
static double* g_scratch_ptr[kMaxDevices] = {nullptr};

hipError_t launch_consensus_static(const float* x, int64_t stride, int L, int64_t P, double* out, hipStream_t s) {
    if (L < 1 || P < 1) return hipErrorInvalidValue;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    double* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = (double*)p;
        }
        ptr = g_scratch_ptr[dev];
    }
    int64_t blocks = (P + 255) / 256;
    if (blocks > kConsensusBlocks) blocks = kConsensusBlocks;
    hipLaunchKernelGGL(consensus_partial_kernel, dim3((unsigned)blocks), dim3(256), 0, s, x, stride, L, P, ptr);
    hipLaunchKernelGGL(consensus_final_kernel, dim3(1), dim3(256), 0, s, (const double*)ptr, (int)blocks, out);
    return hipGetLastError();
}

hipError_t launch_average(const float* x, int64_t stride, int L, int64_t P, float* out, hipStream_t s) {
    hipLaunchKernelGGL(average_kernel, dim3((unsigned)((P + 255) / 256)), dim3(256), 0, s, x, stride, L, P,
                       1.0f / (float)L, out);
    return hipGetLastError();
}

}  // namespace adpsgd
