// Bandwidth-bound helper kernels of the LSTM gradient: staging/casting of the
// minibatch and of the bf16 weight copy, softmax cross-entropy with its
// gradient, and the column sums that give the bias gradients.
#include "kernels.hpp"

namespace adpsgd {

struct StageArgs {
    LearnerMap lmap;
    int64_t rows; int I, ldx;
    void* x0; int64_t sX0; int32_t* y; int64_t sY;
    const float* feats[128];
    const int32_t* labels[128];
};

template <typename T>
__global__ __launch_bounds__(256) void stage_kernel(StageArgs p) {
    const int li = p.lmap.idx[blockIdx.y];
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t n = p.rows * p.ldx;
    if (idx < n) {
        const int64_t r = idx / p.ldx;
        const int c = (int)(idx % p.ldx);
        const float v = c < p.I ? p.feats[li][r * p.I + c] : 0.f;
        ((T*)p.x0)[li * p.sX0 + idx] = Elem<T>::from(v);
    }
    if (idx < p.rows) p.y[li * p.sY + idx] = p.labels[li][idx];
}

hipError_t launch_stage(const StageDesc& d, hipStream_t s) {
    if (d.L < 1 || d.L > 128) return hipErrorInvalidValue;
    StageArgs a;
    a.lmap = d.lmap;
    a.rows = d.rows; a.I = d.I; a.ldx = d.ldx; a.x0 = d.x0; a.sX0 = d.sX0; a.y = d.y; a.sY = d.sY;
    for (int i = 0; i < 128; ++i) { a.feats[i] = d.feats[i]; a.labels[i] = d.labels[i]; }     // indexed by learner
    dim3 grid((unsigned)((d.rows * d.ldx + 255) / 256), (unsigned)d.L);
    if (d.precision == 0) hipLaunchKernelGGL(stage_kernel<float>, grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(stage_kernel<bf16_t>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

// n must be a multiple of 4 and both pointers 16-byte / 8-byte aligned.
__global__ __launch_bounds__(256) void cast_bf16_kernel(const float4* src, uint2* dst, int64_t n4) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < n4; i += stride) {
        const float4 v = src[i];
        uint2 o;
        o.x = pack_bf16(v.x, v.y);
        o.y = pack_bf16(v.z, v.w);
        dst[i] = o;
    }
}

hipError_t launch_cast_bf16(const float* src, bf16_t* dst, int64_t n, hipStream_t s) {
    if (n % 4 != 0 || (uintptr_t)src % 16 != 0 || (uintptr_t)dst % 8 != 0) return hipErrorInvalidValue;
    const int64_t n4 = n / 4;
    int64_t blocks = (n4 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const float4*)src, (uint2*)dst, n4);
    return hipGetLastError();
}

// dst[z][r][0..ld) = bf16(src[z][r][0..cols)) followed by zeros: rows of a weight matrix padded to
// a row length the direct-to-LDS GEMM can load (16-byte aligned rows, whole K stages).
__global__ __launch_bounds__(256) void pad_rows_bf16_kernel(const float* src, int64_t sS, bf16_t* dst, int64_t sD,
                                                            int64_t rows, int cols, int ld) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * ld) return;
    const int64_t r = idx / ld;
    const int c = (int)(idx % ld);
    dst[blockIdx.y * sD + idx] = c < cols ? f32_to_bf16(src[blockIdx.y * sS + r * cols + c]) : (bf16_t)0;
}

hipError_t launch_pad_rows_bf16(const float* src, int64_t sS, bf16_t* dst, int64_t sD, int64_t rows, int cols, int ld,
                                int L, hipStream_t s) {
    dim3 grid((unsigned)((rows * ld + 255) / 256), (unsigned)L);
    hipLaunchKernelGGL(pad_rows_bf16_kernel, grid, dim3(256), 0, s, src, sS, dst, sD, rows, cols, ld);
    return hipGetLastError();
}

// ---- softmax cross-entropy ---------------------------------------------------
// One workgroup per frame (row of logits).  loss_row = -(z_y - max - log sum exp(z - max));
// dlogits = (softmax - onehot) / rows   (mean over the B*T frames of the minibatch).
__device__ inline void lse_merge_(float& m, float& s, float m2, float s2) {
    const float mm = fmaxf(m, m2);
    s = s * expf(m - mm) + s2 * expf(m2 - mm);
    m = mm;
}

// Label of a frame.  A label outside [0, C) is reported through the status word (the host turns it
// into an error) and clamped, so that it is never used as an index.
__device__ inline int checked_label_(const SoftmaxDesc& p, int li, int64_t row) {
    const int y = p.y[li * p.sYi + row];
    if (y >= 0 && y < p.C) return y;
    if (threadIdx.x == 0 && p.status) atomicOr(p.status, kStatusBadLabel);
    return y < 0 ? 0 : p.C - 1;
}

template <typename T>
__global__ __launch_bounds__(256) void softmax_ce_kernel(SoftmaxDesc p) {
    const int li = p.lmap.idx[blockIdx.y];
    const int64_t row = blockIdx.x;
    const float* z = p.logits + li * p.sLi + row * p.C;
    T* dz = (T*)p.dlogits + li * p.sDi + row * p.C;
    const int y = checked_label_(p, li, row);
    float m = -INFINITY, s = 0.f;
    for (int c = threadIdx.x; c < p.C; c += 256) {
        const float v = z[c];
        if (v > m) { s = s * expf(m - v) + 1.f; m = v; }
        else s += expf(v - m);
    }
    // wave reduction, then across the 4 waves through LDS
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off), s2 = __shfl_xor(s, off);
        if (m2 > -INFINITY || m > -INFINITY) lse_merge_(m, s, m2, s2);
    }
    __shared__ float sm[4], ss[4];
    if ((threadIdx.x & 63) == 0) { sm[threadIdx.x >> 6] = m; ss[threadIdx.x >> 6] = s; }
    __syncthreads();
    m = sm[0]; s = ss[0];
    for (int w = 1; w < 4; ++w) lse_merge_(m, s, sm[w], ss[w]);
    const float inv = 1.f / s;
    const float scale = 1.f / (float)p.rows;
    for (int c = threadIdx.x; c < p.C; c += 256) {
        float pr = expf(z[c] - m) * inv;
        if (c == y) pr -= 1.f;
        dz[c] = Elem<T>::from(pr * scale);
    }
    if (threadIdx.x == 0) p.row_loss[li * p.rows + row] = -((z[y] - m) - logf(s));
}

// One workgroup per learner of the handle; a learner that took no part in the iteration reports 0.
__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* row_loss, int64_t rows, float* loss, SoftmaxDesc p) {
    const int li = blockIdx.x;
    if (!((p.active_bits[li >> 5] >> (li & 31)) & 1u)) {
        if (threadIdx.x == 0) loss[li] = 0.f;
        return;
    }
    float s = 0.f;
    for (int64_t r = threadIdx.x; r < rows; r += 256) s += row_loss[li * rows + r];
    __shared__ float sh[256];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) loss[li] = sh[0] / (float)rows;
}

// Single-pass version: the whole row of logits lives in registers (NV float4 per thread, C <= 4*NT*NV),
// so the logits are read from HBM once.
typedef float vf4_t __attribute__((ext_vector_type(4)));
typedef uint32_t vu2_t __attribute__((ext_vector_type(2)));

template <typename T, int NV, int NT = 256>
__global__ __launch_bounds__(NT) void softmax_ce_row_kernel(SoftmaxDesc p) {
    const int li = p.lmap.idx[blockIdx.y];
    const int64_t row = blockIdx.x;
    const float4* z4 = (const float4*)(p.logits + li * p.sLi + row * p.C);
    T* dz = (T*)p.dlogits + li * p.sDi + row * p.C;
    const int C4 = p.C >> 2;
    const int y = checked_label_(p, li, row);
    float4 v[NV];
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c4 = threadIdx.x + NT * j;
        if (c4 < C4) {
            { const vf4_t t4 = __builtin_nontemporal_load((const vf4_t*)z4 + c4); v[j] = make_float4(t4.x, t4.y, t4.z, t4.w); }   // read once
            m = fmaxf(fmaxf(fmaxf(v[j].x, v[j].y), fmaxf(v[j].z, v[j].w)), m);
        }
    }
    __shared__ float red[2][NT / 64];
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    if ((threadIdx.x & 63) == 0) red[0][threadIdx.x >> 6] = m;
    __syncthreads();
    m = red[0][0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) m = fmaxf(m, red[0][w]);
    float zy = 0.f;                      // logit of the label, picked up by the thread that holds it
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c4 = threadIdx.x + NT * j;
        if (c4 < C4) {
            if ((y >> 2) == c4) zy = (y & 3) == 0 ? v[j].x : (y & 3) == 1 ? v[j].y : (y & 3) == 2 ? v[j].z : v[j].w;
            v[j].x = exp_fast_(v[j].x - m); v[j].y = exp_fast_(v[j].y - m); v[j].z = exp_fast_(v[j].z - m); v[j].w = exp_fast_(v[j].w - m);
            s += (v[j].x + v[j].y) + (v[j].z + v[j].w);
        }
    }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    if ((threadIdx.x & 63) == 0) red[1][threadIdx.x >> 6] = s;
    __syncthreads();
    s = red[1][0];
#pragma unroll
    for (int w = 1; w < NT / 64; ++w) s += red[1][w];
    const float inv = 1.f / s;
    const float scale = 1.f / (float)p.rows;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
        const int c4 = threadIdx.x + NT * j;
        if (c4 < C4) {
            float4 pr = make_float4(v[j].x * inv, v[j].y * inv, v[j].z * inv, v[j].w * inv);
            if ((y >> 2) == c4) {
                if ((y & 3) == 0) pr.x -= 1.f; else if ((y & 3) == 1) pr.y -= 1.f; else if ((y & 3) == 2) pr.z -= 1.f; else pr.w -= 1.f;
            }
            pr.x *= scale; pr.y *= scale; pr.z *= scale; pr.w *= scale;
            if constexpr (sizeof(T) == 2) {
                uint2 o;
                o.x = pack_bf16(pr.x, pr.y);
                o.y = pack_bf16(pr.z, pr.w);
                { vu2_t o2; o2.x = o.x; o2.y = o.y; __builtin_nontemporal_store(o2, (vu2_t*)dz + c4); }
            } else {
                { vf4_t o4; o4.x = pr.x; o4.y = pr.y; o4.z = pr.z; o4.w = pr.w; __builtin_nontemporal_store(o4, (vf4_t*)dz + c4); }
            }
        }
    }
    if ((y >> 2) % NT == (int)threadIdx.x) p.row_loss[li * p.rows + row] = -((zy - m) - logf(s));
}

template <typename T>
static void launch_softmax_t(const SoftmaxDesc& d, hipStream_t s) {
    dim3 grid((unsigned)d.rows, (unsigned)d.L);
    const bool vec = d.C % 4 == 0 && d.sLi % 4 == 0 && d.sDi % 4 == 0 && (uintptr_t)d.logits % 16 == 0 &&
                     (uintptr_t)d.dlogits % 16 == 0;
    // long rows: 512 threads per row, so that a thread holds at most 16 float4 (measured on 32 000 classes:
    // 1.55 ms against 2.25 ms with 256 threads x 32 float4, whose 128 registers allow three waves per SIMD only, and
    // 1.78 ms with 1024 threads x 8 float4)
    if (vec && d.C <= 1024) hipLaunchKernelGGL((softmax_ce_row_kernel<T, 1>), grid, dim3(256), 0, s, d);
    else if (vec && d.C <= 4096) hipLaunchKernelGGL((softmax_ce_row_kernel<T, 4>), grid, dim3(256), 0, s, d);
    else if (vec && d.C <= 8192) hipLaunchKernelGGL((softmax_ce_row_kernel<T, 4, 512>), grid, dim3(512), 0, s, d);
    else if (vec && d.C <= 16384) hipLaunchKernelGGL((softmax_ce_row_kernel<T, 8, 512>), grid, dim3(512), 0, s, d);
    else if (vec && d.C <= 32768) hipLaunchKernelGGL((softmax_ce_row_kernel<T, 16, 512>), grid, dim3(512), 0, s, d);
    else hipLaunchKernelGGL(softmax_ce_kernel<T>, grid, dim3(256), 0, s, d);
}

hipError_t launch_softmax_ce(const SoftmaxDesc& d, hipStream_t s) {
    if (d.L < 1 || d.L > d.L_all || d.L_all > 128) return hipErrorInvalidValue;
    if (d.precision == 0) launch_softmax_t<float>(d, s);
    else launch_softmax_t<bf16_t>(d, s);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(loss_reduce_kernel, dim3((unsigned)d.L_all), dim3(256), 0, s, d.row_loss, d.rows, d.loss, d);
    return hipGetLastError();
}

// ---- column sums -----------------------------------------------------------------
// Workgroup = 64 columns x 4 row slices; fixed summation order (deterministic).
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* in, int64_t ld, int64_t sIi, int64_t rows, int N,
                                                     float* out, int64_t sOi, LearnerMap lmap) {
    const int li = lmap.idx[blockIdx.y];
    const int col = blockIdx.x * 64 + (threadIdx.x & 63);
    const int slice = threadIdx.x >> 6;
    const T* src = in + li * sIi;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (col < N) {
        int64_t r = slice;
        for (; r + 12 < rows; r += 16) {
            s0 += Elem<T>::to(__builtin_nontemporal_load(src + r * ld + col));
            s1 += Elem<T>::to(__builtin_nontemporal_load(src + (r + 4) * ld + col));
            s2 += Elem<T>::to(__builtin_nontemporal_load(src + (r + 8) * ld + col));
            s3 += Elem<T>::to(__builtin_nontemporal_load(src + (r + 12) * ld + col));
        }
        for (; r < rows; r += 4) s0 += Elem<T>::to(src[r * ld + col]);
    }
    __shared__ float sh[4][64];
    sh[slice][threadIdx.x & 63] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (slice == 0 && col < N)
        out[li * sOi + col] = (sh[0][threadIdx.x] + sh[1][threadIdx.x]) + (sh[2][threadIdx.x] + sh[3][threadIdx.x]);
}

hipError_t launch_colsum(int precision, const void* in, int64_t ld, int64_t sIi, int64_t rows, int N,
                         float* out, int64_t sOi, int L, const LearnerMap& lmap, hipStream_t s) {
    if (L < 1 || L > 128) return hipErrorInvalidValue;
    dim3 grid((unsigned)((N + 63) / 64), (unsigned)L);
    if (precision == 0)
        hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, s, (const float*)in, ld, sIi, rows, N, out, sOi, lmap);
    else
        hipLaunchKernelGGL(colsum_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t*)in, ld, sIi, rows, N, out, sOi, lmap);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void zero_kernel(float* dst, int64_t sDi, int64_t n, LearnerMap lmap) {
    float* p = dst + lmap.idx[blockIdx.y] * sDi;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) p[i] = 0.f;
}

hipError_t launch_zero(float* dst, int64_t sDi, int64_t n, int L, const LearnerMap& lmap, hipStream_t s) {
    if (L < 1 || L > 128 || n < 1) return hipErrorInvalidValue;
    int64_t blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)blocks, (unsigned)L), dim3(256), 0, s, dst, sDi, n, lmap);
    return hipGetLastError();
}

}  // namespace adpsgd
