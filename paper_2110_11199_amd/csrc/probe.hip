// Measurement probes: what this device attains on the two resources the kernels of the library are bound by,
// so that a kernel's rate can be set against an ATTAINED peak besides the published one.
//   mfma_peak_kernel    a register-only loop of v_mfma_f32_32x32x16_bf16 (the instruction of the GEMM kernels),
//                       eight independent accumulators per wave: the matrix pipe with nothing else in its way
//   stream_probe_kernel a pure streaming pass with a chosen mix of fp32 reads, fp32 writes and bf16 writes per
//                       position, float4 per thread and stream, non-temporal, the access pattern of the update kernels:
//                       1:0:0 a read-only stream, 1:1:0 a copy, 2:1:0 the pairwise update (x, g in; x out),
//                       2:1:1 the update that also writes the bf16 copy of the model (8 bytes read : 6 written)
#include "kernels.hpp"

namespace adpsgd {

__global__ __launch_bounds__(256) void mfma_peak_kernel(float* out, int iters) {
    f32x16_t acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    const uint4 a = make_uint4(threadIdx.x, 1, 2, 3), b = make_uint4(4, 5, 6, threadIdx.x);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

typedef float pvf4_t __attribute__((ext_vector_type(4)));
typedef uint32_t pvu2_t __attribute__((ext_vector_type(2)));

// Streams are consecutive slices of one buffer, `pitch` bytes apart: first the R read streams, then the W4 fp32
// write streams, then the W2 bf16 write streams.  Position e of every stream belongs to one thread.
template <int R, int W4, int W2>
__global__ __launch_bounds__(256) void stream_probe_kernel(char* buf, int64_t pitch, int64_t n4, float* sink) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n4) return;
    pvf4_t s = __builtin_nontemporal_load((const pvf4_t*)buf + e);
#pragma unroll 8
    for (int j = 1; j < R; ++j) s += __builtin_nontemporal_load((const pvf4_t*)(buf + j * pitch) + e);
#pragma unroll 8
    for (int j = 0; j < W4; ++j) __builtin_nontemporal_store(s, (pvf4_t*)(buf + (R + j) * pitch) + e);
#pragma unroll 8
    for (int j = 0; j < W2; ++j) {
        pvu2_t o;
        o.x = pack_bf16(s.x, s.y); o.y = pack_bf16(s.z, s.w);
        __builtin_nontemporal_store(o, (pvu2_t*)(buf + (R + W4 + j) * pitch) + e);
    }
    if (W4 + W2 == 0 && s.x == 123.456f && s.y == -7.f) sink[0] = s.z;      // keeps the loads of a read-only pass alive
}

// Idles until `ticks` of the 100 MHz wall clock have passed, sleeping between looks at the clock: the loop ends by
// construction (the clock advances on its own).
__global__ __launch_bounds__(64) void delay_kernel(unsigned long long ticks) {
    const unsigned long long t0 = wall_clock64();
    while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(64);
}

hipError_t launch_delay(unsigned long long ticks, hipStream_t s) {
    hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, s, ticks);
    return hipGetLastError();
}

hipError_t launch_mfma_peak(float* out, int blocks, int iters, hipStream_t s) {
    if (!out || blocks < 1 || iters < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(mfma_peak_kernel, dim3((unsigned)blocks), dim3(256), 0, s, out, iters);
    return hipGetLastError();
}

hipError_t launch_stream_probe(int reads, int writes_f32, int writes_bf16, void* buf, int64_t pitch, int64_t elems, hipStream_t s) {
    if (!buf || elems < 4 || elems % 4 || pitch % 16 || pitch < elems * 4 || (uintptr_t)buf % 16) return hipErrorInvalidValue;
    const int64_t n4 = elems / 4;
    const dim3 grid((unsigned)((n4 + 255) / 256)), block(256);
    char* b = (char*)buf;
    float* sink = (float*)buf;
    const int key = reads * 10000 + writes_f32 * 100 + writes_bf16;
    switch (key) {
        case 10000: hipLaunchKernelGGL((stream_probe_kernel<1, 0, 0>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 10100: hipLaunchKernelGGL((stream_probe_kernel<1, 1, 0>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 20100: hipLaunchKernelGGL((stream_probe_kernel<2, 1, 0>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 20101: hipLaunchKernelGGL((stream_probe_kernel<2, 1, 1>), grid, block, 0, s, b, pitch, n4, sink); break;
        // the same mixes with more positions' worth of streams owned by one thread (one thread of the update kernels
        // owns an element index of 2 learners (pairwise) or of all L learners (global mean, ring neighbours))
        case 40200: hipLaunchKernelGGL((stream_probe_kernel<4, 2, 0>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 40202: hipLaunchKernelGGL((stream_probe_kernel<4, 2, 2>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 80404: hipLaunchKernelGGL((stream_probe_kernel<8, 4, 4>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 160808: hipLaunchKernelGGL((stream_probe_kernel<16, 8, 8>), grid, block, 0, s, b, pitch, n4, sink); break;
        case 321616: hipLaunchKernelGGL((stream_probe_kernel<32, 16, 16>), grid, block, 0, s, b, pitch, n4, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace adpsgd
