// Grouped MFMA GEMM kernels: the time-batched GEMMs of the LSTM gradient
// (input projections, output layers, weight gradients, input gradients).
#include <type_traits>
#include "gemm_core.hpp"
#include "kernels.hpp"

namespace adpsgd {

template <typename T, bool AKC, bool BKC, bool CELEM, int VB>
__global__ __launch_bounds__(256) void gemm_kernel(GemmDesc p) {
    typedef typename std::conditional<AKC, KcSrc<T>, McSrc<T>>::type ASrc;
    typedef typename std::conditional<BKC, KcSrc<T>, McSrc<T>>::type BSrc;
    typedef GemmCore<T, ASrc, BSrc, 2, 2, 2, 2, VB> Core;
    __shared__ __attribute__((aligned(16))) char lds[Core::LDS_BYTES];

    const int tiles_m = (p.M + Core::BM - 1) / Core::BM;
    const int tm = blockIdx.x % tiles_m, tn = blockIdx.x / tiles_m;
    const int gi = blockIdx.y / p.groupsD, gd = blockIdx.y % p.groupsD;
    const int m0 = tm * Core::BM, n0 = tn * Core::BN;
    const T* A = (const T*)p.A + gi * p.sAi + gd * p.sAd;
    const T* B = (const T*)p.B + gi * p.sBi + gd * p.sBd;

    ASrc a; BSrc b;
    if constexpr (AKC) { a.base = A + (int64_t)m0 * p.lda; } else { a.base = A + m0; }
    a.ld = p.lda; a.R = p.M - m0;
    if constexpr (BKC) { b.base = B + (int64_t)n0 * p.ldb; } else { b.base = B + n0; }
    b.ld = p.ldb; b.R = p.N - n0;

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    Core::run(acc, a, b, p.K, lds);

    const float* bias = p.bias ? p.bias + gi * p.sBiasI + gd * p.sBiasD : nullptr;
    const int64_t coff = gi * p.sCi + gd * p.sCd;
#pragma unroll
    for (int fn = 0; fn < 2; ++fn) {
        const int col = n0 + Core::acc_col(fn);
        if (col >= p.N) continue;
        const float bv = bias ? bias[col] : 0.f;
#pragma unroll
        for (int fm = 0; fm < 2; ++fm) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = m0 + Core::acc_row(fm, i);
                if (row >= p.M) continue;
                const float v = acc[fm][fn][i] + bv;
                const int64_t o = coff + (int64_t)row * p.ldc + col;
                if constexpr (CELEM) ((T*)p.C)[o] = Elem<T>::from(v);
                else ((float*)p.C)[o] = v;
            }
        }
    }
}

template <typename T, bool AKC, bool BKC, bool CELEM, int VB>
static hipError_t launch_t(const GemmDesc& d, hipStream_t s) {
    const int tiles_m = (d.M + 127) / 128, tiles_n = (d.N + 127) / 128;
    dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)(d.groupsI * d.groupsD));
    hipLaunchKernelGGL((gemm_kernel<T, AKC, BKC, CELEM, VB>), grid, dim3(256), 0, s, d);
    return hipGetLastError();
}

template <typename T, int VB>
static hipError_t launch_layout(const GemmDesc& d, hipStream_t s) {
    const int key = (d.a_kc ? 4 : 0) | (d.b_kc ? 2 : 0) | (d.c_elem ? 1 : 0);
    switch (key) {
        case 0: return launch_t<T, false, false, false, VB>(d, s);
        case 1: return launch_t<T, false, false, true, VB>(d, s);
        case 2: return launch_t<T, false, true, false, VB>(d, s);
        case 3: return launch_t<T, false, true, true, VB>(d, s);
        case 4: return launch_t<T, true, false, false, VB>(d, s);
        case 5: return launch_t<T, true, false, true, VB>(d, s);
        case 6: return launch_t<T, true, true, false, VB>(d, s);
        default: return launch_t<T, true, true, true, VB>(d, s);
    }
}

static bool aligned_to(const void* p, int64_t ld, int64_t s1, int64_t s2, int esz, int bytes) {
    return ((uintptr_t)p % bytes == 0) && ((ld * esz) % bytes == 0) && ((s1 * esz) % bytes == 0) &&
           ((s2 * esz) % bytes == 0);
}

hipError_t launch_gemm(const GemmDesc& d, hipStream_t s) {
    if (d.M < 1 || d.N < 1 || d.K < 1 || d.groupsI < 1 || d.groupsD < 1) return hipErrorInvalidValue;
    const int esz = d.precision ? 2 : 4;
    const int quad = 4 * esz;    // every operand must allow loads of 4 elements
    if (!aligned_to(d.A, d.lda, d.sAi, d.sAd, esz, quad) || !aligned_to(d.B, d.ldb, d.sBi, d.sBd, esz, quad))
        return hipErrorInvalidValue;
    if (d.precision == 0) return launch_layout<float, 16>(d, s);
    bool wide = true;
    if (d.a_kc && !aligned_to(d.A, d.lda, d.sAi, d.sAd, esz, 16)) wide = false;
    if (d.b_kc && !aligned_to(d.B, d.ldb, d.sBi, d.sBd, esz, 16)) wide = false;
    return wide ? launch_layout<bf16_t, 16>(d, s) : launch_layout<bf16_t, 8>(d, s);
}

}  // namespace adpsgd
