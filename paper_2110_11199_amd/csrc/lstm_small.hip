// Per-time-step LSTM kernels for small batches (at most 32 segments per learner).
//
// Same operations as lstm.hip (one launch = one frame of one layer for all learners and directions,
// gate non-linearities / cell update / cell backward fused behind the recurrent product), but laid
// out for launches that are bound by latency, not by bytes: with a batch of 32 or fewer rows the
// 32-row tiles of lstm.hip make only L*D*H/128 workgroups (32 on 256 compute units for 8 learners of
// 256 units), and every wave walks the whole contraction in 16 dependent load -> LDS -> MFMA stages.
//
// Here a workgroup of 8 waves owns a 32 x 32 (batch rows x hidden units) tile and SPLITS THE
// CONTRACTION over its waves: wave w takes the k-chunks w, w+8, w+16, ...  Every wave loads its MFMA
// fragments straight from global memory into registers (no LDS staging, no barrier in the loop, all
// loads of up to four or eight chunks in flight at once; the operands are a few MB and live in L2),
// the eight partial products are added through LDS in a fixed order (wave 0, 1, ..., 7), and the
// epilogue is spread over the waves too: wave w finishes accumulator elements 2w and 2w+1 of every
// lane, i.e. 2 of the 16 batch rows a lane holds.
//
// MFMA operand mapping as in gemm_core.hpp: lane (r = lane%32, g = lane/32) supplies the 16 bytes of
// operand row r at k = chunk*CH + g*CH/2; accumulator element i of a lane is row 8*(i/4) + 4*g + i%4,
// column lane%32 of the 32x32 tile.
#include "gemm_core.hpp"
#include "kernels.hpp"

namespace adpsgd {
namespace {

constexpr int kKS = 8;                       // waves of a workgroup = parts the contraction is split in

__device__ inline uint4 zero4_() { return make_uint4(0u, 0u, 0u, 0u); }

// 16 bytes of a K-contiguous operand row
template <typename T> __device__ inline uint4 frag_kc_(const T* row, int k, bool ok) {
    return ok ? *(const uint4*)(row + k) : zero4_();
}
// the same fragment of an operand stored rows-contiguous: elements k, k+1, ... of column `col` lie ld apart
__device__ inline uint4 frag_mc_(const float* col, int64_t ld, int k, bool ok) {
    if (!ok) return zero4_();
    const float* p = col + (int64_t)k * ld;
    return make_uint4(__builtin_bit_cast(uint32_t, p[0]), __builtin_bit_cast(uint32_t, p[ld]),
                      __builtin_bit_cast(uint32_t, p[2 * ld]), __builtin_bit_cast(uint32_t, p[3 * ld]));
}
__device__ inline uint4 frag_mc_(const bf16_t* col, int64_t ld, int k, bool ok) {
    if (!ok) return zero4_();
    const bf16_t* p = col + (int64_t)k * ld;
    uint32_t w[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = (uint32_t)p[(2 * j) * ld] | ((uint32_t)p[(2 * j + 1) * ld] << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

__device__ inline int acc_row_(int i, int g) { return 8 * (i >> 2) + 4 * g + (i & 3); }

// Sum of the eight partial values of accumulator slot `slot` (0..NS-1) of this lane, wave 0 first.
template <int NS> __device__ inline float reduce_slot_(const float* red, int slot, int lane) {
    float v = red[(0 * NS + slot) * 64 + lane];
#pragma unroll
    for (int w = 1; w < kKS; ++w) v += red[(w * NS + slot) * 64 + lane];
    return v;
}

// ---- forward ------------------------------------------------------------------------------------
//   a = W_x x_t + b + W_h h_{t'}     i,f,o = sigmoid(a), g = tanh(a)     c_t = f c_{t'} + i g     h_t = o tanh(c_t)
template <typename T>
__global__ __launch_bounds__(64 * kKS) void rec_forward_small_kernel(RecDesc p) {
    constexpr int EL = 16 / (int)sizeof(T), CH = 2 * EL, UN = 4;
    __shared__ float red[kKS * 64 * 64];                       // [wave][gate*16 + i][lane]
    const int D = p.D, H = p.H, B = p.B;
    const int li = p.lmap.idx[blockIdx.x / D], d = blockIdx.x % D;
    const int t = d == 0 ? p.step : p.T - 1 - p.step;
    const int tp = d == 0 ? t - 1 : t + 1;
    const int u0 = blockIdx.y * 32, b0 = blockIdx.z * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 31, g = lane >> 5;
    const int64_t DH = (int64_t)D * H, G4 = (int64_t)D * 4 * H;
    const int u = u0 + r;
    float* gates = p.gates + li * p.sGi;
    float* cbuf = p.c + li * p.sCi + (int64_t)d * p.T * B * H;
    T* y = (T*)p.y + li * p.sYi;

    // inputs of this lane's part of the epilogue, requested before the product
    float a_in[2][4], c_prev[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int row = b0 + acc_row_(2 * wave + e, g);
        const bool ok = row < B && u < H;
        const float* gp = gates + ((int64_t)t * B + (ok ? row : 0)) * G4 + (int64_t)d * 4 * H + (ok ? u : 0);
#pragma unroll
        for (int q = 0; q < 4; ++q) a_in[e][q] = ok ? gp[(int64_t)q * H] : 0.f;
        c_prev[e] = (ok && p.step > 0) ? cbuf[((int64_t)tp * B + row) * H + u] : 0.f;
    }

    float s[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    if (p.step > 0) {
        f32x16_t acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[q][i] = 0.f;
        const bool ok_a = b0 + r < B, ok_b = u < H;
        const T* arow = y + ((int64_t)tp * B + (ok_a ? b0 + r : 0)) * DH + (int64_t)d * H;
        const T* wrow = (const T*)p.wh + li * p.sWi + d * p.sWd + (int64_t)(ok_b ? u : 0) * H;   // gate q: + q*H*H
        const int nch = (H + CH - 1) / CH;
        for (int c0 = wave; c0 < nch; c0 += kKS * UN) {
            uint4 af[UN], bf[UN][4];
#pragma unroll
            for (int j = 0; j < UN; ++j) {
                const int k = (c0 + j * kKS) * CH + g * EL;
                const bool ok = k < H;                          // H is a multiple of EL: a fragment is whole or absent
                af[j] = frag_kc_(arow, k, ok && ok_a);
#pragma unroll
                for (int q = 0; q < 4; ++q) bf[j][q] = frag_kc_(wrow + (int64_t)q * H * H, k, ok && ok_b);
            }
#pragma unroll
            for (int j = 0; j < UN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) mma_chunk<T>(acc[q], af[j], bf[j][q]);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 16; ++i) red[((wave * 64) + q * 16 + i) * 64 + lane] = acc[q][i];
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
            for (int q = 0; q < 4; ++q) s[e][q] = reduce_slot_<64>(red, q * 16 + 2 * wave + e, lane);
    }

#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int row = b0 + acc_row_(2 * wave + e, g);
        if (row >= B || u >= H) continue;
        const float ig = sigmoidf_(a_in[e][0] + s[e][0]);
        const float fg = sigmoidf_(a_in[e][1] + s[e][1]);
        const float gg = tanhf_(a_in[e][2] + s[e][2]);
        const float og = sigmoidf_(a_in[e][3] + s[e][3]);
        const float cc = fg * c_prev[e] + ig * gg;
        const float hv = og * tanhf_(cc);
        float* gp = gates + ((int64_t)t * B + row) * G4 + (int64_t)d * 4 * H + u;
        gp[0] = ig; gp[H] = fg; gp[2 * (int64_t)H] = gg; gp[3 * (int64_t)H] = og;
        cbuf[((int64_t)t * B + row) * H + u] = cc;
        y[((int64_t)t * B + row) * DH + (int64_t)d * H + u] = Elem<T>::from(hv);
    }
}

// ---- backward -----------------------------------------------------------------------------------
//   dh_t = dY_t + da_{t''} W_h  (t'' = the frame handled by the previous launch)
//   do = dh tanh(c_t)            dc = dc_rec + dh o (1 - tanh^2 c_t)
//   di = dc g, dg = dc i, df = dc c_{t'}, dc_rec <- dc f
//   da = (di i(1-i), df f(1-f), dg (1-g^2), do o(1-o))
template <typename T>
__global__ __launch_bounds__(64 * kKS) void rec_backward_small_kernel(RecDesc p) {
    constexpr int EL = 16 / (int)sizeof(T), CH = 2 * EL, UN = sizeof(T) == 4 ? 8 : 4;
    __shared__ float red[kKS * 16 * 64];                       // [wave][i][lane]
    __shared__ float cred[kKS * 32 * 4];                       // [wave][column][gate]: column sums of da
    const int D = p.D, H = p.H, B = p.B;
    const int li = p.lmap.idx[blockIdx.x / D], d = blockIdx.x % D;
    const int t = d == 0 ? p.T - 1 - p.step : p.step;          // reverse of the forward processing order
    const int tn = d == 0 ? t + 1 : t - 1;                     // frame handled by the previous launch
    const int tp = d == 0 ? t - 1 : t + 1;                     // frame the forward pass processed before t
    const bool has_prev = tp >= 0 && tp < p.T;
    const int u0 = blockIdx.y * 32, b0 = blockIdx.z * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, r = lane & 31, g = lane >> 5;
    const int64_t DH = (int64_t)D * H, G4 = (int64_t)D * 4 * H;
    const int u = u0 + r;
    const float* gates = p.gates + li * p.sGi;
    const float* cbuf = p.c + li * p.sCi + (int64_t)d * p.T * B * H;
    const float* dy = p.dy + li * p.sDYi;
    float* dcb = p.dc + li * p.sDCi + (int64_t)d * B * H;
    T* da = (T*)p.da + li * p.sDAi;

    float dyv[2], gv[2][4], cv[2], cp[2], dcr[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int row = b0 + acc_row_(2 * wave + e, g);
        const bool ok = row < B && u < H;
        const int64_t m = (int64_t)t * B + (ok ? row : 0);
        const int uu = ok ? u : 0;
        const float* gp = gates + m * G4 + (int64_t)d * 4 * H + uu;
        dyv[e] = ok ? dy[m * DH + (int64_t)d * H + uu] : 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) gv[e][q] = ok ? gp[(int64_t)q * H] : 0.f;
        cv[e] = ok ? cbuf[m * H + uu] : 0.f;
        cp[e] = (ok && has_prev) ? cbuf[((int64_t)tp * B + row) * H + uu] : 0.f;
        dcr[e] = (ok && p.step > 0) ? dcb[(int64_t)row * H + uu] : 0.f;
    }

    float s[2] = {0.f, 0.f};
    if (p.step > 0) {
        f32x16_t acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
        const bool ok_a = b0 + r < B, ok_b = u < H;
        const T* arow = da + ((int64_t)tn * B + (ok_a ? b0 + r : 0)) * G4 + (int64_t)d * 4 * H;
        const T* wcol = (const T*)p.wh + li * p.sWi + d * p.sWd + (ok_b ? u : 0);   // W_h[k][u] at wcol[k*H]
        const int K = 4 * H, nch = K / CH;                     // 4H is a multiple of CH (H is a multiple of 4)
        for (int c0 = wave; c0 < nch; c0 += kKS * UN) {
            uint4 af[UN], bf[UN];
#pragma unroll
            for (int j = 0; j < UN; ++j) {
                const int k = (c0 + j * kKS) * CH + g * EL;
                const bool ok = k < K;
                af[j] = frag_kc_(arow, k, ok && ok_a);
                bf[j] = frag_mc_(wcol, (int64_t)H, k, ok && ok_b);
            }
#pragma unroll
            for (int j = 0; j < UN; ++j) mma_chunk<T>(acc, af[j], bf[j]);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) red[(wave * 16 + i) * 64 + lane] = acc[i];
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 2; ++e) s[e] = reduce_slot_<16>(red, 2 * wave + e, lane);
    }

    float cs[4] = {0.f, 0.f, 0.f, 0.f};                        // sums of the four da values over this lane's rows
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int row = b0 + acc_row_(2 * wave + e, g);
        // rows past the batch and units past H: all gates were read as 0, so all four results are 0
        const float dh = dyv[e] + s[e];
        const float ig = gv[e][0], fg = gv[e][1], g2 = gv[e][2], og = gv[e][3];
        const float tc = tanhf_(cv[e]);
        const float dov = dh * tc;
        const float dcv = dcr[e] + dh * og * (1.f - tc * tc);
        const float di = dcv * g2, dg = dcv * ig, df = dcv * cp[e];
        const float a0 = di * ig * (1.f - ig), a1 = df * fg * (1.f - fg), a2 = dg * (1.f - g2 * g2), a3 = dov * og * (1.f - og);
        cs[0] += a0; cs[1] += a1; cs[2] += a2; cs[3] += a3;
        if (row >= B || u >= H) continue;
        dcb[(int64_t)row * H + u] = dcv * fg;
        T* dp = da + ((int64_t)t * B + row) * G4 + (int64_t)d * 4 * H + u;
        dp[0] = Elem<T>::from(a0); dp[H] = Elem<T>::from(a1);
        dp[2 * (int64_t)H] = Elem<T>::from(a2); dp[3 * (int64_t)H] = Elem<T>::from(a3);
    }
    // Bias gradient: column sums of da over the 32 rows of the tile in a fixed order (the two rows of a lane,
    // the lane pair, then the waves 0..7), written as one row of partial sums per (frame, batch tile).
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float v = cs[q] + __shfl_xor(cs[q], 32);
        if (lane < 32) cred[(wave * 32 + r) * 4 + q] = v;
    }
    __syncthreads();
    if (threadIdx.x < 128) {
        const int col = threadIdx.x & 31, q = threadIdx.x >> 5;
        float sum = cred[col * 4 + q];
#pragma unroll
        for (int w = 1; w < kKS; ++w) sum += cred[(w * 32 + col) * 4 + q];
        float* out = p.dbp + li * p.sDBi + ((int64_t)t * gridDim.z + blockIdx.z) * G4 + (int64_t)d * 4 * H;
        if (u0 + col < H) out[(int64_t)q * H + u0 + col] = sum;
    }
}

}  // namespace

// At most 32 batch rows (one row tile, so the partial bias sums keep one row per frame as
// rec_backward_batch_tiles says), whole 16-byte fragments, 16-byte aligned operand rows.
bool rec_small_supported(const RecDesc& d) {
    const int el = d.precision ? 8 : 4;
    const int64_t m = el;
    return d.direct && d.B >= 1 && d.B <= 32 && d.H % el == 0 && d.L >= 1 && d.L <= 128 && d.D >= 1 && d.D <= 2 &&
           (uintptr_t)d.wh % 16 == 0 && d.sWi % m == 0 && d.sWd % m == 0 && (uintptr_t)d.y % 16 == 0 && d.sYi % m == 0 &&
           (d.da == nullptr || ((uintptr_t)d.da % 16 == 0 && d.sDAi % m == 0));
}

hipError_t launch_rec_small(const RecDesc& d, bool backward, hipStream_t s) {
    if (!rec_small_supported(d) || d.step < 0 || d.step >= d.T) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(d.L * d.D), (unsigned)((d.H + 31) / 32), (unsigned)((d.B + 31) / 32));
    const dim3 block(64 * kKS);
    if (d.precision == 0) {
        if (backward) hipLaunchKernelGGL(rec_backward_small_kernel<float>, grid, block, 0, s, d);
        else hipLaunchKernelGGL(rec_forward_small_kernel<float>, grid, block, 0, s, d);
    } else {
        if (backward) hipLaunchKernelGGL(rec_backward_small_kernel<bf16_t>, grid, block, 0, s, d);
        else hipLaunchKernelGGL(rec_forward_small_kernel<bf16_t>, grid, block, 0, s, d);
    }
    return hipGetLastError();
}

}  // namespace adpsgd
