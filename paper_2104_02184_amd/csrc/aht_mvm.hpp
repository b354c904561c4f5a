// Analog matrix-vector product, Eq. (1) of arXiv 2104.02184, and its transposed form for the
// backward pass (Sec. 3):  y_i = f_adc( sum_j (w_ij + s_w xi_ij)(f_dac(x_j) + s_inp xi_j) + s_out xi_i ).
//
//   k_mvm_prepare  per input vector: dynamic scaling alpha = max|x|, DAC (clip, round to the
//                  input grid), input noise, and |xq|_2 for the output-referred weight noise
//   k_mvm_gemm     Z = Xq * W^T (forward) or Xq * W (backward) on the fp32 matrix cores
//                  (v_mfma_f32_32x32x2_f32, 64x64 block tiles staged through LDS), with the
//                  epilogue fused: weight noise, output noise, ADC (clip, round to the output
//                  grid), rescale by alpha.
// Random numbers: input j of vector b takes Gaussian (j & 3) of block (j >> 2, b, call counter,
// tag 7 forward / 9 backward); output i takes Gaussians 2(i & 1) (output noise) and 2(i & 1) + 1
// (weight noise) of block (i >> 1, b, call counter, tag 8 / 10).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "aht_rng.hpp"

namespace aht {

struct IoArgs {
    float inp_res, inp_bound, inp_noise, w_noise, out_noise, out_res, out_bound;
    int noise_management;
};

// one workgroup per input vector
__global__ void __launch_bounds__(256)
k_mvm_prepare(const float* __restrict__ x, int K, IoArgs io, uint32_t k0, uint32_t k1, uint32_t t, uint32_t tag,
              float* __restrict__ xq, float* __restrict__ alpha_out, float* __restrict__ norm_out)
{
    __shared__ float red[4];
    __shared__ double redd[4];
    const int b = blockIdx.x;
    const float* xr = x + (size_t)b * K;
    float alpha = 1.0f;
    if (io.noise_management) {
        float m = 0.0f;
        for (int j = threadIdx.x; j < K; j += 256) {
            const float a = fabsf(xr[j]);
            m = fmaxf(m, (a < __builtin_inff()) ? a : 0.0f);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
        __syncthreads();
        alpha = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    }
    double part = 0.0;
    for (int g = threadIdx.x; g * 4 < K; g += 256) {      // four inputs share one Philox block
        float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (io.inp_noise > 0.0f) gauss4_fast(k0, k1, (uint32_t)g, (uint32_t)b, t, tag, z);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int j = g * 4 + e;
            if (j < K) {
                float v = xr[j];
                if (!(fabsf(v) < __builtin_inff()) || alpha == 0.0f) v = 0.0f;
                float xh = (alpha != 0.0f) ? v / alpha : 0.0f;
                xh = fminf(fmaxf(xh, -io.inp_bound), io.inp_bound);
                if (io.inp_res > 0.0f) xh = rintf(xh / io.inp_res) * io.inp_res;
                if (io.inp_noise > 0.0f) {
                    const float nz = io.inp_noise * z[e];
                    xh = xh + nz;
                }
                xq[(size_t)b * K + j] = xh;
                part += (double)xh * (double)xh;
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
    if ((threadIdx.x & 63) == 0) redd[threadIdx.x >> 6] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
        alpha_out[b] = alpha;
        norm_out[b] = (float)sqrt(redd[0] + redd[1] + redd[2] + redd[3]);
    }
}

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Z[M][N] = A[M][K] * Bm, Bm[k][n] = TRANS ? Wm[k*ldw + n] : Wm[n*ldw + k]; fused analog epilogue.
// Block tile 64 x 64, K step 32; four waves, each a 32 x 32 tile of v_mfma_f32_32x32x2_f32.
template <bool TRANS>
__global__ void __launch_bounds__(256)
k_mvm_gemm(const float* __restrict__ A, const float* __restrict__ Wm, int M, int N, int K, int ldw,
           const float* __restrict__ alpha, const float* __restrict__ norm, IoArgs io, uint32_t k0, uint32_t k1,
           uint32_t t, uint32_t tag, float* __restrict__ y, float* __restrict__ pre)
{
    constexpr int BM = 64, BN = 64, BK = 32, LD = 65;      // LD: padded row length of the k-major LDS tiles
    __shared__ float As[2][BK][LD];
    __shared__ float Bs[2][BK][LD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // staging: every thread moves two groups of four consecutive k (or n) values per operand
    float ra[2][4], rb[2][4];
    // 16-byte loads when every row start and every group of four is aligned and inside the matrix
    const bool vec_a = (K & 3) == 0, vec_w = (ldw & 3) == 0 && (TRANS ? (N & 3) == 0 : (K & 3) == 0);
    auto fetch = [&](int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            {   // A: rows m, k contiguous
                const int row = (tid >> 3) + 32 * h, kk = kc + (tid & 7) * 4;
                const int m = m0 + row;
                if (vec_a && m < M && kk + 3 < K) {
                    const float4 v = *(const float4*)(A + (size_t)m * K + kk);
                    ra[h][0] = v.x; ra[h][1] = v.y; ra[h][2] = v.z; ra[h][3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        ra[h][e] = (m < M && kk + e < K) ? A[(size_t)m * K + kk + e] : 0.0f;
                }
            }
            if (!TRANS) {   // W[n][k], k contiguous
                const int row = (tid >> 3) + 32 * h, kk = kc + (tid & 7) * 4;
                const int n = n0 + row;
                if (vec_w && n < N && kk + 3 < K) {
                    const float4 v = *(const float4*)(Wm + (size_t)n * ldw + kk);
                    rb[h][0] = v.x; rb[h][1] = v.y; rb[h][2] = v.z; rb[h][3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        rb[h][e] = (n < N && kk + e < K) ? Wm[(size_t)n * ldw + kk + e] : 0.0f;
                }
            } else {        // W[k][n], n contiguous
                const int krow = (tid >> 4) + 16 * h, nn = n0 + (tid & 15) * 4;
                const int kk = kc + krow;
                if (vec_w && kk < K && nn + 3 < N) {
                    const float4 v = *(const float4*)(Wm + (size_t)kk * ldw + nn);
                    rb[h][0] = v.x; rb[h][1] = v.y; rb[h][2] = v.z; rb[h][3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        rb[h][e] = (kk < K && nn + e < N) ? Wm[(size_t)kk * ldw + nn + e] : 0.0f;
                }
            }
        }
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int row = (tid >> 3) + 32 * h, kq = (tid & 7) * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) As[buf][kq + e][row] = ra[h][e];
            if (!TRANS) {
#pragma unroll
                for (int e = 0; e < 4; ++e) Bs[buf][kq + e][row] = rb[h][e];
            } else {
                const int krow = (tid >> 4) + 16 * h, nq = (tid & 15) * 4;
#pragma unroll
                for (int e = 0; e < 4; ++e) Bs[buf][krow][nq + e] = rb[h][e];
            }
        }
    };

    floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    fetch(0);
    stage(0);
    __syncthreads();
    const int nchunks = (K + BK - 1) / BK;
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < nchunks) fetch((c + 1) * BK);           // global loads in flight during the MFMAs
        const int arow = wm * 32 + (lane & 31), brow = wn * 32 + (lane & 31), kh = lane >> 5;
#pragma unroll
        for (int s = 0; s < BK / 2; ++s) {
            const float av = As[buf][2 * s + kh][arow];
            const float bv = Bs[buf][2 * s + kh][brow];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
        }
        if (c + 1 < nchunks) stage(buf ^ 1);
        __syncthreads();
    }

    // epilogue: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32 of the wave's tile
    const int n = n0 + wn * 32 + (lane & 31);
    const bool noisy = (io.w_noise > 0.0f) || (io.out_noise > 0.0f);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (m < M && n < N) {
            float z = acc[r];
            if (noisy) {
                float g[4];
                gauss4_fast(k0, k1, (uint32_t)n >> 1, (uint32_t)m, t, tag, g);
                const float g_out = (n & 1) ? g[2] : g[0], g_w = (n & 1) ? g[3] : g[1];
                float wn_ = io.w_noise * norm[m];
                wn_ = wn_ * g_w;
                z = z + wn_;
                const float on = io.out_noise * g_out;
                z = z + on;
            }
            if (pre) pre[(size_t)m * N + n] = z;
            float q = fminf(fmaxf(z, -io.out_bound), io.out_bound);
            if (io.out_res > 0.0f) q = rintf(q / io.out_res) * io.out_res;
            y[(size_t)m * N + n] = alpha[m] * q;
        }
    }
}

}  // namespace aht
