// Analog matrix-vector product, Eq. (1) of arXiv 2104.02184, and its transposed form for the
// backward pass (Sec. 3):  y_i = f_adc( sum_j (w_ij + s_w xi_ij)(f_dac(x_j) + s_inp xi_j) + s_out xi_i ).
//
//   k_mvm_prepare  per input vector: dynamic scaling alpha = max|x|, DAC (clip, round to the
//                  input grid), input noise, and |xq|_2 for the output-referred weight noise
//   k_mvm_gemm     Z = Xq * W^T (forward) or Xq * W (backward) on the fp32 matrix cores
//                  (v_mfma_f32_32x32x2_f32, 64x64 block tiles staged through LDS, the K range
//                  split over several workgroups when there are few tiles)
//   epilogue       weight noise, output noise, ADC (clip, round to the output grid), rescale
//                  by alpha: fused into k_mvm_gemm, or k_mvm_epilogue after a K-split product
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

// one workgroup of 1024 lanes per input vector; a lane handles groups of four neighbouring
// inputs (one Philox block each), with 16-byte accesses when `vec` (K a multiple of 4, aligned)
__global__ void __launch_bounds__(1024)
k_mvm_prepare(const float* __restrict__ x, int K, int vec, IoArgs io, uint32_t k0, uint32_t k1, uint32_t t,
              uint32_t tag, float* __restrict__ xq, float* __restrict__ alpha_out, float* __restrict__ norm_out,
              uint16_t* __restrict__ codes, int nplanes, size_t plane_elems)
{
    __shared__ float red[16];
    __shared__ double redd[16];
    const int b = blockIdx.x, tid = threadIdx.x;
    const float* xr = x + (size_t)b * K;
    float* qr = xq + (size_t)b * K;
    const int groups = (K + 3) >> 2;
    auto load_group = [&](int g, float (&v)[4]) __attribute__((always_inline)) {
        if (vec) {
            const float4 q = *(const float4*)(xr + 4 * (size_t)g);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (4 * g + e < K) ? xr[4 * (size_t)g + e] : 0.0f;
        }
    };
    // up to 4096 inputs every thread has one group of four: read once, kept for both passes
    const bool single = groups <= 1024;
    float kept[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (single && tid < groups) load_group(tid, kept);
    float alpha = 1.0f;
    if (io.noise_management) {
        float m = 0.0f;
        for (int g = tid; g < groups; g += 1024) {
            float v[4];
            if (single) { v[0] = kept[0]; v[1] = kept[1]; v[2] = kept[2]; v[3] = kept[3]; }
            else load_group(g, v);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = fabsf(v[e]);
                m = fmaxf(m, (a < __builtin_inff()) ? a : 0.0f);
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
        if ((tid & 63) == 0) red[tid >> 6] = m;
        __syncthreads();
        alpha = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) alpha = fmaxf(alpha, red[w]);
    }
    double part = 0.0;
    for (int g = tid; g < groups; g += 1024) {            // four inputs share one Philox block
        float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (io.inp_noise > 0.0f) gauss4_fast(k0, k1, (uint32_t)g, (uint32_t)b, t, tag, z);
        float v[4], o[4];
        uint32_t cbits[4] = {0u, 0u, 0u, 0u}, mbits[4] = {0u, 0u, 0u, 0u}, lbits[4] = {0u, 0u, 0u, 0u};
        if (single) { v[0] = kept[0]; v[1] = kept[1]; v[2] = kept[2]; v[3] = kept[3]; }
        else load_group(g, v);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float u = v[e];
            if (!(fabsf(u) < __builtin_inff()) || alpha == 0.0f) u = 0.0f;
            float xh = (alpha != 0.0f) ? u / alpha : 0.0f;
            xh = fminf(fmaxf(xh, -io.inp_bound), io.inp_bound);
            if (io.inp_res > 0.0f) {
                const float code = rintf(xh / io.inp_res);     // the DAC's integer, |code| <= bound / res
                // as bf16 (exact up to 256) for the product on the bf16 matrix cores
                // (operand layout of the matrix instruction: blocks of 16 vectors x 32 inputs, 64 lanes x 8 codes)
                // (the four codes of a group lie side by side there: one 8-byte store after the loop; the
                // path needs K % 32 == 0, so a group is never ragged)
                cbits[e] = __float_as_uint(code) >> 16;
                xh = code * io.inp_res;
            }
            if (io.inp_noise > 0.0f) {
                const float nz = io.inp_noise * z[e];
                xh = xh + nz;
            }
            o[e] = xh;
            if (nplanes == 3) {
                // the value itself as three bf16 terms, xh = h + m + l to the last bit (both subtractions exact)
                const uint32_t hb = __float_as_uint(xh) & 0xFFFF0000u;
                const float r1 = xh - __uint_as_float(hb);
                const uint32_t mb = __float_as_uint(r1) & 0xFFFF0000u;
                const float r2 = r1 - __uint_as_float(mb);
                cbits[e] = hb >> 16;
                mbits[e] = mb >> 16;
                lbits[e] = __float_as_uint(r2) >> 16;
            }
            if (4 * g + e < K) part += (double)xh * (double)xh;
        }
        if (codes) {
            // the product reads the codes: the fp32 values are not stored
            const int kk = 4 * g;
            const size_t block = (size_t)(b >> 4) * (size_t)(K >> 5) + (size_t)(kk >> 5);
            uint16_t* at = codes + (block * 64 + (size_t)(((kk >> 3) & 3) * 16 + (b & 15))) * 8 + (size_t)(kk & 7);
            *(uint2*)at = make_uint2(cbits[0] | (cbits[1] << 16), cbits[2] | (cbits[3] << 16));
            if (nplanes == 3) {
                *(uint2*)(at + plane_elems) = make_uint2(mbits[0] | (mbits[1] << 16), mbits[2] | (mbits[3] << 16));
                *(uint2*)(at + 2 * plane_elems) = make_uint2(lbits[0] | (lbits[1] << 16), lbits[2] | (lbits[3] << 16));
            }
        } else if (vec) {
            *(float4*)(qr + 4 * (size_t)g) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (4 * g + e < K) qr[4 * (size_t)g + e] = o[e];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
    if ((tid & 63) == 0) redd[tid >> 6] = part;
    __syncthreads();
    if (tid == 0) {
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) sum += redd[w];
        alpha_out[b] = alpha;
        norm_out[b] = (float)sqrt(sum);
    }
}

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Noise, ADC and rescaling of one pre-activation z = (Xq W^T)[m][n]; g_out / g_w are the output's
// two Gaussians.
__device__ __forceinline__ void mvm_finish(float z, float g_out, float g_w, bool noisy, const IoArgs& io, float norm_m,
                                           float alpha_m, size_t at, float* __restrict__ y, float* __restrict__ pre)
{
    if (noisy) {
        float wn_ = io.w_noise * norm_m;
        wn_ = wn_ * g_w;
        z = z + wn_;
        const float on = io.out_noise * g_out;
        z = z + on;
    }
    if (pre) pre[at] = z;
    float q = fminf(fmaxf(z, -io.out_bound), io.out_bound);
    if (io.out_res > 0.0f) q = rintf(q / io.out_res) * io.out_res;
    y[at] = alpha_m * q;
}

// Z[M][N] = A[M][K] * Bm, Bm[k][n] = TRANS ? Wm[k*ldw + n] : Wm[n*ldw + k].
// Block tile BM x 64 (BM = 64 or 128), K step 32; four waves, each BM/2 x 32 outputs as one or
// two 32 x 32 tiles of v_mfma_f32_32x32x2_f32.
//
// Operand order inside a K step.  One matrix instruction multiplies, per lane half h = lane/32,
// one k index.  Which of the step's 32 k values a half takes is free as long as both operands
// agree, so half h takes k = 16 h + s at instruction s: a lane then needs 16 consecutive k of
// its row, which are four 16-byte LDS reads from a tile kept in the matrix' own k-contiguous
// order (rows padded to 36 floats: conflict-free for 16-byte accesses).  No transposition on
// the way into LDS either: 16-byte global loads, 16-byte LDS stores.  In the transposed product
// the weights are n-contiguous; their tile is [k][n] (rows of 68 floats) and a lane reads its 16
// k values one by one, 32 lanes side by side.
//
// K split.  The K range is cut into `splits` slices, one workgroup per (tile, slice), so that a
// product with few output tiles (a batch of 256 vectors against 4096 rows gives one 64 x 64 tile
// per compute unit) still puts several workgroups on every compute unit, whose loads, barriers
// and matrix instructions overlap.  splits == 1: the analog epilogue is fused.  splits > 1:
// slice z writes its partial sums to part[z][M][N] and k_mvm_epilogue adds them in slice order.
// (Letting the slice that finishes last do the epilogue saves the second launch but needs a
// device-scope fence in every workgroup, which costs far more on this chip: 0.17 against 0.10 ms.)
//
// Workgroup ids go round-robin to the 8 XCDs; the id -> (tile, slice) map gives each XCD a
// contiguous range with the row blocks of A fastest, so that the workgroups sharing a tile of
// the weights run together on one L2.
//
// ALIGNED: K is a multiple of 32 and every 16-byte group is aligned and inside its row.  Rows
// m >= M and n >= N of a ragged edge tile are read from the last valid row instead (their
// outputs are never stored).  Otherwise elements are loaded one by one with k >= K as zero.
template <bool TRANS, int BM, bool ALIGNED>
__global__ void __launch_bounds__(256)
k_mvm_gemm(const float* __restrict__ A, const float* __restrict__ Wm, int M, int N, int K, int ldw,
           const float* __restrict__ alpha, const float* __restrict__ norm, IoArgs io, uint32_t k0, uint32_t k1,
           uint32_t t, uint32_t tag, float* __restrict__ y, float* __restrict__ pre, float* __restrict__ part,
           int splits, int mb, int nb)
{
    constexpr int BN = 64, BK = 32, LDK = 36, LDN = 68;
    constexpr int AH = BM / 32;                   // 16-byte groups of A per thread and K step (2 or 4)
    constexpr int NACC = BM / 64;                 // 32 x 32 tiles per wave
    constexpr int kBsFloats = TRANS ? BK * LDN : BN * LDK;
    __shared__ __align__(16) float As[2][BM * LDK];
    __shared__ __align__(16) float Bs[2][kBsFloats];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    const uint32_t total = (uint32_t)mb * (uint32_t)nb * (uint32_t)splits;
    const uint32_t per = (total + 7u) >> 3;
    const uint32_t seq = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
    if (seq >= total) return;
    const uint32_t mblk = seq % (uint32_t)mb, rest = seq / (uint32_t)mb;
    const uint32_t z = rest % (uint32_t)splits, nblk = rest / (uint32_t)splits;
    const int m0 = (int)mblk * BM, n0 = (int)nblk * BN;
    const int nchunks = (K + BK - 1) / BK;
    const int cps = (nchunks + splits - 1) / splits;
    const int c_begin = (int)z * cps, c_end = (c_begin + cps < nchunks) ? c_begin + cps : nchunks;

    // element (row, k) of a k-contiguous matrix with `rows` rows of length `ld`; rows are clamped
    auto load4 = [&](const float* __restrict__ base, int row, int rows, int ld, int kk) __attribute__((always_inline)) {
        const int r = row < rows ? row : rows - 1;
        if (ALIGNED) return *(const float4*)(base + (size_t)r * ld + kk);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const bool ok = kk + e < K;
            const float x = base[(size_t)r * ld + (ok ? kk + e : 0)];
            v[e] = ok ? x : 0.0f;
        }
        return make_float4(v[0], v[1], v[2], v[3]);
    };
    // 16-byte group of the transposed product's weights W[k][n] (n contiguous)
    auto load4_t = [&](int kr, int nn) __attribute__((always_inline)) {
        if (ALIGNED) {
            const int nc = nn + 3 < N ? nn : N - 4;                  // N is a multiple of 4 here
            return *(const float4*)(Wm + (size_t)kr * ldw + nc);
        }
        const bool kok = kr < K;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int nc = nn + e < N ? nn + e : N - 1;
            const float x = Wm[(size_t)(kok ? kr : 0) * ldw + nc];
            v[e] = kok ? x : 0.0f;
        }
        return make_float4(v[0], v[1], v[2], v[3]);
    };
    // Software pipeline over the K steps: while the matrix cores work on step c from registers,
    // the operands of step c+1 are read from LDS into a second register set, step c+2 is moved
    // from its staging registers to the LDS buffer step c has left, and the global loads of step
    // c+3 are in flight.  The workgroup barrier only orders LDS (its fences name the local address
    // space), so the global loads stay in flight across it.  (Register sets are plain variables
    // and the steps macros: anything passed by reference here ended up in scratch memory.)
    const int frow = tid >> 3, k_first = c_begin * BK + (tid & 7) * 4;
    auto a_row = [&](int h) __attribute__((always_inline)) {
        const int m = m0 + frow + 32 * h;
        return A + (size_t)(m < M ? m : M - 1) * K + k_first;
    };
    auto w_row = [&](int h) __attribute__((always_inline)) {
        if (!TRANS) {
            const int n = n0 + frow + 32 * h;
            return Wm + (size_t)(n < N ? n : N - 1) * ldw + k_first;
        }
        const int nn = n0 + (tid & 15) * 4;
        return Wm + (size_t)(c_begin * BK + (tid >> 4) + 16 * h) * ldw + (nn + 3 < N ? nn : N - 4);
    };
    // ALIGNED: running pointers, advanced in place (no address temporaries next to the staging registers)
    const float *pa0 = a_row(0), *pa1 = a_row(1), *pa2 = a_row(2), *pa3 = a_row(3);
    const float *pw0 = w_row(0), *pw1 = w_row(1);
    const size_t w_step = TRANS ? (size_t)BK * ldw : (size_t)BK;
    int fetched = 0;                                        // K steps fetched so far
#define AHT_FETCH(G)                                                                       \
    do {                                                                                   \
        if (ALIGNED) {                                                                     \
            G##a0 = *(const float4*)pa0;                                                   \
            G##a1 = *(const float4*)pa1;                                                   \
            if (AH == 4) {                                                                 \
                G##a2 = *(const float4*)pa2;                                               \
                G##a3 = *(const float4*)pa3;                                               \
            }                                                                              \
            G##b0 = *(const float4*)pw0;                                                   \
            G##b1 = *(const float4*)pw1;                                                   \
            pa0 += BK;                                                                     \
            pa1 += BK;                                                                     \
            if (AH == 4) {                                                                 \
                pa2 += BK;                                                                 \
                pa3 += BK;                                                                 \
            }                                                                              \
            pw0 += w_step;                                                                 \
            pw1 += w_step;                                                                 \
        } else {                                                                           \
            const int kc_ = (c_begin + fetched) * BK, kk_ = kc_ + (tid & 7) * 4;           \
            G##a0 = load4(A, m0 + frow, M, K, kk_);                                        \
            G##a1 = load4(A, m0 + frow + 32, M, K, kk_);                                   \
            if (AH == 4) {                                                                 \
                G##a2 = load4(A, m0 + frow + 64, M, K, kk_);                               \
                G##a3 = load4(A, m0 + frow + 96, M, K, kk_);                               \
            }                                                                              \
            if (!TRANS) {                                                                  \
                G##b0 = load4(Wm, n0 + frow, N, ldw, kk_);                                 \
                G##b1 = load4(Wm, n0 + frow + 32, N, ldw, kk_);                            \
            } else {                                                                       \
                G##b0 = load4_t(kc_ + (tid >> 4), n0 + (tid & 15) * 4);                    \
                G##b1 = load4_t(kc_ + (tid >> 4) + 16, n0 + (tid & 15) * 4);               \
            }                                                                              \
        }                                                                                  \
        fetched += 1;                                                                      \
    } while (0)
#define AHT_STAGE(BUF, G)                                                                  \
    do {                                                                                   \
        float* ap_ = &As[BUF][(tid >> 3) * LDK + (tid & 7) * 4];                           \
        *(float4*)ap_ = G##a0;                                                             \
        *(float4*)(ap_ + 32 * LDK) = G##a1;                                                \
        if (AH == 4) {                                                                     \
            *(float4*)(ap_ + 64 * LDK) = G##a2;                                            \
            *(float4*)(ap_ + 96 * LDK) = G##a3;                                            \
        }                                                                                  \
        if (!TRANS) {                                                                      \
            float* bp_ = &Bs[BUF][(tid >> 3) * LDK + (tid & 7) * 4];                       \
            *(float4*)bp_ = G##b0;                                                         \
            *(float4*)(bp_ + 32 * LDK) = G##b1;                                            \
        } else {                                                                           \
            float* bp_ = &Bs[BUF][(tid >> 4) * LDN + (tid & 15) * 4];                      \
            *(float4*)bp_ = G##b0;                                                         \
            *(float4*)(bp_ + 16 * LDN) = G##b1;                                            \
        }                                                                                  \
    } while (0)
    const int kh = lane >> 5, l32 = lane & 31;
#define AHT_LDS_READ(BUF, OA, OB)                                                          \
    do {                                                                                   \
        _Pragma("unroll") for (int i_ = 0; i_ < NACC; ++i_) {                              \
            const float* ap_ = &As[BUF][(wm * (BM / 2) + 32 * i_ + l32) * LDK + 16 * kh];  \
            _Pragma("unroll") for (int q_ = 0; q_ < 4; ++q_) {                             \
                const float4 v_ = *(const float4*)(ap_ + 4 * q_);                          \
                OA[i_][4 * q_] = v_.x; OA[i_][4 * q_ + 1] = v_.y;                          \
                OA[i_][4 * q_ + 2] = v_.z; OA[i_][4 * q_ + 3] = v_.w;                      \
            }                                                                              \
        }                                                                                  \
        if (!TRANS) {                                                                      \
            const float* bp_ = &Bs[BUF][(wn * 32 + l32) * LDK + 16 * kh];                  \
            _Pragma("unroll") for (int q_ = 0; q_ < 4; ++q_) {                             \
                const float4 v_ = *(const float4*)(bp_ + 4 * q_);                          \
                OB[4 * q_] = v_.x; OB[4 * q_ + 1] = v_.y;                                  \
                OB[4 * q_ + 2] = v_.z; OB[4 * q_ + 3] = v_.w;                              \
            }                                                                              \
        } else {                                                                           \
            const float* bp_ = &Bs[BUF][(16 * kh) * LDN + wn * 32 + l32];                  \
            _Pragma("unroll") for (int s_ = 0; s_ < 16; ++s_) OB[s_] = bp_[s_ * LDN];      \
        }                                                                                  \
    } while (0)
    floatx16 acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i) acc[i] = floatx16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#define AHT_MMA(OA, OB)                                                                    \
    do {                                                                                   \
        _Pragma("unroll") for (int s_ = 0; s_ < 16; ++s_)                                  \
            _Pragma("unroll") for (int i_ = 0; i_ < NACC; ++i_)                            \
                acc[i_] = __builtin_amdgcn_mfma_f32_32x32x2f32(OA[i_][s_], OB[s_], acc[i_], 0, 0, 0); \
    } while (0)
    auto lds_sync = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    const int nsteps = c_end - c_begin;                     // block-uniform, as is every branch below
    if (nsteps > 0) {
        float4 g0a0, g0a1, g0a2 = {}, g0a3 = {}, g0b0, g0b1;     // staging registers, two sets
        float4 g1a0 = {}, g1a1 = {}, g1a2 = {}, g1a3 = {}, g1b0 = {}, g1b1 = {};
        float o0a[NACC][16], o0b[16], o1a[NACC][16], o1b[16];    // operands, two sets
        AHT_FETCH(g0);
        if (nsteps > 1) AHT_FETCH(g1);
        AHT_STAGE(0, g0);
        lds_sync();
        AHT_LDS_READ(0, o0a, o0b);
        if (nsteps > 2) AHT_FETCH(g0);
        if (nsteps > 1) AHT_STAGE(1, g1);
        lds_sync();
        int c = 0;
        for (; c + 1 < nsteps; c += 2) {
            // step c: operands in set 0, its LDS buffer 0 is free for step c+2
            if (c + 3 < nsteps) AHT_FETCH(g1);
            AHT_LDS_READ(1, o1a, o1b);
            AHT_MMA(o0a, o0b);
            if (c + 2 < nsteps) AHT_STAGE(0, g0);
            lds_sync();
            // step c+1: operands in set 1, LDS buffer 1 is free for step c+3
            if (c + 4 < nsteps) AHT_FETCH(g0);
            if (c + 2 < nsteps) AHT_LDS_READ(0, o0a, o0b);
            AHT_MMA(o1a, o1b);
            if (c + 3 < nsteps) AHT_STAGE(1, g1);
            lds_sync();
        }
        if (c < nsteps) AHT_MMA(o0a, o0b);                  // odd number of steps: the last one
    }
#undef AHT_FETCH
#undef AHT_STAGE
#undef AHT_LDS_READ
#undef AHT_MMA

    // register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32 of a 32 x 32 tile
    const int n = n0 + wn * 32 + (lane & 31);
    const bool noisy = (io.w_noise > 0.0f) || (io.out_noise > 0.0f);
    float* __restrict__ pz = (splits > 1) ? part + (size_t)z * (size_t)M * (size_t)N : nullptr;
#pragma unroll
    for (int i = 0; i < NACC; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm * (BM / 2) + 32 * i + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
            if (m < M && n < N) {
                if (pz) {
                    pz[(size_t)m * N + n] = acc[i][r];
                } else {
                    float g[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                    if (noisy) gauss4_fast(k0, k1, (uint32_t)n >> 1, (uint32_t)m, t, tag, g);
                    mvm_finish(acc[i][r], (n & 1) ? g[2] : g[0], (n & 1) ? g[3] : g[1], noisy, io, norm[m], alpha[m],
                               (size_t)m * N + n, y, pre);
                }
            }
        }
    }
}

// Product for quantised inputs without input noise: X~ = res * C with integer codes C,
// |c| <= 256, exact in bf16.  Each weight is cut into three bf16 terms (8 + 8 + 8 mantissa bits:
// w = hi + mid + lo up to the last bit of its fp32 value), so that Z = res * (C hi^T + C mid^T +
// C lo^T) takes three passes of the bf16 matrix cores (v_mfma_f32_16x16x32_bf16, fp32 sums) in
// place of one pass of the fp32 ones at an eighth of their rate.  A wave owns 16 outputs x MT * 16
// input vectors x one slice of the inner dimension: it reads its weights once, row-contiguous (eight
// lanes per 128-byte line), turns them into the operand layout (lane = output and one of four groups
// of 8 inner indices) through a little LDS of its own, needs no barrier, and writes its partial sums
// for k_mvm_epilogue.  Needs K % 32 == 0, N % 16 == 0, 16-byte aligned rows.  TRANS: the transposed
// product (the weights of an output are a column: eight 4-byte loads per lane and step).
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

// Eight fp32 weights (o0, o1) as three bf16 terms each, packed two to a register in the order of
// the matrix instruction's B operand: w = hi + mid + lo to the last bit (both subtractions are exact).
__device__ __forceinline__ void split_bf16x3(const float4& o0, const float4& o1, bf16x8_t& bh, bf16x8_t& bm, bf16x8_t& bl)
{
    const float wv[8] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w};
    uint32_t hb[8], mb[8], lb[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        hb[e] = __float_as_uint(wv[e]) & 0xFFFF0000u;
        const float r1 = wv[e] - __uint_as_float(hb[e]);        // exact
        mb[e] = __float_as_uint(r1) & 0xFFFF0000u;
        const float r2 = r1 - __uint_as_float(mb[e]);           // exact
        lb[e] = __float_as_uint(r2);
    }
    auto pack = [](uint32_t even, uint32_t odd) __attribute__((always_inline)) {
        return __builtin_amdgcn_perm(odd, even, 0x07060302u);   // high halves: even element low, odd element high
    };
    const uint4 ph = make_uint4(pack(hb[0], hb[1]), pack(hb[2], hb[3]), pack(hb[4], hb[5]), pack(hb[6], hb[7]));
    const uint4 pm = make_uint4(pack(mb[0], mb[1]), pack(mb[2], mb[3]), pack(mb[4], mb[5]), pack(mb[6], mb[7]));
    const uint4 pl = make_uint4(pack(lb[0], lb[1]), pack(lb[2], lb[3]), pack(lb[4], lb[5]), pack(lb[6], lb[7]));
    bh = __builtin_bit_cast(bf16x8_t, ph);
    bm = __builtin_bit_cast(bf16x8_t, pm);
    bl = __builtin_bit_cast(bf16x8_t, pl);
}

// FUSED: the four waves of a workgroup take four slices of the inner dimension of the same outputs
// (splits == 4), exchange their partial sums through LDS, add them in slice order (the order of
// k_mvm_epilogue: same bits) and apply the analog epilogue themselves, a quarter of the tile rows
// each: no partial sums in memory, no second launch.
struct MvmTail {
    const float* alpha;
    const float* norm;
    IoArgs io;
    uint32_t k0, k1, t, tag;
    float* y;
    float* pre;
};

template <int MT, bool TRANS, bool FUSED>
__global__ void __launch_bounds__(256)
k_mvm_gemm_codes(const uint16_t* __restrict__ xc, const float* __restrict__ W, int B, int N, int K, int ldw,
                 int splits, float inp_res, float* __restrict__ part, MvmTail tail)
{
    extern __shared__ float mvm_exchange[];                        // FUSED: [4 slices][MT tiles][4 registers][64 lanes]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int nslab = N >> 4, mchunks = (B + 16 * MT - 1) / (16 * MT);
    // FUSED: one workgroup per (outputs, vectors), wave = slice; else one wave per (outputs, vectors, slice)
    const int unit = FUSED ? wave * (nslab * mchunks) + (int)blockIdx.x : (int)blockIdx.x * 4 + wave;
    if (FUSED) {
        if ((int)blockIdx.x >= nslab * mchunks) return;            // uniform over the workgroup: its barrier stays safe
    } else {
        if (unit >= nslab * mchunks * splits) return;              // wave-uniform; no barriers on this path
    }
    const int z = unit / (nslab * mchunks), rem = unit - z * (nslab * mchunks);
    const int mc = rem / nslab, slab = rem - mc * nslab;
    const int steps = K >> 5, per = (steps + splits - 1) / splits;
    const int s0 = z * per, s1 = (s0 + per < steps) ? s0 + per : steps;
    const int j = lane & 15, g = lane >> 4;
    // forward: output n is row n of W, its inner indices lie side by side; transposed: output n is
    // column n, inner index k is row k (the lanes of 16 neighbouring outputs read 64 bytes of a row)
    const float* wp = TRANS ? W + (size_t)(8 * g) * ldw + (size_t)(slab * 16 + j)
                            : W + (size_t)(slab * 16 + j) * ldw + 8 * g;
    // forward: the weights are loaded row-contiguous (lane = row lane / 8 (+ 8), 16-byte piece lane % 8)
    // and turned into the operand layout through 2.25 KB of LDS of the wave's own (rows 144 bytes apart)
    const float* wco = W + (size_t)(slab * 16 + (lane >> 3)) * ldw + 4 * (lane & 7);
    __shared__ float wturn[4][16 * 36];
    float* wt_st = &wturn[wave][(lane >> 3) * 36 + 4 * (lane & 7)];
    const float* wt_ld = &wturn[wave][j * 36 + 8 * g];
    // codes: one contiguous 1 KB block per (16 vectors, 32 inputs); blocks past the batch hold zeros
    const uint16_t* ap[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) ap[m] = xc + ((size_t)(mc * MT + m) * (size_t)steps * 64 + (size_t)lane) * 8;
    floatx4_t acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[m][r] = 0.0f;

    // The weights come from HBM once and nothing hides their latency but loads in flight: a ring of
    // DW steps of weights and codes per wave.  (The codes are L2 resident, but loads complete in
    // order: fetched any later than the weights of their step, they would make the wave wait for
    // younger weight loads too.)  Fetches past the slice read its last step again: no branch around
    // a load, so that the compiler can count the loads in flight and wait for the oldest only.
    constexpr int DW = (MT >= 16) ? 3 : 4;
    float4 wq[DW][2];
    uint4 av[DW][MT];
    auto fetch = [&](int s, float4 (&q)[2], uint4 (&v)[MT]) __attribute__((always_inline)) {
        if (TRANS) {
            const float* wr = wp + (size_t)(32 * s) * ldw;
            float e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = __builtin_nontemporal_load(wr + (size_t)i * ldw);
            q[0] = make_float4(e[0], e[1], e[2], e[3]);
            q[1] = make_float4(e[4], e[5], e[6], e[7]);
        } else {
            // row-contiguous: eight lanes read the 128 bytes of one row and step, two loads cover the 16 rows
            typedef float f4_t __attribute__((ext_vector_type(4)));
            const float* wr = wco + 32 * (size_t)s;
            const f4_t u0 = __builtin_nontemporal_load((const f4_t*)wr),
                       u1 = __builtin_nontemporal_load((const f4_t*)(wr + 8 * (size_t)ldw));
            q[0] = make_float4(u0.x, u0.y, u0.z, u0.w);
            q[1] = make_float4(u1.x, u1.y, u1.z, u1.w);
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) v[m] = *(const uint4*)(ap[m] + 512 * (size_t)s);
    };
    const int last = s1 - 1;
    if (s0 < s1) {                                // (an empty slice still writes its zeros)
#pragma unroll
        for (int d = 0; d < DW; ++d) fetch(s0 + d < last ? s0 + d : last, wq[d], av[d]);
    }
    // one step of the inner dimension from ring slot (q, v); then the slot is filled again for step `next`
    auto step = [&](float4 (&q)[2], uint4 (&v)[MT], int next) __attribute__((always_inline)) {
        // three bf16 terms of the eight weights, packed two to a register
        float4 o0 = q[0], o1 = q[1];
        if (!TRANS) {
            *(float4*)wt_st = q[0];
            *(float4*)(wt_st + 8 * 36) = q[1];
            __builtin_amdgcn_wave_barrier();
            o0 = *(const float4*)wt_ld;
            o1 = *(const float4*)(wt_ld + 4);
            __builtin_amdgcn_wave_barrier();
        }
        bf16x8_t bh, bm, bl;
        split_bf16x3(o0, o1, bh, bm, bl);
        bf16x8_t a[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m) a[m] = __builtin_bit_cast(bf16x8_t, v[m]);
        fetch(next < last ? next : last, q, v);
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bl, acc[m], 0, 0, 0);
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bm, acc[m], 0, 0, 0);
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bh, acc[m], 0, 0, 0);
    };
    // Whole turns of the ring in a loop with one way in and one way out (an exit from the middle of a
    // turn would, for the compiler, lead back to the head of the loop, and the head would then wait for
    // every load in flight); what is left of the slice, fewer than DW steps, after it.
    int s = s0;
    for (; s + DW <= s1; s += DW) {
#pragma unroll
        for (int d = 0; d < DW; ++d) step(wq[d], av[d], s + d + DW);
    }
#pragma unroll
    for (int d = 0; d < DW - 1; ++d)
        if (s + d < s1) step(wq[d], av[d], last);                  // wave-uniform
    // partial sums, in units of the input grid; lane = output, register r = row 4 g + r of the tile
    if (FUSED) {
        float* mine = mvm_exchange + (size_t)wave * (MT * 256) + lane;
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) mine[(m * 4 + r) * 64] = acc[m][r] * inp_res;
        __syncthreads();
        const int n = slab * 16 + j;
        const bool noisy = (tail.io.w_noise > 0.0f) || (tail.io.out_noise > 0.0f);
        constexpr int kPerWave = (MT + 3) / 4;                     // tile rows this wave finishes
#pragma unroll
        for (int i = 0; i < kPerWave; ++i) {
            const int m = wave * kPerWave + i;
            if (m >= MT) break;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = (mc * MT + m) * 16 + 4 * g + r;
                if (row >= B) continue;
                float zsum = 0.0f;
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) zsum += mvm_exchange[(size_t)sl * (MT * 256) + (m * 4 + r) * 64 + lane];
                float gq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (noisy) gauss4_fast(tail.k0, tail.k1, (uint32_t)n >> 1, (uint32_t)row, tail.t, tail.tag, gq);
                mvm_finish(zsum, (n & 1) ? gq[2] : gq[0], (n & 1) ? gq[3] : gq[1], noisy, tail.io, tail.norm[row],
                           tail.alpha[row], (size_t)row * N + n, tail.y, tail.pre);
            }
        }
    } else {
        float* pz = part + (size_t)z * B * N + (size_t)(slab * 16 + j);
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = (mc * MT + m) * 16 + 4 * g + r;
                if (row < B) pz[(size_t)row * N] = acc[m][r] * inp_res;
            }
    }
}

// The same product with the codes shared inside a workgroup: its four waves take four neighbouring
// groups of 16 outputs of the SAME vectors and slice of the inner dimension, so that each 1 KB block of
// codes is fetched once per workgroup (a quarter by each wave), passed through LDS (two stages, one
// barrier per step) and read from there by all four.  Without this every wave fetches all the codes of
// its slice itself: at 256 vectors eight times the bytes of its weights.  Needs N % 64 == 0 and
// MT % 4 == 0; always writes partial sums for k_mvm_epilogue.
// NP = 3: inputs of any value, given as three bf16 planes (x~ = h + m + l to the last bit, as the weights
// are cut; planes `plane_elems` apart).  Of the nine products of a term of x~ and a term of w the six
// down to 2^-16 of the largest are formed (l H, m M, h L, m H, h M, h H, small ones first), the three
// left out are each 2^-24 of it: an fp32 product at six sixteenths of the time of the fp32 matrix cores.
template <int MT, bool TRANS, int NP>
__global__ void __launch_bounds__(256, NP == 1 ? 2 : 1)
k_mvm_gemm_codes_shared(const uint16_t* __restrict__ xc, size_t plane_elems, const float* __restrict__ W, int B, int N,
                        int K, int ldw, int splits, float inp_res, float* __restrict__ part)
{
    static_assert(NP == 1 || NP == 3, "one plane of integer codes or three planes of an fp32 value");
    static_assert(MT % 4 == 0, "each wave fetches a quarter of the code blocks of a step");
    constexpr int QT = MT / 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int ngroup = N >> 6, mchunks = (B + 16 * MT - 1) / (16 * MT);
    const int unit = (int)blockIdx.x;
    if (unit >= ngroup * mchunks * splits) return;                 // uniform over the workgroup
    const int z = unit / (ngroup * mchunks), rem = unit - z * (ngroup * mchunks);
    const int mc = rem / ngroup, slab = (rem - mc * ngroup) * 4 + wave;
    const int steps = K >> 5, per = (steps + splits - 1) / splits;
    const int s0 = z * per, s1 = (s0 + per < steps) ? s0 + per : steps;    // the same for the four waves
    const int j = lane & 15, g = lane >> 4;
    const float* wp = TRANS ? W + (size_t)(8 * g) * ldw + (size_t)(slab * 16 + j)
                            : W + (size_t)(slab * 16 + j) * ldw + 8 * g;
    const float* wco = W + (size_t)(slab * 16 + (lane >> 3)) * ldw + 4 * (lane & 7);
    __shared__ float wturn[4][16 * 36];
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    extern __shared__ u32x4_t cstage[];                            // [2 stages][NP][MT][64 lanes]
    auto staged = [&](int buf, int p, int m) __attribute__((always_inline)) -> u32x4_t& {
        return cstage[((buf * NP + p) * MT + m) * 64 + lane];
    };
    float* wt_st = &wturn[wave][(lane >> 3) * 36 + 4 * (lane & 7)];
    const float* wt_ld = &wturn[wave][j * 36 + 8 * g];
    const uint16_t* ap[NP * QT];                                   // this wave's blocks: tiles wave, wave + 4, ... of every plane
#pragma unroll
    for (int p = 0; p < NP; ++p)
#pragma unroll
        for (int i = 0; i < QT; ++i)
            ap[p * QT + i] = xc + (size_t)p * plane_elems +
                             ((size_t)(mc * MT + 4 * i + wave) * (size_t)steps * 64 + (size_t)lane) * 8;
    floatx4_t acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[m][r] = 0.0f;

    constexpr int DW = (NP == 1) ? 4 : 3;
    float4 wq[DW][2];
    uint4 av[DW][NP * QT];
    auto fetch = [&](int s, float4 (&q)[2], uint4 (&v)[NP * QT]) __attribute__((always_inline)) {
        if (TRANS) {
            const float* wr = wp + (size_t)(32 * s) * ldw;
            float e[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) e[i] = __builtin_nontemporal_load(wr + (size_t)i * ldw);
            q[0] = make_float4(e[0], e[1], e[2], e[3]);
            q[1] = make_float4(e[4], e[5], e[6], e[7]);
        } else {
            typedef float f4_t __attribute__((ext_vector_type(4)));
            const float* wr = wco + 32 * (size_t)s;
            const f4_t u0 = __builtin_nontemporal_load((const f4_t*)wr),
                       u1 = __builtin_nontemporal_load((const f4_t*)(wr + 8 * (size_t)ldw));
            q[0] = make_float4(u0.x, u0.y, u0.z, u0.w);
            q[1] = make_float4(u1.x, u1.y, u1.z, u1.w);
        }
#pragma unroll
        for (int i = 0; i < NP * QT; ++i) v[i] = *(const uint4*)(ap[i] + 512 * (size_t)s);
    };
    const int last = s1 - 1;
    if (s0 < s1) {
#pragma unroll
        for (int d = 0; d < DW; ++d) fetch(s0 + d < last ? s0 + d : last, wq[d], av[d]);
    }
    int buf = 0;
    // one step of the inner dimension from ring slot (q, v); then the slot is filled again for step `next`
    auto step = [&](float4 (&q)[2], uint4 (&v)[NP * QT], int next) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < NP; ++p)
#pragma unroll
            for (int i = 0; i < QT; ++i)
                staged(buf, p, 4 * i + wave) = u32x4_t{v[p * QT + i].x, v[p * QT + i].y, v[p * QT + i].z, v[p * QT + i].w};
        float4 o0 = q[0], o1 = q[1];
        if (!TRANS) {
            *(float4*)wt_st = q[0];
            *(float4*)(wt_st + 8 * 36) = q[1];
        }
        // One barrier per step: a stage is written again two steps later, and by then every wave
        // has passed the barrier of the step between, which it reaches after its reads of this one.
        __syncthreads();
        if (!TRANS) {
            o0 = *(const float4*)wt_ld;
            o1 = *(const float4*)(wt_ld + 4);
        }
        bf16x8_t bh, bm, bl;
        split_bf16x3(o0, o1, bh, bm, bl);
        bf16x8_t a[MT];
        if (NP == 3) {
#pragma unroll
            for (int m = 0; m < MT; ++m) a[m] = __builtin_bit_cast(bf16x8_t, staged(buf, 2, m));
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bh, acc[m], 0, 0, 0);
#pragma unroll
            for (int m = 0; m < MT; ++m) a[m] = __builtin_bit_cast(bf16x8_t, staged(buf, 1, m));
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bm, acc[m], 0, 0, 0);
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bh, acc[m], 0, 0, 0);
        }
#pragma unroll
        for (int m = 0; m < MT; ++m) a[m] = __builtin_bit_cast(bf16x8_t, staged(buf, 0, m));
        fetch(next < last ? next : last, q, v);
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bl, acc[m], 0, 0, 0);
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bm, acc[m], 0, 0, 0);
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], bh, acc[m], 0, 0, 0);
        buf ^= 1;
    };
    // Whole turns of the ring in a loop with one way in and one way out (an exit from the middle of a
    // turn would, for the compiler, lead back to the head of the loop, and the head would then wait for
    // every load in flight); what is left of the slice, fewer than DW steps, after it.
    int s = s0;
    for (; s + DW <= s1; s += DW) {
#pragma unroll
        for (int d = 0; d < DW; ++d) step(wq[d], av[d], s + d + DW);
    }
#pragma unroll
    for (int d = 0; d < DW - 1; ++d)
        if (s + d < s1) step(wq[d], av[d], last);                  // uniform over the workgroup
    float* pz = part + (size_t)z * B * N + (size_t)(slab * 16 + j);
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = (mc * MT + m) * 16 + 4 * g + r;
            if (row < B) pz[(size_t)row * N] = acc[m][r] * inp_res;
        }
}

// Second pass of a K-split product: one thread per pair of neighbouring outputs (they share one
// Philox block) adds the slices' partial sums in slice order and applies the analog epilogue.
__global__ void __launch_bounds__(256)
k_mvm_epilogue(const float* __restrict__ part, int splits, int M, int N, const float* __restrict__ alpha,
               const float* __restrict__ norm, IoArgs io, uint32_t k0, uint32_t k1, uint32_t t, uint32_t tag,
               float* __restrict__ y, float* __restrict__ pre)
{
    const int half = (N + 1) >> 1;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)M * half) return;
    const int m = (int)(idx / half), n = 2 * (int)(idx % half);
    const size_t at = (size_t)m * N + n, plane = (size_t)M * N;
    const bool two = n + 1 < N;
    float z0 = 0.0f, z1 = 0.0f;
    for (int s = 0; s < splits; ++s) {
        z0 += part[(size_t)s * plane + at];
        if (two) z1 += part[(size_t)s * plane + at + 1];
    }
    const bool noisy = (io.w_noise > 0.0f) || (io.out_noise > 0.0f);
    float g[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (noisy) gauss4_fast(k0, k1, (uint32_t)n >> 1, (uint32_t)m, t, tag, g);
    mvm_finish(z0, g[0], g[1], noisy, io, norm[m], alpha[m], at, y, pre);
    if (two) mvm_finish(z1, g[2], g[3], noisy, io, norm[m], alpha[m], at + 1, y, pre);
}

// Analog read of one column: the product of W with the one-hot vector e_col when the input
// carries no noise.  Then x~ = xq e_col with xq = DAC(1) (alpha = 1), |x~| = |xq|, and the
// pre-activation of row i is the single product w[i][col] * xq, which is also what the matrix
// kernel's sum reduces to; the epilogue is the common one, so the two paths agree bit for bit.
// Also writes the negated read and the one-hot vector itself (inputs of the pulsed write).
__global__ void __launch_bounds__(256)
k_mvm_column_read(const float* __restrict__ W, int R, int C, int col, IoArgs io, uint32_t k0, uint32_t k1, uint32_t t,
                  uint32_t tag, float* __restrict__ read, float* __restrict__ neg, float* __restrict__ onehot)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < C) onehot[i] = (i == col) ? 1.0f : 0.0f;
    if (i >= R) return;
    float xq = fminf(fmaxf(1.0f, -io.inp_bound), io.inp_bound);
    if (io.inp_res > 0.0f) xq = rintf(xq / io.inp_res) * io.inp_res;
    const float z = W[(size_t)i * C + col] * xq;
    const bool noisy = (io.w_noise > 0.0f) || (io.out_noise > 0.0f);
    float g[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (noisy) gauss4_fast(k0, k1, (uint32_t)i >> 1, 0u, t, tag, g);
    mvm_finish(z, (i & 1) ? g[2] : g[0], (i & 1) ? g[3] : g[1], noisy, io, fabsf(xq), 1.0f, (size_t)i, read, nullptr);
    neg[i] = -read[i];
}

}  // namespace aht
