// HIP kernels of the stochastic pulsed update for gfx950 (wave64).
//
// Steps (arXiv 2104.02184, Sec. 3, Eq. (2) and the paragraphs after it):
//   k_gen_planes     per-cell device planes (device-to-device variation), once per tile
//   k_line_scale     per-sample max|x|, max|d| -> probability factors (update management)
//   k_pulse_words    stochastic pulse trains of every line, bit-packed
//   k_cell_update    coincidence counts (AND + popcount) and sequential device steps for
//                    every update vector of the call, weights resident in registers
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <type_traits>

#include "aht_rng.hpp"

#ifndef AHT_GROUP
#define AHT_GROUP 4
#endif

namespace aht {

// Profiling build only (-DAHT_WAVE_STAMPS, see wave_timeline.py): lane 0 of every wave of the cell kernel
// notes the 100 MHz wall clock at seven points of its life, and where it ran, in eight words of a buffer the
// host hands over.  The default build has none of this.
#ifdef AHT_WAVE_STAMPS
__device__ unsigned long long* g_wave_stamps = nullptr;
#define AHT_STAMP(k)                                                                                          \
    do {                                                                                                      \
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");                                           \
        if (g_wave_stamps && (threadIdx.x & 63) == 0)                                                         \
            g_wave_stamps[((size_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8 + (k)] =                          \
                (k) < 7 ? __builtin_amdgcn_s_memrealtime()                                                    \
                        : ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 4) /* HW_ID */ |        \
                           ((unsigned long long)__builtin_amdgcn_s_getreg((31 << 11) | 20) /* XCC_ID */ << 32)); \
    } while (0)
#else
#define AHT_STAMP(k) ((void)0)
#endif

enum : int { kConstantStep = 0, kLinearStep = 1, kSoftBounds = 2 };

template <typename WordT>
struct WordTraits;
template <>
struct WordTraits<uint32_t> {
    static constexpr int kSignBit = 31;
};
template <>
struct WordTraits<uint64_t> {
    static constexpr int kSignBit = 63;
};

// ------------------------------------------------------------------------------------------
// Per-cell planes.  fp32 arithmetic without contraction on Gaussians evaluated in fp64 and
// rounded once, so that the planes are reproducible to the last bit.
// ------------------------------------------------------------------------------------------
struct PlaneArgs {
    int kind;
    float dw_min, dw_min_dtod, up_down, up_down_dtod, w_max, w_max_dtod, w_min, w_min_dtod;
    float gamma_up, gamma_down, gamma_dtod;
    uint32_t k0, k1;
    int R, C;
    float *dw_up, *dw_down, *b_max, *b_min, *slope_up, *slope_down;  // slopes: LinearStep only
};

__global__ void __launch_bounds__(256) k_gen_planes(PlaneArgs a)
{
    const size_t n = (size_t)a.R * a.C;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n;
         k += (size_t)gridDim.x * blockDim.x) {
        float g[8];
        gauss4_accurate(a.k0, a.k1, (uint32_t)k, 0u, 0u, kTagD2D, g);
        gauss4_accurate(a.k0, a.k1, (uint32_t)k, 1u, 0u, kTagD2D, g + 4);
        const float dw = a.dw_min * fabsf(1.0f + a.dw_min_dtod * g[0]);
        const float asym = a.up_down + a.up_down_dtod * g[1];
        const float bmax = fmaxf(0.0f, a.w_max * (1.0f + a.w_max_dtod * g[2]));
        const float bmin = fminf(0.0f, a.w_min * (1.0f + a.w_min_dtod * g[3]));
        a.dw_up[k] = dw * (1.0f + asym);
        a.dw_down[k] = dw * (1.0f - asym);
        a.b_max[k] = bmax;
        a.b_min[k] = bmin;
        if (a.kind == kLinearStep) {
            const float gu = a.gamma_up * (1.0f + a.gamma_dtod * g[4]);
            const float gd = a.gamma_down * (1.0f + a.gamma_dtod * g[5]);
            a.slope_up[k] = (bmax != 0.0f) ? gu / bmax : 0.0f;
            a.slope_down[k] = (bmin != 0.0f) ? gd / bmin : 0.0f;
        }
    }
}

// slope plane of a SoftBounds tile (1/bound, 0 where the bound is 0); bound == nullptr: zeros
__global__ void __launch_bounds__(256) k_derived_slope(const float* bound, float* out, size_t n)
{
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n;
         k += (size_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        if (bound) {
            const float b = bound[k];
            s = (b != 0.0f) ? 1.0f / b : 0.0f;
        }
        out[k] = s;
    }
}

// transfer between coupled tiles: the one-hot read vector and the negated read-out
__global__ void __launch_bounds__(256) k_one_hot(float* x, int n, int hot)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < n) x[k] = (k == hot) ? 1.0f : 0.0f;
}

// effective weight of a unit cell: out = sum_k gamma_k W_k, added in device order, four cells per thread
struct UnitCellArgs {
    const float* w[8];
    float gamma[8];
    int n;
};
__global__ void __launch_bounds__(256) k_unit_cell_weights(UnitCellArgs u, float* __restrict__ out, size_t cells)
{
    const size_t i4 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i4 >= cells) return;
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const bool whole = i4 + 3 < cells;
    for (int k = 0; k < u.n; ++k) {
        float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (whole) {
            const float4 q = *(const float4*)(u.w[k] + i4);
            v[0] = q.x; v[1] = q.y; v[2] = q.z; v[3] = q.w;
        } else {
            for (int e = 0; e < 4; ++e)
                if (i4 + e < cells) v[e] = u.w[k][i4 + e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float term = u.gamma[k] * v[e];
            acc[e] = acc[e] + term;
        }
    }
    if (whole) {
        *(float4*)(out + i4) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    } else {
        for (int e = 0; e < 4; ++e)
            if (i4 + e < cells) out[i4 + e] = acc[e];
    }
}

__global__ void __launch_bounds__(256) k_negate(const float* in, float* out, int n)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < n) out[k] = -in[k];
}

// ------------------------------------------------------------------------------------------
// Temporal processes, once per mini-batch (Sec. 4, last paragraph of the paper): decay,
// diffusion and reset with per-cell parameters.  The planes use Gaussians 6, 7, 8 of the
// device-to-device stream; the noise of a cell in one temporal step is Gaussian number `cell` of
// that step's stream (index 0, t = temporal step, tag 5 for diffusion, 6 for reset), so that four
// neighbouring cells use the four numbers of one block.
// ------------------------------------------------------------------------------------------
constexpr uint32_t kTagDiffusion = 5u, kTagReset = 6u;

__global__ void __launch_bounds__(256)
k_gen_temporal_planes(float decay_rate, float decay_rate_dtod, float diffusion, float diffusion_dtod, float reset,
                      float reset_dtod, uint32_t k0, uint32_t k1, size_t n, float* decay, float* sdiff, float* rplane)
{
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x) {
        float g1[4], g2[4];
        gauss4_accurate(k0, k1, (uint32_t)k, 1u, 0u, kTagD2D, g1);     // numbers 4..7
        gauss4_accurate(k0, k1, (uint32_t)k, 2u, 0u, kTagD2D, g2);     // numbers 8..11
        float lam = decay_rate * (1.0f + decay_rate_dtod * g1[2]);
        lam = fminf(fmaxf(lam, 0.0f), 1.0f);
        decay[k] = lam;
        sdiff[k] = diffusion * fabsf(1.0f + diffusion_dtod * g1[3]);
        rplane[k] = reset + reset_dtod * g2[0];
    }
}

// HBM bound: 20 bytes read and 4 written per cell.  One thread per four consecutive cells.
__global__ void __launch_bounds__(256)
k_decay_diffuse(float* __restrict__ W, const float* __restrict__ decay, const float* __restrict__ sdiff,
                const float* __restrict__ b_max, const float* __restrict__ b_min, size_t n, uint32_t k0,
                uint32_t k1, uint32_t tau, int with_diffusion)
{
    const size_t g = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t k = g * 4;
    if (k >= n) return;
    float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (with_diffusion) gauss4_fast(k0, k1, 0u, (uint32_t)g, tau, kTagDiffusion, z);
    if (k + 4 <= n) {
        float4 w = *(const float4*)(W + k);
        const float4 la = *(const float4*)(decay + k), sd = *(const float4*)(sdiff + k);
        const float4 hi = *(const float4*)(b_max + k), lo = *(const float4*)(b_min + k);
        w.x = fminf(fmaxf(w.x * (1.0f - la.x) + sd.x * z[0], lo.x), hi.x);
        w.y = fminf(fmaxf(w.y * (1.0f - la.y) + sd.y * z[1], lo.y), hi.y);
        w.z = fminf(fmaxf(w.z * (1.0f - la.z) + sd.z * z[2], lo.z), hi.z);
        w.w = fminf(fmaxf(w.w * (1.0f - la.w) + sd.w * z[3], lo.w), hi.w);
        *(float4*)(W + k) = w;
    } else {
        for (int e = 0; e < 4 && k + e < n; ++e)
            W[k + e] = fminf(fmaxf(W[k + e] * (1.0f - decay[k + e]) + sdiff[k + e] * z[e], b_min[k + e]), b_max[k + e]);
    }
}

__global__ void __launch_bounds__(256)
k_reset_columns(float* __restrict__ W, const float* __restrict__ rplane, float reset_std,
                const float* __restrict__ b_max, const float* __restrict__ b_min, int R, int C, int c0, int ncols,
                uint32_t k0, uint32_t k1, uint32_t tau)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (size_t)R * ncols) return;
    const int i = (int)(t / (size_t)ncols), j = c0 + (int)(t % (size_t)ncols);
    const size_t k = (size_t)i * C + j;
    float z[4];
    gauss4_fast(k0, k1, 0u, (uint32_t)(k >> 2), tau, kTagReset, z);
    const uint32_t e = (uint32_t)k & 3u;
    const float xi = e == 0 ? z[0] : e == 1 ? z[1] : e == 2 ? z[2] : z[3];
    W[k] = fminf(fmaxf(rplane[k] + reset_std * xi, b_min[k]), b_max[k]);
}

// ------------------------------------------------------------------------------------------
// Update vectors of a convolution layer, gathered on the fly (Sec. 3: convolutions accumulate
// their positions' rank-1 updates in analog memory).  With conv.enabled the "x" buffer is the
// input image [N][Cin][H][W] and the "d" buffer the output gradient [N][Cout][OH][OW]; update
// vector b = (n*OH + oy)*OW + ox has x_b[(c*kh + ky)*kw + kx] = img[n][c][oy*stride-pad+ky][ox*stride-pad+kx]
// (0 outside the image) and d_b[i] = grad[n][i][oy][ox].  Otherwise x is [B][C] and d is [B][R].
// ------------------------------------------------------------------------------------------
struct ConvView {
    int enabled;
    int Cin, H, W, kh, kw, stride, pad, OH, OW, Cout;
};

struct ConvPos {
    int n, oy, ox;
};

__device__ __forceinline__ ConvPos conv_pos(const ConvView& v, uint32_t b)
{
    ConvPos p;
    p.ox = (int)(b % (uint32_t)v.OW);
    const uint32_t t = b / (uint32_t)v.OW;
    p.oy = (int)(t % (uint32_t)v.OH);
    p.n = (int)(t / (uint32_t)v.OH);
    return p;
}

__device__ __forceinline__ float view_x(const float* __restrict__ x, const ConvView& v, uint32_t b, int j, int C)
{
    if (!v.enabled) return x[(size_t)b * C + j];
    const int kx = j % v.kw, t = j / v.kw, ky = t % v.kh, c = t / v.kh;
    const ConvPos p = conv_pos(v, b);
    const int iy = p.oy * v.stride - v.pad + ky, ix = p.ox * v.stride - v.pad + kx;
    if (iy < 0 || iy >= v.H || ix < 0 || ix >= v.W) return 0.0f;
    return x[(((size_t)p.n * v.Cin + c) * v.H + iy) * v.W + ix];
}

__device__ __forceinline__ float view_d(const float* __restrict__ d, const ConvView& v, uint32_t b, int i, int R)
{
    if (!v.enabled) return d[(size_t)b * R + i];
    const ConvPos p = conv_pos(v, b);
    return d[(((size_t)p.n * v.Cout + i) * v.OH + p.oy) * v.OW + p.ox];
}

// ------------------------------------------------------------------------------------------
// Line scaling with update management: one workgroup per update vector.
// a_x = A sqrt(m_d/m_x), a_d = A sqrt(m_x/m_d); both 0 when a maximum is 0 (sample skipped).
// With a per-sample train length BL_b = clamp(ceil(lr m_x m_d / dw_min), 1, BL), A uses BL_b.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float finite_abs_or_zero(float v)
{
    const float a = fabsf(v);
    return (a < __builtin_inff()) ? a : 0.0f;   // NaN and Inf compare false
}

// (the body is a device function so that one launch can also take the vectors of several tiles, see
// k_line_scale_group: sample `b`)
__device__ __forceinline__ void line_scale_body(const float* __restrict__ x, const float* __restrict__ d, int R, int C,
                                                double lr, double dw_min, int BL, int update_management,
                                                int dynamic_bl, double* __restrict__ a_x, double* __restrict__ a_d,
                                                int32_t* __restrict__ bl_b, const ConvView& conv, const int b)
{
    __shared__ float red_x[4], red_d[4];
    float mx = 0.0f, md = 0.0f;
    for (int j = threadIdx.x; j < C; j += 256) mx = fmaxf(mx, finite_abs_or_zero(view_x(x, conv, (uint32_t)b, j, C)));
    for (int i = threadIdx.x; i < R; i += 256) md = fmaxf(md, finite_abs_or_zero(view_d(d, conv, (uint32_t)b, i, R)));
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        mx = fmaxf(mx, __shfl_xor(mx, off, 64));
        md = fmaxf(md, __shfl_xor(md, off, 64));
    }
    if ((threadIdx.x & 63) == 0) {
        red_x[threadIdx.x >> 6] = mx;
        red_d[threadIdx.x >> 6] = md;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const double m_x = (double)fmaxf(fmaxf(red_x[0], red_x[1]), fmaxf(red_x[2], red_x[3]));
        const double m_d = (double)fmaxf(fmaxf(red_d[0], red_d[1]), fmaxf(red_d[2], red_d[3]));
        double ax = 0.0, ad = 0.0;
        int bl = BL;
        if (m_x != 0.0 && m_d != 0.0) {
            if (dynamic_bl) {                     // shortest train that keeps the probabilities <= 1
                double need = ceil(lr * m_x * m_d / dw_min);
                if (!(need >= 1.0)) need = 1.0;
                if (need > (double)BL) need = (double)BL;
                bl = (int)need;
            }
            const double A = sqrt(lr / (dw_min * (double)bl));
            if (update_management) {
                ax = A * sqrt(m_d / m_x);
                ad = A * sqrt(m_x / m_d);
            } else {
                ax = A;
                ad = A;
            }
        }
        a_x[b] = ax;
        a_d[b] = ad;
        if (bl_b) bl_b[b] = bl;
    }
}

__global__ void __launch_bounds__(256) k_line_scale(const float* __restrict__ x,
                                                    const float* __restrict__ d, int R, int C,
                                                    double lr, double dw_min, int BL, int update_management,
                                                    int dynamic_bl, double* __restrict__ a_x,
                                                    double* __restrict__ a_d, int32_t* __restrict__ bl_b,
                                                    ConvView conv)
{
    line_scale_body(x, d, R, C, lr, dw_min, BL, update_management, dynamic_bl, a_x, a_d, bl_b, conv, (int)blockIdx.x);
}

// OR of a value over aligned groups of 8 or 16 lanes, in every lane of the group: data-parallel
// primitives of the vector ALU (quad permutes, then mirrors of the half row and of the row), no LDS.
template <int GROUP>
__device__ __forceinline__ uint32_t or_across_lines(uint32_t v)
{
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);      // quad_perm [1,0,3,2]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);      // quad_perm [2,3,0,1]
    v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);     // row_half_mirror
    if (GROUP == 16) v |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true);   // row_mirror
    return v;
}
template <int GROUP>
__device__ __forceinline__ uint64_t or_across_lines(uint64_t v)
{
    return ((uint64_t)or_across_lines<GROUP>((uint32_t)(v >> 32)) << 32) | or_across_lines<GROUP>((uint32_t)v);
}

constexpr int kGroupMax = 16;                    // tiles whose kernels share one launch, at most

// A kernel whose only argument is a group { n, ..., first_block[kGroupMax + 1], e[kGroupMax] } finds the entry
// that owns this workgroup and the workgroup's index inside the entry's range.  The group is read word by word
// from the kernel-argument segment through the constant address space: loads from there at a wave-uniform
// address are scalar loads, so that the entry's pointers and arguments sit in scalar registers as the kernel
// arguments of a single tile's launch do (indexing the by-value struct with a run-time index made the compiler
// treat them as per-lane values).
template <typename Group, typename Entry>
__device__ __forceinline__ Entry group_entry_of_block(uint32_t* block)
{
    static_assert(sizeof(Entry) % 4 == 0 && offsetof(Group, e) % 4 == 0, "copied in 32-bit words");
    typedef __attribute__((address_space(4))) const uint32_t const_u32;
    const_u32* words = (const_u32*)__builtin_amdgcn_kernarg_segment_ptr();
    const uint32_t n = words[offsetof(Group, n) / 4];
    const_u32* first = words + offsetof(Group, first_block) / 4;
    uint32_t i = 0;
    while (i + 1 < n && blockIdx.x >= first[i + 1]) ++i;                     // uniform over the workgroup
    *block = blockIdx.x - first[i];
    const_u32* src = words + (offsetof(Group, e) + (size_t)i * sizeof(Entry)) / 4;
    uint32_t raw[sizeof(Entry) / 4];
#pragma unroll
    for (int k = 0; k < (int)(sizeof(Entry) / 4); ++k) raw[k] = src[k];
    Entry e;
    __builtin_memcpy(&e, raw, sizeof(e));
    return e;
}

// ------------------------------------------------------------------------------------------
// Pulse words.  One thread per line value: threshold T = floor(min(1, a|v|) 2^32) in fp64,
// pulse n set iff Philox word n&3 of block n>>2 is below T; top bit = line value negative.
// Internal layout: xw[B][Cpad] and dw[Rpad][Bpad] (a row's words of consecutive samples lie side by
// side: the cell kernel fetches them a group of samples at a time with one scalar load per row, and
// consecutive groups share a cache line) with Cpad = C rounded up to 64, Rpad = R rounded up to 16
// and Bpad = B rounded up to 16; the padding columns and rows are filled with zero words so that
// the cell kernel needs no edge masks, the padding samples are never read.
// grid.x covers the Cpad + Rpad lines of one sample, grid.y strides over the samples.
// ------------------------------------------------------------------------------------------
// Deterministic trains use no random numbers: pulse n is set iff u_n < T / 2^32 with
// u_n = (n + 1/2) / BL for column lines and the bit-reversed, digitally shifted pulse number
// (brev(n) xor 0xAAAAAAAA) / 2^32 for row lines (a shifted Hammersley point set).
// Stochastic trains need random numbers only for line values with 0 < a|v| < 1: a zero value has
// no pulses and a saturated one has them all.  Where many lanes of a wave need none (activations
// after a rectifier: about half are zero), the lanes that do are listed in LDS and their Philox
// blocks are dealt out over the whole wave, 64 / kBlocks lines at a time with one block per lane;
// the four compare bits of each block are OR-ed together across the lanes of a line and the owner
// of the line fetches the word.  The counters are those of the plain path: same words.
// (The body is a device function so that one launch can also draw the words of several tiles, see
// k_pulse_words_group: workgroup `bx` of the lines, samples `by`, `by + ny`, ...)
template <typename WordT>
__device__ __forceinline__ void
pulse_words_body(const float* __restrict__ x, const float* __restrict__ d, int B, int R, int C, int Rpad, int Cpad,
                 int Bpad, int BL, double A, const double* __restrict__ a_x, const double* __restrict__ a_d,
                 const int32_t* __restrict__ bl_b, int deterministic,
                 uint32_t k0, uint32_t k1, uint32_t t, const uint32_t* step_on_device, WordT* __restrict__ xw,
                 WordT* __restrict__ dw, const ConvView& conv, unsigned long long* __restrict__ row_words_with_pulses,
                 const uint32_t bx, const uint32_t by, const uint32_t ny)
{
    constexpr int kBlocks = (sizeof(WordT) == 4) ? 8 : 16;       // Philox blocks per line value, at most
    constexpr int kLines = 64 / kBlocks;                         // lines served at a time by the shared path
    __shared__ uint32_t needy_list[4][64][2];                    // per wave: lane and threshold of the lines that need random numbers
    const int l = (int)(bx * 256 + threadIdx.x);
    const bool live = l < Cpad + Rpad;                           // (no early exit: the shared path needs whole waves)
    const bool is_x = l < Cpad;                                  // uniform per wave (Cpad % 64 == 0)
    const int idx = is_x ? l : l - Cpad;
    const int len = is_x ? C : R;
    const uint32_t tagw = (is_x ? kTagX : kTagD) << 24;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    if (step_on_device) t = *(const volatile uint32_t*)step_on_device;   // a recorded call: the device's counter
    for (uint32_t b = by; b < (uint32_t)B; b += ny) {
        WordT word = 0;
        const int bl = bl_b ? bl_b[b] : BL;
        const int nblk = (bl + 3) >> 2;
        bool random = false;                                     // this line needs random numbers
        bool negative = false;
        uint32_t Tlo = 0;
        if (live && idx < len) {
            const float v = is_x ? view_x(x, conv, b, idx, C) : view_d(d, conv, b, idx, R);
            const double a = a_x ? (is_x ? a_x[b] : a_d[b]) : A;
            const float av = fabsf(v);
            if (av > 0.0f && av < __builtin_inff() && a > 0.0) {
                double p = a * (double)av;
                if (!(p < 1.0)) p = 1.0;
                const uint64_t T = (uint64_t)(p * 4294967296.0);      // 0 .. 2^32
                if (T != 0) {
                    if (deterministic) {
                        const uint64_t lim = 2ull * (uint64_t)bl * T;
                        for (int n = 0; n < bl; ++n) {
                            const bool set = is_x ? (((uint64_t)(2 * n + 1)) << 32) < lim
                                                  : (uint64_t)(__brev((uint32_t)n) ^ 0xAAAAAAAAu) < T;
                            word |= (WordT)(set ? 1u : 0u) << n;
                        }
                    } else if ((T >> 32) != 0) {
                        word = (((WordT)1 << bl) - 1);                // saturated: every pulse
                    } else {
                        random = true;
                        Tlo = (uint32_t)T;
                    }
                }
                negative = v < 0.0f;
            }
        }
        const unsigned long long need = __ballot(random);
        const int count = __popcll(need);
        // one block per lane and round for ceil(count / kLines) rounds, against nblk blocks per lane
        if (count != 0 && (count + kLines - 1) / kLines * 3 < nblk * 2) {
            const uint32_t rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(need >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)need, 0u));
            if (random) {
                needy_list[wave][rank][0] = lane;
                needy_list[wave][rank][1] = Tlo;
            }
            __builtin_amdgcn_wave_barrier();     // a wave's LDS operations take effect in program order
            const uint32_t blk = lane % kBlocks, slot = lane / kBlocks;
            for (int r0 = 0; r0 < count; r0 += kLines) {
                const uint32_t r = (uint32_t)r0 + slot;              // the listed line this lane works for
                uint32_t part = 0;
                if (r < (uint32_t)count && blk < (uint32_t)nblk) {
                    const uint32_t src = needy_list[wave][r][0], Ts = needy_list[wave][r][1];
                    const uint32_t sidx = (uint32_t)idx - lane + src;
                    const U4 q = philox4x32_10(sidx, b, t, tagw | blk, k0, k1);
                    part = (uint32_t)(q.x < Ts) | ((uint32_t)(q.y < Ts) << 1) | ((uint32_t)(q.z < Ts) << 2) |
                           ((uint32_t)(q.w < Ts) << 3);
                }
                WordT w = (WordT)part << (4 * blk);
                w = or_across_lines<kBlocks>(w);
                // the owner of listed line r0 + s finds its word in the lanes of slot s
                const WordT got = (WordT)__shfl(w, (int)((rank % kLines) * kBlocks), 64);
                if (random && rank >= (uint32_t)r0 && rank < (uint32_t)(r0 + kLines)) word = got;
            }
            __builtin_amdgcn_wave_barrier();     // the list is written again for the next sample
            if (random) word &= (((WordT)1 << bl) - 1);
        } else if (random) {
            for (int blk = 0; blk < nblk; ++blk) {
                const U4 r = philox4x32_10((uint32_t)idx, b, t, tagw | (uint32_t)blk, k0, k1);
                const uint32_t bits = (uint32_t)(r.x < Tlo) | ((uint32_t)(r.y < Tlo) << 1) |
                                      ((uint32_t)(r.z < Tlo) << 2) | ((uint32_t)(r.w < Tlo) << 3);
                word |= (WordT)bits << (4 * blk);
            }
            word &= (((WordT)1 << bl) - 1);
        }
        // how many row trains have a pulse at all, counted on every 16th sample (atomics on one address
        // serialise: counting all 12 544 samples of a long batch cost 0.3 ms): the host reads the sum now and
        // then and, where most trains have none, lets the cell update walk per-row lists of the samples that do
        if (row_words_with_pulses && !is_x && (b & 15u) == 0u) {
            const unsigned long long some = __ballot(word != 0);
            if (lane == 0 && some) atomicAdd(row_words_with_pulses, (unsigned long long)__popcll(some));
        }
        if (negative) word |= (WordT)1 << WordTraits<WordT>::kSignBit;
        if (live) {
            if (is_x) xw[(size_t)b * Cpad + idx] = word;
            else dw[(size_t)idx * Bpad + b] = word;
        }
    }
}

template <typename WordT>
__global__ void __launch_bounds__(256)
k_pulse_words(const float* __restrict__ x, const float* __restrict__ d, int B, int R, int C, int Rpad, int Cpad,
              int Bpad, int BL, double A, const double* __restrict__ a_x, const double* __restrict__ a_d,
              const int32_t* __restrict__ bl_b, int deterministic,
              uint32_t k0, uint32_t k1, uint32_t t, const uint32_t* step_on_device, WordT* __restrict__ xw,
              WordT* __restrict__ dw, ConvView conv, unsigned long long* __restrict__ row_words_with_pulses)
{
    pulse_words_body<WordT>(x, d, B, R, C, Rpad, Cpad, Bpad, BL, A, a_x, a_d, bl_b, deterministic, k0, k1, t, step_on_device,
                            xw, dw, conv, row_words_with_pulses, blockIdx.x, blockIdx.y, gridDim.y);
}

// The pulse words of several tiles in one launch (aht_pulsed_update_many; no convolution view): entry i owns workgroups first_block[i] .. first_block[i + 1] - 1, laid out
// as nbx workgroups of lines times ny strides of samples, as the grid of its own launch would be.
struct WordsGroupEntry {
    const float *x, *d;
    void *xw, *dw;
    unsigned long long* row_stat;
    const double *a_x, *a_d;                      // per-vector factors and train lengths (k_line_scale_group), or null
    const int32_t* bl_b;
    double A;
    int B, R, C, Rpad, Cpad, Bpad, BL, deterministic;
    uint32_t k0, k1, t, nbx, ny, pad_;
    const uint32_t* step_on_device;               // a recorded call: the step is read from the tile's device counter
};
struct WordsGroup {
    uint32_t n, pad_;
    uint32_t first_block[kGroupMax + 1];
    WordsGroupEntry e[kGroupMax];
};

// The per-vector factors of several tiles in one launch: entry i owns workgroups first_block[i] ..
// first_block[i + 1] - 1, one per update vector.
struct LineScaleGroupEntry {
    const float *x, *d;
    double *a_x, *a_d;
    int32_t* bl_b;
    double lr, dw_min;
    int R, C, BL, update_management, dynamic_bl, pad_;
};
struct LineScaleGroup {
    uint32_t n, pad_;
    uint32_t first_block[kGroupMax + 1];
    LineScaleGroupEntry e[kGroupMax];
};
__global__ void __launch_bounds__(256) k_line_scale_group(LineScaleGroup g)
{
    (void)g;
    uint32_t block;
    const LineScaleGroupEntry e = group_entry_of_block<LineScaleGroup, LineScaleGroupEntry>(&block);
    line_scale_body(e.x, e.d, e.R, e.C, e.lr, e.dw_min, e.BL, e.update_management, e.dynamic_bl, e.a_x, e.a_d, e.bl_b,
                    ConvView{}, (int)block);
}

template <typename WordT>
__global__ void __launch_bounds__(256)
k_pulse_words_group(WordsGroup g)
{
    (void)g;
    uint32_t block;
    const WordsGroupEntry e = group_entry_of_block<WordsGroup, WordsGroupEntry>(&block);
    pulse_words_body<WordT>(e.x, e.d, e.B, e.R, e.C, e.Rpad, e.Cpad, e.Bpad, e.BL, e.A, e.a_x, e.a_d, e.bl_b,
                            e.deterministic, e.k0, e.k1, e.t, e.step_on_device, (WordT*)e.xw, (WordT*)e.dw, ConvView{},
                            e.row_stat, block % e.nbx, block / e.nbx, e.ny);
}

// Per row, the samples whose row train has at least one pulse, in sample order: entry k of row i is
// (sample b, row word), rlist[i * stride + k], k < rlen[i]; 16 all-zero entries follow the last one
// (the cell update reads its list a few entries ahead and in groups).  One workgroup per row takes
// 2048 samples at a time, eight loads per lane in flight (a wave per row with one load in flight was
// bound by the latency of its 196 dependent rounds: 64 us for 256 rows of 12 544 samples); the places
// of a round's entries come from the 32 ballots of its (load, wave) pairs, summed in sample order.
constexpr int kRowListPad = 16;
__global__ void __launch_bounds__(256)
k_compact_rows(const uint32_t* __restrict__ dw, int R, int B, int Bpad, uint2* __restrict__ rlist,
               uint32_t* __restrict__ rlen)
{
    constexpr int kLoads = 8;
    __shared__ uint32_t counts[2][kLoads * 4];
    const int row = (int)blockIdx.x;
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const size_t stride = (size_t)Bpad + kRowListPad;
    uint2* __restrict__ out = rlist + (size_t)row * stride;
    const uint32_t* __restrict__ in = dw + (size_t)row * Bpad;
    uint32_t total = 0;
    int buf = 0;
    for (int b0 = 0; b0 < B; b0 += 256 * kLoads, buf ^= 1) {
        uint32_t w[kLoads], before[kLoads];
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const int b = b0 + u * 256 + (int)threadIdx.x;
            w[u] = b < B ? in[b] : 0u;
        }
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            const unsigned long long m = __ballot((w[u] & 0x7FFFFFFFu) != 0u);
            before[u] = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
            if (lane == 0) counts[buf][u * 4 + (int)wave] = (uint32_t)__popcll(m);
        }
        __syncthreads();                          // (two buffers: the next round's counts go elsewhere)
        uint32_t at = total, round = 0;
#pragma unroll
        for (int k = 0; k < kLoads * 4; ++k) {
            const uint32_t c = counts[buf][k];
            round += c;
#pragma unroll
            for (int u = 0; u < kLoads; ++u)
                if (k < u * 4 + (int)wave) before[u] += c;     // the (load, wave) pairs that come earlier in sample order
        }
#pragma unroll
        for (int u = 0; u < kLoads; ++u)
            if ((w[u] & 0x7FFFFFFFu) != 0u) out[at + before[u]] = make_uint2((uint32_t)(b0 + u * 256 + (int)threadIdx.x), w[u]);
        total += round;
    }
    if (threadIdx.x < (uint32_t)kRowListPad) out[total + threadIdx.x] = make_uint2(0u, 0u);
    if (threadIdx.x == 0) rlen[row] = total;
}

// word format conversions for the debug entry points (public format: u64 [B][len], sign in bit 63;
// internal format: WordT [B][lpad], sign in the top bit, zero padding)
// `bpad` > 0: the internal buffer is sample-contiguous, in[idx][bpad] (row words); 0: in[b][lpad]
template <typename WordT>
__global__ void __launch_bounds__(256) k_words_to_public(const WordT* in, uint64_t* out, int B, int len, int lpad, int bpad)
{
    const size_t k = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= (size_t)B * len) return;
    const size_t b = k / (size_t)len, idx = k - b * (size_t)len;
    const WordT w = bpad ? in[idx * (size_t)bpad + b] : in[b * (size_t)lpad + idx];
    const WordT sign = (WordT)1 << WordTraits<WordT>::kSignBit;
    out[k] = (uint64_t)(w & ~sign) | ((w & sign) ? (1ull << 63) : 0ull);
}

template <typename WordT>
__global__ void __launch_bounds__(256) k_words_from_public(const uint64_t* in, WordT* out, int B, int len, int lpad, int bpad,
                                                           int BL)
{
    const size_t k = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= (size_t)B * lpad) return;
    const size_t b = k / (size_t)lpad, idx = k - b * (size_t)lpad;
    WordT r = 0;
    if (idx < (size_t)len) {
        const uint64_t w = in[b * (size_t)len + idx];
        r = (WordT)(w & ((1ull << BL) - 1));
        if (w >> 63) r |= (WordT)1 << WordTraits<WordT>::kSignBit;
    }
    if (bpad) out[idx * (size_t)bpad + b] = r;
    else out[k] = r;
}

// signed coincidence counts of sample b (debug): +n UP (x_j d_i < 0), -n DOWN
__global__ void __launch_bounds__(256) k_counts(const uint64_t* __restrict__ xw, const uint64_t* __restrict__ dw,
                                                int b, int R, int C, int BL, int8_t* __restrict__ out)
{
    const size_t k = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= (size_t)R * C) return;
    const int i = (int)(k / C), j = (int)(k % C);
    const uint64_t xv = xw[(size_t)b * C + j], dv = dw[(size_t)b * R + i];
    const int n = __popcll(xv & dv & ((1ull << BL) - 1));
    const bool up = ((xv ^ dv) >> 63) != 0;
    out[k] = (int8_t)(up ? n : -n);
}

__global__ void __launch_bounds__(256) k_debug_philox(const uint32_t* ctr, const uint32_t* key, int n, uint32_t* out)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    const U4 r = philox4x32_10(ctr[4 * k], ctr[4 * k + 1], ctr[4 * k + 2], ctr[4 * k + 3], key[2 * k], key[2 * k + 1]);
    out[4 * k] = r.x; out[4 * k + 1] = r.y; out[4 * k + 2] = r.z; out[4 * k + 3] = r.w;
}

__global__ void __launch_bounds__(256) k_debug_gauss(uint32_t k0, uint32_t k1, uint32_t index, uint32_t t,
                                                     uint32_t tag, uint32_t q0, int n, int fast, float* out)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= n) return;
    const uint32_t q = q0 + (uint32_t)k;
    float z[4];
    if (fast) gauss4_fast(k0, k1, index, q >> 2, t, tag, z);
    else gauss4_accurate(k0, k1, index, q >> 2, t, tag, z);
    out[k] = z[q & 3];
}

// ------------------------------------------------------------------------------------------
// The cell update.
//
// Work split: lane <-> column j (coalesced rows of W, the row word is wave-uniform and comes
// through scalar loads), each lane owns RPL cells (rows i0 .. i0+RPL-1 of its column); a
// workgroup is 4 independent waves stacked along the rows.  Weights and device parameters are
// loaded once, stay in registers for all B update vectors and are stored once.
//
// A cell sees few coincidences per sample and their number differs from lane to lane, so the
// samples are not applied in lock-step.
//   Phase A walks the samples at full lane occupancy: count = popcount(x word AND d word), and
//   `count` copies of the direction bit (1 = up) are shifted into a per-cell bit stream, one bit
//   per pulse, in sample order.  The newest bits gather in a 32-bit pending word (two 32-bit
//   operations per sample); only when a pending word of the wave would overflow are they moved
//   to a 64-bit register tail, whose full 32-bit words go to LDS (lane-interleaved, free of
//   bank conflicts).
//   Phase B drains the streams: iteration i handles stream bits 4i..4i+3 of every cell with
//   one Philox block = four Gaussians per cell; all cells of the wave run the same number of
//   iterations (the wave's longest stream).
// Bit p of a cell's stream is pulse number (q & ~31) + p of the call, q being the cell's pulse
// count when the stream was (re)started; the stream therefore starts at bit q & 31 and the
// Gaussian block of iteration i is (q >> 5) * 8 + i.  Pulses of one cell stay in sample order,
// which is all the sequential application asks for (cells are independent), and the Gaussian a
// pulse uses is fixed by its number, so the phase split does not change any result.
// Normally the whole call fits one stream; if a stream runs out of LDS room the wave drains
// early and starts new streams.
// ------------------------------------------------------------------------------------------
struct CellArgs {
    int R, C, B, Bpad, Cpad;
    uint32_t nbx, nby;            // tiles along columns / rows
    uint32_t bx0;                 // first column strip of this launch (a caller that knows where x is
                                  // non-zero leaves the other strips out: their cells get no pulses)
    uint32_t k0, k1, t;           // t: the step of the call ...
    float c2c;
    int qwords;                   // 32-bit words of stream storage per cell (>= 5)
    // The tile's step counter also lives in device memory, so that a sequence of update calls can be recorded
    // once in a HIP graph and replayed.  A call made directly takes its step from the host (t) and, if it
    // counts, leaves t + 1 in the device's counter (`publish`; nobody reads the counter while it runs).  A call
    // being recorded reads its step from the device's counter instead (`step_on_device`), and a one-thread
    // kernel after it advances the counter.  (Counting finished waves in the kernel to let the last one
    // advance it cost 1.7 ms on the 4096 x 4096 tile: 65 536 returning atomics on one address, about 30 ns each.)
    const uint32_t* step_on_device;
    uint32_t* publish;
};

// counter = value, or counter += value
__global__ void k_set_step(uint32_t* counter, uint32_t value, int relative)
{
    *counter = relative ? *counter + value : value;
}

// a directly made call that counts: leave the next step in the device's counter
__device__ __forceinline__ void publish_step(const CellArgs& a)
{
    if (a.publish && blockIdx.x == 0 && threadIdx.x == 0) *a.publish = a.t + 1u;
}

// after the body of k_update_small (few workgroups): the last wave to get here advances the counter
// (state[0]; state[1] counts the finished waves)
__device__ __forceinline__ void finish_step(uint32_t* state, uint32_t waves_of_launch)
{
    if ((threadIdx.x & 63u) == 0u) {
        const uint32_t before = atomicAdd(state + 1, 1u);
        if (before + 1u == waves_of_launch) {      // every other wave has read the step long ago
            state[1] = 0u;
            atomicAdd(state, 1u);
        }
    }
}

// select by an all-ones / all-zeros mask: (m & a) | (~m & b), one v_bfi_b32
__device__ __forceinline__ float mask_select(uint32_t m, float a, float b)
{
    return __uint_as_float((m & __float_as_uint(a)) | (~m & __float_as_uint(b)));
}

// One pulse through the response curve.  dmask = ~0 for an UP pulse (dw_up, slope_up), 0 for a
// DOWN pulse (dw_down, slope_down); s_dn_neg is -dw_down so that the direction is one select.
template <int KIND, bool NOISE>
__device__ __forceinline__ float device_step(float w, uint32_t dmask, float z, float c2c, float s_up, float s_dn_neg,
                                             float bmax, float bmin, float sl_up, float sl_dn)
{
    float s = mask_select(dmask, s_up, s_dn_neg);
    if (KIND != kConstantStep) {
        const float sl = mask_select(dmask, sl_up, sl_dn);
        s *= fmaxf(0.0f, fmaf(-sl, w, 1.0f));
    }
    const float noise = NOISE ? fmaf(c2c, z, 1.0f) : 1.0f;
    const float wn = fmaf(s, noise, w);
    return __builtin_amdgcn_fmed3f(wn, bmin, bmax);      // clamp; bmin <= 0 <= bmax
}

// LDS is addressed through 32-bit local pointers kept in registers
typedef __attribute__((address_space(3))) uint32_t lds_u32;
__device__ __forceinline__ void lds_store_u32(uint32_t addr, uint32_t v) { *(lds_u32*)(size_t)addr = v; }
__device__ __forceinline__ uint32_t lds_load_u32(uint32_t addr) { return *(const lds_u32*)(size_t)addr; }
__device__ __forceinline__ void lds_atomic_add_u32(uint32_t addr, uint32_t v)
{
    (void)__hip_atomic_fetch_add((lds_u32*)(size_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ uint32_t lds_atomic_add_rtn_u32(uint32_t addr, uint32_t v)
{
    return __hip_atomic_fetch_add((lds_u32*)(size_t)addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// lane index from the execution mask: valid where all lanes of the wave are active, which holds
// everywhere in the cell kernel (its branches are wave-uniform); costs two instructions and no
// long-lived register
__device__ __forceinline__ uint32_t lane_by_count()
{
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t o = (uint32_t)__shfl_xor((int)v, off, 64);
        v = v > o ? v : o;
    }
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)v);
}

// W [R][C] in/out; planes [R][C]; xw[B][Cpad], dw[Rpad][Bpad]: internal zero-padded pulse words.
// The pointers are separate restrict-qualified parameters so that the wave-uniform row words
// are fetched with scalar loads.
// (The body is a device function of its own so that one launch can run it with two different
// numbers of rows per lane, see k_cell_update_pair; `block` is the workgroup's index in its part.)
// SPARSE (one row per lane, 32-bit words): phase A walks the row's list of samples whose row train has a
// pulse (rlist, rlen: see k_compact_rows) instead of all B samples; a sample left out gives every cell of
// the row the count zero, so the streams, and with them all results, are the same.
template <int KIND, typename WordT, bool NOISE, int RPL, bool SPARSE = false, bool GROUPED = false>
__device__ __forceinline__ void
cell_update_body(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
                 const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
                 const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
                 const WordT* __restrict__ xw, const WordT* __restrict__ dw,
                 unsigned long long* __restrict__ pulse_count, const CellArgs& a, const uint32_t block,
                 const uint2* __restrict__ rlist = nullptr, const uint32_t* __restrict__ rlen = nullptr)
{
    static_assert(!SPARSE || (RPL == 1 && sizeof(WordT) == 4), "row lists: one row per lane, 32-bit words");
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) unsigned char*)lds;
    constexpr int kSign = WordTraits<WordT>::kSignBit;
    constexpr WordT kBits = (WordT)(~((WordT)1 << kSign));
    constexpr int G = AHT_GROUP;                  // samples per group: one load batch, one overflow check
    constexpr uint32_t kWordStride = 64 * 4;      // bytes between consecutive words of one stream

    // XCD-aware tile mapping.  Consecutive workgroup ids go round-robin to the 8 XCDs, so each
    // XCD gets one contiguous range of the tile sequence; the sequence walks super-tiles of
    // kSuperY row blocks x kSuperX column strips so that the x words (per strip) and d words
    // (per row block) a range touches stay resident in that XCD's 4 MB L2.  Super-tiles at the
    // lower and right edges are clipped to the tiles that exist, so that the sequence has no holes
    // and every XCD gets the same number of tiles whatever the shape.
    constexpr uint32_t kSuperY = 64, kSuperX = 8;
    const uint32_t total = a.nby * a.nbx;
    const uint32_t per = (total + 7u) >> 3;
    const uint32_t seq = (block & 7u) * per + (block >> 3);
    if ((block >> 3) >= per || seq >= total) return;
    const uint32_t colsize = a.nby * kSuperX;                        // tiles of a full-width column of super-tiles
    uint32_t sx = seq / colsize;
    const uint32_t full_x = a.nbx / kSuperX;
    if (sx > full_x) sx = full_x;                                    // (the clipped last column is narrower)
    const uint32_t off = seq - sx * colsize;
    const uint32_t wd = sx < full_x ? kSuperX : a.nbx - full_x * kSuperX;    // strips in this column
    const uint32_t rowsize = kSuperY * wd;                           // tiles of a full-height super-tile here
    uint32_t sy = off / rowsize;
    const uint32_t full_y = a.nby / kSuperY;
    if (sy > full_y) sy = full_y;
    const uint32_t in = off - sy * rowsize;
    const uint32_t ht = sy < full_y ? kSuperY : a.nby - full_y * kSuperY;    // row blocks in this super-tile
    const uint32_t by = sy * kSuperY + (in % ht), bxr = sx * kSuperX + (in / ht);
    const uint32_t bx = a.bx0 + bxr;              // the launch covers strips bx0 .. bx0 + nbx - 1

    AHT_STAMP(0);                                 // start
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = (int)bx * 64 + lane;            // < Cpad
    const int i0 = ((int)by * 4 + wave) * RPL;    // i0 + RPL <= Rpad
    if (i0 >= a.R) return;                        // wave-uniform; the kernel has no barriers
    const int R = a.R, C = a.C, B = a.B;
    const size_t xstride = (size_t)a.Cpad, drow = (size_t)a.Bpad;
    const WordT* __restrict__ xp = xw + (size_t)bx * 64;   // wave-uniform: the strip's first column

    float w[RPL];
    uint32_t q[RPL];
    // LDS address of the lane's first stream; stream c starts c * cell_stride bytes further (wave-uniform)
    const uint32_t qb0 = lds0 + (uint32_t)((wave * RPL * a.qwords * 64 + lane) * 4);
    const uint32_t cell_stride = (uint32_t)a.qwords * kWordStride;
    auto qb = [&](int c) __attribute__((always_inline)) { return qb0 + (uint32_t)c * cell_stride; };
    uint32_t acc_lo[RPL], acc_hi[RPL], fill[RPL], wp[RPL];   // stream tail, its length, LDS write pointer
    uint32_t pend[RPL], plen[RPL];                           // bits not yet in the tail (plen <= 31)
    bool cv[RPL];
#pragma unroll
    for (int c = 0; c < RPL; ++c) {
        cv[c] = ((i0 + c) < R) && (j < C);
        const size_t k = cv[c] ? ((size_t)(i0 + c) * C + j) : 0;
        // weights and device parameters are touched once per call: stream them past the L2 so that
        // the pulse words, which every tile of a super-tile re-reads, stay resident
        w[c] = __builtin_nontemporal_load(W + k);
        q[c] = 0;
        acc_lo[c] = 0;
        acc_hi[c] = 0;
        fill[c] = 0;
        wp[c] = qb(c);
        pend[c] = 0;
        plen[c] = 0;
    }

    // At four rows per lane, where registers are short, the pulse counts of a wave's cells rest in its
    // exchange buffer between drains (only the drain uses it), at the cells' home places, and not in
    // registers.
    AHT_STAMP(1);                                 // the weights have arrived
    constexpr bool kParkCounts = RPL == 4;
    if (kParkCounts) {
        const uint32_t xhome = lds0 + (uint32_t)(4 * RPL * 64 * a.qwords * 4) + (uint32_t)wave * 1024u +
                               (uint32_t)(lane * RPL) * 4u;
#pragma unroll
        for (int c = 0; c < RPL; ++c) lds_store_u32(xhome + (uint32_t)c * 4u, 0u);
    }

    // Append `n` (<= 31, and fill + n <= 64) copies of the direction bit to the stream tail.
    auto append = [&](int c, uint32_t n, uint32_t m) __attribute__((always_inline)) {
        const uint64_t acc = (((uint64_t)acc_hi[c] << 32) | acc_lo[c]) << n;
        const uint32_t ones = (1u << n) - 1u;                        // n <= 31; one v_bfm_b32
        acc_lo[c] = (ones & m) | (uint32_t)acc;
        acc_hi[c] = (uint32_t)(acc >> 32);
        fill[c] += n;
    };
    // Move one full word (the oldest 32 bits of the tail) to LDS if there is one.  The store is
    // unconditional; the write pointer only moves when the word was full.
    auto flush = [&](int c) __attribute__((always_inline)) {
        const uint64_t acc = ((uint64_t)acc_hi[c] << 32) | acc_lo[c];
        lds_store_u32(wp[c], (uint32_t)(acc >> ((fill[c] - 32u) & 63u)));
        wp[c] += (fill[c] & 32u) << 3;                               // one word = kWordStride bytes; fill < 64
        fill[c] &= 31u;
    };
    // The bits of several samples are first gathered in a 32-bit word (`pend`: they enter at the top,
    // one funnel shift per sample, so the newest bit is the highest and the bits below the `plen`
    // valid ones are zero) and moved to the tail, newest bit lowest, only when some cell of the wave
    // would overflow it: one bit reversal, one 64-bit shift and one flush per commit instead of per
    // sample.
    auto commit = [&](int c) __attribute__((always_inline)) {
        const uint64_t acc = (((uint64_t)acc_hi[c] << 32) | acc_lo[c]) << plen[c];
        acc_lo[c] = (uint32_t)acc | __builtin_bitreverse32(pend[c]);
        acc_hi[c] = (uint32_t)(acc >> 32);
        fill[c] += plen[c];                                          // < 32 + 32
        flush(c);
        pend[c] = 0;
        plen[c] = 0;
    };

    // ---- phase B: drain the streams ---------------------------------------------------
    // `last`: no more samples follow.  Then the lane's cells may change places: sorted by stream
    // length, the c-th cells of the 64 lanes are more alike, the rows of the wave end closer to
    // their longest stream and fewer of their iterations need masks.
    auto drain = [&](bool last) __attribute__((always_inline)) {
        // The lane index is worked out again and made opaque: whatever the drain derives from it (the
        // cells' indices, the LDS addresses of the dealing, origins) is then formed here and not kept
        // in registers through phase A.
        AHT_STAMP(2);                             // phase A over (of the last drain, if there are several)
        if constexpr (SPARSE) __builtin_amdgcn_s_setprio(0);
        int dlane = (int)lane_by_count();
        asm volatile("" : "+v"(dlane));
        uint32_t tstep = a.t;
        if (a.step_on_device) tstep = *(const volatile uint32_t*)a.step_on_device;   // (a recorded call)
        // The device parameters are needed only here.  Loading them now (normally once per call)
        // keeps 6 registers per cell free during phase A.
        float s_up[RPL], s_dn_neg[RPL], bmax[RPL], bmin[RPL], sl_up[RPL], sl_dn[RPL];
        uint32_t cellid[RPL];                     // index of the cell in the matrix (0 for cells outside it)
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            const int jd = (int)bx * 64 + dlane;
            const uint32_t k = ((i0 + c) < R && jd < C) ? (uint32_t)((size_t)(i0 + c) * C + jd) : 0u;
            cellid[c] = k;
            s_up[c] = __builtin_nontemporal_load(p_dw_up + k);
            s_dn_neg[c] = -__builtin_nontemporal_load(p_dw_down + k);
            bmax[c] = __builtin_nontemporal_load(p_b_max + k);
            bmin[c] = __builtin_nontemporal_load(p_b_min + k);
            sl_up[c] = 0.0f;
            sl_dn[c] = 0.0f;
            if (KIND == kLinearStep) {
                sl_up[c] = __builtin_nontemporal_load(p_slope_up + k);
                sl_dn[c] = __builtin_nontemporal_load(p_slope_down + k);
            } else if (KIND == kSoftBounds) {
                sl_up[c] = (bmax[c] != 0.0f) ? 1.0f / bmax[c] : 0.0f;
                sl_dn[c] = (bmin[c] != 0.0f) ? 1.0f / bmin[c] : 0.0f;
            }
        }
        // Per cell: stream end, Gaussian block of the next iteration, current stream word, the LDS
        // address of its stream, and where it came from (cells may change lanes below).  A stream
        // starts at bit q & 31.
        uint32_t endpos[RPL], blk[RPL], D[RPL], sbase[RPL], origin[RPL];
        if (kParkCounts) {                        // the pulse counts, parked by the previous drain
            const uint32_t xhome = lds0 + (uint32_t)(4 * RPL * 64 * a.qwords * 4) + (uint32_t)wave * 1024u +
                                   (uint32_t)(dlane * RPL) * 4u;
#pragma unroll
            for (int c = 0; c < RPL; ++c) q[c] = lds_load_u32(xhome + (uint32_t)c * 4u);
        }
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            commit(c);
            lds_store_u32(wp[c], acc_lo[c] << ((32u - fill[c]) & 31u));      // left-aligned partial word
            endpos[c] = ((wp[c] - qb(c)) >> 3) + fill[c];                    // 32 bits per 256-byte step
            D[c] = 0;
            sbase[c] = qb(c);
            origin[c] = (uint32_t)(dlane * RPL + c);
        }
        // Several rows per lane: before a drain the wave's cells are dealt out again, the 64
        // shortest streams to slot 0 of the 64 lanes, the next 64 to slot 1, and so on, so that the
        // cells a drain iteration handles together are alike in length and few lanes idle while a
        // row finishes.  A cell's whole state moves through a 1 KB exchange buffer behind the
        // wave's streams.  Positions come from a counting sort on the stream length (buckets of two
        // pulses): histogram, exclusive scan, one returning atomic per cell.  A wave's LDS
        // operations take effect in program order, so the steps need no barrier.
        AHT_STAMP(3);                             // device parameters loaded, streams closed
        const bool sorted = RPL > 1;
        const uint32_t xbuf = lds0 + (uint32_t)(4 * RPL * 64 * a.qwords * 4) + (uint32_t)wave * 1024u;
        if (sorted) {
            constexpr uint32_t kBuckets = 192;                       // 3 per lane
            auto bucket_of = [&](int c) __attribute__((always_inline)) {
                const uint32_t bk = endpos[c] >> 1;
                return bk < kBuckets - 1 ? bk : kBuckets - 1;
            };
#pragma unroll
            for (int k = 0; k < 3; ++k) lds_store_u32(xbuf + (uint32_t)(3 * dlane + k) * 4u, 0u);
#pragma unroll
            for (int c = 0; c < RPL; ++c) lds_atomic_add_u32(xbuf + bucket_of(c) * 4u, 1u);
            uint32_t h[3];
#pragma unroll
            for (int k = 0; k < 3; ++k) h[k] = lds_load_u32(xbuf + (uint32_t)(3 * dlane + k) * 4u);
            const uint32_t mine = h[0] + h[1] + h[2];
            uint32_t incl = mine;                                    // inclusive scan over the lanes
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = (uint32_t)__shfl_up((int)incl, off, 64);
                incl += (dlane >= off) ? up : 0u;
            }
            const uint32_t excl = incl - mine;
            lds_store_u32(xbuf + (uint32_t)(3 * dlane) * 4u, excl);
            lds_store_u32(xbuf + (uint32_t)(3 * dlane + 1) * 4u, excl + h[0]);
            lds_store_u32(xbuf + (uint32_t)(3 * dlane + 2) * 4u, excl + h[0] + h[1]);
            uint32_t pos[RPL];                                       // LDS byte offset of the cell's new place
#pragma unroll
            for (int c = 0; c < RPL; ++c)
                pos[c] = lds_atomic_add_rtn_u32(xbuf + bucket_of(c) * 4u, 1u) * 4u;   // places 0 .. 64 RPL - 1, each once
            // every field: four stores to the cells' new places, four loads of the lane's new cells
            auto move_u32 = [&](uint32_t (&v)[RPL]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < RPL; ++c) lds_store_u32(xbuf + pos[c], v[c]);
#pragma unroll
                for (int c = 0; c < RPL; ++c) v[c] = lds_load_u32(xbuf + (uint32_t)(c * 64 + dlane) * 4u);
            };
            auto move_f32 = [&](float (&v)[RPL]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < RPL; ++c) lds_store_u32(xbuf + pos[c], __float_as_uint(v[c]));
#pragma unroll
                for (int c = 0; c < RPL; ++c) v[c] = __uint_as_float(lds_load_u32(xbuf + (uint32_t)(c * 64 + dlane) * 4u));
            };
            move_u32(endpos); move_u32(q); move_u32(sbase); move_u32(origin); move_u32(cellid);
            move_f32(w); move_f32(s_up); move_f32(s_dn_neg); move_f32(bmax); move_f32(bmin);
            if (KIND != kConstantStep) {
                move_f32(sl_up);
                move_f32(sl_dn);
            }
        }
        AHT_STAMP(4);                             // cells dealt
#pragma unroll
        for (int c = 0; c < RPL; ++c) blk[c] = (q[c] >> 5) << 3;
        // Wave-uniform per row: iterations its longest stream needs, and the iteration from which
        // some stream of the row has fewer than four pulses left.
        int row_iters[RPL], row_plain_end[RPL];
        int niter = 0, plain_end = 0x7FFFFFFF;
        uint32_t last_start = 0;
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            row_iters[c] = (int)((wave_max_u32(endpos[c]) + 3u) >> 2);
            row_plain_end[c] = (int)(~wave_max_u32(~endpos[c]) >> 2);        // wave minimum, rounded down
            niter = niter > row_iters[c] ? niter : row_iters[c];
            plain_end = plain_end < row_plain_end[c] ? plain_end : row_plain_end[c];
            last_start = last_start > (q[c] & 31u) ? last_start : (q[c] & 31u);
        }
        const int plain_begin = (int)((wave_max_u32(last_start) + 3u) >> 2);  // every stream has started
        const float c2c_unit = a.c2c * kGaussUnitScale;              // the Gaussians below come without this factor
        auto load_words = [&](int i) __attribute__((always_inline)) {
            if ((i & 7) == 0) {
#pragma unroll
                for (int c = 0; c < RPL; ++c)
                    D[c] = lds_load_u32(sbase[c] + (uint32_t)(i >> 3) * kWordStride);
            }
        };
        // Stream bits 4i .. 4i+3 of the lanes' c-th cells.  mode 0: all four pulses exist in every
        // lane; 1: head (streams may start after bit 4i); 2: tail (streams may end before bit 4i + 4)
        auto row_step = [&](int i, int c, auto mode_tag) __attribute__((always_inline)) {
            constexpr int mode = decltype(mode_tag)::value;
            float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (NOISE) gauss4_unit(a.k0, a.k1, cellid[c], blk[c], tstep, kTagC2C, z);
            blk[c] += 1;
            const int lo = (int)(q[c] & 31u) - 4 * i, hi = (int)endpos[c] - 4 * i;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t dmask = (uint32_t)__builtin_amdgcn_sbfe((int)D[c], 31 - k, 1);
                const float wn = device_step<KIND, NOISE>(w[c], dmask, z[k], c2c_unit, s_up[c], s_dn_neg[c],
                                                          bmax[c], bmin[c], sl_up[c], sl_dn[c]);
                if (mode == 1) w[c] = ((k >= lo) & (k < hi)) ? wn : w[c];
                else if (mode == 2) w[c] = (k < hi) ? wn : w[c];
                else w[c] = wn;
            }
            D[c] <<= 4;
        };
        int i = 0;
        const int head_end = plain_begin < niter ? plain_begin : niter;
        for (; i < head_end; ++i) {
            load_words(i);
#pragma unroll
            for (int c = 0; c < RPL; ++c)
                if (i < row_iters[c]) row_step(i, c, std::integral_constant<int, 1>{});
        }
        for (; i < plain_end; ++i) {              // all rows in one block
            load_words(i);
#pragma unroll
            for (int c = 0; c < RPL; ++c) row_step(i, c, std::integral_constant<int, 0>{});
        }
        for (; i < niter; ++i) {                  // rows end one after the other
            load_words(i);
#pragma unroll
            for (int c = 0; c < RPL; ++c) {
                if (i >= row_iters[c]) continue;  // all 64 cells of this row are done
                if (i < row_plain_end[c]) row_step(i, c, std::integral_constant<int, 0>{});
                else row_step(i, c, std::integral_constant<int, 2>{});
            }
        }
        AHT_STAMP(5);                             // pulses applied
#pragma unroll
        for (int c = 0; c < RPL; ++c) q[c] += endpos[c] - (q[c] & 31u);      // pulses applied so far
        if (sorted) {
            // The weights go back to where their cells came from; if more samples follow, so do the
            // pulse counts, last of all, so that they stay in the buffer for the next drain (after the
            // last drain only the sum of q is used).
            auto send_home = [&](uint32_t (&v)[RPL]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < RPL; ++c) lds_store_u32(xbuf + origin[c] * 4u, v[c]);
#pragma unroll
                for (int c = 0; c < RPL; ++c) v[c] = lds_load_u32(xbuf + (lane_by_count() * RPL + (uint32_t)c) * 4u);
            };
            uint32_t wbits[RPL];
#pragma unroll
            for (int c = 0; c < RPL; ++c) wbits[c] = __float_as_uint(w[c]);
            send_home(wbits);
#pragma unroll
            for (int c = 0; c < RPL; ++c) w[c] = __uint_as_float(wbits[c]);
            if (!last) send_home(q);
        }
#pragma unroll
        for (int c = 0; c < RPL; ++c) {           // restart the streams at bit q & 31
            acc_lo[c] = 0;
            acc_hi[c] = 0;
            fill[c] = q[c] & 31u;
            wp[c] = qb(c);
        }
        if constexpr (SPARSE) {
            if (!last) __builtin_amdgcn_s_setprio(3);
        }
    };

    // ---- phase A ----------------------------------------------------------------------
    // Walking the lists, a wave in phase A mostly waits for memory (a list entry names the sample whose column
    // words are fetched next), and the few instructions between its waits are worth issuing ahead of the
    // arithmetic of the waves that drain: phase A runs at the highest wave priority, the drain at the lowest
    // (256 x 2304, 12 544 vectors: 1.47 -> 1.37 ms).  The dense walk is left alone: there the same setting
    // costs 7 % on the 4096 x 4096 tile and changes nothing on the small ones, and so does every other
    // assignment tried (drain above phase A: no change anywhere; priority falling with a wave's progress, so that
    // the waves of a SIMD end together: 8 - 15 % slower everywhere).
    if constexpr (SPARSE) __builtin_amdgcn_s_setprio(3);
    const WordT* __restrict__ xcur = xp;          // column words of sample b from the strip's first column on: a
                                                  // scalar base, so that the loads take the lane as a 32-bit
                                                  // offset and need no per-lane address arithmetic
    const uint32_t xlane = (uint32_t)lane;
    uint32_t xoff[G];                             // byte offsets of the lane's words of a group's G samples
#pragma unroll
    for (int u = 0; u < G; ++u) xoff[u] = (uint32_t)(((size_t)u * xstride + xlane) * sizeof(WordT));
    // GROUPED (several tiles in one launch): the pointers come out of a table, not from kernel arguments of their
    // own, and the compiler no longer knows that nothing in this kernel writes the row words; read through the
    // constant address space (an earlier kernel wrote them) they stay scalar loads.
    typedef __attribute__((address_space(4))) const WordT const_word;
    const const_word* dwc = (const const_word*)(size_t)dw;
    auto row_word = [&](size_t at) __attribute__((always_inline)) -> WordT {
        if constexpr (GROUPED) return dwc[at];
        else return dw[at];
    };
    size_t doff = (size_t)i0 * drow;              // dw[doff + c * drow]: row words of sample b (wave-uniform,
                                                  // indexed off the kernel argument so that they stay scalar loads)
    auto load_x = [&](const WordT* __restrict__ p0, WordT (&xg)[G]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < G; ++u) {
            asm volatile("" : "+v"(xoff[u]));     // stays a 32-bit offset beside the scalar base
            xg[u] = *(const WordT*)((const char*)p0 + xoff[u]);
        }
    };
    // ~0 if the word's sign bit is set
    auto sign_mask = [&](WordT v) __attribute__((always_inline)) {
        return (uint32_t)((int32_t)(uint32_t)(v >> (kSign - 31)) >> 31);
    };
    // coincidence counts of one sample for the lane's cells
    auto count = [&](WordT xv, const WordT (&dv)[RPL], uint32_t (&n)[RPL]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            WordT dm = dv[c] & kBits;             // the row word without its sign: on the scalar unit
            if constexpr (sizeof(WordT) == 4 && !SPARSE) asm("" : "+s"(dm)); // (not folded into a three-input vector op)
            const WordT both = xv & dm;
            n[c] = (sizeof(WordT) == 8)
                       ? (uint32_t)__popc((uint32_t)((uint64_t)both >> 32)) + (uint32_t)__popc((uint32_t)both)
                       : (uint32_t)__popc((uint32_t)both);
        }
    };
    // direction masks of one sample: ~0 where x_j d_i < 0, an UP pulse.  The row part is
    // wave-uniform and stays on the scalar unit.
    auto direction_of = [&](uint32_t xm, const WordT (&dv)[RPL], uint32_t (&m)[RPL]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < RPL; ++c) m[c] = xm ^ sign_mask(dv[c]);
    };
    auto direction = [&](WordT xv, const WordT (&dv)[RPL], uint32_t (&m)[RPL]) __attribute__((always_inline)) {
        uint32_t xm = sign_mask(xv);
        asm volatile("" : "+v"(xm));
        direction_of(xm, dv, m);
    };
    // a sample with any count: at most 16 bits at a time, flushing in between
    auto append_slow = [&](const uint32_t (&n)[RPL], const uint32_t (&m)[RPL]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            uint32_t left = n[c];
#pragma unroll
            for (int part = 0; part < 4; ++part) {                   // 4 x 16 >= 63
                const uint32_t take = left < 16u ? left : 16u;
                append(c, take, m[c]);
                flush(c);
                left -= take;
            }
        }
    };

    // A stream may be extended while the word under its write pointer has index <= qwords - 3:
    // a commit adds at most one word, a sample on the slow path at most two, and the drain
    // commits once more and stores the partial word under the pointer.
    const uint32_t last_ok = (uint32_t)(a.qwords - 3) * kWordStride;
    auto nearly_full = [&]() __attribute__((always_inline)) {
        bool nf = false;
#pragma unroll
        for (int c = 0; c < RPL; ++c) nf |= (wp[c] - qb(c)) > last_ok;
        return __any(nf) != 0;
    };
    WordT xg[G];                                  // column words of the group in hand
    if constexpr (SPARSE) {
        // The row's list: entries `pos` .. of (sample, row word).  The loop keeps the entries of the group
        // in hand (e), of the next one (e1) and, on their way, of the one after (e2); the column words of
        // the next group are requested, by the samples e1 names, as soon as the counts and sign masks of
        // this group are taken, into the same registers.
        const size_t lstride = drow + (size_t)kRowListPad;
        const size_t lbase = (size_t)i0 * lstride;
        const int n_list = (int)rlen[i0];
        uint32_t xoff0 = (uint32_t)(xlane * sizeof(WordT));
        const uint32_t xrow_bytes = (uint32_t)(xstride * sizeof(WordT));   // (the host keeps B * xrow_bytes below 2^32)
        auto x_of = [&](uint32_t sample) __attribute__((always_inline)) {
            asm volatile("" : "+v"(xoff0));
            return *(const WordT*)((const char*)xp + (size_t)(sample * xrow_bytes) + xoff0);
        };
        // (read through the constant address space: the lists were written by an earlier kernel and nothing
        // in this one writes them, and a wave-uniform load from there is always a scalar load)
        typedef __attribute__((address_space(4))) const uint32_t const_u32;
        const const_u32* rwords = (const const_u32*)(size_t)rlist;
        auto entry = [&](int at) __attribute__((always_inline)) {
            const size_t k = 2 * (lbase + (size_t)at);
            return make_uint2(rwords[k], rwords[k + 1]);
        };
        uint2 e[G], e1[G], e2[G];
        int pos = 0;
        bool primed = false, done_s = false;
        do {
            bool full = false;
            while (!full && pos < n_list) {
                if (!primed) {                    // (re)start the pipeline at pos
#pragma unroll
                    for (int u = 0; u < G; ++u) {
                        e[u] = entry(pos + u);
                        e1[u] = entry(pos + G + u);
                    }
#pragma unroll
                    for (int u = 0; u < G; ++u) xg[u] = x_of(e[u].x);
                    primed = true;
                }
                uint32_t n[G][RPL], xm[G], sum = 0;
                bool stopped = false, big = false;
                for (;;) {
#pragma unroll
                    for (int u = 0; u < G; ++u) e2[u] = entry(pos + 2 * G + u);
#pragma unroll
                    for (int u = 0; u < G; ++u) {
                        const WordT dv[RPL] = {(WordT)e[u].y};
                        count(xg[u], dv, n[u]);
                        xm[u] = sign_mask(xg[u]);
                        asm volatile("" : "+v"(xm[u]));
                    }
                    asm volatile("" ::: "memory");         // the loads below stay below the last use of xg
#pragma unroll
                    for (int u = 0; u < G; ++u) xg[u] = x_of(e1[u].x);
                    sum = 0;
#pragma unroll
                    for (int u = 0; u < G; ++u) sum += n[u][0];
                    asm volatile("v_add_u32_e32 %0, %0, %1" : "+v"(plen[0]) : "v"(sum));
                    big = sum > 31u;
                    if (__any(plen[0] > 31u)) {
                        stopped = true;
                        break;
                    }
#pragma unroll
                    for (int u = 0; u < G; ++u) {
                        const WordT dv[RPL] = {(WordT)e[u].y};
                        uint32_t m1[RPL];
                        direction_of(xm[u], dv, m1);
                        pend[0] = __builtin_amdgcn_alignbit(m1[0], pend[0], n[u][0]);
                    }
                    pos += G;
#pragma unroll
                    for (int u = 0; u < G; ++u) {
                        e[u] = e1[u];
                        e1[u] = e2[u];
                    }
                    if (pos >= n_list) break;
                }
                if (stopped) {                    // empty the pending word, then deal with the group in hand
                    plen[0] -= sum;
                    commit(0);
                    if (nearly_full()) {          // drain first, then take this group again
                        full = true;
                        primed = false;
                    } else if (__any(big)) {      // a group with a large count: sample by sample while room lasts
                        primed = false;
#pragma unroll
                        for (int u = 0; u < G; ++u) {
                            const WordT dv[RPL] = {(WordT)e[u].y};
                            uint32_t m1[RPL];
                            direction_of(xm[u], dv, m1);
                            append_slow(n[u], m1);
                            pos += 1;
                            if (nearly_full()) {
                                full = true;
                                break;
                            }
                        }
                    } else {                      // fits now: the counts and sign masks are still in hand
                        plen[0] += sum;
#pragma unroll
                        for (int u = 0; u < G; ++u) {
                            const WordT dv[RPL] = {(WordT)e[u].y};
                            uint32_t m1[RPL];
                            direction_of(xm[u], dv, m1);
                            pend[0] = __builtin_amdgcn_alignbit(m1[0], pend[0], n[u][0]);
                        }
                        pos += G;
#pragma unroll
                        for (int u = 0; u < G; ++u) {
                            e[u] = e1[u];
                            e1[u] = e2[u];
                        }
                    }
                }
            }
            done_s = pos >= n_list;
            drain(done_s);
        } while (!done_s);
    } else {
    bool have_x = false;                          // xg holds (or is about to receive) the words of samples b .. b+G-1
    bool more = false;
    int b = 0;
    bool done = false;
    do {
        bool full = false;
        while (!full && b < B) {
            if (b + G <= B) {
                WordT dg[G][RPL];                 // row words of the group (scalar registers)
                uint32_t n[G][RPL], xm[G], sum[RPL];
                bool big = false;
                // the group's bits join the pending words (whose lengths the caller has advanced); then
                // on to the next group, whose column words are already on their way into xg
                auto take_group = [&]() __attribute__((always_inline)) {
#pragma unroll
                    for (int u = 0; u < G; ++u) {
                        uint32_t m1[RPL];
                        direction_of(xm[u], dg[u], m1);
#pragma unroll
                        for (int c = 0; c < RPL; ++c)       // n (<= 31) copies of the direction enter at the top
                            pend[c] = __builtin_amdgcn_alignbit(m1[c], pend[c], n[u][c]);
                    }
                    b += G;
                    xcur += (size_t)G * xstride;
                    doff += (size_t)G;
                    have_x = more;
                };
                // Straight path: groups are taken until some pending word of the wave would overflow.
                // All that a group needs from its column words are the counts and the sign masks; once
                // these are taken, the next group's words load into the same registers and arrive while
                // the bits of this group are appended.
                bool stopped = false;
                if (!have_x) load_x(xcur, xg);
                have_x = true;
                for (;;) {
#pragma unroll
                    for (int u = 0; u < G; ++u)
#pragma unroll
                        for (int c = 0; c < RPL; ++c) dg[u][c] = row_word(doff + (size_t)c * drow + u);
                    __builtin_amdgcn_sched_barrier(0);        // all row words requested before the first is waited for
#pragma unroll
                    for (int u = 0; u < G; ++u) {
                        count(xg[u], dg[u], n[u]);
                        xm[u] = sign_mask(xg[u]);
                        asm volatile("" : "+v"(xm[u]));
                    }
                    more = b + 2 * G <= B;
                    // the loads must not move above the last use of xg (they would need registers of
                    // their own and copies); without a next group the same words are read again
                    asm volatile("" ::: "memory");
                    load_x(more ? xcur + (size_t)G * xstride : xcur, xg);
                    bool over = false;
                    big = false;
#pragma unroll
                    for (int c = 0; c < RPL; ++c) {
                        sum[c] = 0;
#pragma unroll
                        for (int u = 0; u < G; ++u) sum[c] += n[u][c];
                        // in place: the old length need not stay live (it is worked out again if needed)
                        asm volatile("v_add_u32_e32 %0, %0, %1" : "+v"(plen[c]) : "v"(sum[c]));
                        over |= plen[c] > 31u;
                        big |= sum[c] > 31u;
                    }
                    if (__any(over)) {
                        stopped = true;
                        break;
                    }
                    take_group();
                    if (!more) break;             // fewer than G samples left
                }
                if (stopped) {                    // empty the pending words, then deal with the group in hand
#pragma unroll
                    for (int c = 0; c < RPL; ++c) {
                        plen[c] -= sum[c];        // the group was not taken: the lengths before it
                        commit(c);
                    }
                    if (nearly_full()) {          // drain first, then take this group again (its words have
                        full = true;              // been overwritten: they are loaded once more)
                        have_x = false;
                    } else if (__any(big)) {      // a group with a large count: sample by sample while room lasts
                        have_x = false;
#pragma unroll
                        for (int u = 0; u < G; ++u) {
                            uint32_t m1[RPL];
                            direction_of(xm[u], dg[u], m1);
                            append_slow(n[u], m1);
                            b += 1;
                            xcur += xstride;
                            doff += 1;
                            if (nearly_full()) {
                                full = true;
                                break;
                            }
                        }
                    } else {
#pragma unroll
                        for (int c = 0; c < RPL; ++c) plen[c] += sum[c];
                        take_group();
                    }
                }
            } else {                              // fewer than G samples left
#pragma unroll
                for (int c = 0; c < RPL; ++c) commit(c);
                if (nearly_full()) {
                    full = true;
                    break;
                }
                WordT dv[RPL];
#pragma unroll
                for (int c = 0; c < RPL; ++c) dv[c] = row_word(doff + (size_t)c * drow);
                uint32_t n1[RPL], m1[RPL];
                const WordT xv = *(const WordT*)((const char*)xcur + xoff[0]);
                count(xv, dv, n1);
                direction(xv, dv, m1);
                append_slow(n1, m1);
                b += 1;
                xcur += xstride;
                doff += 1;
                full = nearly_full();
            }
        }
        done = b >= B;
        drain(done);
    } while (!done);
    }

    unsigned long long pulses = 0;
    // the column is worked out again (lane index from the execution mask), so that neither the
    // thread index nor a store address has to stay in registers from the start of the kernel to here
    const int j_out = (int)bx * 64 + (int)lane_by_count();
#pragma unroll
    for (int c = 0; c < RPL; ++c) {
        if ((i0 + c) < R && j_out < C) __builtin_nontemporal_store(w[c], W + (size_t)(i0 + c) * C + j_out);
        pulses += q[c];                           // cells outside the matrix see zero words: no pulses
    }
    if (pulse_count) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) pulses += __shfl_xor(pulses, off, 64);
        if (lane == 0 && pulses) atomicAdd(pulse_count, pulses);
    }
    AHT_STAMP(6);                                 // weights stored
    AHT_STAMP(7);                                 // where the wave ran
}

// Register budget: four waves per SIMD (128 registers) at four rows per lane, the variant of large
// tiles, where the host also keeps the LDS streams short enough for four workgroups per compute unit
// (the fourth wave gains more than the dozen spills outside the inner loops cost); five (96
// registers) for 32-bit words at two rows per lane, the variant long batches on small tiles run;
// three otherwise.
template <typename WordT, int RPL>
struct CellOccupancy {
    static constexpr int kWorkgroups = (sizeof(WordT) == 4 && RPL == 2) ? 5 : (RPL == 4) ? 4 : 3;
};

template <int KIND, typename WordT, bool NOISE, int RPL>
__global__ void __launch_bounds__(256, (CellOccupancy<WordT, RPL>::kWorkgroups))
k_cell_update(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
              const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
              const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
              const WordT* __restrict__ xw, const WordT* __restrict__ dw,
              unsigned long long* __restrict__ pulse_count, CellArgs a)
{
    cell_update_body<KIND, WordT, NOISE, RPL>(W, p_dw_up, p_dw_down, p_b_max, p_b_min, p_slope_up, p_slope_down, xw, dw,
                                              pulse_count, a, blockIdx.x);
    publish_step(a);
}

// The cell update along per-row sample lists (one row per lane, 32-bit words), for long batches whose row
// trains are mostly empty.
template <int KIND, bool NOISE>
__global__ void __launch_bounds__(256, 4)
k_cell_update_rowlists(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
                       const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
                       const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
                       const uint32_t* __restrict__ xw, const uint32_t* __restrict__ dw,
                       unsigned long long* __restrict__ pulse_count, CellArgs a, const uint2* __restrict__ rlist,
                       const uint32_t* __restrict__ rlen)
{
    cell_update_body<KIND, uint32_t, NOISE, 1, true>(W, p_dw_up, p_dw_down, p_b_max, p_b_min, p_slope_up, p_slope_down,
                                                     xw, dw, pulse_count, a, blockIdx.x, rlist, rlen);
    publish_step(a);
}

// One launch, two shapes: the first `main_blocks` workgroups work on their range of column strips at RPL
// rows per lane (arguments `a`), the others on theirs at SIDE rows per lane (arguments `b`), so that a
// tile whose waves would not fill the SIMDs a whole number of times ends evenly without a second
// launch.  Registers and LDS are those of the larger shape.
template <int KIND, typename WordT, bool NOISE, int RPL, int SIDE>
__global__ void __launch_bounds__(256, (CellOccupancy<WordT, RPL>::kWorkgroups))
k_cell_update_pair(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
                   const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
                   const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
                   const WordT* __restrict__ xw, const WordT* __restrict__ dw,
                   unsigned long long* __restrict__ pulse_count, CellArgs a, CellArgs b, uint32_t main_blocks)
{
    if (blockIdx.x < main_blocks)
        cell_update_body<KIND, WordT, NOISE, RPL>(W, p_dw_up, p_dw_down, p_b_max, p_b_min, p_slope_up, p_slope_down, xw,
                                                  dw, pulse_count, a, blockIdx.x);
    else
        cell_update_body<KIND, WordT, NOISE, SIDE>(W, p_dw_up, p_dw_down, p_b_max, p_b_min, p_slope_up, p_slope_down, xw,
                                                   dw, pulse_count, b, blockIdx.x - main_blocks);
    publish_step(a);
}

// The cell updates of several tiles in one launch (aht_pulsed_update_many): tiles of the same device kind, word
// width, noise setting and rows per lane, each with its own weights, planes, pulse words and arguments.  The
// workgroups of entry i are blocks first_block[i] .. first_block[i + 1] - 1 (multiples of 8, so that a tile's
// blocks keep their round-robin places on the 8 XCDs); inside its range a workgroup does exactly what it does in
// a launch of the tile's own.  What this buys small tiles: one round of waves per SIMD from each of several
// tiles instead of one round in all, so that a SIMD holds waves at different points of their lives and none of
// them ends alone.
struct CellGroupEntry {
    float* W;
    const float *dw_up, *dw_down, *b_max, *b_min, *slope_up, *slope_down;
    const void *xw, *dw;
    unsigned long long* pulse_count;
    CellArgs a;
};
struct CellGroup {
    uint32_t n;
    uint32_t first_block[kGroupMax + 1];
    CellGroupEntry e[kGroupMax];
};

template <int KIND, typename WordT, bool NOISE, int RPL>
__global__ void __launch_bounds__(256, (CellOccupancy<WordT, RPL>::kWorkgroups))
k_cell_update_group(CellGroup g)
{
    (void)g;
    uint32_t block;
    const CellGroupEntry e = group_entry_of_block<CellGroup, CellGroupEntry>(&block);
    cell_update_body<KIND, WordT, NOISE, RPL, false, true>(e.W, e.dw_up, e.dw_down, e.b_max, e.b_min, e.slope_up,
                                                           e.slope_down, (const WordT*)e.xw, (const WordT*)e.dw,
                                                           e.pulse_count, e.a, block);
    if (e.a.publish && block == 0 && threadIdx.x == 0) *e.a.publish = e.a.t + 1u;
}

// after a recorded shared launch: the device-side step counters of its tiles move on
struct StepGroup {
    uint32_t n, pad_;
    uint32_t* state[kGroupMax];
};
__global__ void k_advance_steps(StepGroup g)
{
    if (threadIdx.x < g.n) *g.state[threadIdx.x] += 1u;
}

// ------------------------------------------------------------------------------------------
// The whole update call in one launch, for tiny tiles and a few update vectors (an on-line update of
// a small layer: 64 x 64, one vector): two dependent launches cost more than the work itself.  A
// workgroup owns 4 rows x 64 columns (one cell per lane), draws the pulse words of its 64 columns and
// 4 rows for all B samples into LDS -- the words of a line are drawn again by every workgroup that
// needs them, which is why this is for small tiles only -- and applies the samples in order, pulse
// by pulse.  Same counters, same arithmetic per pulse (device_step, gauss4_unit) as the two-kernel
// path: same bits.  No update management and no per-sample train length (they need a reduction over
// the whole vector first).
// ------------------------------------------------------------------------------------------
template <typename WordT>
__device__ __forceinline__ WordT line_word(float v, double a, int bl, int deterministic, bool is_x, uint32_t idx,
                                           uint32_t b, uint32_t t, uint32_t k0, uint32_t k1)
{
    const float av = fabsf(v);
    if (!(av > 0.0f && av < __builtin_inff() && a > 0.0)) return 0;
    WordT word = 0;
    double p = a * (double)av;
    if (!(p < 1.0)) p = 1.0;
    const uint64_t T = (uint64_t)(p * 4294967296.0);              // 0 .. 2^32
    if (T != 0) {
        if (deterministic) {
            const uint64_t lim = 2ull * (uint64_t)bl * T;
            for (int n = 0; n < bl; ++n) {
                const bool set = is_x ? (((uint64_t)(2 * n + 1)) << 32) < lim
                                      : (uint64_t)(__brev((uint32_t)n) ^ 0xAAAAAAAAu) < T;
                word |= (WordT)(set ? 1u : 0u) << n;
            }
        } else if ((T >> 32) != 0) {
            word = (((WordT)1 << bl) - 1);
        } else {
            const uint32_t Tlo = (uint32_t)T, tagw = (is_x ? kTagX : kTagD) << 24;
            for (int blk = 0; blk < ((bl + 3) >> 2); ++blk) {
                const U4 r = philox4x32_10(idx, b, t, tagw | (uint32_t)blk, k0, k1);
                const uint32_t bits = (uint32_t)(r.x < Tlo) | ((uint32_t)(r.y < Tlo) << 1) |
                                      ((uint32_t)(r.z < Tlo) << 2) | ((uint32_t)(r.w < Tlo) << 3);
                word |= (WordT)bits << (4 * blk);
            }
            word &= (((WordT)1 << bl) - 1);
        }
    }
    if (v < 0.0f) word |= (WordT)1 << WordTraits<WordT>::kSignBit;
    return word;
}

constexpr int kSmallMaxB = 8;                     // update vectors one launch of k_update_small takes

// (the body is a device function so that one launch can also take several tiny tiles, see
// k_update_small_group: workgroup `block` of the `nblocks` the tile has)
template <int KIND, typename WordT, bool NOISE>
__device__ __forceinline__ void
update_small_body(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
                  const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
                  const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
                  const float* __restrict__ x, const float* __restrict__ d, int B, int R, int C, int BL, double A,
                  int deterministic, uint32_t k0, uint32_t k1, float c2c, unsigned long long* __restrict__ pulse_count,
                  uint32_t t, uint32_t* step_state, int recorded, const ConvView& conv, const uint32_t block,
                  const uint32_t nblocks)
{
    // (a call made directly: the step is t and t + 1 is left in the device's counter; a recorded call reads
    // the counter, and the last wave advances it)
    __shared__ WordT xs[kSmallMaxB][64], ds[kSmallMaxB][4];
    constexpr int kSign = WordTraits<WordT>::kSignBit;
    if (recorded) t = *(const volatile uint32_t*)step_state;
    const int strips = (C + 63) / 64;
    const int j0 = (int)(block % (uint32_t)strips) * 64, i0 = (int)(block / (uint32_t)strips) * 4;
    for (int item = (int)threadIdx.x; item < B * 68; item += 256) {
        const int b = item / 68, l = item % 68;
        if (l < 64) {
            const int j = j0 + l;
            xs[b][l] = j < C ? line_word<WordT>(view_x(x, conv, (uint32_t)b, j, C), A, BL, deterministic, true, (uint32_t)j,
                                                (uint32_t)b, t, k0, k1)
                             : (WordT)0;
        } else {
            const int i = i0 + (l - 64);
            ds[b][l - 64] = i < R ? line_word<WordT>(view_d(d, conv, (uint32_t)b, i, R), A, BL, deterministic, false,
                                                     (uint32_t)i, (uint32_t)b, t, k0, k1)
                                  : (WordT)0;
        }
    }
    __syncthreads();
    const int lane = (int)(threadIdx.x & 63u), wave = (int)(threadIdx.x >> 6);
    const int i = i0 + wave, j = j0 + lane;
    uint32_t q = 0;
    if (i < R && j < C) {
        const size_t k = (size_t)i * C + j;
        float w = W[k];
        const float s_up = p_dw_up[k], s_dn_neg = -p_dw_down[k], bmax = p_b_max[k], bmin = p_b_min[k];
        float sl_up = 0.0f, sl_dn = 0.0f;
        if (KIND == kLinearStep) {
            sl_up = p_slope_up[k];
            sl_dn = p_slope_down[k];
        } else if (KIND == kSoftBounds) {
            sl_up = (bmax != 0.0f) ? 1.0f / bmax : 0.0f;
            sl_dn = (bmin != 0.0f) ? 1.0f / bmin : 0.0f;
        }
        const float c2c_unit = c2c * kGaussUnitScale;
        float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int b = 0; b < B; ++b) {
            const WordT xv = xs[b][lane], dv = ds[b][wave];
            const WordT both = xv & dv & (WordT)(~((WordT)1 << kSign));
            const int n = (sizeof(WordT) == 8) ? __popcll((unsigned long long)both) : __popc((uint32_t)both);
            const uint32_t dmask = (((xv ^ dv) >> kSign) & 1) ? ~0u : 0u;     // x_j d_i < 0: an UP pulse
            for (int p = 0; p < n; ++p) {
                if (NOISE && (q & 3u) == 0u) gauss4_unit(k0, k1, (uint32_t)k, q >> 2, t, kTagC2C, z);
                const uint32_t e = q & 3u;
                const float zq = e == 0 ? z[0] : e == 1 ? z[1] : e == 2 ? z[2] : z[3];
                w = device_step<KIND, NOISE>(w, dmask, zq, c2c_unit, s_up, s_dn_neg, bmax, bmin, sl_up, sl_dn);
                ++q;
            }
        }
        W[k] = w;
    }
    unsigned long long pulses = q;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) pulses += __shfl_xor(pulses, off, 64);
    if (lane == 0 && pulses) atomicAdd(pulse_count, pulses);
    if (recorded) finish_step(step_state, nblocks * 4u);
    else if (block == 0 && threadIdx.x == 0) step_state[0] = t + 1u;
}

template <int KIND, typename WordT, bool NOISE>
__global__ void __launch_bounds__(256)
k_update_small(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
               const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
               const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
               const float* __restrict__ x, const float* __restrict__ d, int B, int R, int C, int BL, double A,
               int deterministic, uint32_t k0, uint32_t k1, float c2c, unsigned long long* __restrict__ pulse_count,
               uint32_t t, uint32_t* step_state, int recorded, ConvView conv)
{
    update_small_body<KIND, WordT, NOISE>(W, p_dw_up, p_dw_down, p_b_max, p_b_min, p_slope_up, p_slope_down, x, d, B, R, C,
                                          BL, A, deterministic, k0, k1, c2c, pulse_count, t, step_state, recorded, conv,
                                          blockIdx.x, gridDim.x);
}

// The one-launch updates of several tiny tiles in one launch (aht_pulsed_update_many; calls made directly, no
// convolution view): entry i owns workgroups first_block[i] .. first_block[i + 1] - 1.
struct SmallGroupEntry {
    float* W;
    const float *dw_up, *dw_down, *b_max, *b_min, *slope_up, *slope_down, *x, *d;
    unsigned long long* pulse_count;
    uint32_t* step_state;
    double A;
    int B, R, C, BL, deterministic;
    uint32_t k0, k1, t;
    float c2c;
    int recorded;                                 // the step is read from step_state[0], and the last wave advances it
};
struct SmallGroup {
    uint32_t n, pad_;
    uint32_t first_block[kGroupMax + 1];
    SmallGroupEntry e[kGroupMax];
};

template <int KIND, typename WordT, bool NOISE>
__global__ void __launch_bounds__(256)
k_update_small_group(SmallGroup g)
{
    (void)g;
    uint32_t block;
    const SmallGroupEntry e = group_entry_of_block<SmallGroup, SmallGroupEntry>(&block);
    const uint32_t nblocks = (uint32_t)((e.C + 63) / 64) * (uint32_t)((e.R + 3) / 4);
    update_small_body<KIND, WordT, NOISE>(e.W, e.dw_up, e.dw_down, e.b_max, e.b_min, e.slope_up, e.slope_down, e.x, e.d, e.B,
                                          e.R, e.C, e.BL, e.A, e.deterministic, e.k0, e.k1, e.c2c, e.pulse_count, e.t,
                                          e.step_state, e.recorded, ConvView{}, block, nblocks);
}

}  // namespace aht
