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
#include <stdint.h>

#include "aht_rng.hpp"

namespace aht {

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

// ------------------------------------------------------------------------------------------
// Line scaling with update management: one workgroup per update vector.
// a_x = A sqrt(m_d/m_x), a_d = A sqrt(m_x/m_d); both 0 when a maximum is 0 (sample skipped).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float finite_abs_or_zero(float v)
{
    const float a = fabsf(v);
    return (a < __builtin_inff()) ? a : 0.0f;   // NaN and Inf compare false
}

__global__ void __launch_bounds__(256) k_line_scale(const float* __restrict__ x,
                                                    const float* __restrict__ d, int R, int C,
                                                    double A, double* __restrict__ a_x,
                                                    double* __restrict__ a_d)
{
    __shared__ float red_x[4], red_d[4];
    const int b = blockIdx.x;
    float mx = 0.0f, md = 0.0f;
    for (int j = threadIdx.x; j < C; j += 256) mx = fmaxf(mx, finite_abs_or_zero(x[(size_t)b * C + j]));
    for (int i = threadIdx.x; i < R; i += 256) md = fmaxf(md, finite_abs_or_zero(d[(size_t)b * R + i]));
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
        if (m_x != 0.0 && m_d != 0.0) {
            ax = A * sqrt(m_d / m_x);
            ad = A * sqrt(m_x / m_d);
        }
        a_x[b] = ax;
        a_d[b] = ad;
    }
}

// ------------------------------------------------------------------------------------------
// Pulse words.  One thread per line value: threshold T = floor(min(1, a|v|) 2^32) in fp64,
// pulse n set iff Philox word n&3 of block n>>2 is below T; top bit = line value negative.
// Internal layout: xw[B][Cpad], dw[B][Rpad] with Cpad = C rounded up to 64 and Rpad = R rounded
// up to 16, the padding filled with zero words so that the cell kernel needs no edge masks.
// grid.x covers the Cpad + Rpad lines of one sample, grid.y strides over the samples.
// ------------------------------------------------------------------------------------------
template <typename WordT>
__global__ void __launch_bounds__(256)
k_pulse_words(const float* __restrict__ x, const float* __restrict__ d, int B, int R, int C, int Rpad, int Cpad,
              int BL, double A, const double* __restrict__ a_x, const double* __restrict__ a_d,
              uint32_t k0, uint32_t k1, uint32_t t, WordT* __restrict__ xw, WordT* __restrict__ dw)
{
    const int l = (int)(blockIdx.x * 256 + threadIdx.x);
    if (l >= Cpad + Rpad) return;
    const bool is_x = l < Cpad;                         // uniform per wave (Cpad % 64 == 0)
    const int idx = is_x ? l : l - Cpad;
    const int len = is_x ? C : R;
    const uint32_t tagw = (is_x ? kTagX : kTagD) << 24;
    const int nblk = (BL + 3) >> 2;
    for (uint32_t b = blockIdx.y; b < (uint32_t)B; b += gridDim.y) {
        WordT word = 0;
        if (idx < len) {
            const float v = is_x ? x[(size_t)b * C + idx] : d[(size_t)b * R + idx];
            const double a = a_x ? (is_x ? a_x[b] : a_d[b]) : A;
            const float av = fabsf(v);
            if (av > 0.0f && av < __builtin_inff() && a > 0.0) {
                double p = a * (double)av;
                if (!(p < 1.0)) p = 1.0;
                const uint64_t T = (uint64_t)(p * 4294967296.0);      // 0 .. 2^32
                if (T != 0) {
                    const bool sat = (T >> 32) != 0;
                    const uint32_t Tlo = (uint32_t)T;
                    for (int blk = 0; blk < nblk; ++blk) {
                        const U4 r = philox4x32_10((uint32_t)idx, b, t, tagw | (uint32_t)blk, k0, k1);
                        const uint32_t bits = (uint32_t)(sat | (r.x < Tlo)) | ((uint32_t)(sat | (r.y < Tlo)) << 1) |
                                              ((uint32_t)(sat | (r.z < Tlo)) << 2) | ((uint32_t)(sat | (r.w < Tlo)) << 3);
                        word |= (WordT)bits << (4 * blk);
                    }
                    word &= (((WordT)1 << BL) - 1);
                }
                if (v < 0.0f) word |= (WordT)1 << WordTraits<WordT>::kSignBit;
            }
        }
        if (is_x) xw[(size_t)b * Cpad + idx] = word;
        else dw[(size_t)b * Rpad + idx] = word;
    }
}

// word format conversions for the debug entry points (public format: u64 [B][len], sign in bit 63;
// internal format: WordT [B][lpad], sign in the top bit, zero padding)
template <typename WordT>
__global__ void __launch_bounds__(256) k_words_to_public(const WordT* in, uint64_t* out, int B, int len, int lpad)
{
    const size_t k = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (k >= (size_t)B * len) return;
    const size_t b = k / (size_t)len, idx = k - b * (size_t)len;
    const WordT w = in[b * (size_t)lpad + idx];
    const WordT sign = (WordT)1 << WordTraits<WordT>::kSignBit;
    out[k] = (uint64_t)(w & ~sign) | ((w & sign) ? (1ull << 63) : 0ull);
}

template <typename WordT>
__global__ void __launch_bounds__(256) k_words_from_public(const uint64_t* in, WordT* out, int B, int len, int lpad, int BL)
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
    out[k] = r;
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
// Work split: lane <-> column j (coalesced rows of W, the row word is wave-uniform), each lane
// owns RPL cells (rows i0 .. i0+RPL-1 of its column); a workgroup is 4 independent waves
// stacked along the rows.  Weights and device parameters are loaded once, stay in registers
// for all B update vectors and are stored once.
//
// A cell's coincidences are few per sample and their number differs from lane to lane, so the
// samples are not applied in lock-step.  Phase A walks the samples at full lane occupancy and
// appends one byte (count | direction<<7) per non-empty sample to a per-cell queue in LDS;
// when a queue in the wave is (nearly) full, or after the last sample, phase B drains the
// queues: every iteration draws one Philox block = four Gaussians per cell and applies up to
// four pulses.  Pulses of one cell stay in sample order, which is all the sequential
// application asks for (cells are independent).  The Gaussian a pulse uses is fixed by the
// cell's running pulse counter q, so the split into phases does not change any result.
// ------------------------------------------------------------------------------------------
struct CellArgs {
    int R, C, B, Rpad, Cpad;
    uint32_t nbx, nby;            // tiles along columns / rows
    uint32_t k0, k1, t;
    float c2c;
    int qcap;                     // queue capacity (entries) per cell, multiple of 4
    int qstride;                  // bytes between the queues of neighbouring lanes
};

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

// LDS bytes are addressed through 32-bit local pointers kept in registers
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) uint32_t lds_u32;
__device__ __forceinline__ void lds_store_u8(uint32_t addr, uint32_t v) { *(lds_u8*)(size_t)addr = (unsigned char)v; }
__device__ __forceinline__ uint32_t lds_load_u32(uint32_t addr) { return *(const lds_u32*)(size_t)addr; }

// W [R][C] in/out; planes [R][C]; xw[B][Cpad], dw[B][Rpad]: internal zero-padded pulse words.
// The pointers are separate restrict-qualified parameters so that the wave-uniform row words
// are fetched with scalar loads.
template <int KIND, typename WordT, bool NOISE, int RPL>
__global__ void __launch_bounds__(256)
k_cell_update(float* __restrict__ W, const float* __restrict__ p_dw_up, const float* __restrict__ p_dw_down,
              const float* __restrict__ p_b_max, const float* __restrict__ p_b_min,
              const float* __restrict__ p_slope_up, const float* __restrict__ p_slope_down,
              const WordT* __restrict__ xw, const WordT* __restrict__ dw,
              unsigned long long* __restrict__ pulse_count, CellArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const uint32_t lds0 = (uint32_t)(size_t)(lds_u8*)lds;
    constexpr int kSign = WordTraits<WordT>::kSignBit;
    constexpr WordT kBits = (WordT)(~((WordT)1 << kSign));
    constexpr int G = 4;                          // samples per group (prefetch depth, fill check)

    // XCD-aware tile mapping: consecutive workgroup ids go round-robin to the 8 XCDs, so give
    // each XCD one contiguous range of tiles; tiles of one column strip are neighbours and
    // share their x words in that XCD's L2.
    const uint32_t total = a.nbx * a.nby;
    const uint32_t per = (total + 7u) >> 3;
    const uint32_t tile = (blockIdx.x & 7u) * per + (blockIdx.x >> 3);
    if (tile >= total) return;
    const uint32_t bx = tile / a.nby, by = tile - bx * a.nby;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = (int)bx * 64 + lane;            // < Cpad
    const int i0 = ((int)by * 4 + wave) * RPL;    // i0 + RPL <= Rpad
    if (i0 >= a.R) return;                        // wave-uniform; the kernel has no barriers
    const int R = a.R, C = a.C, B = a.B;
    const size_t xstride = (size_t)a.Cpad, dstride = (size_t)a.Rpad;
    const WordT* __restrict__ xp = xw + j;
    const WordT* __restrict__ dp = dw + i0;

    float w[RPL], s_up[RPL], s_dn_neg[RPL], bmax[RPL], bmin[RPL], sl_up[RPL], sl_dn[RPL];
    uint32_t q[RPL], wr[RPL], qb[RPL], cellid[RPL];
    bool cv[RPL];
#pragma unroll
    for (int c = 0; c < RPL; ++c) {
        cv[c] = ((i0 + c) < R) && (j < C);
        const size_t k = cv[c] ? ((size_t)(i0 + c) * C + j) : 0;
        cellid[c] = (uint32_t)k;
        w[c] = W[k];
        s_up[c] = p_dw_up[k];
        s_dn_neg[c] = -p_dw_down[k];
        bmax[c] = p_b_max[k];
        bmin[c] = p_b_min[k];
        sl_up[c] = 0.0f;
        sl_dn[c] = 0.0f;
        if (KIND == kLinearStep) {
            sl_up[c] = p_slope_up[k];
            sl_dn[c] = p_slope_down[k];
        } else if (KIND == kSoftBounds) {
            sl_up[c] = (bmax[c] != 0.0f) ? 1.0f / bmax[c] : 0.0f;
            sl_dn[c] = (bmin[c] != 0.0f) ? 1.0f / bmin[c] : 0.0f;
        }
        q[c] = 0;
        qb[c] = lds0 + (uint32_t)(((wave * RPL + c) * 64 + lane) * a.qstride);
        wr[c] = qb[c];
    }

    // ---- phase B: drain the queues ----------------------------------------------------
    auto drain = [&]() __attribute__((always_inline)) {
        uint32_t rd[RPL], nrem[RPL], dmask[RPL];
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            lds_store_u8(wr[c], 0);               // terminator: an entry with count 0
            rd[c] = qb[c];
            nrem[c] = 0;
            dmask[c] = 0;
        }
        for (;;) {
            bool pending = false;
#pragma unroll
            for (int c = 0; c < RPL; ++c) pending |= (rd[c] != wr[c]) | (nrem[c] != 0);
            if (!__any(pending)) break;
#pragma unroll
            for (int c = 0; c < RPL; ++c) {
                const uint32_t ph = q[c] & 3u;
                float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (NOISE) gauss4_fast(a.k0, a.k1, cellid[c], q[c] >> 2, a.t, kTagC2C, z);
                // the next four queue bytes, fetched as two aligned dwords
                const uint32_t al = rd[c] & ~3u;
                const uint32_t lo = lds_load_u32(al);
                const uint32_t hi = lds_load_u32(al + 4);
                uint32_t E = __builtin_amdgcn_alignbyte(hi, lo, rd[c] & 3u);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    // branch-free: fetch the next entry when the current one is used up; the
                    // terminator (count 0) is never stepped over
                    const bool need = nrem[c] == 0;
                    const uint32_t n_new = E & 0x7Fu;
                    const uint32_t d_new = (uint32_t)__builtin_amdgcn_sbfe((int)E, 7, 1);
                    const bool adv = need & (n_new != 0);
                    nrem[c] = need ? n_new : nrem[c];
                    dmask[c] = need ? d_new : dmask[c];
                    E = adv ? (E >> 8) : E;
                    rd[c] += adv ? 1u : 0u;
                    const bool act = (nrem[c] != 0) & ((uint32_t)k >= ph);
                    const float wn = device_step<KIND, NOISE>(w[c], dmask[c], z[k], a.c2c, s_up[c], s_dn_neg[c],
                                                              bmax[c], bmin[c], sl_up[c], sl_dn[c]);
                    w[c] = act ? wn : w[c];
                    nrem[c] -= act ? 1u : 0u;
                    q[c] += act ? 1u : 0u;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < RPL; ++c) wr[c] = qb[c];
    };

    // ---- phase A: counts of one sample, appended to the queues --------------------------
    // entry byte = count + 128 * (x_j d_i < 0); the byte is always stored, the write pointer
    // only moves past it when the count is non-zero.  Seven vector instructions per cell and
    // sample: two ANDs, one XOR for the direction, two popcounts that accumulate on top of the
    // direction bit, a compare and an add-with-carry.  The empty asm statements only stop the
    // compiler from re-associating the direction bit into per-cell shifts.
    auto sample = [&](WordT xv, const WordT (&dv)[RPL]) __attribute__((always_inline)) {
        uint32_t xs = (uint32_t)(xv >> (kSign - 7)) & 0x80u;
        asm volatile("" : "+v"(xs));
#pragma unroll
        for (int c = 0; c < RPL; ++c) {
            const uint32_t dsg = (uint32_t)(dv[c] >> (kSign - 7)) & 0x80u;     // wave-uniform
            const WordT both = xv & (dv[c] & kBits);
            uint32_t xd = xs ^ dsg;
            asm volatile("" : "+v"(xd));
            uint32_t e;
            if (sizeof(WordT) == 8)
                e = (uint32_t)__popc((uint32_t)((uint64_t)both >> 32)) + ((uint32_t)__popc((uint32_t)both) + xd);
            else
                e = (uint32_t)__popc((uint32_t)both) + xd;
            lds_store_u8(wr[c], e);
            wr[c] += (e != xd) ? 1u : 0u;
        }
    };
    auto load_x = [&](int b0, WordT (&xg)[G]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < G; ++u) xg[u] = xp[(size_t)(b0 + u) * xstride];
    };

    const uint32_t limit = (uint32_t)(a.qcap - G);
    WordT xg[G];
    int b = 0;
    if (G <= B) load_x(0, xg);
    bool done = false;
    do {
        bool full = false;
        while (!full && b + G <= B) {
            WordT dg[G][RPL];                     // row words of this group (scalar registers)
#pragma unroll
            for (int u = 0; u < G; ++u)
#pragma unroll
                for (int c = 0; c < RPL; ++c) dg[u][c] = dp[(size_t)(b + u) * dstride + c];
            WordT xn[G];
            const bool more = b + 2 * G <= B;
            if (more) load_x(b + G, xn);          // next group's column words in flight meanwhile
#pragma unroll
            for (int u = 0; u < G; ++u) sample(xg[u], dg[u]);
            b += G;
            bool nearly_full = false;
#pragma unroll
            for (int c = 0; c < RPL; ++c) nearly_full |= (wr[c] - qb[c]) > limit;
            full = __any(nearly_full) != 0;
            if (more) {
#pragma unroll
                for (int u = 0; u < G; ++u) xg[u] = xn[u];
            }
        }
        if (!full) {                              // fewer than G samples left and room for them
            for (; b < B; ++b) {
                WordT dv[RPL];
#pragma unroll
                for (int c = 0; c < RPL; ++c) dv[c] = dp[(size_t)b * dstride + c];
                sample(xp[(size_t)b * xstride], dv);
            }
            done = true;
        }
        drain();
    } while (!done);

    unsigned long long pulses = 0;
#pragma unroll
    for (int c = 0; c < RPL; ++c) {
        if (cv[c]) {
            W[(size_t)(i0 + c) * C + j] = w[c];
            pulses += q[c];
        }
    }
    if (pulse_count) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) pulses += __shfl_xor(pulses, off, 64);
        if (lane == 0 && pulses) atomicAdd(pulse_count, pulses);
    }
}

}  // namespace aht
