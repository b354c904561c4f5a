/*
 * CPU oracle for the analog tile's stochastic pulsed rank-update.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, scalar
 * reference that only the test-suite, the smoke check and the benchmark's
 * "cpu_baseline" leg may call.  It shares no source, header, table or helper
 * with the HIP library; the two are compared against each other.
 *
 * What it follows (arXiv 2104.02184, Sec. 3 "Analog tile model simulation"):
 *   - Eq. (2): the rank update w_ij <- w_ij + lambda d_i x_j that the pulsed
 *     scheme realises in the mean (sign convention below).
 *   - Sec. 3, paragraph after Eq. (2): stochastic pulse sequences of fixed
 *     length on every row and column, pulse probability proportional to
 *     |x_j| and |d_i|; a coincidence at cross-point ij changes w_ij by a
 *     finite step.
 *   - Sec. 3, next paragraph: the step varies from device to device, can be
 *     biased between up and down pulses, and can depend on the present
 *     weight; pulse-to-pulse variation on top.
 *   - Sec. 3, paragraph on batches/convolutions: the p rank-1 updates of a
 *     mini-batch act on the analog weights one after the other, never as a
 *     digital sum.
 *   - Sec. 3, paragraph on the update kernels: the pulse trains are drawn
 *     and the coincidences are applied SEQUENTIALLY through the device
 *     response curve.
 *
 * The paper fixes the structure only.  Every constant, formula and tie-break
 * it leaves open is a reading of this build (readings R1..R12 listed in the
 * project's design notes); the ones that matter here:
 *   R1  sign: d is the back-propagated error and the tile descends,
 *       W -= lr * d x^T; a coincidence with x_j*d_i > 0 is a DOWN pulse.
 *   R2  p = min(1, a*|v|), a = sqrt(lr / (dw_min * BL)) (nominal dw_min).
 *   R3  update management: a_x = a*sqrt(m_d/m_x), a_d = a*sqrt(m_x/m_d)
 *       with m = per-sample max |.| over finite entries; m_x==0 or m_d==0
 *       skips the sample.
 *   R4  a line value that is zero or not finite produces the all-zero word.
 *   R5  threshold T = floor(min(1,a|v|) * 2^32) in fp64; bit n is set iff
 *       (32-bit random) < T.
 *   R6  Philox4x32-10, key = 64-bit seed, counter words
 *       (line index, sample, step, tag<<24 | n>>2), output word n&3.
 *       tags: 1 = x trains, 2 = d trains, 3 = pulse-to-pulse noise,
 *       4 = device-to-device planes.
 *   R7  the k-th coincidence a cell sees within one call uses Gaussian k of
 *       the cell's (cell, step) stream.
 *   R8  Gaussian = Box-Muller on 24-bit uniforms, evaluated in fp64, rounded
 *       once to fp32.
 *   R9  device step in fp32, clip after every pulse.
 *   R14 variable-length trains: the length is chosen per sample (orc_line_scale_ex).
 *   R15 deterministic trains: evenly spaced / bit-reversed pulses (orc_pulse_word_deterministic).
 *
 * Parity pins: see tests/test_oracle_*.py.  The SHAPE of the response curves
 * against measured ReRAM data (the paper's Fig. 2B) is "parity unpinned": the
 * figure's data is not available.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_CONSTANT_STEP = 0, ORC_LINEAR_STEP = 1, ORC_SOFT_BOUNDS = 2 };
enum { ORC_TAG_X = 1, ORC_TAG_D = 2, ORC_TAG_C2C = 3, ORC_TAG_D2D = 4 };

/* ------------------------------------------------------------------------
 * Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): ten rounds of
 *   (c0,c1,c2,c3) <- (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0))
 * with the key advanced by the Weyl constants between rounds.
 * ---------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void seed_key(uint64_t seed, uint32_t key[2])
{
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
}

/* ------------------------------------------------------------------------
 * Gaussian stream (R8).  Block `blk` of stream (index, t, tag) holds four
 * N(0,1) numbers: words (r0,r1) give numbers 0,1 and (r2,r3) give 2,3 via
 *   u1 = ((ra>>8)+1) * 2^-24 in (0,1],  u2 = (rb>>8) * 2^-24 in [0,1)
 *   z_even = sqrt(-2 ln u1) cos(2 pi u2),  z_odd = sqrt(-2 ln u1) sin(2 pi u2)
 * ---------------------------------------------------------------------- */
void orc_gauss_block_f64(uint64_t seed, uint32_t index, uint32_t t, uint32_t blk,
                         uint32_t tag, double z[4])
{
    uint32_t key[2], ctr[4], r[4];
    seed_key(seed, key);
    ctr[0] = index; ctr[1] = blk; ctr[2] = t; ctr[3] = tag << 24;
    orc_philox4x32_10(ctr, key, r);
    const double two_pi = 6.283185307179586476925286766559;
    for (int pair = 0; pair < 2; ++pair) {
        double u1 = ((double)(r[2 * pair] >> 8) + 1.0) / 16777216.0;
        double u2 = (double)(r[2 * pair + 1] >> 8) / 16777216.0;
        double rad = sqrt(-2.0 * log(u1));
        z[2 * pair] = rad * cos(two_pi * u2);
        z[2 * pair + 1] = rad * sin(two_pi * u2);
    }
}

/* Gaussian number q of stream (index, t, tag), rounded once to fp32. */
float orc_gauss(uint64_t seed, uint32_t index, uint32_t t, uint32_t q, uint32_t tag)
{
    double z[4];
    orc_gauss_block_f64(seed, index, t, q >> 2, tag, z);
    return (float)z[q & 3];
}

/* ------------------------------------------------------------------------
 * Per-cell device planes (device-to-device variation; drawn once at tile
 * creation, Sec. 3 paragraph on device-to-device variations).  Gaussians
 * g1..g6 are numbers 0..5 of stream (cell, t=0, tag 4).  Arithmetic in fp32
 * on the fp32-rounded Gaussians.
 *   dw      = dw_min * |1 + dw_min_dtod*g1|
 *   a       = up_down + up_down_dtod*g2
 *   dw_up   = dw*(1+a),  dw_down = dw*(1-a)
 *   b_max   = max(0, w_max*(1 + w_max_dtod*g3))
 *   b_min   = min(0, w_min*(1 + w_min_dtod*g4))
 *   LinearStep: slope_up = gamma_up*(1+gamma_dtod*g5) / b_max   (0 if b_max==0)
 *               slope_down = gamma_down*(1+gamma_dtod*g6) / b_min (0 if b_min==0)
 *   SoftBounds: slope_up = 1/b_max, slope_down = 1/b_min (0 if the bound is 0)
 *   ConstantStep: slopes are 0.
 * ---------------------------------------------------------------------- */
void orc_device_planes(int kind, float dw_min, float dw_min_dtod, float up_down,
                       float up_down_dtod, float w_max, float w_max_dtod, float w_min,
                       float w_min_dtod, float gamma_up, float gamma_down, float gamma_dtod,
                       uint64_t seed, int R, int C, float *dw_up, float *dw_down,
                       float *b_max, float *b_min, float *slope_up, float *slope_down)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < R; ++i) {
        for (int j = 0; j < C; ++j) {
            uint32_t cell = (uint32_t)i * (uint32_t)C + (uint32_t)j;
            float g[6];
            for (uint32_t q = 0; q < 6; ++q) g[q] = orc_gauss(seed, cell, 0u, q, ORC_TAG_D2D);
            float dw = dw_min * fabsf(1.0f + dw_min_dtod * g[0]);
            float a = up_down + up_down_dtod * g[1];
            float bmax = fmaxf(0.0f, w_max * (1.0f + w_max_dtod * g[2]));
            float bmin = fminf(0.0f, w_min * (1.0f + w_min_dtod * g[3]));
            float su = 0.0f, sd = 0.0f;
            if (kind == ORC_LINEAR_STEP) {
                float gu = gamma_up * (1.0f + gamma_dtod * g[4]);
                float gd = gamma_down * (1.0f + gamma_dtod * g[5]);
                su = (bmax != 0.0f) ? gu / bmax : 0.0f;
                sd = (bmin != 0.0f) ? gd / bmin : 0.0f;
            } else if (kind == ORC_SOFT_BOUNDS) {
                su = (bmax != 0.0f) ? 1.0f / bmax : 0.0f;
                sd = (bmin != 0.0f) ? 1.0f / bmin : 0.0f;
            }
            size_t k = (size_t)i * C + j;
            dw_up[k] = dw * (1.0f + a);
            dw_down[k] = dw * (1.0f - a);
            b_max[k] = bmax;
            b_min[k] = bmin;
            slope_up[k] = su;
            slope_down[k] = sd;
        }
    }
}

/* ------------------------------------------------------------------------
 * Line scaling (R2, R3).  a_x[b], a_d[b] are the fp64 factors that turn a
 * line value into a pulse probability; both 0 marks a skipped sample.
 * ---------------------------------------------------------------------- */
static int is_active(float v) { return isfinite(v) && v != 0.0f; }

/* Extended form: dynamic_bl != 0 chooses the train length per sample (the paper names
 * variable-length trains without a rule): BL_b = clamp(ceil(lr*m_x*m_d/dw_min), 1, BL), the
 * shortest train whose largest pulse probabilities stay <= 1 under update management; the
 * factor A uses BL_b.  bl_b may be NULL when dynamic_bl == 0. */
void orc_line_scale_ex(const float *x, const float *d, int B, int R, int C, float lr, float dw_min,
                       int BL, int update_management, int dynamic_bl, double *a_x, double *a_d,
                       int32_t *bl_b)
{
    for (int b = 0; b < B; ++b) {
        int bl = BL;
        double m_x = 0.0, m_d = 0.0;
        if (update_management || dynamic_bl) {
            for (int j = 0; j < C; ++j) {
                float v = x[(size_t)b * C + j];
                if (is_active(v) && fabs((double)v) > m_x) m_x = fabs((double)v);
            }
            for (int i = 0; i < R; ++i) {
                float v = d[(size_t)b * R + i];
                if (is_active(v) && fabs((double)v) > m_d) m_d = fabs((double)v);
            }
            if (m_x == 0.0 || m_d == 0.0) {
                a_x[b] = 0.0; a_d[b] = 0.0;
                if (bl_b) bl_b[b] = BL;
                continue;
            }
        }
        if (dynamic_bl) {
            double need = ceil((double)lr * m_x * m_d / (double)dw_min);
            if (!(need >= 1.0)) need = 1.0;
            if (need > (double)BL) need = (double)BL;
            bl = (int)need;
        }
        if (bl_b) bl_b[b] = bl;
        double A = sqrt((double)lr / ((double)dw_min * (double)bl));
        if (update_management) {
            a_x[b] = A * sqrt(m_d / m_x);
            a_d[b] = A * sqrt(m_x / m_d);
        } else {
            a_x[b] = A;
            a_d[b] = A;
        }
    }
}

void orc_line_scale(const float *x, const float *d, int B, int R, int C, float lr,
                    float dw_min, int BL, int update_management, double *a_x, double *a_d)
{
    orc_line_scale_ex(x, d, B, R, C, lr, dw_min, BL, update_management, 0, a_x, a_d, NULL);
}

/* 33-bit threshold (R5): 0 .. 2^32 inclusive. */
uint64_t orc_threshold(double a, float v)
{
    if (!is_active(v)) return 0;
    double p = a * fabs((double)v);
    if (!(p < 1.0)) p = 1.0;          /* min(1, p); also catches +inf */
    return (uint64_t)floor(p * 4294967296.0);
}

/* One pulse word (R4..R6): bit n (n < BL) = pulse n, bit 63 = (v < 0). */
uint64_t orc_pulse_word(uint64_t seed, uint32_t t, uint32_t tag, uint32_t index, uint32_t b,
                        double a, float v, int BL)
{
    if (!is_active(v) || !(a > 0.0)) return 0;    /* R4; a == 0 marks a skipped sample (R3) */
    uint64_t T = orc_threshold(a, v);
    uint32_t key[2], ctr[4], r[4];
    seed_key(seed, key);
    uint64_t word = 0;
    for (int n = 0; n < BL; ++n) {
        ctr[0] = index; ctr[1] = b; ctr[2] = t; ctr[3] = (tag << 24) | (uint32_t)(n >> 2);
        orc_philox4x32_10(ctr, key, r);
        if ((uint64_t)r[n & 3] < T) word |= (uint64_t)1 << n;
    }
    if (v < 0.0f) word |= (uint64_t)1 << 63;
    return word;
}

/* Deterministic train (reading R15; Sec. 3 names trains without randomness beside the
 * stochastic ones, and gives no rule): no random numbers; pulse n of a line is set iff u_n < T/2^32 with
 *   column lines:  u_n = (n + 1/2) / BL        (evenly spaced pulses)
 *   row lines:     u_n = (bit-reversal of n  XOR  0xAAAAAAAA) / 2^32
 *                  (van der Corput sequence with an alternating digital shift)
 * so that the pairs (u_n^x, u_n^d), n < BL, form a digitally shifted Hammersley point set: the
 * number of coincidences is BL*p_x*p_d up to its discrepancy, and the alternating shift removes
 * the positive mean error (log2(BL)/8) of the unshifted set.  All in integer arithmetic. */
static uint32_t bit_reverse32(uint32_t v)
{
    uint32_t r = 0;
    for (int k = 0; k < 32; ++k) { r = (r << 1) | (v & 1u); v >>= 1; }
    return r;
}

uint64_t orc_pulse_word_deterministic(uint32_t tag, double a, float v, int BL)
{
    if (!is_active(v) || !(a > 0.0)) return 0;
    uint64_t T = orc_threshold(a, v);
    uint64_t word = 0;
    for (int n = 0; n < BL; ++n) {
        int set;
        if (tag == ORC_TAG_X) set = (((uint64_t)(2 * n + 1)) << 32) < 2u * (uint64_t)BL * T;
        else set = (uint64_t)(bit_reverse32((uint32_t)n) ^ 0xAAAAAAAAu) < T;
        if (set) word |= (uint64_t)1 << n;
    }
    if (v < 0.0f) word |= (uint64_t)1 << 63;
    return word;
}

/* All pulse words of one call: xw[B][C], dw[B][R].
 * train_kind 0 = stochastic, 1 = deterministic; dynamic_bl as in orc_line_scale_ex. */
void orc_pulse_words_ex(const float *x, const float *d, int B, int R, int C, float lr, float dw_min,
                        int BL, int update_management, int train_kind, int dynamic_bl, uint64_t seed,
                        uint32_t t, uint64_t *xw, uint64_t *dw)
{
    double *a_x = (double *)malloc(sizeof(double) * (size_t)(B > 0 ? B : 1));
    double *a_d = (double *)malloc(sizeof(double) * (size_t)(B > 0 ? B : 1));
    int32_t *bl_b = (int32_t *)malloc(sizeof(int32_t) * (size_t)(B > 0 ? B : 1));
    orc_line_scale_ex(x, d, B, R, C, lr, dw_min, BL, update_management, dynamic_bl, a_x, a_d, bl_b);
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < C; ++j) {
            float v = x[(size_t)b * C + j];
            xw[(size_t)b * C + j] = train_kind
                ? orc_pulse_word_deterministic(ORC_TAG_X, a_x[b], v, bl_b[b])
                : orc_pulse_word(seed, t, ORC_TAG_X, (uint32_t)j, (uint32_t)b, a_x[b], v, bl_b[b]);
        }
        for (int i = 0; i < R; ++i) {
            float v = d[(size_t)b * R + i];
            dw[(size_t)b * R + i] = train_kind
                ? orc_pulse_word_deterministic(ORC_TAG_D, a_d[b], v, bl_b[b])
                : orc_pulse_word(seed, t, ORC_TAG_D, (uint32_t)i, (uint32_t)b, a_d[b], v, bl_b[b]);
        }
    }
    free(a_x);
    free(a_d);
    free(bl_b);
}

void orc_pulse_words(const float *x, const float *d, int B, int R, int C, float lr, float dw_min,
                     int BL, int update_management, uint64_t seed, uint32_t t, uint64_t *xw,
                     uint64_t *dw)
{
    orc_pulse_words_ex(x, d, B, R, C, lr, dw_min, BL, update_management, 0, 0, seed, t, xw, dw);
}

/* Coincidences of cell (i,j) in one sample: count and direction. */
static int coincidences(uint64_t xword, uint64_t dword, int BL, int *up)
{
    uint64_t mask = ((uint64_t)1 << BL) - 1;      /* BL <= 63 */
    uint64_t both = xword & dword & mask;
    int n = 0;
    while (both) { n += (int)(both & 1); both >>= 1; }
    *up = (int)(((xword ^ dword) >> 63) & 1);     /* x_j*d_i < 0  =>  UP (R1) */
    return n;
}

/* Signed counts of sample b: +n for UP pulses, -n for DOWN pulses. */
void orc_counts(const uint64_t *xw, const uint64_t *dw, int b, int R, int C, int BL,
                int8_t *signed_counts)
{
    for (int i = 0; i < R; ++i)
        for (int j = 0; j < C; ++j) {
            int up;
            int n = coincidences(xw[(size_t)b * C + j], dw[(size_t)b * R + i], BL, &up);
            signed_counts[(size_t)i * C + j] = (int8_t)(up ? n : -n);
        }
}

/* One pulse through the device response curve (R9), all in fp32. */
float orc_device_step(int kind, float w, int up, float xi, float c2c, float s_up, float s_dn,
                      float bmax, float bmin, float slope_up, float slope_dn)
{
    float s = up ? s_up : s_dn;
    float f = 1.0f;
    if (kind != ORC_CONSTANT_STEP) {
        float slope = up ? slope_up : slope_dn;
        float prod = slope * w;
        f = fmaxf(0.0f, 1.0f - prod);
    }
    float step = s * f;
    float cx = c2c * xi;
    float noise = 1.0f + cx;
    float delta = step * noise;
    float wn = up ? (w + delta) : (w - delta);
    wn = fmaxf(wn, bmin);
    wn = fminf(wn, bmax);
    return wn;
}

/* Apply the B samples' coincidences, in sample order, to the selected cells.
 * cells == NULL: every cell.  Returns the number of applied pulses. */
int64_t orc_apply_words(float *W, const float *dw_up, const float *dw_down, const float *b_max,
                        const float *b_min, const float *slope_up, const float *slope_down,
                        int kind, float c2c, const uint64_t *xw, const uint64_t *dw, int B,
                        int R, int C, int BL, uint64_t seed, uint32_t t, const int64_t *cells,
                        int64_t n_cells)
{
    /* lookup copies with the sample index innermost (cells walk over b) */
    uint64_t *xwT = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)C * (size_t)(B > 0 ? B : 1));
    uint64_t *dwT = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)R * (size_t)(B > 0 ? B : 1));
    for (int b = 0; b < B; ++b) {
        for (int j = 0; j < C; ++j) xwT[(size_t)j * B + b] = xw[(size_t)b * C + j];
        for (int i = 0; i < R; ++i) dwT[(size_t)i * B + b] = dw[(size_t)b * R + i];
    }
    int64_t total = cells ? n_cells : (int64_t)R * C;
    int64_t pulses = 0;
#pragma omp parallel for schedule(dynamic, 256) reduction(+ : pulses)
    for (int64_t idx = 0; idx < total; ++idx) {
        int64_t k = cells ? cells[idx] : idx;
        int i = (int)(k / C), j = (int)(k % C);
        uint32_t cell = (uint32_t)k;
        float w = W[k];
        uint32_t q = 0;                     /* pulse counter of this call (R7) */
        double zblk[4] = {0, 0, 0, 0};
        for (int b = 0; b < B; ++b) {
            int up;
            int n = coincidences(xwT[(size_t)j * B + b], dwT[(size_t)i * B + b], BL, &up);
            for (int p = 0; p < n; ++p) {
                float xi = 0.0f;
                if (c2c > 0.0f) {
                    if ((q & 3) == 0) orc_gauss_block_f64(seed, cell, t, q >> 2, ORC_TAG_C2C, zblk);
                    xi = (float)zblk[q & 3];
                }
                w = orc_device_step(kind, w, up, xi, c2c, dw_up[k], dw_down[k], b_max[k],
                                    b_min[k], slope_up[k], slope_down[k]);
                ++q;
            }
        }
        W[k] = w;
        pulses += q;
    }
    free(xwT);
    free(dwT);
    return pulses;
}

/* The whole update call at step t: words, then cells.  Returns applied pulses. */
int64_t orc_pulsed_update_ex(float *W, const float *dw_up, const float *dw_down, const float *b_max,
                             const float *b_min, const float *slope_up, const float *slope_down,
                             int kind, float c2c, float dw_min, int BL, int update_management,
                             int train_kind, int dynamic_bl, const float *x, const float *d, int B,
                             int R, int C, float lr, uint64_t seed, uint32_t t, const int64_t *cells,
                             int64_t n_cells)
{
    if (B <= 0 || !(lr > 0.0f)) return 0;
    uint64_t *xw = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)B * C);
    uint64_t *dw = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)B * R);
    orc_pulse_words_ex(x, d, B, R, C, lr, dw_min, BL, update_management, train_kind, dynamic_bl, seed,
                       t, xw, dw);
    int64_t pulses = orc_apply_words(W, dw_up, dw_down, b_max, b_min, slope_up, slope_down, kind,
                                     c2c, xw, dw, B, R, C, BL, seed, t, cells, n_cells);
    free(xw);
    free(dw);
    return pulses;
}

int64_t orc_pulsed_update(float *W, const float *dw_up, const float *dw_down, const float *b_max,
                          const float *b_min, const float *slope_up, const float *slope_down,
                          int kind, float c2c, float dw_min, int BL, int update_management,
                          const float *x, const float *d, int B, int R, int C, float lr,
                          uint64_t seed, uint32_t t, const int64_t *cells, int64_t n_cells)
{
    return orc_pulsed_update_ex(W, dw_up, dw_down, b_max, b_min, slope_up, slope_down, kind, c2c, dw_min,
                                BL, update_management, 0, 0, x, d, B, R, C, lr, seed, t, cells, n_cells);
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Bulk draw for the statistical tests: out[k*nq + q] = gauss(seed, index0+k, t, q, tag). */
void orc_gauss_fill(uint64_t seed, uint32_t index0, int n_index, uint32_t t, int nq, uint32_t tag,
                    float *out)
{
    for (int k = 0; k < n_index; ++k)
        for (int q = 0; q < nq; ++q)
            out[(size_t)k * nq + q] = orc_gauss(seed, index0 + (uint32_t)k, t, (uint32_t)q, tag);
}

/* ------------------------------------------------------------------------
 * Temporal processes (Sec. 4 of the paper, last paragraph: conductance
 * decay, reset and diffusion with systematic device-to-device variability,
 * applied once per mini-batch).  The paper names them only; readings:
 *   planes (fixed at set-up; Gaussians 6, 7, 8 of stream (cell, t=0, tag 4)):
 *     lambda_ij = clamp(decay_rate * (1 + decay_rate_dtod*g7), 0, 1)
 *     sdiff_ij  = diffusion * |1 + diffusion_dtod*g8|
 *     reset_ij  = reset + reset_dtod*g9
 *   once per mini-batch (temporal step tau):
 *     w <- w * (1 - lambda_ij)                      (decay toward 0)
 *     w <- w + sdiff_ij * xi,  xi = Gaussian number `cell` of the step's one stream
 *          (index 0, t = tau, tag 5): the cells of the tile number the stream's Gaussians
 *     w <- clamp(w, b_min, b_max)
 *   reset of columns [c0, c0+n): w <- clamp(reset_ij + reset_std * xi', ...),
 *     xi' = Gaussian number `cell` of stream (index 0, t = tau, tag 6).
 * fp32 arithmetic, every operation rounded separately.
 * ---------------------------------------------------------------------- */
enum { ORC_TAG_DIFFUSION = 5, ORC_TAG_RESET = 6 };

void orc_temporal_planes(float decay_rate, float decay_rate_dtod, float diffusion, float diffusion_dtod,
                         float reset, float reset_dtod, uint64_t seed, int R, int C, float *lambda,
                         float *sdiff, float *reset_plane)
{
#pragma omp parallel for schedule(static)
    for (int i = 0; i < R; ++i)
        for (int j = 0; j < C; ++j) {
            uint32_t cell = (uint32_t)i * (uint32_t)C + (uint32_t)j;
            float g7 = orc_gauss(seed, cell, 0u, 6u, ORC_TAG_D2D);
            float g8 = orc_gauss(seed, cell, 0u, 7u, ORC_TAG_D2D);
            float g9 = orc_gauss(seed, cell, 0u, 8u, ORC_TAG_D2D);
            float lam = decay_rate * (1.0f + decay_rate_dtod * g7);
            lam = fminf(fmaxf(lam, 0.0f), 1.0f);
            size_t k = (size_t)i * C + j;
            lambda[k] = lam;
            sdiff[k] = diffusion * fabsf(1.0f + diffusion_dtod * g8);
            reset_plane[k] = reset + reset_dtod * g9;
        }
}

static float temporal_gauss(uint64_t seed, uint32_t cell, uint32_t tau, uint32_t tag)
{
    return orc_gauss(seed, 0u, tau, cell, tag);
}

void orc_decay_diffuse(float *W, const float *lambda, const float *sdiff, const float *b_max,
                       const float *b_min, uint64_t seed, uint32_t tau, int R, int C)
{
    size_t n = (size_t)R * C;
#pragma omp parallel for schedule(static)
    for (int64_t k = 0; k < (int64_t)n; ++k) {
        float w = W[k];
        float keep = 1.0f - lambda[k];
        w = w * keep;
        float xi = temporal_gauss(seed, (uint32_t)k, tau, ORC_TAG_DIFFUSION);
        float dz = sdiff[k] * xi;
        w = w + dz;
        w = fmaxf(w, b_min[k]);
        w = fminf(w, b_max[k]);
        W[k] = w;
    }
}

void orc_reset_columns(float *W, const float *reset_plane, float reset_std, const float *b_max,
                       const float *b_min, uint64_t seed, uint32_t tau, int R, int C, int c0, int ncols)
{
    for (int i = 0; i < R; ++i)
        for (int j = c0; j < c0 + ncols && j < C; ++j) {
            size_t k = (size_t)i * C + j;
            float xi = temporal_gauss(seed, (uint32_t)k, tau, ORC_TAG_RESET);
            float dz = reset_std * xi;
            float w = reset_plane[k] + dz;
            w = fmaxf(w, b_min[k]);
            w = fminf(w, b_max[k]);
            W[k] = w;
        }
}

/* ------------------------------------------------------------------------
 * Analog matrix-vector product, Eq. (1) of the paper:
 *   y_i = f_adc( sum_j (w_ij + s_w xi_ij)(f_dac(x_j) + s_inp xi_j) + s_out xi_i )
 * and its transposed form for the backward pass (Sec. 3, paragraph on the backward
 * pass).  The paper leaves f_dac, f_adc ("discretization ... dynamic scaling and
 * clipping") and the noise bookkeeping open; readings (F1..F7):
 *   F1 dynamic scaling: alpha = max |x| over the finite entries of the vector
 *      (non-finite entries count as 0); alpha == 0 gives the zero vector.
 *   F2 f_dac: xh = x/alpha clipped to +-inp_bound; with inp_res > 0
 *      xq = rint(xh / inp_res) * inp_res (round half to even), all fp32.
 *   F3 input noise: xq_j += s_inp * Gaussian (j & 3) of block (index j>>2, word b,
 *      t = call counter, tag 7 forward / 9 backward).
 *   F4 weight noise, output referred: the sum over j of s_w xi_ij xq_j of fresh
 *      independent xi_ij is N(0, s_w^2 |xq|^2) and independent across i, so it is
 *      drawn as s_w * |xq|_2 * one Gaussian per output.  orc_analog_mvm_cellwise is
 *      Eq. (1) as printed, with a fresh xi_ij for every cell and vector (Gaussian 0 of
 *      block (index = cell i*C+j, word b, t, tag 11 forward / 12 backward)); the tests
 *      hold the output-referred form against it in law.
 *   F5 output noise: s_out * one Gaussian per output.  Output i takes Gaussians
 *      2(i&1) (output noise) and 2(i&1)+1 (weight noise) of block (index i>>1,
 *      word b, t, tag 8 forward / 10 backward).
 *   F6 f_adc: z clipped to +-out_bound; with out_res > 0 rint(z/out_res)*out_res;
 *      y = alpha * that.
 *   F7 the product itself is accumulated in fp64 and rounded once to fp32; the
 *      noise terms are added in fp32 in the order product, weight noise, output noise.
 * transposed == 0: x[B][C] -> y[B][R] with W[R][C];  != 0: x[B][R] -> y[B][C].
 * pre (optional) receives the value entering f_adc.
 * ---------------------------------------------------------------------- */
static void analog_mvm(const float *W, int R, int C, int transposed, const float *x, int B, float inp_res,
                       float inp_bound, float inp_noise, float w_noise, float out_noise, float out_res,
                       float out_bound, int noise_management, uint64_t seed, uint32_t t, float *y, float *pre,
                       int cellwise)
{
    const int K = transposed ? R : C;      /* input length */
    const int N = transposed ? C : R;      /* output length */
    const uint32_t tag_in = transposed ? 9u : 7u, tag_out = transposed ? 10u : 8u;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        float *xq = (float *)malloc(sizeof(float) * (size_t)K);
        float alpha = 1.0f;
        if (noise_management) {
            alpha = 0.0f;
            for (int j = 0; j < K; ++j) {
                float v = x[(size_t)b * K + j];
                if (isfinite(v) && fabsf(v) > alpha) alpha = fabsf(v);
            }
        }
        double norm2 = 0.0;
        for (int j = 0; j < K; ++j) {
            float v = x[(size_t)b * K + j];
            if (!isfinite(v) || alpha == 0.0f) v = 0.0f;
            float xh = (alpha != 0.0f) ? v / alpha : 0.0f;
            xh = fminf(fmaxf(xh, -inp_bound), inp_bound);
            if (inp_res > 0.0f) xh = rintf(xh / inp_res) * inp_res;
            xq[j] = xh;
        }
        if (inp_noise > 0.0f) {
            for (int j = 0; j < K; ++j) {
                double zb[4];                     /* counter (j>>2, b, t, tag): the sample is word 1 */
                orc_gauss_block_f64(seed, (uint32_t)j >> 2, t, (uint32_t)b, tag_in, zb);
                float xi = (float)zb[j & 3];
                float nz = inp_noise * xi;
                xq[j] = xq[j] + nz;
            }
        }
        for (int j = 0; j < K; ++j) norm2 += (double)xq[j] * (double)xq[j];
        float norm = (float)sqrt(norm2);
        for (int i = 0; i < N; ++i) {
            double acc = 0.0;
            for (int j = 0; j < K; ++j) {
                size_t cell = transposed ? (size_t)j * C + i : (size_t)i * C + j;
                double w = (double)W[cell];
                if (cellwise && w_noise > 0.0f) {  /* Eq. (1) as printed: w_ij + s_w xi_ij */
                    double zc[4];
                    orc_gauss_block_f64(seed, (uint32_t)cell, t, (uint32_t)b, transposed ? 12u : 11u, zc);
                    w += (double)w_noise * zc[0];
                }
                acc += w * (double)xq[j];
            }
            float z = (float)acc;
            if (w_noise > 0.0f || out_noise > 0.0f) {
                double zb[4];                     /* counter (i>>1, b, t, tag) */
                orc_gauss_block_f64(seed, (uint32_t)i >> 1, t, (uint32_t)b, tag_out, zb);
                float g_out = (float)zb[2 * (i & 1)], g_w = (float)zb[2 * (i & 1) + 1];
                if (!cellwise) {                  /* F4: the same law, one Gaussian per output */
                    float wn = w_noise * norm;
                    wn = wn * g_w;
                    z = z + wn;
                }
                float on = out_noise * g_out;
                z = z + on;
            }
            if (pre) pre[(size_t)b * N + i] = z;
            float q = fminf(fmaxf(z, -out_bound), out_bound);
            if (out_res > 0.0f) q = rintf(q / out_res) * out_res;
            y[(size_t)b * N + i] = alpha * q;
        }
        free(xq);
    }
}

void orc_analog_mvm(const float *W, int R, int C, int transposed, const float *x, int B, float inp_res,
                    float inp_bound, float inp_noise, float w_noise, float out_noise, float out_res,
                    float out_bound, int noise_management, uint64_t seed, uint32_t t, float *y, float *pre)
{
    analog_mvm(W, R, C, transposed, x, B, inp_res, inp_bound, inp_noise, w_noise, out_noise, out_res, out_bound,
               noise_management, seed, t, y, pre, 0);
}

/* Eq. (1) with the weight noise drawn per cell and vector, as printed (R*C Gaussians per vector). */
void orc_analog_mvm_cellwise(const float *W, int R, int C, int transposed, const float *x, int B, float inp_res,
                             float inp_bound, float inp_noise, float w_noise, float out_noise, float out_res,
                             float out_bound, int noise_management, uint64_t seed, uint32_t t, float *y,
                             float *pre)
{
    analog_mvm(W, R, C, transposed, x, B, inp_res, inp_bound, inp_noise, w_noise, out_noise, out_res, out_bound,
               noise_management, seed, t, y, pre, 1);
}

/* ------------------------------------------------------------------------
 * Convolution layers (Sec. 3, paragraph on batch sizes larger than one and convolutions: their
 * rank-1 updates, too, are summed up by the analog weights themselves, one after the other).  A
 * convolution maps on a tile with one row per output channel and one column per
 * (input channel, kernel row, kernel column); every output position of every image is one
 * update vector.  These two functions write the update vectors out explicitly:
 *   x[b][j],  b = (n*OH + oy)*OW + ox,  j = (c*kh + ky)*kw + kx
 *           = img[n][c][oy*stride - pad + ky][ox*stride - pad + kx]   (0 outside the image)
 *   d[b][i] = dgrad[n][i][oy][ox]
 * with OH = (H + 2 pad - kh)/stride + 1, OW likewise.  The update itself is the ordinary one.
 * ---------------------------------------------------------------------- */
void orc_conv_patches(const float *img, int N, int Cin, int H, int Wd, int kh, int kw, int stride,
                      int pad, float *x)
{
    int OH = (H + 2 * pad - kh) / stride + 1, OW = (Wd + 2 * pad - kw) / stride + 1;
    int J = Cin * kh * kw;
    for (int n = 0; n < N; ++n)
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                size_t b = ((size_t)n * OH + oy) * OW + ox;
                for (int c = 0; c < Cin; ++c)
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            int iy = oy * stride - pad + ky, ix = ox * stride - pad + kx;
                            float v = 0.0f;
                            if (iy >= 0 && iy < H && ix >= 0 && ix < Wd)
                                v = img[(((size_t)n * Cin + c) * H + iy) * Wd + ix];
                            x[b * J + ((size_t)c * kh + ky) * kw + kx] = v;
                        }
            }
}

void orc_conv_rows(const float *dgrad, int N, int Cout, int OH, int OW, float *d)
{
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < Cout; ++i)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    size_t b = ((size_t)n * OH + oy) * OW + ox;
                    d[b * Cout + i] = dgrad[(((size_t)n * Cout + i) * OH + oy) * OW + ox];
                }
}
