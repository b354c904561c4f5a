/*
 * aht.h -- C ABI of the analog-tile stochastic pulsed update for AMD MI355X (gfx950).
 *
 * One tile = one 2-D weight matrix W[rows][cols] (row-major, fp32, y_i = sum_j w_ij x_j)
 * living on a simulated resistive crossbar, configured at creation (arXiv 2104.02184,
 * Sec. 3, first paragraph).  The library implements the tile's in-situ parallel update:
 * the rank update of Eq. (2) carried out with stochastic pulse trains whose coincidences
 * step each cross-point through a device response model (Sec. 3, paragraphs after Eq. (2)),
 * the update vectors of a mini-batch or convolution acting on the analog weights one after
 * the other (Sec. 3, paragraph on batch sizes larger than one and convolutions).
 *
 * Conventions
 *   - every pointer named *_dev is a DEVICE pointer on the current HIP device; the caller
 *     owns x, d and every output buffer; the tile owns W, the device planes and scratch;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); calls are
 *     asynchronous on it and do not synchronise the host, except create/destroy and a call
 *     that has to grow the tile's scratch memory (the first call, or the first with a larger
 *     batch: hipFree / hipMalloc, which wait for the device);
 *   - every function returns aht_status and never throws or aborts; aht_last_error() gives a
 *     thread-local message.  Arguments are checked before anything is launched: after
 *     INVALID_ARG or UNSUPPORTED the tile is unchanged.  OOM and DEVICE can come from the
 *     runtime in the middle of a call (a scratch buffer that cannot grow, a launch that
 *     fails); then no call counter of the tile has advanced, but kernels launched before the
 *     failure may have run, so the weights are to be taken as undefined;
 *   - one tile must not be used from two streams or two host threads at the same time
 *     (different tiles may be);
 *   - all quantities are in the paper's normalised units (Sec. 3, after Eq. (1)).
 */
#ifndef AHT_H
#define AHT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aht_tile aht_tile; /* opaque */

typedef enum {
    AHT_OK = 0,
    AHT_ERR_INVALID_ARG = 1,
    AHT_ERR_UNSUPPORTED = 2,
    AHT_ERR_OOM = 3,
    AHT_ERR_DEVICE = 4
} aht_status;

/* Device response models (Sec. 3: the step per coincidence may depend on the direction and,
 * non-linearly, on the present weight):
 *   CONSTANT_STEP  step independent of w
 *   LINEAR_STEP    step * max(0, 1 - gamma * w / bound)   (per direction)
 *   SOFT_BOUNDS    step * max(0, 1 - w / bound)           (= LINEAR_STEP with gamma == 1) */
typedef enum { AHT_CONSTANT_STEP = 0, AHT_LINEAR_STEP = 1, AHT_SOFT_BOUNDS = 2 } aht_device_kind;

/* Scalar description of the device population.  *_dtod = relative std of the device-to-
 * device (per cross-point, fixed at creation) Gaussian variation; dw_min_std = relative std
 * of the pulse-to-pulse Gaussian variation of every single step (names as in the paper's
 * device-configuration listing: dw_min, dw_min_dtod, dw_min_std). */
typedef struct {
    int32_t kind;        /* aht_device_kind */
    float dw_min;        /* nominal step per coincidence, > 0 */
    float dw_min_dtod;   /* >= 0 */
    float dw_min_std;    /* >= 0 */
    float up_down;       /* mean asymmetry: dw_up = dw*(1+a), dw_down = dw*(1-a) */
    float up_down_dtod;  /* absolute std of the asymmetry a */
    float w_max;         /* upper bound, >= 0 */
    float w_max_dtod;
    float w_min;         /* lower bound, <= 0 */
    float w_min_dtod;
    float gamma_up;      /* LINEAR_STEP only */
    float gamma_down;    /* LINEAR_STEP only */
    float gamma_dtod;    /* LINEAR_STEP only, relative */
} aht_device_params;

typedef struct {
    int32_t bl;                /* pulse-train length, 1..63 */
    int32_t update_management; /* 0/1: per update vector, rescale the two pulse probabilities
                                  by sqrt(max|d| / max|x|) and its inverse */
} aht_update_params;

/* Indices of the per-cell planes (fp32 [rows][cols]). */
enum {
    AHT_PLANE_DW_UP = 0,
    AHT_PLANE_DW_DOWN = 1,
    AHT_PLANE_B_MAX = 2,
    AHT_PLANE_B_MIN = 3,
    AHT_PLANE_SLOPE_UP = 4,   /* gamma_up_ij / b_max_ij   (1 / b_max_ij for SOFT_BOUNDS) */
    AHT_PLANE_SLOPE_DOWN = 5, /* gamma_down_ij / b_min_ij (1 / b_min_ij for SOFT_BOUNDS) */
    AHT_NUM_PLANES = 6
};

/* Create a tile on the current HIP device: allocates W (zeros), draws the device planes
 * from (params, seed) with the library's counter-based random stream (device-to-device
 * variation, Sec. 3), sets the step counter to 0.  May synchronise.
 * Errors: INVALID_ARG for null pointers, rows/cols <= 0, rows*cols >= 2^32, bl outside
 * 1..63, dw_min <= 0, negative std, w_min > 0 or w_max < 0, unknown kind; OOM; DEVICE. */
aht_status aht_tile_create(aht_tile** out, int32_t rows, int32_t cols,
                           const aht_device_params* device, const aht_update_params* update,
                           uint64_t seed);

/* Frees everything the tile owns.  Synchronises the device.  NULL is accepted. */
aht_status aht_tile_destroy(aht_tile* tile);

/* Copy weights in / out (device to device, fp32 [rows][cols]).  aht_set_weights stores the
 * values as given (the caller keeps them inside the per-cell bounds if that matters). */
aht_status aht_set_weights(aht_tile* tile, const float* w_dev, void* stream);
aht_status aht_get_weights(const aht_tile* tile, float* w_dev_out, void* stream);

/* The stochastic pulsed update (Sec. 3, Eq. (2) and the paragraphs after it):
 *   for b = 0..B-1, in order:   W <- W - lr * d[b] x[b]^T   in the mean,
 * realised by drawing a pulse train of `bl` pulses for every column j (probability
 * min(1, a_x |x[b][j]|)) and every row i (probability min(1, a_d |d[b][i]|)),
 * a_x a_d = lr / (dw_min * bl), and stepping cell ij once per coincidence, sequentially,
 * through its device response with pulse-to-pulse noise and clipping to the cell's bounds.
 * A coincidence with x_j * d_i > 0 is a DOWN pulse, < 0 an UP pulse.
 *   x_dev  [B][cols] fp32, d_dev [B][rows] fp32 (zero, NaN and Inf entries send no pulses)
 *   B >= 0 update vectors (B == 0 or lr == 0: weights unchanged; the step counter still
 *   advances), lr >= 0.
 * Every random draw is a pure function of (seed, step counter, line or cell index, sample,
 * pulse number), so a sequence of calls is reproducible and resumable.  Increments the
 * tile's step counter.  Asynchronous on `stream`; x and d must stay valid until the
 * stream has passed the call.
 * Errors: INVALID_ARG (null pointers with B > 0, B < 0, lr < 0 or NaN); OOM (scratch for
 * the pulse words could not be grown); DEVICE. */
aht_status aht_pulsed_update(aht_tile* tile, const float* x_dev, const float* d_dev, int32_t B,
                             float lr, void* stream);

/* aht_pulsed_update for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, semantics, kernels and
 * results (bit for bit) as aht_pulsed_update, but the pulse words and per-vector factors of the
 * call live in a static device array of AHT_NOALLOC_SCRATCH_BYTES that the library holds on every
 * GPU it runs on until the process ends; the call itself never calls hipMalloc, hipFree or any
 * other allocating routine, records no events and issues no copy to the host.  (Its address on a
 * device is looked up when the first tile is created there.)
 *   Needs 3 * align256(8 B) + B * cols64 * w + B16 * rows16 * w bytes, cols64 / rows16 / B16 = cols /
 *   rows / B rounded up to 64 / 16 / 16, w = 4 for bl <= 31 else 8: a 4096 x 4096 tile with bl = 63
 *   takes up to 511 update vectors, a 1024 x 1024 tile with bl = 31 up to 4095.
 * Errors: those of aht_pulsed_update, and UNSUPPORTED if the call needs more scratch than that
 * (then nothing has been launched and the step counter has not advanced).
 * Every call on one GPU uses the same array: calls that overlap in time on one GPU -- two streams,
 * two tiles, two threads -- race; order them on one stream or with events.  Nothing in the array
 * has to start at zero (each call writes every word it reads, padding included). */
#define AHT_NOALLOC_SCRATCH_BYTES (32u << 20)
aht_status aht_pulsed_update_noalloc(aht_tile* tile, const float* x_dev, const float* d_dev, int32_t B,
                                     float lr, void* stream);

/* The updates of several tiles in one call: the layers of a network after one backward pass (Sec. 3: each
 * layer's weights sit on a tile of their own, and every tile does its rank update in place, independently of
 * the others).  Tile i gets exactly what aht_pulsed_update(tiles[i], x_dev[i], d_dev[i], B[i], lr[i], .) gives
 * it, bit for bit -- a tile's result depends on its own inputs, seed and step counter only -- but tiles too
 * small to fill the chip on their own share the chip: the pulse-train kernels of up to 16 tiles of one word width
 * are one launch (behind one for the per-vector factors of update management and per-vector train lengths), and so
 * are the cell-update kernels of up to 16 tiles of one device kind, word width, noise setting and launch shape;
 * what cannot share a launch (sparse long batches that walk row lists, tiles being profiled) runs on a few streams
 * of the library's own, forked from `stream` and joined to it again with events, all at the default priority.  Tiny tiles whose whole update is one short launch share launches as well (sixteen
 * 64 x 64 tiles with one vector each: 2.2 us per tile against 6.4, what is left being the host's part: 0.4 us
 * replayed from a recorded graph).
 * Eight 512 x 512 tiles with 64 vectors each take 43 us per tile this way, 66 us one after the other; eight
 * 1024 x 1024 tiles with 128 vectors 108 against 129 us.
 *   tiles, x_dev, d_dev, B, lr: host arrays of n entries; x_dev[i] [B[i]][cols_i], d_dev[i] [B[i]][rows_i] device
 *   pointers as for aht_pulsed_update; n >= 0.  Work queued on `stream` before the call is waited for by all
 *   of it, and work queued on `stream` after the call waits for all of it.  Calls from several host threads
 *   are issued one at a time.
 * Errors: INVALID_ARG if any entry would be rejected by aht_pulsed_update, if a tile appears twice, or if the
 * tiles do not all live on the current device -- checked for every entry before anything is launched; OOM,
 * DEVICE as for aht_pulsed_update (some of the tiles may then have been updated, others not).
 * The call may be recorded into a HIP graph (`stream` being captured): its kernels then read every tile's step
 * from the tile's device-side counter and a small kernel advances the counters, as for a recorded
 * aht_pulsed_update_noalloc (see aht_sync_step); nothing is allocated and no counters are sent to the host, so
 * UNSUPPORTED if a tile's scratch is too small for its entry (make the same call once outside the recording
 * first) or a tile is being profiled -- checked before anything is recorded.
 * AHT_GROUP=0 in the environment keeps every tile's kernels in launches of their own (on the streams). */
aht_status aht_pulsed_update_many(aht_tile* const* tiles, const float* const* x_dev, const float* const* d_dev,
                                  const int32_t* B, const float* lr, int32_t n, void* stream);

/* The pulsed update of a convolution layer mapped on the tile (Sec. 3: convolutions accumulate
 * their rank-1 updates in analog memory): rows = output channels, cols = Cin * kh * kw, and
 * every output position of every image is one update vector, applied in the order
 * b = (n * OH + oy) * OW + ox.  The patches are gathered inside the pulse-train kernel; no
 * [B][cols] matrix is materialised.
 *   img_dev  [N][Cin][H][W] fp32 (zero padding `pad` on both sides of H and W)
 *   grad_dev [N][rows][OH][OW] fp32, OH = (H + 2 pad - kh) / stride + 1, OW likewise
 * Same semantics, counters and errors as aht_pulsed_update with B = N * OH * OW; additionally
 * INVALID_ARG if Cin * kh * kw != cols, a size is <= 0, pad < 0, or OH, OW <= 0.
 * aht_debug_pulse_words_conv2d is the test hook corresponding to aht_debug_pulse_words. */
aht_status aht_pulsed_update_conv2d(aht_tile* tile, const float* img_dev, const float* grad_dev, int32_t N,
                                    int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t stride,
                                    int32_t pad, float lr, void* stream);
aht_status aht_debug_pulse_words_conv2d(aht_tile* tile, const float* img_dev, const float* grad_dev, int32_t N,
                                        int32_t Cin, int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t stride,
                                        int32_t pad, float lr, uint64_t* xw_dev, uint64_t* dw_dev, void* stream);

/* Alternative pulse-train generators (Sec. 3 mentions deterministic trains and trains of
 * variable length beside the stochastic fixed-length ones, without giving their rules).
 *   train_kind  AHT_TRAIN_STOCHASTIC (default): Bernoulli pulses from the counter-based stream.
 *               AHT_TRAIN_DETERMINISTIC: no random numbers; a column line with probability p
 *               fires its first round(bl p) pulses ((n + 1/2)/bl < p), a row line fires pulse n
 *               iff (bit-reversed n xor 0xAAAAAAAA) / 2^32 < p, so that coincidences number
 *               bl p_x p_d up to the discrepancy of that point set (at most 2 for bl <= 63).
 *   dynamic_bl  0 (default): every update vector uses `bl` pulses.  1: vector b uses
 *               bl_b = clamp(ceil(lr max|x_b| max|d_b| / dw_min), 1, bl) pulses, the shortest
 *               train whose probabilities need no clipping; the probability factor uses bl_b.
 * Takes effect from the next aht_pulsed_update.  Errors: INVALID_ARG. */
enum { AHT_TRAIN_STOCHASTIC = 0, AHT_TRAIN_DETERMINISTIC = 1 };
aht_status aht_set_pulse_mode(aht_tile* tile, int32_t train_kind, int32_t dynamic_bl);

/* Step counter (number of aht_pulsed_update calls so far); together with the weights, the
 * planes and the seed it makes a run resumable bit for bit.
 * The counter is kept on the host and, equal to it, in device memory.  A call made directly passes
 * the host's count to its kernels.  aht_pulsed_update and aht_pulsed_update_noalloc notice when their
 * stream is being recorded into a HIP graph: the kernels then read the device's counter, and a
 * one-thread kernel after them advances it, so that a sequence of update calls can be recorded once
 * and replayed, each replay continuing the random streams where the counter stands (record
 * aht_pulsed_update_noalloc: it allocates nothing, records no events and issues no copies).
 * aht_get_step returns the host's count without touching the device.  Recording counts the recorded
 * calls on the host although nothing ran, and a replay does not count there at all: after recording
 * and after replays aht_sync_step reads the device's counter back into the host's (it waits for
 * `stream`), before the next call made directly.  Other calls that use the step (transfers, unit
 * cells, convolution updates are fine; the debug hooks) are not meant to be recorded.
 * aht_set_step waits for the device. */
aht_status aht_get_step(const aht_tile* tile, uint32_t* step);
aht_status aht_set_step(aht_tile* tile, uint32_t step);
aht_status aht_sync_step(aht_tile* tile, uint32_t* step /* nullable */, void* stream);

/* Number of coincidence pulses applied by all calls so far on this tile (device counter,
 * read back with a synchronising copy on `stream`). */
aht_status aht_get_pulse_count(const aht_tile* tile, uint64_t* pulses, void* stream);

/* Per-cell device planes, `plane` = AHT_PLANE_*; fp32 [rows][cols] device buffers.
 * Planes 4,5 exist for every kind (all-zero for CONSTANT_STEP). */
aht_status aht_get_device_planes(const aht_tile* tile, int32_t plane, float* dev_out, void* stream);
aht_status aht_set_device_planes(aht_tile* tile, int32_t plane, const float* dev_in, void* stream);

/* Test hooks for the bit-exact part of the contract.
 * aht_debug_pulse_words: the pulse words aht_pulsed_update would draw at the CURRENT step
 *   for (x, d, B, lr); no state change.  Word layout: bit n (n < bl) = pulse n, bit 63 = the
 *   line value is negative.  xw_dev [B][cols], dw_dev [B][rows] uint64.
 * aht_debug_counts: signed coincidence counts of sample b from given words:
 *   +n for n UP pulses (x_j d_i < 0), -n for n DOWN pulses; int8 [rows][cols].
 * aht_debug_apply_words: applies given words (B samples, in order) to the tile as step
 *   `step` without touching the step counter. */
aht_status aht_debug_pulse_words(aht_tile* tile, const float* x_dev, const float* d_dev, int32_t B,
                                 float lr, uint64_t* xw_dev, uint64_t* dw_dev, void* stream);
aht_status aht_debug_counts(aht_tile* tile, const uint64_t* xw_dev, const uint64_t* dw_dev,
                            int32_t B, int32_t b, int8_t* signed_counts_dev, void* stream);
aht_status aht_debug_apply_words(aht_tile* tile, const uint64_t* xw_dev, const uint64_t* dw_dev,
                                 int32_t B, uint32_t step, void* stream);

/* Raw streams of the library's random generator, for pinning it from tests:
 * out_dev[4*k..4*k+3] = Philox4x32-10 block of counter ctr_dev[4*k..] under key_dev[2*k..];
 * gauss_dev[k] = fp32 Gaussian number q0+k of stream (index, t, tag) as the update kernel
 * evaluates it (fast = 1) or as tile creation evaluates it (fast = 0). */
aht_status aht_debug_philox(const uint32_t* ctr_dev, const uint32_t* key_dev, int32_t n,
                            uint32_t* out_dev, void* stream);
aht_status aht_debug_gauss(uint64_t seed, uint32_t index, uint32_t t, uint32_t tag, uint32_t q0,
                           int32_t n, int32_t fast, float* gauss_dev, void* stream);

/* Analog matrix-vector product, Eq. (1) of the paper, and its transposed form for the backward
 * pass (Sec. 3):  y_i = f_adc( sum_j (w_ij + s_w xi_ij)(f_dac(x_j) + s_inp xi_j) + s_out xi_i ).
 *   f_dac: with noise_management the vector is divided by alpha = max|x| (finite entries only;
 *          alpha == 0 gives y == 0), clipped to +-inp_bound and rounded (half to even) to
 *          multiples of inp_res (0 = no rounding); input noise s_inp is added after it.
 *   weight noise is drawn output-referred: s_w |f_dac(x)|_2 times one Gaussian per output
 *          (equal in law to fresh independent xi_ij).
 *   f_adc: clipped to +-out_bound, rounded to multiples of out_res (0 = none), times alpha.
 * aht_forward:  x_dev [B][cols] -> y_dev [B][rows];  aht_backward: d_dev [B][rows] -> g_dev [B][cols].
 * pre_dev (nullable, test hook) receives the values entering f_adc.  Each call uses the tile's
 * forward (backward) call counter for its random stream and increments it.  fp32 product on the
 * matrix cores; asynchronous on `stream`.  Errors: INVALID_ARG (null pointers, B <= 0, negative
 * or non-finite parameters), OOM (scratch), DEVICE. */
typedef struct {
    float inp_res, inp_bound, inp_noise;
    float w_noise;
    float out_noise, out_res, out_bound;
    int32_t noise_management;
} aht_io_params;
aht_status aht_forward(aht_tile* tile, const aht_io_params* io, const float* x_dev, float* y_dev,
                       float* pre_dev, int32_t B, void* stream);
aht_status aht_backward(aht_tile* tile, const aht_io_params* io, const float* d_dev, float* g_dev,
                        float* pre_dev, int32_t B, void* stream);
aht_status aht_get_mvm_steps(const aht_tile* tile, uint32_t* forward_calls, uint32_t* backward_calls);
aht_status aht_set_mvm_steps(aht_tile* tile, uint32_t forward_calls, uint32_t backward_calls);

/* Transfer between two coupled tiles (Sec. 4, the Tiki-Taka compound that the paper's second
 * listing configures: a fast tile takes the gradient updates and hands its content, column by
 * column, to a slow tile).  One transfer event reads column `col` of the
 * fast tile `src` with an analog forward pass of the one-hot vector e_col (non-idealities `io`)
 * and writes it onto the slow tile `dst` with one pulsed update: dst[:, col] += lr * read, in
 * the mean, through dst's own device model.  Both tiles must have the same shape and live on
 * the same device.  Uses and advances src's forward counter and dst's step counter; asynchronous
 * on `stream`; scratch is owned by `dst`.  Without input noise the product reduces to the column
 * itself, which is then read directly (same values bit for bit); the pulsed write only visits the
 * 64 columns around `col`.  Errors: INVALID_ARG (null, shape mismatch, col out
 * of range, lr < 0), OOM, DEVICE. */
aht_status aht_transfer_column(aht_tile* src, aht_tile* dst, int32_t col, float lr, const aht_io_params* io,
                               void* stream);

/* Unit cells of several devices (Sec. 4: a cross-point may hold several conductive elements, each
 * with its own material properties, updated one by one or all together).  A unit cell is given as
 * an array of 1..8 distinct tiles of the same shape, GPU and train length; device k holds the
 * conductances w^(k), and the cell's weight is sum_k gamma_k w^(k).  `gamma` is a HOST array.
 *
 * aht_unit_cell_update: the devices of a cell sit on the same row and column lines, so one set of
 *   pulse trains is drawn -- with device 0's seed, update parameters and pulse mode at device 0's
 *   step count -- and applied to every device (which = -1) or to device `which` only, each through
 *   its own response model and pulse-to-pulse noise stream.  The step counters of all devices are
 *   set to device 0's count + 1.  B = 0 and lr = 0 as for aht_pulsed_update.  With which = -1 the
 *   devices after the first are updated on streams of their own tiles, which `stream` waits for.
 * aht_unit_cell_weights: w_out[rows][cols] = sum_k gamma_k w^(k), added in device order in fp32.
 * aht_unit_cell_forward / _backward: aht_forward / aht_backward on that effective weight (it is
 *   formed in scratch owned by device 0, whose call counters and seed serve the product; a call on
 *   the same stream with the same devices and factors, none of them written since the last product,
 *   multiplies the matrix formed then instead of forming it again).
 * Errors: INVALID_ARG (null, n out of range, a tile twice, mismatched devices, which out of range,
 * non-finite gamma or lr), OOM, DEVICE. */
aht_status aht_unit_cell_update(aht_tile* const* devices, int32_t n, int32_t which, const float* x_dev,
                                const float* d_dev, int32_t B, float lr, void* stream);
aht_status aht_unit_cell_weights(aht_tile* const* devices, const float* gamma, int32_t n, float* w_out_dev,
                                 void* stream);
aht_status aht_unit_cell_forward(aht_tile* const* devices, const float* gamma, int32_t n, const aht_io_params* io,
                                 const float* x_dev, float* y_dev, float* pre_dev, int32_t B, void* stream);
aht_status aht_unit_cell_backward(aht_tile* const* devices, const float* gamma, int32_t n, const aht_io_params* io,
                                  const float* d_dev, float* g_dev, float* pre_dev, int32_t B, void* stream);

/* Once-per-mini-batch temporal processes with device-to-device variability (Sec. 4, last
 * paragraph: conductance decay, reset and diffusion).  Per-cell planes are drawn at
 * aht_set_temporal from the tile's seed:
 *   decay_ij = clamp(decay_rate (1 + decay_rate_dtod g), 0, 1),  diffusion_ij = diffusion |1 + diffusion_dtod g|,
 *   reset_ij = reset + reset_dtod g.
 * aht_decay_diffuse: w <- clamp(w (1 - decay_ij) + diffusion_ij xi, b_min, b_max) for every cell,
 *   xi fresh per cell and temporal step; uses the temporal step counter, then increments it.
 * aht_reset_columns: w <- clamp(reset_ij + reset_std xi, b_min, b_max) for the cells of columns
 *   [c0, c0 + ncols) (clipped to the tile); uses the current temporal step, does not advance it.
 * aht_set_temporal allocates three planes and may synchronise; the other calls are asynchronous
 * on `stream`.  Errors: INVALID_ARG (null, negative or non-finite rates, c0 < 0, ncols < 0,
 * processes used before aht_set_temporal), OOM, DEVICE. */
typedef struct {
    float decay_rate;       /* fraction of the weight lost per mini-batch, 0..1 */
    float decay_rate_dtod;  /* relative std */
    float diffusion;        /* std of the per-mini-batch Gaussian step */
    float diffusion_dtod;   /* relative std */
    float reset;            /* mean reset value */
    float reset_dtod;       /* absolute std of the per-cell reset value */
    float reset_std;        /* std of the reset noise of every reset event */
} aht_temporal_params;
enum { AHT_TPLANE_DECAY = 0, AHT_TPLANE_DIFFUSION = 1, AHT_TPLANE_RESET = 2, AHT_NUM_TPLANES = 3 };
aht_status aht_set_temporal(aht_tile* tile, const aht_temporal_params* params);
aht_status aht_decay_diffuse(aht_tile* tile, void* stream);
aht_status aht_reset_columns(aht_tile* tile, int32_t c0, int32_t ncols, void* stream);
aht_status aht_get_temporal_plane(const aht_tile* tile, int32_t which, float* dev_out, void* stream);
aht_status aht_get_temporal_step(const aht_tile* tile, uint32_t* step);
aht_status aht_set_temporal_step(aht_tile* tile, uint32_t step);

/* Measurement hook.  While enabled, every aht_pulsed_update records HIP events on its stream
 * before the pulse-train kernels, between them and the cell-update kernel, and after it.
 * aht_profile_read waits for the recorded events, returns the summed durations in
 * milliseconds (line scaling + pulse words; cell update) and the number of calls they cover,
 * and clears the record.  At most 4096 calls are recorded between two reads. */
aht_status aht_profile_enable(aht_tile* tile, int32_t enable);
aht_status aht_profile_read(aht_tile* tile, double* ms_words, double* ms_cells, int32_t* calls);

/* What the library chose for the tile's most recent full update and its most recent analog product
 * (measurement aid: results do not depend on any of it beyond the summation order of the product). */
typedef struct {
    int32_t rows_per_lane;       /* cell update: rows per lane of the launch (1, 2 or 4); 0: no update yet */
    int32_t side_rows_per_lane;  /* rows per lane of the launch's second shape, 0 if it had one shape */
    int32_t row_lists;           /* 1: the update walked per-row lists of the samples whose row train has a pulse */
    int32_t stream_words;        /* 32-bit words of pulse-stream storage per cell */
    int32_t mvm_path;            /* product: 0 none yet, 1 fp32 matrix cores, 2 bf16 matrix cores on DAC codes (three
                                    passes), 3 bf16 matrix cores on three input planes (six passes) */
    int32_t mvm_splits;          /* slices of the product's inner dimension */
    double pulse_rate;           /* applied pulses per cell and full update as the host last saw it; < 0: not yet */
    double row_fill;             /* share of the row trains that had a pulse, likewise */
} aht_launch_info;
aht_status aht_get_launch_info(const aht_tile* tile, aht_launch_info* out);

/* Tuning overrides, read from the environment at every call (measurement aids; results do not
 * depend on them beyond the summation order of the analog product):
 *   AHT_RPL         rows per lane of the cell-update kernel (1, 2 or 4); without it the library
 *                   chooses from the tile size and, from 400 000 cells on, from the tile's own
 *                   pulse rate: some update calls are followed by an asynchronous 8-byte copy of
 *                   the pulse counter to pinned host memory on the caller's stream (one in flight
 *                   at most; the host reads it when it has arrived and never waits)
 *   AHT_FUSED       0 / 1: never / always (at most 8 update vectors, no update management, fixed train length)
 *                   take the whole update in one launch, every workgroup drawing the pulse words it needs;
 *                   without it: when rows x cols x B <= 32 768
 *   AHT_QWORDS      32-bit words of pulse-stream storage per cell in LDS
 *   AHT_ROWLISTS    0 / 1: never / always (32-bit pulse words only) let the cell update walk per-row lists of
 *                   the samples whose row train has a pulse; without it: for batches of 256 vectors and more once
 *                   the host has seen that fewer than 55 % of the tile's row trains have one
 *   AHT_GROUP       0: aht_pulsed_update_many keeps every tile's kernels in launches of their own
 *   AHT_EVEN_ROUND  0: never give some column strips fewer rows per lane than the others to fill
 *                   the chip's last round of waves evenly, nor update the devices of a unit cell
 *                   beside each other (on streams of their own tiles, between events); 2: the
 *                   former whenever the shape allows, however short the call
 *   AHT_MVM_BM      block height of the analog product (64 or 128 input vectors)
 *   AHT_MVM_SPLITS  number of slices the product's inner dimension is cut into (1..16)
 *   AHT_MVM_CODES   0: keep products of quantised inputs off the bf16 matrix cores
 *   AHT_MVM_MT      16-vector tiles per wave on that path (2, 4, 8 or 16)
 *   AHT_MVM_FUSED   0: always add the slices' partial sums in a second kernel
 *   AHT_MVM_SHARED  0: never share the input codes among the waves of a workgroup through LDS
 *   AHT_MVM_PLANES  0: products of other inputs (input noise, no or a finer DAC) on the fp32 matrix cores */

const char* aht_status_string(aht_status s);
const char* aht_last_error(void);
/* Library version string; also tells which architecture the kernels were built for. */
const char* aht_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AHT_H */
