// Host side of the C ABI declared in include/aht.h: argument checks, tile state, scratch
// management and kernel launches.  All arithmetic of the update runs in the kernels of
// aht_kernels.hpp; nothing here computes on the host and there is no CPU fallback.
#include "../../include/aht.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "aht_kernels.hpp"
#include "aht_mvm.hpp"

using namespace aht;

struct aht_tile {
    int rows = 0, cols = 0;
    aht_device_params dev{};
    aht_update_params upd{};
    uint64_t seed = 0;
    // The step counter is kept twice: `step` on the host, which every call made directly passes to its
    // kernels by value, and step_state[0] in device memory, which those calls keep equal to it (the cell
    // kernel leaves step + 1 there) and which calls that are being recorded into a HIP graph read instead,
    // so that a replay continues where the counter stands ([1] counts the finished waves of a recorded
    // one-launch update).  After a replay aht_sync_step brings the host's copy up to date.
    uint32_t step = 0;
    uint32_t* step_state = nullptr;
    int device = 0;
    float* W = nullptr;
    float* planes[AHT_NUM_PLANES] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    // scratch owned by the tile, grown on demand
    void* xw = nullptr;
    void* dw = nullptr;
    size_t xw_bytes = 0, dw_bytes = 0;
    double* a_x = nullptr;
    double* a_d = nullptr;
    int a_cap = 0;
    int32_t* bl_b = nullptr;
    int bl_cap = 0;
    int train_kind = AHT_TRAIN_STOCHASTIC;
    int dynamic_bl = 0;
    // device counters: applied pulses [0] by full updates (aht_pulsed_update and its variants on the whole
    // tile), [1] by everything else (transfers, unit-cell updates, injected words); [2] row trains of full
    // updates that had a pulse at all
    unsigned long long* pulse_count = nullptr;
    // Feedback for the launch shape of the cell update: a pinned host copy of counter [0], refreshed by an
    // asynchronous copy behind some full updates of a tile large enough to have a choice.  One copy is in
    // flight at most: before it is issued the host marks the pinned word as empty, and the next copy is
    // issued only after the host has seen this one's value, so a value always belongs to the number of
    // full updates noted when its copy was issued.  The host reads what has arrived; it never waits.
    unsigned long long* pulses_seen = nullptr;
    uint64_t full_updates = 0;                    // full updates issued so far
    uint64_t row_trains = 0;                      // row trains looked at by them (rows x every 16th update vector)
    bool copy_pending = false;                    // a copy has been issued and its value not yet seen
    uint64_t copy_index = 0;                      // full updates counted by the copy in flight
    uint64_t copy_row_trains = 0;                 // row trains counted by it
    double pulse_rate = -1.0;                     // pulses per cell and full update; < 0: not known yet
    double row_fill = -1.0;                       // share of the row trains that had a pulse; < 0: not known yet
    // per-row lists of the samples whose row train has a pulse (k_compact_rows), for long sparse batches
    uint2* rlist = nullptr;
    uint32_t* rlen = nullptr;
    size_t rlist_entries = 0;
    int rlen_cap = 0;
    // stream and events for the update of a unit cell, whose devices run beside each other
    hipStream_t side_stream = nullptr;
    hipEvent_t side_fork = nullptr, side_join = nullptr;
    // analog matrix-vector product: scratch and call counters
    float* mvm_xq = nullptr;
    float* mvm_alpha = nullptr;
    float* mvm_norm = nullptr;
    size_t mvm_xq_floats = 0;
    float* mvm_part = nullptr;    // partial sums of a K-split product [splits][B][N]
    uint16_t* mvm_codes = nullptr;   // DAC integers of the quantised inputs as bf16 [B][K]
    size_t mvm_codes_elems = 0;
    // Effective weights of the unit cell this tile leads [rows][cols], and what they were formed from:
    // the devices, their weight versions, the factors and the stream.  A product on the same stream with
    // all of these unchanged multiplies the stored matrix again instead of re-forming it.
    float* ucell_w = nullptr;
    int ucell_n = 0;
    const aht_tile* ucell_dev[8] = {};
    uint64_t ucell_ver[8] = {};
    float ucell_gamma[8] = {};
    hipStream_t ucell_stream = nullptr;
    // Changes with every write to W (any tile's new value is one no tile has had before).
    uint64_t w_version = 0;
    size_t mvm_part_floats = 0;
    int mvm_b_cap = 0;
    uint32_t fwd_step = 0, bwd_step = 0;
    // transfer scratch: one-hot input, read-out, negated read-out
    float* xfer = nullptr;
    // temporal processes
    bool has_temporal = false;
    aht_temporal_params temporal{};
    float* tplanes[AHT_NUM_TPLANES] = {nullptr, nullptr, nullptr};
    uint32_t tstep = 0;
    // what the most recent full update and analog product chose (aht_get_launch_info)
    aht_launch_info info{};
    // measurement hook: three events per recorded call
    bool profiling = false;
    std::vector<hipEvent_t> events;
    size_t events_used = 0;
};

namespace {

thread_local std::string g_last_error;

std::atomic<uint64_t> g_w_versions{0};
inline void weights_written(aht_tile* t) { t->w_version = ++g_w_versions; }

aht_status fail(aht_status s, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof(buf), fmt, ap);
    va_end(ap);
    g_last_error = buf;
    return s;
}

aht_status hip_fail(hipError_t e, const char* what)
{
    return fail(e == hipErrorOutOfMemory ? AHT_ERR_OOM : AHT_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

#define AHT_HIP(call)                                       \
    do {                                                    \
        hipError_t e_ = (call);                             \
        if (e_ != hipSuccess) return hip_fail(e_, #call);   \
    } while (0)

inline bool use_u32(const aht_tile* t) { return t->upd.bl <= 31; }
inline size_t word_bytes(const aht_tile* t) { return use_u32(t) ? 4 : 8; }
inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }
// internal word buffers are padded so that the cell kernel needs no edge masks
inline int cpad(const aht_tile* t) { return (t->cols + 63) & ~63; }
inline int rpad(const aht_tile* t) { return (t->rows + 15) & ~15; }
inline int bpad(int B) { return (B + 15) & ~15; }       // samples per row of the row-word buffer
// tiles from this size on choose the launch shape of the cell update from their pulse rate
constexpr size_t kAdaptMinCells = 400000;

int env_int(const char* name, int dflt)
{
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    return atoi(v);
}

aht_status check_device(const aht_tile* t)
{
    int cur = -1;
    AHT_HIP(hipGetDevice(&cur));
    if (cur != t->device)
        return fail(AHT_ERR_INVALID_ARG, "tile lives on device %d but the current device is %d", t->device, cur);
    return AHT_OK;
}

aht_status ensure_scratch(aht_tile* t, int B)
{
    const size_t need_x = (size_t)B * cpad(t) * word_bytes(t);
    const size_t need_d = (size_t)bpad(B) * rpad(t) * word_bytes(t);
    if (need_x > t->xw_bytes) {
        if (t->xw) AHT_HIP(hipFree(t->xw));
        t->xw = nullptr; t->xw_bytes = 0;
        AHT_HIP(hipMalloc(&t->xw, need_x));
        t->xw_bytes = need_x;
    }
    if (need_d > t->dw_bytes) {
        if (t->dw) AHT_HIP(hipFree(t->dw));
        t->dw = nullptr; t->dw_bytes = 0;
        AHT_HIP(hipMalloc(&t->dw, need_d));
        t->dw_bytes = need_d;
    }
    if (t->dynamic_bl && B > t->bl_cap) {
        if (t->bl_b) AHT_HIP(hipFree(t->bl_b));
        t->bl_b = nullptr; t->bl_cap = 0;
        AHT_HIP(hipMalloc((void**)&t->bl_b, sizeof(int32_t) * (size_t)B));
        t->bl_cap = B;
    }
    if ((t->upd.update_management || t->dynamic_bl) && B > t->a_cap) {
        if (t->a_x) AHT_HIP(hipFree(t->a_x));
        if (t->a_d) AHT_HIP(hipFree(t->a_d));
        t->a_x = t->a_d = nullptr; t->a_cap = 0;
        AHT_HIP(hipMalloc((void**)&t->a_x, sizeof(double) * (size_t)B));
        AHT_HIP(hipMalloc((void**)&t->a_d, sizeof(double) * (size_t)B));
        t->a_cap = B;
    }
    return AHT_OK;
}

// Device memory between the pulse-train kernels and the cell update: the pulse words of the call,
// the per-sample probability factors and train lengths.  Normally the tile's own (grown on demand);
// the allocation-free entry point carves it out of a static device array instead.
struct WordBufs {
    void* xw = nullptr;
    void* dw = nullptr;
    double* a_x = nullptr;
    double* a_d = nullptr;
    int32_t* bl_b = nullptr;
};

inline WordBufs tile_bufs(const aht_tile* t) { return WordBufs{t->xw, t->dw, t->a_x, t->a_d, t->bl_b}; }

// Whether the calls on `s` are being recorded into a HIP graph: then the kernels read the tile's step from the
// device's counter, and something on the device advances it, so that every replay finds the right step.
bool being_recorded(hipStream_t s)
{
    hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &status) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return status == hipStreamCaptureStatusActive;
}

// Scratch of aht_pulsed_update_noalloc: one array per GPU (every device that loads the library
// holds its own copy at its own address until the process ends).  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and copies take the address that call returns.
constexpr size_t kStaticScratchBytes = AHT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (asked for once per device, with that device
// current: the caller has checked that `device` is the current one).
aht_status static_scratch(int device, unsigned char** out)
{
    if (device < 0 || device >= kMaxDevices) return fail(AHT_ERR_UNSUPPORTED, "device index %d out of range", device);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        AHT_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(AHT_ERR_DEVICE, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[device] = (unsigned char*)p;
    }
    *out = g_scratch_ptr[device];
    return AHT_OK;
}

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Bytes of static scratch a call with B update vectors needs, and where its parts lie.
size_t static_scratch_layout(const aht_tile* t, int B, unsigned char* base, WordBufs* bufs)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t at = off; off += align256(bytes); return base ? base + at : nullptr; };
    unsigned char* ax = take(sizeof(double) * (size_t)B);
    unsigned char* ad = take(sizeof(double) * (size_t)B);
    unsigned char* bl = take(sizeof(int32_t) * (size_t)B);
    unsigned char* xw = take((size_t)B * cpad(t) * word_bytes(t));
    unsigned char* dw = take((size_t)bpad(B) * rpad(t) * word_bytes(t));
    if (bufs) *bufs = WordBufs{xw, dw, (double*)ax, (double*)ad, (int32_t*)bl};
    return off;
}

// pulse trains of the call at step `step` into `w`
// `row_stat`: device counter that receives the number of row trains with a pulse (nullable)
// `recorded`: the kernels read the step from the tile's device counter instead of `step`
// whether ensure_scratch(t, B) would find everything large enough already (a call being recorded cannot allocate)
bool scratch_fits(const aht_tile* t, int B)
{
    if ((size_t)B * cpad(t) * word_bytes(t) > t->xw_bytes || (size_t)bpad(B) * rpad(t) * word_bytes(t) > t->dw_bytes) return false;
    if (t->dynamic_bl && B > t->bl_cap) return false;
    if ((t->upd.update_management || t->dynamic_bl) && B > t->a_cap) return false;
    return true;
}

aht_status launch_words(aht_tile* t, const WordBufs& w, const float* x, const float* d, int B, float lr, uint32_t step,
                        hipStream_t s, const ConvView& conv = ConvView{}, unsigned long long* row_stat = nullptr,
                        bool recorded = false)
{
    const uint32_t* step_ptr = recorded ? t->step_state : nullptr;
    const double A = std::sqrt((double)lr / ((double)t->dev.dw_min * (double)t->upd.bl));
    const double *ax = nullptr, *ad = nullptr;
    const int32_t* blb = nullptr;
    if (t->upd.update_management || t->dynamic_bl) {
        hipLaunchKernelGGL(k_line_scale, dim3((unsigned)B), dim3(256), 0, s, x, d, t->rows, t->cols, (double)lr,
                           (double)t->dev.dw_min, t->upd.bl, t->upd.update_management, t->dynamic_bl, w.a_x, w.a_d,
                           t->dynamic_bl ? w.bl_b : nullptr, conv);
        ax = w.a_x;
        ad = w.a_d;
        blb = t->dynamic_bl ? w.bl_b : nullptr;
    }
    const uint32_t k0 = (uint32_t)t->seed, k1 = (uint32_t)(t->seed >> 32);
    const int Cp = cpad(t), Rp = rpad(t);
    const dim3 grid(blocks_for((size_t)Cp + Rp), (unsigned)(B < 32768 ? B : 32768));
    if (use_u32(t))
        hipLaunchKernelGGL(k_pulse_words<uint32_t>, grid, dim3(256), 0, s, x, d, B, t->rows, t->cols, Rp, Cp, bpad(B),
                           t->upd.bl, A, ax, ad, blb, t->train_kind, k0, k1, step, step_ptr, (uint32_t*)w.xw, (uint32_t*)w.dw, conv,
                           row_stat);
    else
        hipLaunchKernelGGL(k_pulse_words<uint64_t>, grid, dim3(256), 0, s, x, d, B, t->rows, t->cols, Rp, Cp, bpad(B),
                           t->upd.bl, A, ax, ad, blb, t->train_kind, k0, k1, step, step_ptr, (uint64_t*)w.xw, (uint64_t*)w.dw, conv,
                           row_stat);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

struct CellPtrs {
    float* W;
    const float *dw_up, *dw_down, *b_max, *b_min, *slope_up, *slope_down;
    const void *xw, *dw;
    unsigned long long* pulse_count;
};

template <int KIND, typename WordT, bool NOISE, int RPL>
void launch_cells_one(dim3 grid, size_t lds, hipStream_t s, const CellPtrs& p, const CellArgs& a)
{
    if (lds > 64 * 1024)     // more dynamic LDS than the default limit: opt in (gfx950 has 160 KB per CU);
                             // per call, because the attribute belongs to the current device's copy of the kernel
        (void)hipFuncSetAttribute((const void*)k_cell_update<KIND, WordT, NOISE, RPL>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL((k_cell_update<KIND, WordT, NOISE, RPL>), grid, dim3(256), lds, s, p.W, p.dw_up, p.dw_down,
                       p.b_max, p.b_min, p.slope_up, p.slope_down, (const WordT*)p.xw, (const WordT*)p.dw,
                       p.pulse_count, a);
}

template <int KIND, typename WordT, bool NOISE>
void launch_cells_rpl(int rpl, dim3 grid, size_t lds, hipStream_t s, const CellPtrs& p, const CellArgs& a)
{
    switch (rpl) {
        case 1: launch_cells_one<KIND, WordT, NOISE, 1>(grid, lds, s, p, a); break;
        case 2: launch_cells_one<KIND, WordT, NOISE, 2>(grid, lds, s, p, a); break;
        default: launch_cells_one<KIND, WordT, NOISE, 4>(grid, lds, s, p, a); break;
    }
}

template <int KIND, typename WordT>
void launch_cells_noise(bool noise, int rpl, dim3 grid, size_t lds, hipStream_t s, const CellPtrs& p, const CellArgs& a)
{
    if (noise) launch_cells_rpl<KIND, WordT, true>(rpl, grid, lds, s, p, a);
    else launch_cells_rpl<KIND, WordT, false>(rpl, grid, lds, s, p, a);
}

template <typename WordT>
void launch_cells_kind(int kind, bool noise, int rpl, dim3 grid, size_t lds, hipStream_t s, const CellPtrs& p,
                       const CellArgs& a)
{
    switch (kind) {
        case AHT_CONSTANT_STEP: launch_cells_noise<kConstantStep, WordT>(noise, rpl, grid, lds, s, p, a); break;
        case AHT_LINEAR_STEP: launch_cells_noise<kLinearStep, WordT>(noise, rpl, grid, lds, s, p, a); break;
        default: launch_cells_noise<kSoftBounds, WordT>(noise, rpl, grid, lds, s, p, a); break;
    }
}

// one launch for the cell updates of several tiles of one signature (k_cell_update_group)
template <int KIND, typename WordT, bool NOISE, int RPL>
void launch_group_one(const CellGroup& g, unsigned blocks, size_t lds, hipStream_t s)
{
    if (lds > 64 * 1024)
        (void)hipFuncSetAttribute((const void*)k_cell_update_group<KIND, WordT, NOISE, RPL>,
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipLaunchKernelGGL((k_cell_update_group<KIND, WordT, NOISE, RPL>), dim3(blocks), dim3(256), lds, s, g);
}

template <int KIND, typename WordT, bool NOISE>
void launch_group_rpl(int rpl, const CellGroup& g, unsigned blocks, size_t lds, hipStream_t s)
{
    switch (rpl) {
        case 1: launch_group_one<KIND, WordT, NOISE, 1>(g, blocks, lds, s); break;
        case 2: launch_group_one<KIND, WordT, NOISE, 2>(g, blocks, lds, s); break;
        default: launch_group_one<KIND, WordT, NOISE, 4>(g, blocks, lds, s); break;
    }
}

template <typename WordT>
void launch_group_kind(int kind, bool noise, int rpl, const CellGroup& g, unsigned blocks, size_t lds, hipStream_t s)
{
#define AHT_GROUP_KIND(K)                                                                  \
    do {                                                                                  \
        if (noise) launch_group_rpl<K, WordT, true>(rpl, g, blocks, lds, s);              \
        else launch_group_rpl<K, WordT, false>(rpl, g, blocks, lds, s);                   \
    } while (0)
    switch (kind) {
        case AHT_CONSTANT_STEP: AHT_GROUP_KIND(kConstantStep); break;
        case AHT_LINEAR_STEP: AHT_GROUP_KIND(kLinearStep); break;
        default: AHT_GROUP_KIND(kSoftBounds); break;
    }
#undef AHT_GROUP_KIND
}

// Rows per lane: enough waves to fill 256 CUs x 4 SIMDs several times over, otherwise as many
// cells per lane as possible (reuse of the x word, independent chains for the scheduler).
int choose_rpl(const aht_tile* t)
{
    const int forced = env_int("AHT_RPL", 0);
    if (forced == 1 || forced == 2 || forced == 4) return forced;
    const size_t cells = (size_t)t->rows * t->cols;
    if (cells < 180000) return 1;                 // measured: crossover between 384 x 384 and 448 x 448
    if (cells < kAdaptMinCells) return 2;
    // Four rows per lane (with 9-word streams) pay when streams stay short: from 0.4 M cells on at
    // about 110 pulses per cell and call, from 2.3 M at about 160, never at 200 (measured on three
    // input laws).  The rate is the tile's own, from the pulse counter as last seen on the host.
    if (t->pulse_rate >= 0.0) {
        if (t->pulse_rate < 130.0) return 4;
        if (t->pulse_rate < 185.0) return cells >= 2300000 ? 4 : 2;
        return 2;
    }
    return cells >= (size_t)4 * 1024 * 1024 ? 4 : 2;      // no feedback yet
}

// Called before a full update is launched: takes note of the counter value of the copy in flight
// if it has arrived.
constexpr unsigned long long kNoValueYet = ~0ull;
void refresh_pulse_rate(aht_tile* t)
{
    if (!t->pulses_seen || !t->copy_pending) return;
    const volatile unsigned long long* seen = (const volatile unsigned long long*)t->pulses_seen;
    const unsigned long long v = seen[0], v2 = seen[2];
    if (v == kNoValueYet || seen[1] == kNoValueYet || v2 == kNoValueYet) return;    // (every word marked: all have arrived)
    t->copy_pending = false;
    t->pulse_rate = (double)v / ((double)t->rows * (double)t->cols * (double)t->copy_index);
    if (t->copy_row_trains > 0)
        t->row_fill = (double)v2 / (double)t->copy_row_trains;
}

// Long batches whose row trains are mostly empty (small error signals: a convolution layer's many output
// positions) walk per-row lists of the samples that have a pulse.  Measured on 256 x 2304 with 12 544 update
// vectors, 35 % of the row trains with a pulse: see the cell kernel's notes.  AHT_ROWLISTS = 0 / 1 forces it
// off / on (where the word width allows).
bool use_row_lists(const aht_tile* t, int B)
{
    if (!use_u32(t) || (uint64_t)B * (uint64_t)cpad(t) * 4u >= (1ull << 32)) return false;   // (32-bit byte offsets of the column words)
    const int forced = env_int("AHT_ROWLISTS", -1);
    if (forced == 0) return false;
    if (forced == 1) return true;
    return B >= 256 && t->row_fill >= 0.0 && t->row_fill < 0.55;
}

aht_status ensure_row_lists(aht_tile* t, int B)
{
    const size_t need = (size_t)rpad(t) * ((size_t)bpad(B) + kRowListPad);
    if (need > t->rlist_entries) {
        if (t->rlist) AHT_HIP(hipFree(t->rlist));
        t->rlist = nullptr; t->rlist_entries = 0;
        AHT_HIP(hipMalloc((void**)&t->rlist, need * sizeof(uint2)));
        t->rlist_entries = need;
    }
    if (!t->rlen) AHT_HIP(hipMalloc((void**)&t->rlen, sizeof(uint32_t) * (size_t)rpad(t)));
    return AHT_OK;
}

// the cell update of step `step` from the words in the tile's scratch
// `strip0`, `strips`: the range of 64-column strips to work on (the caller knows that x is zero elsewhere)
// `words`: where the pulse words are (the tile's own scratch, that of the first device of its unit cell, or
// the static scratch)
// `full`: a full update of the tile (counted by pulse counter [0], whose rate chooses the launch shape)
// `rowlists`: walk the tile's per-row sample lists (already built from `words`), one row per lane
// `counts`: the call advances the tile's step counter; `recorded`: it is being recorded into a graph (the step
// is then read from the device's counter, which the caller advances with a kernel of its own afterwards)
struct CellLaunch {
    CellPtrs p;
    CellArgs a;
    unsigned blocks;
    size_t lds;
    int rpl;
};

// pointers, arguments, grid and LDS of the cell update of one tile (see launch_cells for the parameters)
aht_status build_cell_launch(aht_tile* t, int B, uint32_t step, uint32_t strip0, uint32_t strips, const WordBufs& words,
                             bool full, bool rowlists, bool counts, bool recorded, CellLaunch* out)
{
    const int rpl = rowlists ? 1 : choose_rpl(t);
    // stream storage per cell: 12 words hold 320 pulses before an early drain is needed; at 4 rows
    // per lane, 9 words (224 pulses) let four workgroups share a compute unit's LDS
    int qwords = env_int("AHT_QWORDS", 0);
    // (walking row lists: 24 words; measured on 256 x 2304 with 12 544 vectors, kernel ms at 12 / 16 / 24 / 32 /
    // 40 / 53 words: 1.58 / 1.56 / 1.52 / 1.60 / 1.59 / 2.13 -- longer streams mean fewer drains and lanes
    // that idle less in them, until too few workgroups fit a compute unit)
    if (qwords < 5 || qwords > 160) qwords = rowlists ? 24 : (rpl == 4) ? 9 : 12;
    const size_t lds_extra = (rpl > 1) ? 4 * 1024 : 0;       // exchange buffers of the last drain, 1 KB per wave
    while (qwords > 5 && (size_t)4 * rpl * 64 * qwords * 4 + lds_extra > 160 * 1024) --qwords;   // LDS of one CU
    CellPtrs& p = out->p;
    p = CellPtrs{};
    p.W = t->W;
    weights_written(t);
    p.dw_up = t->planes[AHT_PLANE_DW_UP];
    p.dw_down = t->planes[AHT_PLANE_DW_DOWN];
    p.b_max = t->planes[AHT_PLANE_B_MAX];
    p.b_min = t->planes[AHT_PLANE_B_MIN];
    p.slope_up = t->planes[AHT_PLANE_SLOPE_UP];
    p.slope_down = t->planes[AHT_PLANE_SLOPE_DOWN];
    p.xw = words.xw;
    p.dw = words.dw;
    p.pulse_count = t->pulse_count + (full ? 0 : 1);
    CellArgs& a = out->a;
    a = CellArgs{};
    a.R = t->rows;
    a.C = t->cols;
    a.B = B;
    a.Bpad = bpad(B);
    a.Cpad = cpad(t);
    a.nbx = strips;
    a.bx0 = strip0;
    a.nby = (uint32_t)((t->rows + 4 * rpl - 1) / (4 * rpl));
    a.k0 = (uint32_t)t->seed;
    a.k1 = (uint32_t)(t->seed >> 32);
    a.t = step;
    a.c2c = t->dev.dw_min_std;
    a.qwords = qwords;
    a.step_on_device = recorded ? t->step_state : nullptr;
    a.publish = (counts && !recorded) ? t->step_state : nullptr;
    // one workgroup per tile of 4 * rpl rows x 64 columns, in equal shares for the 8 XCDs
    const uint64_t total = (uint64_t)a.nby * a.nbx;
    const uint64_t per = (total + 7) / 8;
    if (per * 8 > 0x7FFFFFFFull) return fail(AHT_ERR_UNSUPPORTED, "tile too large for one launch");
    out->blocks = (unsigned)(per * 8);
    out->lds = (size_t)4 * rpl * 64 * qwords * 4 + lds_extra;
    out->rpl = rpl;
    if (full) {
        t->info.rows_per_lane = rpl;
        t->info.side_rows_per_lane = 0;
        t->info.row_lists = rowlists ? 1 : 0;
        t->info.stream_words = qwords;
    }
    return AHT_OK;
}

aht_status launch_cells(aht_tile* t, int B, uint32_t step, hipStream_t s, uint32_t strip0, uint32_t strips,
                        const WordBufs& words, bool full, bool rowlists = false, bool counts = false,
                        bool recorded = false)
{
    CellLaunch cl;
    aht_status st = build_cell_launch(t, B, step, strip0, strips, words, full, rowlists, counts, recorded, &cl);
    if (st != AHT_OK) return st;
    const CellPtrs& p = cl.p;
    const CellArgs& a = cl.a;
    const dim3 grid(cl.blocks);
    const size_t lds = cl.lds;
    const int rpl = cl.rpl;
    const bool noise = t->dev.dw_min_std > 0.0f;
    if (rowlists) {
#define AHT_ROWLISTS_LAUNCH(K, N)                                                                                  \
    hipLaunchKernelGGL((k_cell_update_rowlists<K, N>), grid, dim3(256), lds, s, p.W, p.dw_up, p.dw_down, p.b_max,    \
                       p.b_min, p.slope_up, p.slope_down, (const uint32_t*)p.xw, (const uint32_t*)p.dw,             \
                       p.pulse_count, a, t->rlist, t->rlen)
#define AHT_ROWLISTS_KIND(K)                                                                                       \
    do {                                                                                                          \
        if (noise) AHT_ROWLISTS_LAUNCH(K, true); else AHT_ROWLISTS_LAUNCH(K, false);                               \
    } while (0)
        switch (t->dev.kind) {
            case AHT_CONSTANT_STEP: AHT_ROWLISTS_KIND(kConstantStep); break;
            case AHT_LINEAR_STEP: AHT_ROWLISTS_KIND(kLinearStep); break;
            default: AHT_ROWLISTS_KIND(kSoftBounds); break;
        }
#undef AHT_ROWLISTS_KIND
#undef AHT_ROWLISTS_LAUNCH
    } else if (use_u32(t)) launch_cells_kind<uint32_t>(t->dev.kind, noise, rpl, grid, lds, s, p, a);
    else launch_cells_kind<uint64_t>(t->dev.kind, noise, rpl, grid, lds, s, p, a);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

// A tile whose waves fill the chip's 1024 SIMDs a few times only, and not a whole number of times,
// ends with part of the chip idle (256 x 2304 at two rows per lane: 4 608 waves, five on half of the
// SIMDs and four on the others).  Looks for a division of the column strips, `*strips_main` of them at
// `*rpl_main` rows per lane and the rest at `*rpl_side` (half or a quarter as many), under which the
// busiest compute unit has at least 7 % fewer rows to work through; else leaves *strips_main = strips.
// Both shapes then run in one launch (k_cell_update_pair).  Measured: 2.77 -> 2.40 ms for 256 x 2304 with
// 12 544 vectors, 2.98 -> 2.49 ms for 500 x 784 with 2 048 dense ones, 0.095 -> 0.076 ms with 128 sparse
// ones; very short calls lose (0.053 -> 0.059 ms for 256 x 768 with 128 sparse vectors: the waves with
// fewer rows per lane then take longer than the others), so the call's length is estimated first, from
// the batch and the tile's pulse rate as far as the host has seen it.
void even_round(const aht_tile* t, int B, uint32_t strips, uint32_t* strips_main, int* rpl_main, int* rpl_side)
{
    *strips_main = strips;
    *rpl_main = *rpl_side = 0;
    if (env_int("AHT_EVEN_ROUND", 1) == 0 || env_int("AHT_RPL", 0) != 0) return;
    const int r = choose_rpl(t);
    if (r < 2) return;
    // lane operations of the call at a quarter of the chip's rate, which is what tiles of this size reach
    // (one pulse per cell and sample where the tile's own rate is not known: small tiles never report it)
    const double cells = (double)t->rows * (double)t->cols;
    const double est_s = cells * (4.0 * B + 21.0 * (t->pulse_rate >= 0.0 ? t->pulse_rate : (double)B)) / (39.3e12 * 0.25);
    if (est_s < 0.12e-3 && env_int("AHT_EVEN_ROUND", 1) != 2) return;         // (2: whatever the length, for tests)
    // Workgroups (four waves, 4 * rows-per-lane rows of a strip) spread evenly over the 256 compute
    // units; the call lasts as long as the unit with the most rows.  A row on the side launch is counted
    // as 1.15 rows: fewer rows per lane reuse the column words less.
    const uint64_t cus = 256, R = (uint64_t)t->rows;
    auto groups = [&](int rows_per_lane, uint64_t nstrips) { return (R + 4 * rows_per_lane - 1) / (4 * rows_per_lane) * nstrips; };
    const uint64_t all = groups(r, strips);
    if (all <= cus || all >= 8 * cus) return;                     // less than a wave per SIMD, or several rounds anyway
    const double single = (double)((all + cus - 1) / cus) * (4.0 * r);
    double best = single;
    for (int side = r / 2; side >= 1; side /= 2)
        for (uint32_t sb = 1; sb < strips; ++sb) {
            const uint64_t ga = groups(r, strips - sb), gb = groups(side, sb);
            const double m = (double)((ga + cus - 1) / cus) * (4.0 * r) + (double)((gb + cus - 1) / cus) * (4.0 * side) * 1.15;
            if (m < best - 1e-9) {
                best = m;
                *strips_main = strips - sb;
                *rpl_main = r;
                *rpl_side = side;
            }
        }
    if (best > 0.93 * single) {                                  // too little to gain
        *strips_main = strips;
        *rpl_main = *rpl_side = 0;
    }
}

// The cell update of step `step` as ONE launch of two shapes: strips 0 .. strips_main - 1 at rpl_main
// rows per lane, the others at rpl_side (see even_round and k_cell_update_pair).
template <int KIND, typename WordT, bool NOISE>
void launch_pair_shape(int rpl_main, int rpl_side, dim3 grid, size_t lds, hipStream_t s, const CellPtrs& p,
                       const CellArgs& a, const CellArgs& b, uint32_t main_blocks)
{
#define AHT_PAIR(RM, RS)                                                                                          \
    do {                                                                                                         \
        if (lds > 64 * 1024)                                                                                     \
            (void)hipFuncSetAttribute((const void*)k_cell_update_pair<KIND, WordT, NOISE, RM, RS>,               \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                     \
        hipLaunchKernelGGL((k_cell_update_pair<KIND, WordT, NOISE, RM, RS>), grid, dim3(256), lds, s, p.W, p.dw_up, \
                           p.dw_down, p.b_max, p.b_min, p.slope_up, p.slope_down, (const WordT*)p.xw,            \
                           (const WordT*)p.dw, p.pulse_count, a, b, main_blocks);                                \
    } while (0)
    if (rpl_main == 2) AHT_PAIR(2, 1);
    else if (rpl_side == 2) AHT_PAIR(4, 2);
    else AHT_PAIR(4, 1);
#undef AHT_PAIR
}

template <typename WordT>
void launch_pair_kind(int kind, bool noise, int rpl_main, int rpl_side, dim3 grid, size_t lds, hipStream_t s,
                      const CellPtrs& p, const CellArgs& a, const CellArgs& b, uint32_t main_blocks)
{
#define AHT_PAIR_KIND(K)                                                                                          \
    do {                                                                                                         \
        if (noise) launch_pair_shape<K, WordT, true>(rpl_main, rpl_side, grid, lds, s, p, a, b, main_blocks);    \
        else launch_pair_shape<K, WordT, false>(rpl_main, rpl_side, grid, lds, s, p, a, b, main_blocks);         \
    } while (0)
    switch (kind) {
        case AHT_CONSTANT_STEP: AHT_PAIR_KIND(kConstantStep); break;
        case AHT_LINEAR_STEP: AHT_PAIR_KIND(kLinearStep); break;
        default: AHT_PAIR_KIND(kSoftBounds); break;
    }
#undef AHT_PAIR_KIND
}

aht_status launch_cells_pair(aht_tile* t, int B, uint32_t step, hipStream_t s, uint32_t strips, uint32_t strips_main,
                             int rpl_main, int rpl_side, const WordBufs& words, bool full, bool counts = false,
                             bool recorded = false)
{
    CellPtrs p{};
    p.W = t->W;
    weights_written(t);
    p.dw_up = t->planes[AHT_PLANE_DW_UP];
    p.dw_down = t->planes[AHT_PLANE_DW_DOWN];
    p.b_max = t->planes[AHT_PLANE_B_MAX];
    p.b_min = t->planes[AHT_PLANE_B_MIN];
    p.slope_up = t->planes[AHT_PLANE_SLOPE_UP];
    p.slope_down = t->planes[AHT_PLANE_SLOPE_DOWN];
    p.xw = words.xw;
    p.dw = words.dw;
    p.pulse_count = t->pulse_count + (full ? 0 : 1);
    size_t lds = 0;
    auto shape = [&](int rpl, uint32_t strip0, uint32_t nstrips) {
        int qwords = env_int("AHT_QWORDS", 0);
        if (qwords < 5 || qwords > 160) qwords = (rpl == 4) ? 9 : 12;
        const size_t lds_extra = (rpl > 1) ? 4 * 1024 : 0;
        while (qwords > 5 && (size_t)4 * rpl * 64 * qwords * 4 + lds_extra > 160 * 1024) --qwords;
        const size_t need = (size_t)4 * rpl * 64 * qwords * 4 + lds_extra;
        lds = need > lds ? need : lds;
        CellArgs a{};
        a.R = t->rows;
        a.C = t->cols;
        a.B = B;
        a.Bpad = bpad(B);
        a.Cpad = cpad(t);
        a.nbx = nstrips;
        a.bx0 = strip0;
        a.nby = (uint32_t)((t->rows + 4 * rpl - 1) / (4 * rpl));
        a.k0 = (uint32_t)t->seed;
        a.k1 = (uint32_t)(t->seed >> 32);
        a.t = step;
        a.c2c = t->dev.dw_min_std;
        a.qwords = qwords;
        a.step_on_device = recorded ? t->step_state : nullptr;
        a.publish = (counts && !recorded) ? t->step_state : nullptr;
        return a;
    };
    const CellArgs a = shape(rpl_main, 0u, strips_main), b = shape(rpl_side, strips_main, strips - strips_main);
    const uint64_t main_blocks = ((uint64_t)a.nby * a.nbx + 7) / 8 * 8, side_blocks = ((uint64_t)b.nby * b.nbx + 7) / 8 * 8;
    if (main_blocks + side_blocks > 0x7FFFFFFFull) return fail(AHT_ERR_UNSUPPORTED, "tile too large for one launch");
    const dim3 grid((unsigned)(main_blocks + side_blocks));
    if (full) {
        t->info.rows_per_lane = rpl_main;
        t->info.side_rows_per_lane = rpl_side;
        t->info.row_lists = 0;
        t->info.stream_words = a.qwords;
    }
    const bool noise = t->dev.dw_min_std > 0.0f;
    if (use_u32(t)) launch_pair_kind<uint32_t>(t->dev.kind, noise, rpl_main, rpl_side, grid, lds, s, p, a, b, (uint32_t)main_blocks);
    else launch_pair_kind<uint64_t>(t->dev.kind, noise, rpl_main, rpl_side, grid, lds, s, p, a, b, (uint32_t)main_blocks);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

// Tiny tiles with a few update vectors take the whole call in one launch (k_update_small): every workgroup
// draws the pulse words it needs itself, which costs about one extra microsecond per 4 096 cells and update
// vector and saves a launch.  AHT_FUSED = 0 / 1 forces it off / on (where the call qualifies at all).
bool use_small_kernel(const aht_tile* t, int B)
{
    if (B > kSmallMaxB || t->upd.update_management || t->dynamic_bl) return false;
    const int forced = env_int("AHT_FUSED", -1);
    if (forced == 0) return false;
    if (forced == 1) return true;
    return (uint64_t)t->rows * (uint64_t)t->cols * (uint64_t)B <= 32768u;
}

aht_status launch_small(aht_tile* t, const float* x, const float* d, int B, float lr, hipStream_t s, const ConvView& conv,
                        bool recorded)
{
    const double A = std::sqrt((double)lr / ((double)t->dev.dw_min * (double)t->upd.bl));
    const dim3 grid((unsigned)((t->cols + 63) / 64) * (unsigned)((t->rows + 3) / 4));
    const bool noise = t->dev.dw_min_std > 0.0f;
    weights_written(t);
#define AHT_SMALL_LAUNCH(K, WT, N)                                                                                  \
    hipLaunchKernelGGL((k_update_small<K, WT, N>), grid, dim3(256), 0, s, t->W, t->planes[AHT_PLANE_DW_UP],          \
                       t->planes[AHT_PLANE_DW_DOWN], t->planes[AHT_PLANE_B_MAX], t->planes[AHT_PLANE_B_MIN],        \
                       t->planes[AHT_PLANE_SLOPE_UP], t->planes[AHT_PLANE_SLOPE_DOWN], x, d, B, t->rows, t->cols,   \
                       t->upd.bl, A, t->train_kind, (uint32_t)t->seed, (uint32_t)(t->seed >> 32), t->dev.dw_min_std, \
                       t->pulse_count, t->step, t->step_state, recorded ? 1 : 0, conv)
#define AHT_SMALL_NOISE(K, WT)                                                                                      \
    do {                                                                                                           \
        if (noise) AHT_SMALL_LAUNCH(K, WT, true); else AHT_SMALL_LAUNCH(K, WT, false);                              \
    } while (0)
#define AHT_SMALL_KIND(WT)                                                                                          \
    switch (t->dev.kind) {                                                                                         \
        case AHT_CONSTANT_STEP: AHT_SMALL_NOISE(kConstantStep, WT); break;                                          \
        case AHT_LINEAR_STEP: AHT_SMALL_NOISE(kLinearStep, WT); break;                                              \
        default: AHT_SMALL_NOISE(kSoftBounds, WT); break;                                                           \
    }
    if (use_u32(t)) { AHT_SMALL_KIND(uint32_t) } else { AHT_SMALL_KIND(uint64_t) }
#undef AHT_SMALL_KIND
#undef AHT_SMALL_NOISE
#undef AHT_SMALL_LAUNCH
    AHT_HIP(hipGetLastError());
    t->info.rows_per_lane = 1;
    t->info.side_rows_per_lane = 0;
    t->info.row_lists = 0;
    t->info.stream_words = 0;                     // (no pulse streams: the samples are applied pulse by pulse)
    return AHT_OK;
}

bool finite_nonneg(float v) { return std::isfinite(v) && v >= 0.0f; }

}  // namespace

extern "C" {

const char* aht_status_string(aht_status s)
{
    switch (s) {
        case AHT_OK: return "AHT_OK";
        case AHT_ERR_INVALID_ARG: return "AHT_ERR_INVALID_ARG";
        case AHT_ERR_UNSUPPORTED: return "AHT_ERR_UNSUPPORTED";
        case AHT_ERR_OOM: return "AHT_ERR_OOM";
        case AHT_ERR_DEVICE: return "AHT_ERR_DEVICE";
    }
    return "AHT_ERR_UNKNOWN";
}

const char* aht_last_error(void) { return g_last_error.c_str(); }

const char* aht_version(void) { return "aht 0.1 (HIP, gfx950, wave64)"; }

aht_status aht_tile_create(aht_tile** out, int32_t rows, int32_t cols, const aht_device_params* dev,
                           const aht_update_params* upd, uint64_t seed)
{
    if (!out || !dev || !upd) return fail(AHT_ERR_INVALID_ARG, "null argument");
    *out = nullptr;
    if (rows <= 0 || cols <= 0) return fail(AHT_ERR_INVALID_ARG, "rows and cols must be positive");
    if ((uint64_t)rows * (uint64_t)cols >= (1ull << 32))
        return fail(AHT_ERR_INVALID_ARG, "rows*cols must stay below 2^32");
    if (upd->bl < 1 || upd->bl > 63) return fail(AHT_ERR_INVALID_ARG, "bl must be in 1..63");
    if (dev->kind < AHT_CONSTANT_STEP || dev->kind > AHT_SOFT_BOUNDS)
        return fail(AHT_ERR_INVALID_ARG, "unknown device kind %d", dev->kind);
    if (!(dev->dw_min > 0.0f) || !std::isfinite(dev->dw_min)) return fail(AHT_ERR_INVALID_ARG, "dw_min must be > 0");
    if (!finite_nonneg(dev->dw_min_dtod) || !finite_nonneg(dev->dw_min_std) || !finite_nonneg(dev->up_down_dtod) ||
        !finite_nonneg(dev->w_max_dtod) || !finite_nonneg(dev->w_min_dtod) || !finite_nonneg(dev->gamma_dtod))
        return fail(AHT_ERR_INVALID_ARG, "standard deviations must be finite and >= 0");
    if (!(dev->w_max >= 0.0f) || !(dev->w_min <= 0.0f) || !std::isfinite(dev->w_max) || !std::isfinite(dev->w_min))
        return fail(AHT_ERR_INVALID_ARG, "need w_min <= 0 <= w_max");
    if (!std::isfinite(dev->up_down) || !std::isfinite(dev->gamma_up) || !std::isfinite(dev->gamma_down))
        return fail(AHT_ERR_INVALID_ARG, "non-finite device parameter");

    aht_tile* t = new (std::nothrow) aht_tile();
    if (!t) return fail(AHT_ERR_OOM, "host allocation failed");
    t->rows = rows;
    t->cols = cols;
    t->dev = *dev;
    t->upd = *upd;
    t->upd.update_management = upd->update_management ? 1 : 0;
    t->seed = seed;
    aht_status st = AHT_OK;
    const size_t n = (size_t)rows * cols;
    const int nplanes = (dev->kind == AHT_LINEAR_STEP) ? 6 : 4;
    auto cleanup = [&](aht_status s) { aht_tile_destroy(t); return s; };
    hipError_t e = hipGetDevice(&t->device);
    if (e != hipSuccess) return cleanup(hip_fail(e, "hipGetDevice"));
    if ((e = hipMalloc((void**)&t->W, n * sizeof(float))) != hipSuccess) return cleanup(hip_fail(e, "hipMalloc(W)"));
    for (int p = 0; p < nplanes; ++p)
        if ((e = hipMalloc((void**)&t->planes[p], n * sizeof(float))) != hipSuccess)
            return cleanup(hip_fail(e, "hipMalloc(plane)"));
    if ((e = hipMalloc((void**)&t->pulse_count, 3 * sizeof(unsigned long long))) != hipSuccess)
        return cleanup(hip_fail(e, "hipMalloc(counter)"));
    if ((e = hipMemset(t->W, 0, n * sizeof(float))) != hipSuccess) return cleanup(hip_fail(e, "hipMemset"));
    weights_written(t);
    if ((e = hipMemset(t->pulse_count, 0, 3 * sizeof(unsigned long long))) != hipSuccess)
        return cleanup(hip_fail(e, "hipMemset"));
    if ((e = hipMalloc((void**)&t->step_state, 4 * sizeof(uint32_t))) != hipSuccess)
        return cleanup(hip_fail(e, "hipMalloc(step)"));
    if ((e = hipMemset(t->step_state, 0, 4 * sizeof(uint32_t))) != hipSuccess) return cleanup(hip_fail(e, "hipMemset"));
    // the pinned words of the feedback; without them the static choices stay
    if (hipHostMalloc((void**)&t->pulses_seen, 64, hipHostMallocDefault) == hipSuccess) std::memset(t->pulses_seen, 0, 64);
    else { t->pulses_seen = nullptr; (void)hipGetLastError(); }
    PlaneArgs pa{};
    pa.kind = dev->kind;
    pa.dw_min = dev->dw_min; pa.dw_min_dtod = dev->dw_min_dtod;
    pa.up_down = dev->up_down; pa.up_down_dtod = dev->up_down_dtod;
    pa.w_max = dev->w_max; pa.w_max_dtod = dev->w_max_dtod;
    pa.w_min = dev->w_min; pa.w_min_dtod = dev->w_min_dtod;
    pa.gamma_up = dev->gamma_up; pa.gamma_down = dev->gamma_down; pa.gamma_dtod = dev->gamma_dtod;
    pa.k0 = (uint32_t)seed; pa.k1 = (uint32_t)(seed >> 32);
    pa.R = rows; pa.C = cols;
    pa.dw_up = t->planes[0]; pa.dw_down = t->planes[1]; pa.b_max = t->planes[2]; pa.b_min = t->planes[3];
    pa.slope_up = t->planes[4]; pa.slope_down = t->planes[5];
    unsigned nb = blocks_for(n);
    if (nb > 65536u) nb = 65536u;
    hipLaunchKernelGGL(k_gen_planes, dim3(nb), dim3(256), 0, 0, pa);
    if ((e = hipGetLastError()) != hipSuccess) return cleanup(hip_fail(e, "k_gen_planes launch"));
    if ((e = hipDeviceSynchronize()) != hipSuccess) return cleanup(hip_fail(e, "k_gen_planes"));
    unsigned char* primed = nullptr;              // the device's static scratch, looked up once per device here
    if ((st = static_scratch(t->device, &primed)) != AHT_OK) return cleanup(st);
    *out = t;
    return AHT_OK;
}

aht_status aht_tile_destroy(aht_tile* t)
{
    if (!t) return AHT_OK;
    hipError_t first = hipDeviceSynchronize();
    auto rel = [&](void* p) {
        if (p) {
            hipError_t e = hipFree(p);
            if (first == hipSuccess) first = e;
        }
    };
    rel(t->W);
    for (auto* p : t->planes) rel(p);
    rel(t->xw); rel(t->dw); rel(t->a_x); rel(t->a_d); rel(t->bl_b); rel(t->pulse_count); rel(t->rlist); rel(t->rlen); rel(t->step_state);
    for (auto* p : t->tplanes) rel(p);
    rel(t->mvm_xq); rel(t->mvm_part); rel(t->mvm_codes); rel(t->ucell_w); rel(t->mvm_alpha); rel(t->mvm_norm); rel(t->xfer);
    for (hipEvent_t e : t->events) (void)hipEventDestroy(e);
    if (t->side_fork) (void)hipEventDestroy(t->side_fork);
    if (t->side_join) (void)hipEventDestroy(t->side_join);
    if (t->side_stream) (void)hipStreamDestroy(t->side_stream);
    if (t->pulses_seen) (void)hipHostFree(t->pulses_seen);
    delete t;
    if (first != hipSuccess) return hip_fail(first, "aht_tile_destroy");
    return AHT_OK;
}

aht_status aht_set_weights(aht_tile* t, const float* w_dev, void* stream)
{
    if (!t || !w_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    weights_written(t);
    AHT_HIP(hipMemcpyAsync(t->W, w_dev, (size_t)t->rows * t->cols * sizeof(float), hipMemcpyDeviceToDevice,
                           (hipStream_t)stream));
    return AHT_OK;
}

aht_status aht_get_weights(const aht_tile* t, float* w_dev_out, void* stream)
{
    if (!t || !w_dev_out) return fail(AHT_ERR_INVALID_ARG, "null argument");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    AHT_HIP(hipMemcpyAsync(w_dev_out, t->W, (size_t)t->rows * t->cols * sizeof(float), hipMemcpyDeviceToDevice,
                           (hipStream_t)stream));
    return AHT_OK;
}

// `col_lo .. col_hi`: columns outside this range are known to be zero in every x (all columns if col_hi < 0)
// `static_scratch_only`: the allocation-free variant (see aht_pulsed_update_noalloc)
// whether this tile's full updates are worth watching: large enough for a choice of rows per lane, or long
// batches of 32-bit words, which may turn out sparse
static bool watched_update(const aht_tile* t, int B)
{
    return t->pulses_seen && ((size_t)t->rows * t->cols >= kAdaptMinCells || (use_u32(t) && B >= 256));
}

// after the kernels of a full update are on stream s: counts it and, if `may_report`, sends the device's counters
// to the host when no earlier report is still on its way: after each of the first eight updates, then sixteen
// updates after the last report
static aht_status full_update_done(aht_tile* t, int B, bool watched, bool may_report, hipStream_t s)
{
    t->full_updates += 1;
    if (watched) t->row_trains += (uint64_t)t->rows * (uint64_t)((B + 15) / 16);    // every 16th sample is counted
    if (may_report && watched && !t->copy_pending &&
        (t->full_updates <= 8 || t->full_updates >= t->copy_index + 16)) {
        for (int k = 0; k < 3; ++k) ((volatile unsigned long long*)t->pulses_seen)[k] = kNoValueYet;
        AHT_HIP(hipMemcpyAsync(t->pulses_seen, t->pulse_count, 3 * sizeof(unsigned long long),
                               hipMemcpyDeviceToHost, s));
        t->copy_pending = true;
        t->copy_index = t->full_updates;
        t->copy_row_trains = t->row_trains;
    }
    return AHT_OK;
}

// what every update call checks before it launches anything
static aht_status check_update_args(const aht_tile* t, const float* x_dev, const float* d_dev, int64_t B64, float lr)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    if (B64 < 0) return fail(AHT_ERR_INVALID_ARG, "B must be >= 0");
    if (B64 > 0x7FFFFFF0) return fail(AHT_ERR_INVALID_ARG, "too many update vectors for one call");
    if (!(lr >= 0.0f) || !std::isfinite(lr)) return fail(AHT_ERR_INVALID_ARG, "lr must be finite and >= 0");
    if (B64 > 0 && (!x_dev || !d_dev)) return fail(AHT_ERR_INVALID_ARG, "null x or d");
    return check_device(t);
}

static aht_status pulsed_update_impl(aht_tile* t, const float* x_dev, const float* d_dev, int64_t B64, float lr,
                                     void* stream, const ConvView& conv, int col_lo = 0, int col_hi = -1,
                                     bool static_scratch_only = false)
{
    aht_status st = check_update_args(t, x_dev, d_dev, B64, lr);
    if (st != AHT_OK) return st;
    const int B = (int)B64;
    const bool full = col_hi < 0;                 // the whole tile
    const bool recorded = being_recorded((hipStream_t)stream);
    if (B > 0 && lr > 0.0f && full && use_small_kernel(t, B)) {
        hipStream_t s = (hipStream_t)stream;
        hipEvent_t* ev = nullptr;
        if (!static_scratch_only && t->profiling && t->events_used + 3 <= 3 * 4096) {
            while (t->events.size() < t->events_used + 3) {
                hipEvent_t e;
                AHT_HIP(hipEventCreate(&e));
                t->events.push_back(e);
            }
            ev = &t->events[t->events_used];
            AHT_HIP(hipEventRecord(ev[0], s));
            AHT_HIP(hipEventRecord(ev[1], s));      // (no separate pulse-train kernel)
        }
        if ((st = launch_small(t, x_dev, d_dev, B, lr, s, conv, recorded)) != AHT_OK) return st;
        if (ev) {
            AHT_HIP(hipEventRecord(ev[2], s));
            t->events_used += 3;
        }
        t->full_updates += 1;
    } else if (B > 0 && lr > 0.0f) {
        WordBufs bufs;
        if (static_scratch_only) {
            const size_t need = static_scratch_layout(t, B, nullptr, nullptr);
            if (need > kStaticScratchBytes)
                return fail(AHT_ERR_UNSUPPORTED, "%d update vectors on a %d x %d tile need %zu bytes of scratch; the static "
                            "scratch of aht_pulsed_update_noalloc holds %zu (use aht_pulsed_update)", B, t->rows, t->cols,
                            need, kStaticScratchBytes);
            unsigned char* base = nullptr;
            if ((st = static_scratch(t->device, &base)) != AHT_OK) return st;
            (void)static_scratch_layout(t, B, base, &bufs);
        } else {
            if ((st = ensure_scratch(t, B)) != AHT_OK) return st;
            bufs = tile_bufs(t);
        }
        hipStream_t s = (hipStream_t)stream;
        hipEvent_t* ev = nullptr;
        if (!static_scratch_only && t->profiling && t->events_used + 3 <= 3 * 4096) {
            while (t->events.size() < t->events_used + 3) {
                hipEvent_t e;
                AHT_HIP(hipEventCreate(&e));
                t->events.push_back(e);
            }
            ev = &t->events[t->events_used];
        }
        if (ev) AHT_HIP(hipEventRecord(ev[0], s));
        if (col_hi < 0) refresh_pulse_rate(t);
        const bool watched = col_hi < 0 && watched_update(t, B);
        const bool rowlists = col_hi < 0 && !static_scratch_only && use_row_lists(t, B);
        if (rowlists && (st = ensure_row_lists(t, B)) != AHT_OK) return st;
        if ((st = launch_words(t, bufs, x_dev, d_dev, B, lr, t->step, s, conv, watched ? t->pulse_count + 2 : nullptr,
                               recorded)) != AHT_OK)
            return st;
        if (ev) AHT_HIP(hipEventRecord(ev[1], s));
        const uint32_t strip0 = col_hi < 0 ? 0u : (uint32_t)(col_lo / 64);
        const uint32_t strips = (col_hi < 0 ? (uint32_t)((t->cols + 63) / 64) : (uint32_t)(col_hi / 64 + 1)) - strip0;
        uint32_t strips_main = strips;
        int rpl_main = 0, rpl_side = 0;
        if (rowlists) {
            hipLaunchKernelGGL(k_compact_rows, dim3((unsigned)t->rows), dim3(256), 0, s, (const uint32_t*)bufs.dw,
                               t->rows, B, bpad(B), t->rlist, t->rlen);
            AHT_HIP(hipGetLastError());
            if ((st = launch_cells(t, B, t->step, s, strip0, strips, bufs, true, true, true, recorded)) != AHT_OK) return st;
        } else {
        if (col_hi < 0) even_round(t, B, strips, &strips_main, &rpl_main, &rpl_side);
        if (strips_main < strips) {
            if ((st = launch_cells_pair(t, B, t->step, s, strips, strips_main, rpl_main, rpl_side, bufs, true, true, recorded)) != AHT_OK)
                return st;
        } else if ((st = launch_cells(t, B, t->step, s, strip0, strips, bufs, full, false, true, recorded)) != AHT_OK) return st;
        }
        if (ev) {
            AHT_HIP(hipEventRecord(ev[2], s));
            t->events_used += 3;
        }
        if (col_hi < 0 && (st = full_update_done(t, B, watched, !static_scratch_only && !recorded, s)) != AHT_OK) return st;
        if (recorded) {                           // the kernels above read the device's counter: now it moves on
            hipLaunchKernelGGL(k_set_step, dim3(1), dim3(1), 0, s, t->step_state, 1u, 1);
            AHT_HIP(hipGetLastError());
        }
    } else {
        // nothing to apply: the call still counts
        hipLaunchKernelGGL(k_set_step, dim3(1), dim3(1), 0, (hipStream_t)stream, t->step_state, 1u, 1);
        AHT_HIP(hipGetLastError());
    }
    t->step += 1;
    return AHT_OK;
}

aht_status aht_pulsed_update(aht_tile* t, const float* x_dev, const float* d_dev, int32_t B, float lr, void* stream)
{
    return pulsed_update_impl(t, x_dev, d_dev, B, lr, stream, ConvView{});
}

aht_status aht_pulsed_update_noalloc(aht_tile* t, const float* x_dev, const float* d_dev, int32_t B, float lr,
                                     void* stream)
{
    return pulsed_update_impl(t, x_dev, d_dev, B, lr, stream, ConvView{}, 0, -1, true);
}

// Streams and events of aht_pulsed_update_many, per device, made on first use and kept until the process ends
// (default priority: streams of different priorities are not used anywhere in the library).
namespace {
constexpr int kManyStreams = 4;                   // hardware queues a process gets by default
struct ManyLanes {
    bool ready = false;
    hipStream_t stream[kManyStreams];
    hipEvent_t fork, join[kManyStreams];
};
std::mutex g_many_mutex;
ManyLanes g_many[64];
}  // namespace

static aht_status many_lanes(int device, ManyLanes** out)
{
    if (device < 0 || device >= 64) return fail(AHT_ERR_UNSUPPORTED, "device index %d", device);
    std::lock_guard<std::mutex> lock(g_many_mutex);
    ManyLanes& m = g_many[device];
    if (!m.ready) {
        AHT_HIP(hipEventCreateWithFlags(&m.fork, hipEventDisableTiming));
        for (int i = 0; i < kManyStreams; ++i) {
            AHT_HIP(hipStreamCreateWithFlags(&m.stream[i], hipStreamNonBlocking));
            AHT_HIP(hipEventCreateWithFlags(&m.join[i], hipEventDisableTiming));
        }
        m.ready = true;
    }
    *out = &m;
    return AHT_OK;
}

aht_status aht_pulsed_update_many(aht_tile* const* tiles, const float* const* x_dev, const float* const* d_dev,
                                  const int32_t* B, const float* lr, int32_t n, void* stream)
{
    if (n < 0) return fail(AHT_ERR_INVALID_ARG, "n must be >= 0");
    if (n == 0) return AHT_OK;
    if (!tiles || !x_dev || !d_dev || !B || !lr) return fail(AHT_ERR_INVALID_ARG, "null argument");
    aht_status st;
    for (int i = 0; i < n; ++i) {
        if ((st = check_update_args(tiles[i], x_dev[i], d_dev[i], B[i], lr[i])) != AHT_OK) return st;
        for (int k = 0; k < i; ++k)
            if (tiles[k] == tiles[i]) return fail(AHT_ERR_INVALID_ARG, "entries %d and %d name the same tile", k, i);
    }
    hipStream_t caller = (hipStream_t)stream;
    if (n == 1) return pulsed_update_impl(tiles[0], x_dev[0], d_dev[0], B[0], lr[0], stream, ConvView{});
    // A call being recorded into a graph: the kernels read every tile's step from its device counter and a small
    // kernel advances the counters afterwards; nothing may be allocated, no counters are sent to the host.
    const bool recorded = being_recorded(caller);
    if (recorded) {
        for (int i = 0; i < n; ++i) {
            const aht_tile* t = tiles[i];
            if (B[i] == 0 || lr[i] == 0.0f || use_small_kernel(t, B[i])) continue;
            if (t->profiling || !scratch_fits(t, B[i]) ||
                (use_row_lists(t, B[i]) && ((size_t)rpad(t) * ((size_t)bpad(B[i]) + kRowListPad) > t->rlist_entries || !t->rlen)))
                return fail(AHT_ERR_UNSUPPORTED, "entry %d: a recorded call cannot allocate scratch or time its kernels; make "
                            "the same call once outside the recording first (and switch profiling off)", i);
        }
    }
    ManyLanes* m = nullptr;
    if ((st = many_lanes(tiles[0]->device, &m)) != AHT_OK) return st;
    static std::mutex issue;                      // one call at a time forks and joins through the lanes' events
    std::lock_guard<std::mutex> lock(issue);

    // Four kinds of entries.  `in_turn`: nothing to apply: on the caller's stream (one tiny kernel that advances
    // the step).  `tiny`: tiles whose whole update is one short launch (k_update_small): on the caller's stream,
    // sharing launches per signature (forking would cost more than they take).  `grouped`: dense updates
    // whose kernels can share launches with those of other tiles: per-vector factors, pulse words and cell updates,
    // one launch per signature each, on the caller's stream (the cell updates after the lanes have joined).
    // `whole`: everything else (row lists, tiles being profiled): the whole update on a lane.
    const bool grouping = env_int("AHT_GROUP", 1) != 0;
    std::vector<int> in_turn, tiny, grouped, whole;
    for (int i = 0; i < n; ++i) {
        aht_tile* t = tiles[i];
        if (B[i] == 0 || lr[i] == 0.0f) {
            in_turn.push_back(i);
            continue;
        }
        if (use_small_kernel(t, B[i])) {
            if (grouping && !t->profiling) tiny.push_back(i);
            else in_turn.push_back(i);
            continue;
        }
        refresh_pulse_rate(t);                    // (the choices below follow the tile's latest counters)
        if (grouping && !t->profiling && !use_row_lists(t, B[i])) grouped.push_back(i);
        else whole.push_back(i);
    }
    if (grouped.size() == 1) {                    // nothing to share a launch with
        whole.push_back(grouped[0]);
        grouped.clear();
    }
    if (tiny.size() == 1) {
        in_turn.push_back(tiny[0]);
        tiny.clear();
    }
    auto cells_work = [&](int i) { return (double)tiles[i]->rows * tiles[i]->cols * ((double)B[i] + 8.0); };
    // The pulse words of the grouped entries share launches too (k_pulse_words_group, per word width, on the
    // caller's stream), behind one launch for the per-vector factors of those that need them (update management,
    // per-vector train lengths: k_line_scale_group).
    AHT_HIP(hipEventRecord(m->fork, caller));     // (before the caller's stream gets work of this call)
    std::vector<char> watched(n, 0);
    for (int width = 4; width <= 8; width += 4) {
        WordsGroup g{};
        LineScaleGroup ls{};
        unsigned blocks = 0, ls_blocks = 0;
        auto flush = [&]() -> aht_status {
            if (g.n == 0) return AHT_OK;
            if (ls.n != 0) {
                for (uint32_t k = ls.n; k <= (uint32_t)kGroupMax; ++k) ls.first_block[k] = ls_blocks;
                hipLaunchKernelGGL(k_line_scale_group, dim3(ls_blocks), dim3(256), 0, caller, ls);
                AHT_HIP(hipGetLastError());
                ls = LineScaleGroup{};
                ls_blocks = 0;
            }
            for (uint32_t k = g.n; k <= (uint32_t)kGroupMax; ++k) g.first_block[k] = blocks;
            if (width == 4) hipLaunchKernelGGL(k_pulse_words_group<uint32_t>, dim3(blocks), dim3(256), 0, caller, g);
            else hipLaunchKernelGGL(k_pulse_words_group<uint64_t>, dim3(blocks), dim3(256), 0, caller, g);
            AHT_HIP(hipGetLastError());
            g = WordsGroup{};
            blocks = 0;
            return AHT_OK;
        };
        for (int i : grouped) {
            aht_tile* t = tiles[i];
            if ((int)word_bytes(t) != width) continue;
            if ((st = ensure_scratch(t, B[i])) != AHT_OK) return st;
            watched[i] = watched_update(t, B[i]);
            const WordBufs w = tile_bufs(t);
            const unsigned nbx = (unsigned)blocks_for((size_t)cpad(t) + rpad(t)), ny = (unsigned)(B[i] < 32768 ? B[i] : 32768);
            if ((uint64_t)blocks + (uint64_t)nbx * ny > 0x7FFFFFFFull || g.n == (uint32_t)kGroupMax)
                if ((st = flush()) != AHT_OK) return st;
            WordsGroupEntry& e = g.e[g.n];
            e.x = x_dev[i]; e.d = d_dev[i]; e.xw = w.xw; e.dw = w.dw;
            e.row_stat = watched[i] ? t->pulse_count + 2 : nullptr;
            if (t->upd.update_management || t->dynamic_bl) {
                LineScaleGroupEntry& q = ls.e[ls.n];
                q.x = x_dev[i]; q.d = d_dev[i]; q.a_x = w.a_x; q.a_d = w.a_d; q.bl_b = t->dynamic_bl ? w.bl_b : nullptr;
                q.lr = (double)lr[i]; q.dw_min = (double)t->dev.dw_min;
                q.R = t->rows; q.C = t->cols; q.BL = t->upd.bl; q.update_management = t->upd.update_management;
                q.dynamic_bl = t->dynamic_bl;
                ls.first_block[ls.n] = ls_blocks;
                ls_blocks += (unsigned)B[i];
                ls.n += 1;
                e.a_x = w.a_x; e.a_d = w.a_d; e.bl_b = q.bl_b;
            }
            e.A = std::sqrt((double)lr[i] / ((double)t->dev.dw_min * (double)t->upd.bl));
            e.B = B[i]; e.R = t->rows; e.C = t->cols; e.Rpad = rpad(t); e.Cpad = cpad(t); e.Bpad = bpad(B[i]);
            e.BL = t->upd.bl; e.deterministic = t->train_kind;
            e.k0 = (uint32_t)t->seed; e.k1 = (uint32_t)(t->seed >> 32); e.t = t->step;
            e.nbx = nbx; e.ny = ny;
            e.step_on_device = recorded ? t->step_state : nullptr;
            g.first_block[g.n] = blocks;
            blocks += nbx * ny;
            g.n += 1;
        }
        if ((st = flush()) != AHT_OK) return st;
    }
    // the tiny tiles: their one-launch updates share launches per signature (device kind, word width, noise)
    {
        std::vector<char> done(n, 0);
        for (size_t a0 = 0; a0 < tiny.size(); ++a0) {
            const int i0 = tiny[a0];
            if (done[i0]) continue;
            const aht_tile* t0 = tiles[i0];
            SmallGroup g{};
            unsigned blocks = 0;
            for (size_t a1 = a0; a1 < tiny.size() && g.n < (uint32_t)kGroupMax; ++a1) {
                const int i = tiny[a1];
                aht_tile* t = tiles[i];
                if (done[i] || t->dev.kind != t0->dev.kind || use_u32(t) != use_u32(t0) ||
                    (t->dev.dw_min_std > 0.0f) != (t0->dev.dw_min_std > 0.0f))
                    continue;
                SmallGroupEntry& e = g.e[g.n];
                e.W = t->W;
                weights_written(t);
                e.dw_up = t->planes[AHT_PLANE_DW_UP]; e.dw_down = t->planes[AHT_PLANE_DW_DOWN];
                e.b_max = t->planes[AHT_PLANE_B_MAX]; e.b_min = t->planes[AHT_PLANE_B_MIN];
                e.slope_up = t->planes[AHT_PLANE_SLOPE_UP]; e.slope_down = t->planes[AHT_PLANE_SLOPE_DOWN];
                e.x = x_dev[i]; e.d = d_dev[i];
                e.pulse_count = t->pulse_count; e.step_state = t->step_state;
                e.A = std::sqrt((double)lr[i] / ((double)t->dev.dw_min * (double)t->upd.bl));
                e.B = B[i]; e.R = t->rows; e.C = t->cols; e.BL = t->upd.bl; e.deterministic = t->train_kind;
                e.k0 = (uint32_t)t->seed; e.k1 = (uint32_t)(t->seed >> 32); e.t = t->step;
                e.c2c = t->dev.dw_min_std;
                e.recorded = recorded ? 1 : 0;
                g.first_block[g.n] = blocks;
                blocks += (unsigned)((t->cols + 63) / 64) * (unsigned)((t->rows + 3) / 4);
                g.n += 1;
                done[i] = 1;
                t->info.rows_per_lane = 1;
                t->info.side_rows_per_lane = 0;
                t->info.row_lists = 0;
                t->info.stream_words = 0;
                t->full_updates += 1;
                t->step += 1;
            }
            for (uint32_t k = g.n; k <= (uint32_t)kGroupMax; ++k) g.first_block[k] = blocks;
            const bool noise = t0->dev.dw_min_std > 0.0f;
#define AHT_SMALL_GROUP(K, WT)                                                                                       \
    do {                                                                                                            \
        if (noise) hipLaunchKernelGGL((k_update_small_group<K, WT, true>), dim3(blocks), dim3(256), 0, caller, g);  \
        else hipLaunchKernelGGL((k_update_small_group<K, WT, false>), dim3(blocks), dim3(256), 0, caller, g);       \
    } while (0)
#define AHT_SMALL_GROUP_KIND(WT)                                                    \
    switch (t0->dev.kind) {                                                         \
        case AHT_CONSTANT_STEP: AHT_SMALL_GROUP(kConstantStep, WT); break;          \
        case AHT_LINEAR_STEP: AHT_SMALL_GROUP(kLinearStep, WT); break;              \
        default: AHT_SMALL_GROUP(kSoftBounds, WT); break;                           \
    }
            if (use_u32(t0)) { AHT_SMALL_GROUP_KIND(uint32_t) } else { AHT_SMALL_GROUP_KIND(uint64_t) }
#undef AHT_SMALL_GROUP_KIND
#undef AHT_SMALL_GROUP
            AHT_HIP(hipGetLastError());
        }
    }
    // the whole updates that go to the lanes, largest first, each to the lane with the least work so far
    struct Item { int i; double work; };
    std::vector<Item> items;
    for (int i : whole) items.push_back({i, cells_work(i)});
    std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) { return a.work > b.work; });
    double load[kManyStreams] = {0.0, 0.0, 0.0, 0.0};
    bool used[kManyStreams] = {false, false, false, false};
    aht_status result = AHT_OK;

    for (size_t k = 0; k < items.size() && result == AHT_OK; ++k) {
        const int i = items[k].i;
        aht_tile* t = tiles[i];
        int lane = 0;
        for (int l = 1; l < kManyStreams; ++l)
            if (load[l] < load[lane]) lane = l;
        if (!used[lane]) {
            AHT_HIP(hipStreamWaitEvent(m->stream[lane], m->fork, 0));
            used[lane] = true;
        }
        load[lane] += items[k].work;
        result = pulsed_update_impl(t, x_dev[i], d_dev[i], B[i], lr[i], (void*)m->stream[lane], ConvView{});
    }
    for (size_t k = 0; k < in_turn.size() && result == AHT_OK; ++k) {
        const int i = in_turn[k];
        result = pulsed_update_impl(tiles[i], x_dev[i], d_dev[i], B[i], lr[i], stream, ConvView{});
    }
    for (int l = 0; l < kManyStreams; ++l) {       // (also after a failure: what was launched is joined)
        if (!used[l]) continue;
        AHT_HIP(hipEventRecord(m->join[l], m->stream[l]));
        AHT_HIP(hipStreamWaitEvent(caller, m->join[l], 0));
    }
    if (result != AHT_OK) return result;

    // the cell updates of the grouped entries: one launch per signature (device kind, word width, noise, rows
    // per lane, hence also stream length and LDS), up to kGroupMax tiles each
    std::vector<CellLaunch> cl(n);
    for (int i : grouped) {
        aht_tile* t = tiles[i];
        if ((st = build_cell_launch(t, B[i], t->step, 0u, (uint32_t)((t->cols + 63) / 64), tile_bufs(t), true, false, true,
                                    recorded, &cl[i])) != AHT_OK)
            return st;
    }
    std::vector<char> done(n, 0);
    for (size_t a0 = 0; a0 < grouped.size(); ++a0) {
        const int i0 = grouped[a0];
        if (done[i0]) continue;
        const aht_tile* t0 = tiles[i0];
        CellGroup g{};
        unsigned blocks = 0;
        for (size_t a1 = a0; a1 < grouped.size() && g.n < (uint32_t)kGroupMax; ++a1) {
            const int i = grouped[a1];
            const aht_tile* t = tiles[i];
            if (done[i] || t->dev.kind != t0->dev.kind || use_u32(t) != use_u32(t0) ||
                (t->dev.dw_min_std > 0.0f) != (t0->dev.dw_min_std > 0.0f) || cl[i].rpl != cl[i0].rpl ||
                cl[i].lds != cl[i0].lds || (uint64_t)blocks + cl[i].blocks > 0x7FFFFFFFull)
                continue;
            CellGroupEntry& e = g.e[g.n];
            const CellPtrs& p = cl[i].p;
            e.W = p.W; e.dw_up = p.dw_up; e.dw_down = p.dw_down; e.b_max = p.b_max; e.b_min = p.b_min;
            e.slope_up = p.slope_up; e.slope_down = p.slope_down; e.xw = p.xw; e.dw = p.dw; e.pulse_count = p.pulse_count;
            e.a = cl[i].a;
            g.first_block[g.n] = blocks;
            blocks += cl[i].blocks;               // (a multiple of 8)
            g.n += 1;
            done[i] = 1;
        }
        for (uint32_t k = g.n; k <= (uint32_t)kGroupMax; ++k) g.first_block[k] = blocks;
        if (use_u32(t0)) launch_group_kind<uint32_t>(t0->dev.kind, t0->dev.dw_min_std > 0.0f, cl[i0].rpl, g, blocks, cl[i0].lds, caller);
        else launch_group_kind<uint64_t>(t0->dev.kind, t0->dev.dw_min_std > 0.0f, cl[i0].rpl, g, blocks, cl[i0].lds, caller);
        AHT_HIP(hipGetLastError());
        if (recorded) {                           // the kernels above read the devices' counters: now they move on
            StepGroup sg{};
            for (uint32_t k = 0; k < g.n; ++k) sg.state[k] = g.e[k].a.publish ? nullptr : const_cast<uint32_t*>(g.e[k].a.step_on_device);
            sg.n = g.n;
            hipLaunchKernelGGL(k_advance_steps, dim3(1), dim3(64), 0, caller, sg);
            AHT_HIP(hipGetLastError());
        }
    }
    for (int i : grouped) {
        aht_tile* t = tiles[i];
        if ((st = full_update_done(t, B[i], watched[i] != 0, !recorded, caller)) != AHT_OK) return st;
        t->step += 1;
    }
    return AHT_OK;
}

// checks the convolution geometry against the tile and fills the view; B = number of update vectors
static aht_status make_conv_view(const aht_tile* t, int32_t N, int32_t Cin, int32_t H, int32_t W, int32_t kh,
                                 int32_t kw, int32_t stride, int32_t pad, ConvView* v, int64_t* B)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    if (N < 0 || Cin <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0)
        return fail(AHT_ERR_INVALID_ARG, "convolution sizes must be positive (pad >= 0)");
    if ((int64_t)Cin * kh * kw != t->cols)
        return fail(AHT_ERR_INVALID_ARG, "Cin*kh*kw = %lld does not match the tile's %d columns",
                    (long long)Cin * kh * kw, t->cols);
    const int OH = (H + 2 * pad - kh) / stride + 1, OW = (W + 2 * pad - kw) / stride + 1;
    if (H + 2 * pad < kh || W + 2 * pad < kw || OH <= 0 || OW <= 0)
        return fail(AHT_ERR_INVALID_ARG, "kernel larger than the padded image");
    *v = ConvView{1, Cin, H, W, kh, kw, stride, pad, OH, OW, t->rows};
    *B = (int64_t)N * OH * OW;
    return AHT_OK;
}

aht_status aht_pulsed_update_conv2d(aht_tile* t, const float* img_dev, const float* grad_dev, int32_t N, int32_t Cin,
                                    int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                    float lr, void* stream)
{
    ConvView v{};
    int64_t B = 0;
    aht_status st = make_conv_view(t, N, Cin, H, W, kh, kw, stride, pad, &v, &B);
    if (st != AHT_OK) return st;
    return pulsed_update_impl(t, img_dev, grad_dev, B, lr, stream, v);
}

// `w_eff`: weights to multiply with instead of the tile's own (the effective weights of a unit cell)
static aht_status analog_mvm(aht_tile* t, const aht_io_params* io, const float* x, float* y, float* pre, int32_t B,
                             bool transposed, hipStream_t s, const float* w_eff = nullptr)
{
    if (!t || !io || !x || !y) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (B <= 0) return fail(AHT_ERR_INVALID_ARG, "B must be > 0");
    if (!finite_nonneg(io->inp_res) || !finite_nonneg(io->inp_noise) || !finite_nonneg(io->w_noise) ||
        !finite_nonneg(io->out_noise) || !finite_nonneg(io->out_res) || !(io->inp_bound > 0.0f) ||
        !(io->out_bound > 0.0f))
        return fail(AHT_ERR_INVALID_ARG, "io parameters must be finite and >= 0, bounds > 0");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    const int K = transposed ? t->rows : t->cols, N = transposed ? t->cols : t->rows;
    const size_t need = (size_t)B * K;
    if (need > t->mvm_xq_floats) {
        if (t->mvm_xq) AHT_HIP(hipFree(t->mvm_xq));
        t->mvm_xq = nullptr; t->mvm_xq_floats = 0;
        AHT_HIP(hipMalloc((void**)&t->mvm_xq, need * sizeof(float)));
        t->mvm_xq_floats = need;
    }
    if (B > t->mvm_b_cap) {
        if (t->mvm_alpha) AHT_HIP(hipFree(t->mvm_alpha));
        if (t->mvm_norm) AHT_HIP(hipFree(t->mvm_norm));
        t->mvm_alpha = t->mvm_norm = nullptr; t->mvm_b_cap = 0;
        AHT_HIP(hipMalloc((void**)&t->mvm_alpha, sizeof(float) * (size_t)B));
        AHT_HIP(hipMalloc((void**)&t->mvm_norm, sizeof(float) * (size_t)B));
        t->mvm_b_cap = B;
    }
    IoArgs a{io->inp_res, io->inp_bound, io->inp_noise, io->w_noise, io->out_noise, io->out_res, io->out_bound,
             io->noise_management ? 1 : 0};
    const uint32_t k0 = (uint32_t)t->seed, k1 = (uint32_t)(t->seed >> 32);
    const uint32_t step = transposed ? t->bwd_step : t->fwd_step;
    const uint32_t tag_in = transposed ? 9u : 7u, tag_out = transposed ? 10u : 8u;
    const int vec_in = (K % 4 == 0) && (((uintptr_t)x | (uintptr_t)t->mvm_xq) % 16 == 0);
    // Quantised inputs without input noise are integers times the input grid: the product then
    // runs on the bf16 matrix cores (integer codes exact in bf16, weights cut into three bf16 terms).
    const float* wmat = w_eff ? w_eff : t->W;
    const bool codes_path = env_int("AHT_MVM_CODES", 1) != 0 && io->inp_res > 0.0f &&
                            io->inp_noise == 0.0f && io->inp_bound / io->inp_res <= 256.0f && K % 32 == 0 &&
                            N % 16 == 0 && ((uintptr_t)wmat % 16 == 0);
    // Any other input (input noise, no or a finer DAC) as three bf16 planes of its fp32 value: the same
    // matrix cores, six passes instead of three.
    const bool planes_path = !codes_path && env_int("AHT_MVM_PLANES", 1) != 0 && K % 32 == 0 && N % 64 == 0 &&
                             ((uintptr_t)wmat % 16 == 0);
    // codes in blocks of 32 vectors; whole groups of 8 blocks (the most a wave takes), zero where no vector is
    const size_t plane_elems = (size_t)((B + 255) / 256) * 256 * (size_t)K;
    const size_t cneed = plane_elems * (planes_path ? 3 : 1);
    if ((codes_path || planes_path) && cneed > t->mvm_codes_elems) {
        if (t->mvm_codes) AHT_HIP(hipFree(t->mvm_codes));
        t->mvm_codes = nullptr; t->mvm_codes_elems = 0;
        AHT_HIP(hipMalloc((void**)&t->mvm_codes, cneed * sizeof(uint16_t)));
        AHT_HIP(hipMemset(t->mvm_codes, 0, cneed * sizeof(uint16_t)));
        AHT_HIP(hipDeviceSynchronize());          // (the caller's stream may not wait for the null stream)
        t->mvm_codes_elems = cneed;
    }
    t->info.mvm_path = codes_path ? 2 : planes_path ? 3 : 1;
    t->info.mvm_splits = 1;
    hipLaunchKernelGGL(k_mvm_prepare, dim3((unsigned)B), dim3(1024), 0, s, x, K, vec_in, a, k0, k1, step, tag_in,
                       t->mvm_xq, t->mvm_alpha, t->mvm_norm, (codes_path || planes_path) ? t->mvm_codes : nullptr,
                       planes_path ? 3 : 1, plane_elems);
    if (codes_path || planes_path) {
        int mt = B > 128 ? 16 : B > 64 ? 8 : B > 32 ? 4 : 2;    // 16-vector tiles per wave
        // (three planes: 8 at most, so that two workgroups fit a compute unit's LDS; 247 against 280 us at 1024 vectors)
        if (planes_path) mt = B > 64 ? 8 : 4;
        if (const int e = env_int("AHT_MVM_MT", 0)) mt = (e == 16 || e == 8 || e == 4 || e == 2) ? e : mt;
        if (planes_path && mt < 4) mt = 4;
        const int mchunks = (B + 16 * mt - 1) / (16 * mt), nslab = N / 16, steps = K / 32;
        // Small products (up to 0.6 GFLOP: a 1024 x 1024 tile with 256 vectors) are bound by the chain of
        // launches: a launch saved is 2.5 us of about 15, so they finish in the product kernel wherever
        // they can.  Larger ones, from 65 vectors on (and whole groups of 64 outputs): the four waves of a
        // workgroup share the codes of their vectors through LDS and write partial sums (measured at
        // 4096 x 4096: 47 against 54 us per call at 256 vectors, 72 against 92 at 512; no gain below).
        const bool small = 2.0 * (double)B * (double)N * (double)K <= 6e8;
        const bool fuse_ok = env_int("AHT_MVM_FUSED", 1) != 0;
        bool shared = planes_path || (mt >= 8 && N % 64 == 0 && env_int("AHT_MVM_SHARED", 1) != 0);
        int splits = env_int("AHT_MVM_SPLITS", 0);
        if (splits <= 0) {
            const long units = (long)mchunks * nslab;
            splits = (int)((1024 + units - 1) / units);                 // one wave per SIMD (measured optimum)
            if (splits > steps / 4) splits = steps / 4;
            if (!planes_path && small && fuse_ok && splits >= 3 && splits <= 8) shared = false;   // four slices, finished in the kernel
            if (shared && units >= 1024 && units < 2048 && steps >= 8) splits = 2;  // two waves per SIMD, where the sharing kernel has room
            if (!shared && splits >= 3 && splits <= (small ? 8 : 6)) splits = 4;
        } else if (!planes_path && small && fuse_ok && splits == 4) {
            shared = false;
        }
        if (splits > 16) splits = 16;
        if (splits < 1) splits = 1;
        t->info.mvm_splits = splits;
        // With four slices the four waves of a workgroup take one each and finish the product
        // themselves.  For large transposed products this loses: there two neighbouring groups of 16
        // outputs share every 128-byte line of the weights, and they share it best as waves of one
        // workgroup (measured at 4096 x 4096: 64 us per call with partial sums, 68 us fused).
        const bool fused = !shared && splits == 4 && (!transposed || small) && fuse_ok;
        if (!fused) {
            const size_t pneed = (size_t)splits * (size_t)B * (size_t)N;
            if (pneed > t->mvm_part_floats) {
                if (t->mvm_part) AHT_HIP(hipFree(t->mvm_part));
                t->mvm_part = nullptr; t->mvm_part_floats = 0;
                AHT_HIP(hipMalloc((void**)&t->mvm_part, pneed * sizeof(float)));
                t->mvm_part_floats = pneed;
            }
        }
        if (shared) {
            if (mt < 4) mt = 4;
            const dim3 sgrid((unsigned)((B + 16 * mt - 1) / (16 * mt)) * (unsigned)(N / 64) * (unsigned)splits);
            const size_t slds = (size_t)2 * (planes_path ? 3 : 1) * mt * 64 * 16;      // two stages of the planes of a step
#define AHT_SHARED_LAUNCH(MTV, TR, NPV)                                                                           \
    do {                                                                                                         \
        if (slds > 48 * 1024)                                                                                    \
            (void)hipFuncSetAttribute((const void*)k_mvm_gemm_codes_shared<MTV, TR, NPV>,                        \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)slds);                    \
        hipLaunchKernelGGL((k_mvm_gemm_codes_shared<MTV, TR, NPV>), sgrid, dim3(256), slds, s, t->mvm_codes,      \
                           plane_elems, wmat, B, N, K, t->cols, splits, planes_path ? 1.0f : io->inp_res,        \
                           t->mvm_part);                                                                         \
    } while (0)
#define AHT_SHARED_PICK(TR, NPV)                                                                                  \
    switch (mt) {                                                                                                \
        case 16: AHT_SHARED_LAUNCH(16, TR, NPV); break;                                                          \
        case 8: AHT_SHARED_LAUNCH(8, TR, NPV); break;                                                            \
        default: AHT_SHARED_LAUNCH(4, TR, NPV); break;                                                           \
    }
            if (planes_path) {
                if (transposed) { AHT_SHARED_PICK(true, 3) } else { AHT_SHARED_PICK(false, 3) }
            } else {
                if (transposed) { AHT_SHARED_PICK(true, 1) } else { AHT_SHARED_PICK(false, 1) }
            }
#undef AHT_SHARED_PICK
#undef AHT_SHARED_LAUNCH
            AHT_HIP(hipGetLastError());
            const size_t pairs = (size_t)B * (size_t)((N + 1) / 2);
            hipLaunchKernelGGL(k_mvm_epilogue, dim3(blocks_for(pairs)), dim3(256), 0, s, t->mvm_part, splits, B, N,
                               t->mvm_alpha, t->mvm_norm, a, k0, k1, step, tag_out, y, pre);
            AHT_HIP(hipGetLastError());
            if (transposed) t->bwd_step += 1; else t->fwd_step += 1;
            return AHT_OK;
        }
        const unsigned waves = (unsigned)mchunks * (unsigned)nslab * (unsigned)splits;
        const dim3 cgrid(fused ? (unsigned)mchunks * (unsigned)nslab : (waves + 3u) / 4u);
        const MvmTail tail{t->mvm_alpha, t->mvm_norm, a, k0, k1, step, tag_out, y, pre};
        const size_t xlds = fused ? (size_t)4 * mt * 256 * sizeof(float) : 0;
#define AHT_CODES_LAUNCH(MTV, TR, FU)                                                                            \
    do {                                                                                                         \
        if (xlds > 48 * 1024)                                                                                    \
            (void)hipFuncSetAttribute((const void*)k_mvm_gemm_codes<MTV, TR, FU>,                                \
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)xlds);                    \
        hipLaunchKernelGGL((k_mvm_gemm_codes<MTV, TR, FU>), cgrid, dim3(256), xlds, s, t->mvm_codes, wmat, B, N,  \
                           K, t->cols, splits, io->inp_res, t->mvm_part, tail);                                  \
    } while (0)
#define AHT_CODES_PICK(TR, FU)                                                                                   \
    switch (mt) {                                                                                                \
        case 16: AHT_CODES_LAUNCH(16, TR, FU); break;                                                            \
        case 8: AHT_CODES_LAUNCH(8, TR, FU); break;                                                              \
        case 4: AHT_CODES_LAUNCH(4, TR, FU); break;                                                              \
        default: AHT_CODES_LAUNCH(2, TR, FU); break;                                                             \
    }
        if (fused) {
            if (transposed) { AHT_CODES_PICK(true, true) } else { AHT_CODES_PICK(false, true) }
        } else {
            if (transposed) { AHT_CODES_PICK(true, false) } else { AHT_CODES_PICK(false, false) }
        }
#undef AHT_CODES_PICK
#undef AHT_CODES_LAUNCH
        AHT_HIP(hipGetLastError());
        if (!fused) {
            const size_t pairs = (size_t)B * (size_t)((N + 1) / 2);
            hipLaunchKernelGGL(k_mvm_epilogue, dim3(blocks_for(pairs)), dim3(256), 0, s, t->mvm_part, splits, B, N,
                               t->mvm_alpha, t->mvm_norm, a, k0, k1, step, tag_out, y, pre);
            AHT_HIP(hipGetLastError());
        }
        if (transposed) t->bwd_step += 1; else t->fwd_step += 1;
        return AHT_OK;
    }
    // K split aiming at two workgroups per compute unit (measured optimum at 4096 x 4096, B = 256:
    // more slices only add partial-sum traffic), at least four K steps per slice.
    // Blocks of 64 vectors keep three workgroups resident per compute unit; when there are more
    // tiles than that, blocks of 128 halve their number and read the weights half as often.
    int bm = ((long)((B + 63) / 64) * ((N + 63) / 64) > 3L * 256) ? 128 : 64;
    if (const int e = env_int("AHT_MVM_BM", 0)) bm = (e == 128) ? 128 : 64;
    const int mb = (B + bm - 1) / bm, nb = (N + 63) / 64, nchunks = (K + 31) / 32;
    int splits = env_int("AHT_MVM_SPLITS", 0);
    if (splits <= 0) {
        const long tiles = (long)mb * nb, want = (bm == 128) ? 256 : 512;     // 256 compute units
        splits = (int)((want + tiles - 1) / tiles);
        if (splits > nchunks / 4) splits = nchunks / 4;
    }
    if (splits > 16) splits = 16;
    if (splits < 1) splits = 1;
    t->info.mvm_splits = splits;
    if (splits > 1) {
        const size_t pneed = (size_t)splits * (size_t)B * (size_t)N;
        if (pneed > t->mvm_part_floats) {
            if (t->mvm_part) AHT_HIP(hipFree(t->mvm_part));
            t->mvm_part = nullptr; t->mvm_part_floats = 0;
            AHT_HIP(hipMalloc((void**)&t->mvm_part, pneed * sizeof(float)));
            t->mvm_part_floats = pneed;
        }
    }
    const unsigned total = (unsigned)mb * (unsigned)nb * (unsigned)splits;
    const dim3 grid(((total + 7u) / 8u) * 8u);
    // 16-byte accesses need aligned rows and whole groups; the tile's weights start 256-byte aligned
    const bool aligned = (K % 32 == 0) && (t->cols % 4 == 0) && (N % 4 == 0) &&
                         (((uintptr_t)t->mvm_xq | (uintptr_t)wmat) % 16 == 0);
#define AHT_MVM_LAUNCH(TR, BMV, AL)                                                                              \
    hipLaunchKernelGGL((k_mvm_gemm<TR, BMV, AL>), grid, dim3(256), 0, s, t->mvm_xq, wmat, B, N, K, t->cols,       \
                       t->mvm_alpha, t->mvm_norm, a, k0, k1, step, tag_out, y, pre, t->mvm_part, splits, mb, nb)
#define AHT_MVM_PICK(TR)                                                                                         \
    do {                                                                                                         \
        if (bm == 128) { if (aligned) AHT_MVM_LAUNCH(TR, 128, true); else AHT_MVM_LAUNCH(TR, 128, false); }      \
        else { if (aligned) AHT_MVM_LAUNCH(TR, 64, true); else AHT_MVM_LAUNCH(TR, 64, false); }                  \
    } while (0)
    if (transposed) AHT_MVM_PICK(true); else AHT_MVM_PICK(false);
#undef AHT_MVM_PICK
#undef AHT_MVM_LAUNCH
    if (splits > 1) {
        AHT_HIP(hipGetLastError());
        const size_t pairs = (size_t)B * (size_t)((N + 1) / 2);
        hipLaunchKernelGGL(k_mvm_epilogue, dim3(blocks_for(pairs)), dim3(256), 0, s, t->mvm_part, splits, B, N,
                           t->mvm_alpha, t->mvm_norm, a, k0, k1, step, tag_out, y, pre);
    }
    AHT_HIP(hipGetLastError());
    if (transposed) t->bwd_step += 1; else t->fwd_step += 1;
    return AHT_OK;
}

aht_status aht_forward(aht_tile* t, const aht_io_params* io, const float* x_dev, float* y_dev, float* pre_dev,
                       int32_t B, void* stream)
{
    return analog_mvm(t, io, x_dev, y_dev, pre_dev, B, false, (hipStream_t)stream);
}

aht_status aht_backward(aht_tile* t, const aht_io_params* io, const float* d_dev, float* g_dev, float* pre_dev,
                        int32_t B, void* stream)
{
    return analog_mvm(t, io, d_dev, g_dev, pre_dev, B, true, (hipStream_t)stream);
}

aht_status aht_transfer_column(aht_tile* src, aht_tile* dst, int32_t col, float lr, const aht_io_params* io, void* stream)
{
    if (!src || !dst || !io) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (src == dst) return fail(AHT_ERR_INVALID_ARG, "source and destination must be different tiles");
    if (src->rows != dst->rows || src->cols != dst->cols || src->device != dst->device)
        return fail(AHT_ERR_INVALID_ARG, "tiles must have the same shape and device");
    if (col < 0 || col >= src->cols) return fail(AHT_ERR_INVALID_ARG, "column %d out of range", col);
    if (!(lr >= 0.0f) || !std::isfinite(lr)) return fail(AHT_ERR_INVALID_ARG, "lr must be finite and >= 0");
    aht_status st = check_device(dst);
    if (st != AHT_OK) return st;
    const int R = dst->rows, C = dst->cols;
    if (!dst->xfer) AHT_HIP(hipMalloc((void**)&dst->xfer, sizeof(float) * ((size_t)C + 2 * (size_t)R)));
    float* onehot = dst->xfer;
    float* read = dst->xfer + C;
    float* neg = read + R;
    hipStream_t s = (hipStream_t)stream;
    if (io->inp_noise == 0.0f) {
        // without input noise only the column itself enters the product: read it directly
        if (!finite_nonneg(io->inp_res) || !finite_nonneg(io->w_noise) || !finite_nonneg(io->out_noise) ||
            !finite_nonneg(io->out_res) || !(io->inp_bound > 0.0f) || !(io->out_bound > 0.0f))
            return fail(AHT_ERR_INVALID_ARG, "io parameters must be finite and >= 0, bounds > 0");
        if ((st = check_device(src)) != AHT_OK) return st;
        IoArgs a{io->inp_res, io->inp_bound, io->inp_noise, io->w_noise, io->out_noise, io->out_res, io->out_bound,
                 io->noise_management ? 1 : 0};
        hipLaunchKernelGGL(k_mvm_column_read, dim3(blocks_for((size_t)(R > C ? R : C))), dim3(256), 0, s, src->W, R, C,
                           col, a, (uint32_t)src->seed, (uint32_t)(src->seed >> 32), src->fwd_step, 8u, read, neg, onehot);
        AHT_HIP(hipGetLastError());
        src->fwd_step += 1;
    } else {
        hipLaunchKernelGGL(k_one_hot, dim3(blocks_for((size_t)C)), dim3(256), 0, s, onehot, C, col);
        AHT_HIP(hipGetLastError());
        if ((st = analog_mvm(src, io, onehot, read, nullptr, 1, false, s)) != AHT_OK) return st;
        hipLaunchKernelGGL(k_negate, dim3(blocks_for((size_t)R)), dim3(256), 0, s, read, neg, R);
        AHT_HIP(hipGetLastError());
    }
    // dst -= lr * (-read) e_col^T; only the strip of 64 columns that holds `col` can receive pulses
    return pulsed_update_impl(dst, onehot, neg, 1, lr, stream, ConvView{}, col, col);
}

static aht_status check_unit_cell(aht_tile* const* dev, int32_t n)
{
    if (!dev || n < 1 || n > 8) return fail(AHT_ERR_INVALID_ARG, "a unit cell has 1..8 devices");
    for (int k = 0; k < n; ++k) {
        if (!dev[k]) return fail(AHT_ERR_INVALID_ARG, "null device");
        for (int j = 0; j < k; ++j)
            if (dev[j] == dev[k]) return fail(AHT_ERR_INVALID_ARG, "a tile appears twice in the unit cell");
        if (dev[k]->rows != dev[0]->rows || dev[k]->cols != dev[0]->cols || dev[k]->device != dev[0]->device ||
            dev[k]->upd.bl != dev[0]->upd.bl)
            return fail(AHT_ERR_INVALID_ARG, "devices of a unit cell must agree in shape, device and train length");
    }
    return check_device(dev[0]);
}

aht_status aht_unit_cell_update(aht_tile* const* dev, int32_t n, int32_t which, const float* x_dev, const float* d_dev,
                                int32_t B, float lr, void* stream)
{
    aht_status st = check_unit_cell(dev, n);
    if (st != AHT_OK) return st;
    if (which < -1 || which >= n) return fail(AHT_ERR_INVALID_ARG, "device index %d out of range", which);
    if (B < 0) return fail(AHT_ERR_INVALID_ARG, "B must be >= 0");
    if (!(lr >= 0.0f) || !std::isfinite(lr)) return fail(AHT_ERR_INVALID_ARG, "lr must be finite and >= 0");
    if (B > 0 && (!x_dev || !d_dev)) return fail(AHT_ERR_INVALID_ARG, "null x or d");
    aht_tile* lead = dev[0];
    const uint32_t step = lead->step;
    if (B > 0 && lr > 0.0f) {
        if ((st = ensure_scratch(lead, B)) != AHT_OK) return st;
        hipStream_t s = (hipStream_t)stream;
        const WordBufs bufs = tile_bufs(lead);
        if ((st = launch_words(lead, bufs, x_dev, d_dev, B, lr, step, s, ConvView{})) != AHT_OK) return st;
        const uint32_t strips = (uint32_t)((lead->cols + 63) / 64);
        // The devices are tiles of their own, fed from the same words: those after the first run beside
        // it, each on its own tile's side stream (measured, all devices updated: two devices of 512 x 512
        // with 512 vectors 0.90 -> 0.78 ms, four of 256 x 256 with 1 024 vectors 1.40 -> 0.83 ms, two of
        // 2048 x 2048 5.66 -> 5.50 ms, short calls 0.126 -> 0.118 ms: never slower than one after the other).
        // Better still, where the devices have one signature (device kind, word width, noise, launch shape): all
        // of them in one launch (k_cell_update_group), as aht_pulsed_update_many does with the tiles of a step.
        // (Measured, one launch against side streams: four devices of 512 x 512 with 64 vectors 0.185 / 0.208 ms;
        // long calls the same: 0.769 / 0.771, 0.812 / 0.810, 0.277 / 0.277 ms.)
        bool together = which < 0 && n > 1 && n <= kGroupMax && env_int("AHT_GROUP", 1) != 0 &&
                        env_int("AHT_EVEN_ROUND", 1) != 0 && !being_recorded(s);
        if (together) {
            std::vector<CellLaunch> cl(n);
            for (int k = 0; k < n; ++k) {
                if ((st = build_cell_launch(dev[k], B, step, 0u, strips, bufs, false, false, true, false, &cl[k])) != AHT_OK)
                    return st;
                const aht_tile* t = dev[k];
                together = together && t->dev.kind == lead->dev.kind && use_u32(t) == use_u32(lead) &&
                           (t->dev.dw_min_std > 0.0f) == (lead->dev.dw_min_std > 0.0f) && cl[k].rpl == cl[0].rpl &&
                           cl[k].lds == cl[0].lds;
            }
            uint64_t blocks = 0;
            for (int k = 0; k < n; ++k) blocks += cl[k].blocks;
            // (devices whose own launch already brings eight rounds of workgroups per compute unit gain nothing
            // from sharing one: two of 2048 x 2048 measured 1.39 ms in one launch, 1.35 ms beside each other)
            together = together && blocks <= 0x7FFFFFFFull && cl[0].blocks <= 256u * 8u;
            if (together) {
                CellGroup g{};
                unsigned at = 0;
                for (int k = 0; k < n; ++k) {
                    CellGroupEntry& e = g.e[k];
                    const CellPtrs& p = cl[k].p;
                    e.W = p.W; e.dw_up = p.dw_up; e.dw_down = p.dw_down; e.b_max = p.b_max; e.b_min = p.b_min;
                    e.slope_up = p.slope_up; e.slope_down = p.slope_down; e.xw = p.xw; e.dw = p.dw;
                    e.pulse_count = p.pulse_count;
                    e.a = cl[k].a;
                    g.first_block[k] = at;
                    at += cl[k].blocks;
                }
                g.n = (uint32_t)n;
                for (int k = n; k <= kGroupMax; ++k) g.first_block[k] = at;
                if (use_u32(lead)) launch_group_kind<uint32_t>(lead->dev.kind, lead->dev.dw_min_std > 0.0f, cl[0].rpl, g, at, cl[0].lds, s);
                else launch_group_kind<uint64_t>(lead->dev.kind, lead->dev.dw_min_std > 0.0f, cl[0].rpl, g, at, cl[0].lds, s);
                AHT_HIP(hipGetLastError());
            }
        }
        const bool beside = !together && which < 0 && n > 1 && env_int("AHT_EVEN_ROUND", 1) != 0;
        if (beside) {
            if (!lead->side_fork) AHT_HIP(hipEventCreateWithFlags(&lead->side_fork, hipEventDisableTiming));
            AHT_HIP(hipEventRecord(lead->side_fork, s));
        }
        for (int k = 0; k < n && !together; ++k) {
            if (which >= 0 && k != which) continue;
            hipStream_t sk = s;
            if (beside && k > 0) {
                if (!dev[k]->side_stream) AHT_HIP(hipStreamCreateWithFlags(&dev[k]->side_stream, hipStreamNonBlocking));
                if (!dev[k]->side_join) AHT_HIP(hipEventCreateWithFlags(&dev[k]->side_join, hipEventDisableTiming));
                sk = dev[k]->side_stream;
                AHT_HIP(hipStreamWaitEvent(sk, lead->side_fork, 0));
            }
            uint32_t strips_main = strips;
            int rpl_main = 0, rpl_side = 0;
            even_round(dev[k], B, strips, &strips_main, &rpl_main, &rpl_side);
            if (strips_main < strips) {
                if ((st = launch_cells_pair(dev[k], B, step, sk, strips, strips_main, rpl_main, rpl_side, bufs, false, true)) != AHT_OK)
                    return st;
            } else if ((st = launch_cells(dev[k], B, step, sk, 0u, strips, bufs, false, false, true)) != AHT_OK) return st;
            if (sk != s) {
                AHT_HIP(hipEventRecord(dev[k]->side_join, sk));
                AHT_HIP(hipStreamWaitEvent(s, dev[k]->side_join, 0));
            }
        }
    }
    for (int k = 0; k < n; ++k) {                             // the cell's devices count calls together
        dev[k]->step = step + 1;
        // (a device that was updated has left the new count in its device-side counter itself)
        const bool updated = B > 0 && lr > 0.0f && (which < 0 || k == which);
        if (!updated) hipLaunchKernelGGL(k_set_step, dim3(1), dim3(1), 0, (hipStream_t)stream, dev[k]->step_state, step + 1u, 0);
    }
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

static aht_status unit_cell_weights(aht_tile* const* dev, const float* gamma, int32_t n, float* w_out_dev, hipStream_t s)
{
    UnitCellArgs u{};
    u.n = n;
    for (int k = 0; k < n; ++k) {
        if (!std::isfinite(gamma[k])) return fail(AHT_ERR_INVALID_ARG, "gamma must be finite");
        u.w[k] = dev[k]->W;
        u.gamma[k] = gamma[k];
    }
    const size_t cells = (size_t)dev[0]->rows * dev[0]->cols;
    hipLaunchKernelGGL(k_unit_cell_weights, dim3(blocks_for((cells + 3) / 4)), dim3(256), 0, s, u, w_out_dev, cells);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

aht_status aht_unit_cell_weights(aht_tile* const* dev, const float* gamma, int32_t n, float* w_out_dev, void* stream)
{
    aht_status st = check_unit_cell(dev, n);
    if (st != AHT_OK) return st;
    if (!gamma || !w_out_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    return unit_cell_weights(dev, gamma, n, w_out_dev, (hipStream_t)stream);
}

static aht_status unit_cell_mvm(aht_tile* const* dev, const float* gamma, int32_t n, const aht_io_params* io,
                                const float* x_dev, float* y_dev, float* pre_dev, int32_t B, bool transposed, void* stream)
{
    aht_status st = check_unit_cell(dev, n);
    if (st != AHT_OK) return st;
    if (!gamma) return fail(AHT_ERR_INVALID_ARG, "null gamma");
    aht_tile* lead = dev[0];
    if (!lead->ucell_w)
        AHT_HIP(hipMalloc((void**)&lead->ucell_w, sizeof(float) * (size_t)lead->rows * lead->cols));
    bool same = lead->ucell_n == n && lead->ucell_stream == (hipStream_t)stream;
    for (int k = 0; same && k < n; ++k)
        same = lead->ucell_dev[k] == dev[k] && lead->ucell_ver[k] == dev[k]->w_version &&
               std::memcmp(&lead->ucell_gamma[k], &gamma[k], sizeof(float)) == 0;
    if (!same) {
        lead->ucell_n = 0;
        if ((st = unit_cell_weights(dev, gamma, n, lead->ucell_w, (hipStream_t)stream)) != AHT_OK) return st;
        for (int k = 0; k < n; ++k) {
            lead->ucell_dev[k] = dev[k];
            lead->ucell_ver[k] = dev[k]->w_version;
            lead->ucell_gamma[k] = gamma[k];
        }
        lead->ucell_stream = (hipStream_t)stream;
        lead->ucell_n = n;
    }
    return analog_mvm(lead, io, x_dev, y_dev, pre_dev, B, transposed, (hipStream_t)stream, lead->ucell_w);
}

aht_status aht_unit_cell_forward(aht_tile* const* dev, const float* gamma, int32_t n, const aht_io_params* io,
                                 const float* x_dev, float* y_dev, float* pre_dev, int32_t B, void* stream)
{
    return unit_cell_mvm(dev, gamma, n, io, x_dev, y_dev, pre_dev, B, false, stream);
}

aht_status aht_unit_cell_backward(aht_tile* const* dev, const float* gamma, int32_t n, const aht_io_params* io,
                                  const float* d_dev, float* g_dev, float* pre_dev, int32_t B, void* stream)
{
    return unit_cell_mvm(dev, gamma, n, io, d_dev, g_dev, pre_dev, B, true, stream);
}

aht_status aht_get_mvm_steps(const aht_tile* t, uint32_t* f, uint32_t* b)
{
    if (!t || !f || !b) return fail(AHT_ERR_INVALID_ARG, "null argument");
    *f = t->fwd_step;
    *b = t->bwd_step;
    return AHT_OK;
}

aht_status aht_set_mvm_steps(aht_tile* t, uint32_t f, uint32_t b)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    t->fwd_step = f;
    t->bwd_step = b;
    return AHT_OK;
}

aht_status aht_set_temporal(aht_tile* t, const aht_temporal_params* p)
{
    if (!t || !p) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (!(p->decay_rate >= 0.0f && p->decay_rate <= 1.0f)) return fail(AHT_ERR_INVALID_ARG, "decay_rate must be in 0..1");
    if (!finite_nonneg(p->decay_rate_dtod) || !finite_nonneg(p->diffusion) || !finite_nonneg(p->diffusion_dtod) ||
        !finite_nonneg(p->reset_dtod) || !finite_nonneg(p->reset_std) || !std::isfinite(p->reset))
        return fail(AHT_ERR_INVALID_ARG, "temporal parameters must be finite, spreads >= 0");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    const size_t n = (size_t)t->rows * t->cols;
    for (auto*& pl : t->tplanes)
        if (!pl) AHT_HIP(hipMalloc((void**)&pl, n * sizeof(float)));
    unsigned nb = blocks_for(n);
    if (nb > 65536u) nb = 65536u;
    hipLaunchKernelGGL(k_gen_temporal_planes, dim3(nb), dim3(256), 0, 0, p->decay_rate, p->decay_rate_dtod, p->diffusion,
                       p->diffusion_dtod, p->reset, p->reset_dtod, (uint32_t)t->seed, (uint32_t)(t->seed >> 32), n,
                       t->tplanes[0], t->tplanes[1], t->tplanes[2]);
    AHT_HIP(hipGetLastError());
    AHT_HIP(hipDeviceSynchronize());
    t->temporal = *p;
    t->has_temporal = true;
    return AHT_OK;
}

aht_status aht_decay_diffuse(aht_tile* t, void* stream)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    if (!t->has_temporal) return fail(AHT_ERR_INVALID_ARG, "aht_set_temporal has not been called");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    const size_t n = (size_t)t->rows * t->cols;
    weights_written(t);
    hipLaunchKernelGGL(k_decay_diffuse, dim3(blocks_for((n + 3) / 4)), dim3(256), 0, (hipStream_t)stream, t->W,
                       t->tplanes[0], t->tplanes[1], t->planes[AHT_PLANE_B_MAX], t->planes[AHT_PLANE_B_MIN], n,
                       (uint32_t)t->seed, (uint32_t)(t->seed >> 32), t->tstep, t->temporal.diffusion > 0.0f ? 1 : 0);
    AHT_HIP(hipGetLastError());
    t->tstep += 1;
    return AHT_OK;
}

aht_status aht_reset_columns(aht_tile* t, int32_t c0, int32_t ncols, void* stream)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    if (!t->has_temporal) return fail(AHT_ERR_INVALID_ARG, "aht_set_temporal has not been called");
    if (c0 < 0 || ncols < 0) return fail(AHT_ERR_INVALID_ARG, "c0 and ncols must be >= 0");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    if (c0 >= t->cols || ncols == 0) return AHT_OK;
    if (ncols > t->cols - c0) ncols = t->cols - c0;
    weights_written(t);
    hipLaunchKernelGGL(k_reset_columns, dim3(blocks_for((size_t)t->rows * ncols)), dim3(256), 0, (hipStream_t)stream, t->W,
                       t->tplanes[2], t->temporal.reset_std, t->planes[AHT_PLANE_B_MAX], t->planes[AHT_PLANE_B_MIN],
                       t->rows, t->cols, c0, ncols, (uint32_t)t->seed, (uint32_t)(t->seed >> 32), t->tstep);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

aht_status aht_get_temporal_plane(const aht_tile* t, int32_t which, float* dev_out, void* stream)
{
    if (!t || !dev_out) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (which < 0 || which >= AHT_NUM_TPLANES) return fail(AHT_ERR_INVALID_ARG, "plane index %d out of range", which);
    if (!t->has_temporal) return fail(AHT_ERR_INVALID_ARG, "aht_set_temporal has not been called");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    AHT_HIP(hipMemcpyAsync(dev_out, t->tplanes[which], (size_t)t->rows * t->cols * sizeof(float),
                           hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return AHT_OK;
}

aht_status aht_get_temporal_step(const aht_tile* t, uint32_t* step)
{
    if (!t || !step) return fail(AHT_ERR_INVALID_ARG, "null argument");
    *step = t->tstep;
    return AHT_OK;
}

aht_status aht_set_temporal_step(aht_tile* t, uint32_t step)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    t->tstep = step;
    return AHT_OK;
}

aht_status aht_profile_enable(aht_tile* t, int32_t enable)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    t->profiling = enable != 0;
    return AHT_OK;
}

aht_status aht_profile_read(aht_tile* t, double* ms_words, double* ms_cells, int32_t* calls)
{
    if (!t || !ms_words || !ms_cells || !calls) return fail(AHT_ERR_INVALID_ARG, "null argument");
    double w = 0.0, c = 0.0;
    for (size_t k = 0; k + 3 <= t->events_used; k += 3) {
        AHT_HIP(hipEventSynchronize(t->events[k + 2]));
        float a = 0.0f, b = 0.0f;
        AHT_HIP(hipEventElapsedTime(&a, t->events[k], t->events[k + 1]));
        AHT_HIP(hipEventElapsedTime(&b, t->events[k + 1], t->events[k + 2]));
        w += a;
        c += b;
    }
    *ms_words = w;
    *ms_cells = c;
    *calls = (int32_t)(t->events_used / 3);
    t->events_used = 0;
    return AHT_OK;
}

aht_status aht_set_pulse_mode(aht_tile* t, int32_t train_kind, int32_t dynamic_bl)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    if (train_kind != AHT_TRAIN_STOCHASTIC && train_kind != AHT_TRAIN_DETERMINISTIC)
        return fail(AHT_ERR_INVALID_ARG, "unknown train kind %d", train_kind);
    t->train_kind = train_kind;
    t->dynamic_bl = dynamic_bl ? 1 : 0;
    return AHT_OK;
}

aht_status aht_get_launch_info(const aht_tile* t, aht_launch_info* out)
{
    if (!t || !out) return fail(AHT_ERR_INVALID_ARG, "null argument");
    *out = t->info;
    out->pulse_rate = t->pulse_rate;
    out->row_fill = t->row_fill;
    return AHT_OK;
}

aht_status aht_get_step(const aht_tile* t, uint32_t* step)
{
    if (!t || !step) return fail(AHT_ERR_INVALID_ARG, "null argument");
    *step = t->step;
    return AHT_OK;
}

aht_status aht_set_step(aht_tile* t, uint32_t step)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    const uint32_t state[2] = {step, 0u};
    AHT_HIP(hipDeviceSynchronize());              // (no stream is given: nothing of the tile may be in flight)
    AHT_HIP(hipMemcpy(t->step_state, state, sizeof(state), hipMemcpyHostToDevice));
    t->step = step;
    return AHT_OK;
}

aht_status aht_sync_step(aht_tile* t, uint32_t* step, void* stream)
{
    if (!t) return fail(AHT_ERR_INVALID_ARG, "null tile");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    uint32_t v = 0;
    AHT_HIP(hipMemcpyAsync(&v, t->step_state, sizeof(v), hipMemcpyDeviceToHost, (hipStream_t)stream));
    AHT_HIP(hipStreamSynchronize((hipStream_t)stream));
    t->step = v;
    if (step) *step = v;
    return AHT_OK;
}

aht_status aht_get_pulse_count(const aht_tile* t, uint64_t* pulses, void* stream)
{
    if (!t || !pulses) return fail(AHT_ERR_INVALID_ARG, "null argument");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    unsigned long long v[2] = {0, 0};
    AHT_HIP(hipMemcpyAsync(v, t->pulse_count, sizeof(v), hipMemcpyDeviceToHost, (hipStream_t)stream));
    AHT_HIP(hipStreamSynchronize((hipStream_t)stream));
    *pulses = v[0] + v[1];
    return AHT_OK;
}

aht_status aht_get_device_planes(const aht_tile* t, int32_t plane, float* dev_out, void* stream)
{
    if (!t || !dev_out) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (plane < 0 || plane >= AHT_NUM_PLANES) return fail(AHT_ERR_INVALID_ARG, "plane index %d out of range", plane);
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    const size_t n = (size_t)t->rows * t->cols;
    hipStream_t s = (hipStream_t)stream;
    if (t->planes[plane]) {
        AHT_HIP(hipMemcpyAsync(dev_out, t->planes[plane], n * sizeof(float), hipMemcpyDeviceToDevice, s));
        return AHT_OK;
    }
    // slope planes that are not stored: 1/bound for SoftBounds, 0 for ConstantStep
    const float* bound = nullptr;
    if (t->dev.kind == AHT_SOFT_BOUNDS)
        bound = t->planes[plane == AHT_PLANE_SLOPE_UP ? AHT_PLANE_B_MAX : AHT_PLANE_B_MIN];
    unsigned nb = blocks_for(n);
    if (nb > 65536u) nb = 65536u;
    hipLaunchKernelGGL(k_derived_slope, dim3(nb), dim3(256), 0, s, bound, dev_out, n);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

aht_status aht_set_device_planes(aht_tile* t, int32_t plane, const float* dev_in, void* stream)
{
    if (!t || !dev_in) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (plane < 0 || plane >= AHT_NUM_PLANES) return fail(AHT_ERR_INVALID_ARG, "plane index %d out of range", plane);
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    if (!t->planes[plane])
        return fail(AHT_ERR_UNSUPPORTED, "slope planes can only be set on a LINEAR_STEP tile (they are derived otherwise)");
    AHT_HIP(hipMemcpyAsync(t->planes[plane], dev_in, (size_t)t->rows * t->cols * sizeof(float),
                           hipMemcpyDeviceToDevice, (hipStream_t)stream));
    return AHT_OK;
}

static aht_status debug_pulse_words_impl(aht_tile* t, const float* x_dev, const float* d_dev, int64_t B64, float lr,
                                         uint64_t* xw_dev, uint64_t* dw_dev, void* stream, const ConvView& conv)
{
    if (!t || !x_dev || !d_dev || !xw_dev || !dw_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (B64 <= 0 || B64 > 0x7FFFFFF0) return fail(AHT_ERR_INVALID_ARG, "B must be > 0");
    const int B = (int)B64;
    if (!(lr >= 0.0f) || !std::isfinite(lr)) return fail(AHT_ERR_INVALID_ARG, "lr must be finite and >= 0");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    if ((st = ensure_scratch(t, B)) != AHT_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    if ((st = launch_words(t, tile_bufs(t), x_dev, d_dev, B, lr, t->step, s, conv)) != AHT_OK) return st;
    const size_t nx = (size_t)B * t->cols, nd = (size_t)B * t->rows;
    if (use_u32(t)) {
        hipLaunchKernelGGL(k_words_to_public<uint32_t>, dim3(blocks_for(nx)), dim3(256), 0, s, (const uint32_t*)t->xw, xw_dev, B, t->cols, cpad(t), 0);
        hipLaunchKernelGGL(k_words_to_public<uint32_t>, dim3(blocks_for(nd)), dim3(256), 0, s, (const uint32_t*)t->dw, dw_dev, B, t->rows, rpad(t), bpad(B));
    } else {
        hipLaunchKernelGGL(k_words_to_public<uint64_t>, dim3(blocks_for(nx)), dim3(256), 0, s, (const uint64_t*)t->xw, xw_dev, B, t->cols, cpad(t), 0);
        hipLaunchKernelGGL(k_words_to_public<uint64_t>, dim3(blocks_for(nd)), dim3(256), 0, s, (const uint64_t*)t->dw, dw_dev, B, t->rows, rpad(t), bpad(B));
    }
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

aht_status aht_debug_pulse_words(aht_tile* t, const float* x_dev, const float* d_dev, int32_t B, float lr,
                                 uint64_t* xw_dev, uint64_t* dw_dev, void* stream)
{
    return debug_pulse_words_impl(t, x_dev, d_dev, B, lr, xw_dev, dw_dev, stream, ConvView{});
}

aht_status aht_debug_pulse_words_conv2d(aht_tile* t, const float* img_dev, const float* grad_dev, int32_t N, int32_t Cin,
                                        int32_t H, int32_t W, int32_t kh, int32_t kw, int32_t stride, int32_t pad,
                                        float lr, uint64_t* xw_dev, uint64_t* dw_dev, void* stream)
{
    ConvView v{};
    int64_t B = 0;
    aht_status st = make_conv_view(t, N, Cin, H, W, kh, kw, stride, pad, &v, &B);
    if (st != AHT_OK) return st;
    return debug_pulse_words_impl(t, img_dev, grad_dev, B, lr, xw_dev, dw_dev, stream, v);
}

aht_status aht_debug_counts(aht_tile* t, const uint64_t* xw_dev, const uint64_t* dw_dev, int32_t B, int32_t b,
                            int8_t* out_dev, void* stream)
{
    if (!t || !xw_dev || !dw_dev || !out_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (B <= 0 || b < 0 || b >= B) return fail(AHT_ERR_INVALID_ARG, "sample index out of range");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    const size_t n = (size_t)t->rows * t->cols;
    hipLaunchKernelGGL(k_counts, dim3(blocks_for(n)), dim3(256), 0, (hipStream_t)stream, xw_dev, dw_dev, b, t->rows,
                       t->cols, t->upd.bl, out_dev);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

aht_status aht_debug_apply_words(aht_tile* t, const uint64_t* xw_dev, const uint64_t* dw_dev, int32_t B,
                                 uint32_t step, void* stream)
{
    if (!t || !xw_dev || !dw_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (B <= 0) return fail(AHT_ERR_INVALID_ARG, "B must be > 0");
    aht_status st = check_device(t);
    if (st != AHT_OK) return st;
    if ((st = ensure_scratch(t, B)) != AHT_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const size_t nx = (size_t)B * cpad(t), nd = (size_t)B * rpad(t);
    if (use_u32(t)) {
        hipLaunchKernelGGL(k_words_from_public<uint32_t>, dim3(blocks_for(nx)), dim3(256), 0, s, xw_dev, (uint32_t*)t->xw, B, t->cols, cpad(t), 0, t->upd.bl);
        hipLaunchKernelGGL(k_words_from_public<uint32_t>, dim3(blocks_for(nd)), dim3(256), 0, s, dw_dev, (uint32_t*)t->dw, B, t->rows, rpad(t), bpad(B), t->upd.bl);
    } else {
        hipLaunchKernelGGL(k_words_from_public<uint64_t>, dim3(blocks_for(nx)), dim3(256), 0, s, xw_dev, (uint64_t*)t->xw, B, t->cols, cpad(t), 0, t->upd.bl);
        hipLaunchKernelGGL(k_words_from_public<uint64_t>, dim3(blocks_for(nd)), dim3(256), 0, s, dw_dev, (uint64_t*)t->dw, B, t->rows, rpad(t), bpad(B), t->upd.bl);
    }
    AHT_HIP(hipGetLastError());
    return launch_cells(t, B, step, s, 0u, (uint32_t)((t->cols + 63) / 64), tile_bufs(t), false);
}

aht_status aht_debug_philox(const uint32_t* ctr_dev, const uint32_t* key_dev, int32_t n, uint32_t* out_dev, void* stream)
{
    if (!ctr_dev || !key_dev || !out_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (n <= 0) return fail(AHT_ERR_INVALID_ARG, "n must be > 0");
    hipLaunchKernelGGL(k_debug_philox, dim3(blocks_for((size_t)n)), dim3(256), 0, (hipStream_t)stream, ctr_dev, key_dev, n, out_dev);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

aht_status aht_debug_gauss(uint64_t seed, uint32_t index, uint32_t t, uint32_t tag, uint32_t q0, int32_t n,
                           int32_t fast, float* gauss_dev, void* stream)
{
    if (!gauss_dev) return fail(AHT_ERR_INVALID_ARG, "null argument");
    if (n <= 0) return fail(AHT_ERR_INVALID_ARG, "n must be > 0");
    hipLaunchKernelGGL(k_debug_gauss, dim3(blocks_for((size_t)n)), dim3(256), 0, (hipStream_t)stream,
                       (uint32_t)seed, (uint32_t)(seed >> 32), index, t, tag, q0, n, fast, gauss_dev);
    AHT_HIP(hipGetLastError());
    return AHT_OK;
}

#ifdef AHT_WAVE_STAMPS
// Profiling build only: the cell kernel's waves write their time stamps to `stamps_dev`
// (8 words per wave, 4 waves per workgroup of the launch; nullptr switches the stamps off).
int aht_debug_set_wave_stamps(unsigned long long* stamps_dev)
{
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(aht::g_wave_stamps), &stamps_dev, sizeof(stamps_dev));
}
#endif

}  // extern "C"
