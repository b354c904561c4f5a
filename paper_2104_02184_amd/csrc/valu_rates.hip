// Issue-rate microbenchmark for single vector-ALU instructions on gfx950.
//
// Each kernel runs eight independent dependency chains of one instruction, 4096 iterations,
// from 2048 workgroups of 256 lanes (8 waves per SIMD), timed with HIP events.  The result is
// the sustained rate in lane-ops per second, which calibrates the ALU roofline of the
// cell-update kernel: v_fma_f32 defines the nominal rate (256 CUs x 64 lanes x 2.4 GHz),
// transcendentals run at about half of it, simple two-operand integer ops faster.
// Build: python -m paper_2104_02184_amd.build valu_rates ; run: paper_2104_02184_amd/valu_rates
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
#define ITERS 4096
#define CHK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n", hipGetErrorString(e), __LINE__); return 1;}}while(0)

#define KERNEL(NAME, ASMSTR, CONSTRAINT_T)                                                 \
__global__ void __launch_bounds__(256) NAME(uint32_t* out, uint32_t seed) {                \
    CONSTRAINT_T a0 = (CONSTRAINT_T)(threadIdx.x + seed), a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3,           \
                 a4 = a0 + 4, a5 = a0 + 5, a6 = a0 + 6, a7 = a0 + 7;                     \
    CONSTRAINT_T b = (CONSTRAINT_T)(seed | 3);                                                              \
    for (int i = 0; i < ITERS; ++i) {                                                      \
        asm volatile(ASMSTR : "+v"(a0) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a1) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a2) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a3) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a4) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a5) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a6) : "v"(b));                                        \
        asm volatile(ASMSTR : "+v"(a7) : "v"(b));                                        \
    }                                                                                      \
    CONSTRAINT_T s = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;                                \
    if (s == (CONSTRAINT_T)12345) out[0] = 1;                                              \
}

KERNEL(k_and, "v_and_b32 %0, %0, %1", uint32_t)
KERNEL(k_add, "v_add_u32 %0, %0, %1", uint32_t)
KERNEL(k_bcnt, "v_bcnt_u32_b32 %0, %1, %0", uint32_t)
KERNEL(k_mul_lo, "v_mul_lo_u32 %0, %0, %1", uint32_t)
KERNEL(k_mul_hi, "v_mul_hi_u32 %0, %0, %1", uint32_t)
KERNEL(k_mul24, "v_mul_u32_u24 %0, %0, %1", uint32_t)
KERNEL(k_bitop3, "v_bitop3_b32 %0, %0, %1, %1 bitop3:0x96", uint32_t)
KERNEL(k_cndmask, "v_cndmask_b32 %0, %0, %1, vcc", uint32_t)
KERNEL(k_bfi, "v_bfi_b32 %0, %1, %0, %1", uint32_t)
KERNEL(k_fma, "v_fma_f32 %0, %0, %1, %1", float)
KERNEL(k_mulf, "v_mul_f32 %0, %0, %1", float)
KERNEL(k_log, "v_log_f32 %0, %0", float)
KERNEL(k_sin, "v_sin_f32 %0, %0", float)
KERNEL(k_sqrt, "v_sqrt_f32 %0, %0", float)
KERNEL(k_rcp, "v_rcp_f32 %0, %0", float)
KERNEL(k_cvt, "v_cvt_f32_u32 %0, %0", uint32_t)
KERNEL(k_med3, "v_med3_f32 %0, %0, %1, %1", float)
KERNEL(k_lshr, "v_lshrrev_b32 %0, 1, %0", uint32_t)
KERNEL(k_cmp, "v_cmp_ne_u32 vcc, %0, %1", uint32_t)
KERNEL(k_addc, "v_addc_co_u32 %0, vcc, %0, %1, vcc", uint32_t)


KERNEL(k_bfm, "v_bfm_b32 %0, %0, %1", uint32_t)
KERNEL(k_andor, "v_and_or_b32 %0, %0, %1, %1", uint32_t)
KERNEL(k_bfei, "v_bfe_i32 %0, %0, 3, 1", uint32_t)
KERNEL(k_lshladd, "v_lshl_add_u32 %0, %0, 2, %1", uint32_t)
KERNEL(k_max3, "v_max3_u32 %0, %0, %1, %1", uint32_t)
KERNEL(k_ashr, "v_ashrrev_i32 %0, 31, %0", uint32_t)
KERNEL(k_xor, "v_xor_b32 %0, %0, %1", uint32_t)
KERNEL(k_or, "v_or_b32 %0, %0, %1", uint32_t)
KERNEL(k_sub, "v_sub_u32 %0, %0, %1", uint32_t)
KERNEL(k_maxf, "v_max_f32 %0, %0, %1", float)
KERNEL(k_cmpgt, "v_cmp_gt_i32 vcc, %0, %1", uint32_t)
KERNEL(k_cnd64, "v_cndmask_b32_e64 %0, %0, %1, s[8:9]", uint32_t)
KERNEL(k_alignbit, "v_alignbit_b32 %0, %0, %1, %1", uint32_t)
KERNEL(k_logfma, "v_log_f32 %0, %0\n v_fma_f32 %1, %1, %1, %1", float)
KERNEL(k_logfma2, "v_log_f32 %0, %0\n v_fma_f32 %1, %1, %1, %1\n v_fma_f32 %1, %1, %1, %1", float)
KERNEL(k_logand2, "v_log_f32 %0, %0\n v_and_b32 %1, %1, %1\n v_and_b32 %1, %1, %1", float)
__global__ void __launch_bounds__(256) k_lshl64(uint32_t* out, uint32_t seed) {
    uint64_t a0 = threadIdx.x + seed, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0+4, a5=a0+5, a6=a0+6, a7=a0+7;
    uint32_t b = seed & 3;
    for (int i = 0; i < ITERS; ++i) {
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a0) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a1) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a2) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a3) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a4) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a5) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a6) : "v"(b));
        asm volatile("v_lshlrev_b64 %0, %1, %0" : "+v"(a7) : "v"(b));
    }
    uint64_t s = a0+a1+a2+a3+a4+a5+a6+a7;
    if (s == 12345) out[0] = 1;
}
__global__ void __launch_bounds__(256) k_mad64(uint32_t* out, uint32_t seed) {
    uint64_t a0 = threadIdx.x + seed, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0+4, a5=a0+5, a6=a0+6, a7=a0+7;
    uint32_t b = seed | 3;
    for (int i = 0; i < ITERS; ++i) {
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a0) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a1) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a2) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a3) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a4) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a5) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a6) : "v"(b) : "vcc");
        asm volatile("v_mad_u64_u32 %0, vcc, %1, %1, %0" : "+v"(a7) : "v"(b) : "vcc");
    }
    uint64_t s = a0+a1+a2+a3+a4+a5+a6+a7;
    if (s == 12345) out[0] = 1;
}
// mad64 with a zero addend (as the Philox round uses it): "v_mad_u64_u32 d, vcc, a, b, 0"
__global__ void __launch_bounds__(256) k_mad64z(uint32_t* out, uint32_t seed) {
    uint32_t x0 = threadIdx.x + seed, x1 = x0+1, x2=x0+2, x3=x0+3, x4=x0+4,x5=x0+5,x6=x0+6,x7=x0+7;
    uint32_t b = seed | 3;
    for (int i = 0; i < ITERS; ++i) {
        uint64_t t;
#define ONE(X) asm volatile("v_mad_u64_u32 %0, vcc, %1, %2, 0" : "=v"(t) : "v"(X), "v"(b) : "vcc"); X = (uint32_t)(t >> 32) ^ (uint32_t)t;
        ONE(x0) ONE(x1) ONE(x2) ONE(x3) ONE(x4) ONE(x5) ONE(x6) ONE(x7)
    }
    uint32_t s = x0+x1+x2+x3+x4+x5+x6+x7;
    if (s == 12345) out[0] = 1;
}
__global__ void __launch_bounds__(256) k_ldsw8(uint32_t* out, uint32_t seed) {
    __shared__ unsigned char buf[256*68];
    uint32_t a = threadIdx.x * 68;
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u) { asm volatile("ds_write_b8 %0, %1 offset:%2" :: "v"(a), "v"(seed), "n"(u)); }
    }
    __syncthreads();
    if (buf[threadIdx.x*68] == 77 && seed == 99999) out[0] = 1;
}

// fp32 matrix-core rate: v_mfma_f32_32x32x2_f32 (4096 flops per wave instruction), NCHAIN
// independent accumulators per wave.  Calibrates the roofline of the analog product.
typedef float floatx16 __attribute__((ext_vector_type(16)));
// Placement of 8-byte (VOP3) instructions: the same run of eight, once starting at an address that
// is a multiple of 8 and once 4 bytes further (both variants execute two s_nop per iteration).
#define KPLACE(NAME, PRE, POST, INSTR)                                                     \
__global__ void __launch_bounds__(256) NAME(uint32_t* out, uint32_t seed) {                \
    uint32_t a0 = threadIdx.x + seed, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0 + 4, a5 = a0 + 5,      \
             a6 = a0 + 6, a7 = a0 + 7;                                                     \
    uint32_t b = seed | 3;                                                                 \
    for (int i = 0; i < ITERS; ++i) {                                                      \
        asm volatile(".p2align 3\n" PRE                                                    \
                     INSTR(0) INSTR(1) INSTR(2) INSTR(3) INSTR(4) INSTR(5) INSTR(6) INSTR(7) POST           \
                     : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7)      \
                     : "v"(b));                                                            \
    }                                                                                      \
    uint32_t s = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7;                                    \
    if (s == 12345u) out[0] = 1;                                                           \
}
#define I_BITOP3(k) "v_bitop3_b32 %" #k ", %" #k ", %8, %8 bitop3:0x96\n"
#define I_FMA64(k) "v_fma_f32 %" #k ", %" #k ", %8, %8\n"
KPLACE(k_place_bitop3_2, "s_nop 0\ns_nop 0\n", "", I_BITOP3)
KPLACE(k_place_bitop3_3, "s_nop 0\ns_nop 0\ns_nop 0\n", "", I_BITOP3)
KPLACE(k_place_bitop3_4, "s_nop 0\ns_nop 0\ns_nop 0\ns_nop 0\n", "", I_BITOP3)
KPLACE(k_place_bitop3_5, "s_nop 0\ns_nop 0\ns_nop 0\ns_nop 0\ns_nop 0\n", "", I_BITOP3)
KPLACE(k_place_fma_2, "s_nop 0\ns_nop 0\n", "", I_FMA64)
KPLACE(k_place_fma_3, "s_nop 0\ns_nop 0\ns_nop 0\n", "", I_FMA64)
KPLACE(k_place_fma_4, "s_nop 0\ns_nop 0\ns_nop 0\ns_nop 0\n", "", I_FMA64)
KPLACE(k_place_fma_5, "s_nop 0\ns_nop 0\ns_nop 0\ns_nop 0\ns_nop 0\n", "", I_FMA64)

template <int NCHAIN>
__global__ void __launch_bounds__(256) k_mfma(uint32_t* out, uint32_t seed) {
    floatx16 acc[NCHAIN];
    for (int c = 0; c < NCHAIN; ++c)
        for (int r = 0; r < 16; ++r) acc[c][r] = (float)(threadIdx.x + c + r);
    const float a = (float)(seed | 1), b = 1.0f / (float)(seed | 3);
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
        for (int c = 0; c < NCHAIN; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
    for (int c = 0; c < NCHAIN; ++c)
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 12345.0f) out[0] = 1;
}
// bf16 matrix-core rate: v_mfma_f32_16x16x32_bf16 (16 384 flops per wave instruction) and
// v_mfma_f32_32x32x16_bf16 (32 768), NCHAIN independent accumulators per wave.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
template <int NCHAIN>
__global__ void __launch_bounds__(256) k_mfma_bf16_16(uint32_t* out, uint32_t seed) {
    floatx4 acc[NCHAIN];
    for (int c = 0; c < NCHAIN; ++c)
        for (int r = 0; r < 4; ++r) acc[c][r] = (float)(threadIdx.x + c + r);
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((seed | 1) + e); b[e] = (__bf16)(1.0f / (float)((seed | 3) + e)); }
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
        for (int c = 0; c < NCHAIN; ++c) acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
    for (int c = 0; c < NCHAIN; ++c)
        for (int r = 0; r < 4; ++r) s += acc[c][r];
    if (s == 12345.0f) out[0] = 1;
}
template <int NCHAIN>
__global__ void __launch_bounds__(256) k_mfma_bf16_32(uint32_t* out, uint32_t seed) {
    floatx16 acc[NCHAIN];
    for (int c = 0; c < NCHAIN; ++c)
        for (int r = 0; r < 16; ++r) acc[c][r] = (float)(threadIdx.x + c + r);
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((seed | 1) + e); b[e] = (__bf16)(1.0f / (float)((seed | 3) + e)); }
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
        for (int c = 0; c < NCHAIN; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.0f;
    for (int c = 0; c < NCHAIN; ++c)
        for (int r = 0; r < 16; ++r) s += acc[c][r];
    if (s == 12345.0f) out[0] = 1;
}
// What a single wave overlaps with its matrix instructions: per iteration 16 independent
// v_mfma_f32_16x16x32_bf16 (256 cycles of the matrix pipeline) and, interleaved with them,
// MODE 1: 32 independent vector-ALU instructions; 2: 8 LDS reads of 16 bytes per lane;
// 3: 4 global loads of 16 bytes per lane from a 64 KB buffer (cache resident); 0: nothing.
template <int MODE>
__global__ void __launch_bounds__(256) k_mfma_mix(uint32_t* out, uint32_t seed, const uint4* gbuf) {
    __shared__ uint4 lbuf[1024];
    for (int i = threadIdx.x; i < 1024; i += 256) lbuf[i] = make_uint4(i, seed, i, seed);
    __syncthreads();
    floatx4 acc[16];
    for (int c = 0; c < 16; ++c)
        for (int r = 0; r < 4; ++r) acc[c][r] = (float)(threadIdx.x + c + r);
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(float)((seed | 1) + e); b[e] = (__bf16)(1.0f / (float)((seed | 3) + e)); }
    uint32_t v[32];
    for (int k = 0; k < 32; ++k) v[k] = threadIdx.x * 7 + k + seed;
    uint4 ld[8];
    for (int k = 0; k < 8; ++k) ld[k] = make_uint4(k, k, k, k);
    const uint32_t lane = threadIdx.x;
    for (int i = 0; i < ITERS; ++i) {
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[c], 0, 0, 0);
            if (MODE == 1) {
                asm volatile("v_and_b32 %0, %0, %2\nv_and_b32 %1, %1, %2" : "+v"(v[2 * c]), "+v"(v[2 * c + 1]) : "v"(seed | 0xFFFFFFF0u));
            } else if (MODE == 2) {
                if (c % 2 == 0) {
                    const uint4 t = lbuf[(lane + 64 * (c / 2) + (uint32_t)i) & 1023];
                    ld[c / 2].x ^= t.x; ld[c / 2].y ^= t.y; ld[c / 2].z ^= t.z; ld[c / 2].w ^= t.w;
                }
            } else if (MODE == 3) {
                if (c % 4 == 0) {
                    const uint4 t = gbuf[(lane + 256 * (c / 4) + 1024u * (blockIdx.x & 3u) + (uint32_t)i * 64u) & 4095u];
                    ld[c / 4].x ^= t.x; ld[c / 4].y ^= t.y; ld[c / 4].z ^= t.z; ld[c / 4].w ^= t.w;
                }
            }
        }
    }
    float s = 0.0f;
    for (int c = 0; c < 16; ++c)
        for (int r = 0; r < 4; ++r) s += acc[c][r];
    uint32_t u = 0;
    for (int k = 0; k < 32; ++k) u += v[k];
    for (int k = 0; k < 8; ++k) u += ld[k].x + ld[k].y + ld[k].z + ld[k].w;
    if (s == 12345.0f && u == 77u) out[0] = 1;
}
template <typename K> int run_mix(const char* name, K kern, int wg_per_cu, uint32_t* out, const uint4* gbuf) {
    const int blocks = 256 * wg_per_cu, threads = 256;
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u, gbuf);
    CHK(hipDeviceSynchronize());
    CHK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u, gbuf);
    CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
    float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
    // cycles of one SIMD per iteration of one wave, at 2.4 GHz, had the waves of a SIMD run one after the other
    printf("%-34s %8.3f ms  %7.1f cycles per iteration and wave (matrix pipeline alone: 256)\n", name, ms,
           ms * 1e-3 * 2.4e9 / ITERS / wg_per_cu);
    fflush(stdout);
    return 0;
}

template <typename K> int run_mfma_bf16(const char* name, K kern, int nchain, int wg_per_cu, double flops_per_instr, uint32_t* out) {
    const int blocks = 256 * wg_per_cu, threads = 256;
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u);
    CHK(hipDeviceSynchronize());
    CHK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u);
    CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
    float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
    const double flops = (double)blocks * (threads / 64) * ITERS * nchain * flops_per_instr;
    printf("%-26s %8.3f ms  %8.2f TFLOP/s  (%.3f of 2500)\n", name, ms, flops / ms / 1e9, flops / ms / 1e9 / 2500.0);
    fflush(stdout);
    return 0;
}

template <typename K> int run_mfma(const char* name, K kern, int nchain, int wg_per_cu, uint32_t* out) {
    const int blocks = 256 * wg_per_cu, threads = 256;
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u);
    CHK(hipDeviceSynchronize());
    CHK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u);
    CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
    float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
    const double flops = (double)blocks * (threads / 64) * ITERS * nchain * 4096.0;
    printf("%-22s %8.3f ms  %8.2f TFLOP/s  (%.3f of 157.3)\n", name, ms, flops / ms / 1e9, flops / ms / 1e9 / 157.3);
    fflush(stdout);
    return 0;
}

template <typename K> int run(const char* name, K kern, double ops_per_thread_iter, uint32_t* out) {
    const int blocks = 256 * 8, threads = 256;  // 8 WG/CU -> 8 waves per SIMD
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u);
    CHK(hipDeviceSynchronize());
    CHK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(threads), 0, 0, out, 1u);
    CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
    float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
    double ops = (double)blocks * threads * ITERS * ops_per_thread_iter;
    printf("%-10s %8.3f ms  %8.2f Tlane-op/s  (%.3f of 39.3)\n", name, ms, ops / ms / 1e9, ops / ms / 1e9 / 39.32);
    fflush(stdout);
    return 0;
}

// Dependent issue: NCH independent chains per wave, each instruction of a chain needing the result of the
// one before it; W waves per SIMD.  Cycles (at the 2.4 GHz nominal clock) between two instructions of one
// wave tell how much independent work a SIMD needs in flight to issue every cycle it could.
template <int NCH, int OP>
__global__ void __launch_bounds__(256) k_dep(uint32_t* out, uint32_t seed)
{
    float f[NCH];
    uint32_t u[NCH];
    const float b = 1.0f + 1e-7f * (float)seed;
    const uint32_t m = 0xD2511F53u + seed;
#pragma unroll
    for (int c = 0; c < NCH; ++c) { f[c] = (float)(threadIdx.x + c) + 1.5f; u[c] = threadIdx.x * 2654435761u + c; }
#pragma unroll 1
    for (int it = 0; it < ITERS; ++it) {
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                if (OP == 0) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(f[c]) : "v"(b));
                else if (OP == 1) asm volatile("v_mul_hi_u32 %0, %0, %1" : "+v"(u[c]) : "v"(m));
                else if (OP == 2) asm volatile("v_log_f32 %0, %0" : "+v"(f[c]));
                else asm volatile("v_xor_b32 %0, %0, %1" : "+v"(u[c]) : "v"(m));
            }
    }
    float sf = 0.0f; uint32_t su = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) { sf += f[c]; su += u[c]; }
    if (sf == 12345.0f && su == 77u) out[0] = 1;
}
template <typename K> int run_dep(const char* name, K kern, int nch, int waves_per_simd, uint32_t* out)
{
    hipEvent_t e0, e1; CHK(hipEventCreate(&e0)); CHK(hipEventCreate(&e1));
    hipLaunchKernelGGL(kern, dim3(256 * waves_per_simd), dim3(256), 0, 0, out, 1u);
    CHK(hipDeviceSynchronize());
    CHK(hipEventRecord(e0));
    hipLaunchKernelGGL(kern, dim3(256 * waves_per_simd), dim3(256), 0, 0, out, 1u);
    CHK(hipEventRecord(e1)); CHK(hipEventSynchronize(e1));
    float ms; CHK(hipEventElapsedTime(&ms, e0, e1));
    const double instr_per_simd = (double)ITERS * 8 * nch * waves_per_simd;
    printf("dependent %-10s %d chain(s) x %d wave(s) per SIMD: %7.3f ms, %5.2f cycles (2.4 GHz) per instruction of the SIMD, %5.2f per step of a chain\n",
           name, nch, waves_per_simd, ms, ms * 1e-3 * 2.4e9 / instr_per_simd, ms * 1e-3 * 2.4e9 / ((double)ITERS * 8));
    fflush(stdout);
    return 0;
}
// Instruction fetch: 2048 independent 8-byte v_fma_f32 in a straight line (16 KB of code), walked
// three times by every wave; lane 0 of each wave notes the shader clock before and after each pass.
// The first pass of the first launch finds the code nowhere near the compute unit, the first pass of
// the second launch shows what a launch keeps of it, the later passes run from the instruction cache.
__global__ void __launch_bounds__(64) k_ifetch(unsigned long long* stamps, float seed)
{
    float a0 = seed + threadIdx.x, a1 = a0 + 1.0f, a2 = a0 + 2.0f, a3 = a0 + 3.0f, b = seed;
    unsigned long long t[4];
    t[0] = clock64();
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        asm volatile(".rept 512\n v_fma_f32 %0, %0, %4, %4\n v_fma_f32 %1, %1, %4, %4\n v_fma_f32 %2, %2, %4, %4\n"
                     " v_fma_f32 %3, %3, %4, %4\n .endr"
                     : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(b));
        asm volatile("s_nop 0" ::: "memory");
        t[pass + 1] = clock64();
    }
    if (threadIdx.x == 0)
        for (int k = 0; k < 4; ++k) stamps[(size_t)blockIdx.x * 4 + k] = t[k];
    if (a0 + a1 + a2 + a3 == 12345.0f) stamps[0] = 1;
}

static int run_ifetch()
{
    const int waves[2] = {256, 1024};                   // one wave per compute unit; one per SIMD
    for (int w : waves) {
        unsigned long long* st; CHK(hipMalloc(&st, (size_t)w * 4 * sizeof(unsigned long long)));
        unsigned long long* host = new unsigned long long[(size_t)w * 4];
        for (int launch = 0; launch < 3; ++launch) {
            hipLaunchKernelGGL(k_ifetch, dim3(w), dim3(64), 0, 0, st, 1.0f);
            CHK(hipDeviceSynchronize());
            CHK(hipMemcpy(host, st, (size_t)w * 4 * sizeof(unsigned long long), hipMemcpyDeviceToHost));
            double pass[3] = {0, 0, 0};
            for (int k = 0; k < w; ++k)
                for (int p = 0; p < 3; ++p) pass[p] += (double)(host[4 * k + p + 1] - host[4 * k + p]);
            printf("ifetch 16 KB straight line, %4d waves, launch %d: clock ticks per instruction, pass 1 / 2 / 3: %.2f / %.2f / %.2f\n",
                   w, launch + 1, pass[0] / w / 2048, pass[1] / w / 2048, pass[2] / w / 2048);
        }
        delete[] host;
        CHK(hipFree(st));
    }
    return 0;
}

int main() {
    if (run_ifetch()) return 1;
    uint32_t* out; CHK(hipMalloc(&out, 64));
    for (int w = 1; w <= 4; w *= 2) {
        run_dep("v_fma_f32", k_dep<1, 0>, 1, w, out); run_dep("v_fma_f32", k_dep<2, 0>, 2, w, out); run_dep("v_fma_f32", k_dep<4, 0>, 4, w, out);
        run_dep("v_mul_hi", k_dep<1, 1>, 1, w, out); run_dep("v_mul_hi", k_dep<2, 1>, 2, w, out);
        run_dep("v_log_f32", k_dep<1, 2>, 1, w, out); run_dep("v_log_f32", k_dep<2, 2>, 2, w, out);
        run_dep("v_xor_b32", k_dep<1, 3>, 1, w, out); run_dep("v_xor_b32", k_dep<2, 3>, 2, w, out);
    }
    hipDeviceProp_t p; CHK(hipGetDeviceProperties(&p, 0));
    printf("%s CUs=%d clock=%d kHz lds/block=%zu\n", p.name, p.multiProcessorCount, p.clockRate, p.sharedMemPerBlock);
    run("v_and", k_and, 8, out); run("v_add", k_add, 8, out); run("v_bcnt", k_bcnt, 8, out);
    run("v_mul_lo", k_mul_lo, 8, out); run("v_mul_hi", k_mul_hi, 8, out); run("v_mul24", k_mul24, 8, out);
    run("v_mad64", k_mad64, 8, out); run("v_mad64z+2", k_mad64z, 8, out);
    run("v_bitop3", k_bitop3, 8, out); run("v_cndmask", k_cndmask, 8, out); run("v_bfi", k_bfi, 8, out);
    run("v_fma", k_fma, 8, out); run("v_mul_f32", k_mulf, 8, out); run("v_med3", k_med3, 8, out);
    run("v_log", k_log, 8, out); run("v_sin", k_sin, 8, out); run("v_sqrt", k_sqrt, 8, out); run("v_rcp", k_rcp, 8, out);
    run("v_cvt", k_cvt, 8, out); run("v_lshr", k_lshr, 8, out); run("v_cmp", k_cmp, 8, out); run("v_addc", k_addc, 8, out);
    run("ds_write8", k_ldsw8, 8, out);
    run("v_bfm", k_bfm, 8, out); run("v_and_or", k_andor, 8, out); run("v_bfe_i32", k_bfei, 8, out);
    run("v_lshl_add", k_lshladd, 8, out); run("v_max3_u32", k_max3, 8, out); run("v_ashr", k_ashr, 8, out);
    run("v_xor", k_xor, 8, out); run("v_or", k_or, 8, out); run("v_sub", k_sub, 8, out); run("v_max_f32", k_maxf, 8, out);
    run("v_cmp_gt", k_cmpgt, 8, out); run("v_cnd_e64", k_cnd64, 8, out); run("v_alignbit", k_alignbit, 8, out);
    run("v_lshl_b64", k_lshl64, 8, out);
    run_mfma("mfma32x32x2 1ch 1wg/cu", k_mfma<1>, 1, 1, out);
    run_mfma("mfma32x32x2 1ch 4wg/cu", k_mfma<1>, 1, 4, out);
    run_mfma("mfma32x32x2 2ch 2wg/cu", k_mfma<2>, 2, 2, out);
    run_mfma("mfma32x32x2 4ch 1wg/cu", k_mfma<4>, 4, 1, out);
    run_mfma_bf16("mfma16x16x32bf16 1ch 1wg", k_mfma_bf16_16<1>, 1, 1, 16384.0, out);
    run_mfma_bf16("mfma16x16x32bf16 4ch 1wg", k_mfma_bf16_16<4>, 4, 1, 16384.0, out);
    run_mfma_bf16("mfma16x16x32bf16 16ch 1wg", k_mfma_bf16_16<16>, 16, 1, 16384.0, out);
    run_mfma_bf16("mfma16x16x32bf16 4ch 2wg", k_mfma_bf16_16<4>, 4, 2, 16384.0, out);
    run_mfma_bf16("mfma32x32x16bf16 1ch 1wg", k_mfma_bf16_32<1>, 1, 1, 32768.0, out);
    run_mfma_bf16("mfma32x32x16bf16 4ch 1wg", k_mfma_bf16_32<4>, 4, 1, 32768.0, out);
    run_mfma_bf16("mfma32x32x16bf16 4ch 2wg", k_mfma_bf16_32<4>, 4, 2, 32768.0, out);
    {
        uint4* gbuf; CHK(hipMalloc(&gbuf, 4096 * sizeof(uint4))); CHK(hipMemset(gbuf, 1, 4096 * sizeof(uint4)));
        for (int wg = 1; wg <= 2; ++wg) {
            run_mix(wg == 1 ? "16 mfma alone, 1 wave/SIMD" : "16 mfma alone, 2 waves/SIMD", k_mfma_mix<0>, wg, out, gbuf);
            run_mix(wg == 1 ? "16 mfma + 32 valu, 1 wave/SIMD" : "16 mfma + 32 valu, 2 waves/SIMD", k_mfma_mix<1>, wg, out, gbuf);
            run_mix(wg == 1 ? "16 mfma + 8 ds_read_b128, 1 wave" : "16 mfma + 8 ds_read_b128, 2 waves", k_mfma_mix<2>, wg, out, gbuf);
            run_mix(wg == 1 ? "16 mfma + 4 global x4, 1 wave" : "16 mfma + 4 global x4, 2 waves", k_mfma_mix<3>, wg, out, gbuf);
        }
        CHK(hipFree(gbuf));
    }
    // runs of eight 8-byte instructions after 2..5 s_nop from an 8-byte boundary: an even number
    // puts every instruction of the run on a multiple of 8, an odd number 4 bytes past one
    run("bitop3 +8", k_place_bitop3_2, 8, out); run("bitop3 +12", k_place_bitop3_3, 8, out);
    run("bitop3 +16", k_place_bitop3_4, 8, out); run("bitop3 +20", k_place_bitop3_5, 8, out);
    run("fma64 +8", k_place_fma_2, 8, out); run("fma64 +12", k_place_fma_3, 8, out);
    run("fma64 +16", k_place_fma_4, 8, out); run("fma64 +20", k_place_fma_5, 8, out);
    run("log+fma", k_logfma, 16, out); run("log+2fma", k_logfma2, 24, out); run("log+2and", k_logand2, 24, out);
    return 0;
}
