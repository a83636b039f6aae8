// Measurement aids for bench.py (built into lib/libparo_probe.so, NOT into the product library):
//
//   paro_probe_mfma   the matrix-instruction rate this GPU sustains (register operands, no memory);
//   paro_probe_issue  what one wavefront instruction of a given kind costs a SIMD, in shader-clock
//                     cycles, with 1..4 wavefronts resident per SIMD, alone or next to a wavefront
//                     that issues matrix instructions back to back;
//   paro_probe_copy   the rate of a plain streaming copy (1:1 and 2:1 read:write), the yardstick of the
//                     path's bandwidth-bound kernels;
//   paro_probe_block  a register-only replica of the vector-ALU and matrix work of ONE live block of
//                     the INT8 attention kernel (no global memory, LDS or barrier), to tell issue
//                     cost from memory and synchronisation cost.
//
// Occupancy is set by the launch, without any call that changes a kernel's attributes: a workgroup of
// 256 threads puts one wavefront on each SIMD of its compute unit and asks for so much LDS (64, 48 or
// 36 KB of the unit's 160 KB) that exactly W = 2, 3 or 4 workgroups fit, and the grid holds W workgroups
// per unit, so all are resident at once with W wavefronts per SIMD.  The runs with a matrix companion
// use one workgroup of 1024 threads per unit (three timed wavefronts and one companion per SIMD; the
// kernel's register count keeps a second such workgroup out).  Every wavefront records the shader-clock
// cycles (s_memtime) and the constant 100 MHz ticks it took.  Instruction streams are written as
// inline assembly on independent registers so that exactly the named instruction is timed; the
// values computed are meaningless.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kErrInval = -1;
constexpr int kErrHip = -3;
char g_error[256] = "";  // text of the last failure (single-threaded measurement tool)

int hip_failed(const char* what, hipError_t e) {
    snprintf(g_error, sizeof(g_error), "%s: %s", what, hipGetErrorString(e));
    return kErrHip;
}
// LDS request that lets exactly w workgroups share a compute unit's 160 KB
constexpr int lds_for(int w) { return w == 2 ? 64 * 1024 : w == 3 ? 48 * 1024 : 36 * 1024; }
constexpr int kUnroll = 32;           // instructions of the timed kind per loop iteration

// ---- the matrix-rate probe --------------------------------------------------------------------
constexpr int kProbeGroups = 1024;  // workgroups of 256 threads: 4096 wavefronts = 4 per SIMD on 256 CUs

template <int KIND>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int seed, int* __restrict__ out) {
    int result = 0;
    if constexpr (KIND == 0) {
        v4i a = {seed, 1, 2, 3}, b = {4, 5, 6, seed};
        v16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
        }
        for (int r = 0; r < 16; ++r) result += c0[r] + c1[r] + c2[r] + c3[r];
    } else {
        v8bf a, b;
        for (int r = 0; r < 8; ++r) {
            a[r] = (__bf16)(float)(seed + r);
            b[r] = (__bf16)(float)(r - seed);
        }
        v16f c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
        }
        for (int r = 0; r < 16; ++r) result += (int)(c0[r] + c1[r] + c2[r] + c3[r]);
    }
    if ((threadIdx.x & 63) == 0) out[blockIdx.x * 4 + (threadIdx.x >> 6)] = result;
}

// ---- one instruction kind, W wavefronts per SIMD ---------------------------------------------
enum Kind {
    K_FMA_F32 = 0, K_ADD_F32, K_MUL_F32, K_MAX3_I32, K_CVT_PKNORM_U16, K_PERM_B32, K_EXP_F32, K_CVT_F32_I32,
    K_PK_FMA_F16, K_PK_ADD_F16, K_EXP_F16, K_FMA_MIXLO_F16, K_DOT2_F32_F16, K_CVT_PKRTZ_F16, K_MOV_DPP, K_PERMLANE32_SWAP,
    K_CNDMASK, K_ADD_U32, K_LSHL_OR, K_MFMA_I8_32, K_MFMA_I8_16, K_SOFTMAX_MIX,
    K_MFMA_WITH_ADD, K_MFMA_WITH_FMA, K_MFMA_WITH_EXP, K_MFMA_WITH_MIX, K_COUNT
};

const char* const kKindNames[K_COUNT] = {
    "v_fma_f32", "v_add_f32", "v_mul_f32", "v_max3_i32", "v_cvt_pknorm_u16_f32", "v_perm_b32", "v_exp_f32", "v_cvt_f32_i32",
    "v_pk_fma_f16", "v_pk_add_f16", "v_exp_f16", "v_fma_mixlo_f16", "v_dot2_f32_f16", "v_cvt_pkrtz_f16_f32", "v_mov_b32 dpp quad_perm",
    "v_permlane32_swap_b32", "v_cndmask_b32", "v_add_u32", "v_lshl_or_b32", "v_mfma_i32_32x32x32_i8", "v_mfma_i32_16x16x64_i8",
    "softmax mix (fma, exp, add, 1/2 cvt_pknorm, 1/4 perm, 1/2 max3)",
    "one wavefront: 4 x (v_mfma_i32_32x32x32_i8 + 12 v_add_f32), per 32 = 1/8 of that", "one wavefront: 4 x (mfma + 12 v_fma_f32), per 32",
    "one wavefront: 4 x (mfma + 4 v_exp_f32), per 32", "one wavefront: 4 x (mfma + 2 x (fma, exp, add) + max3), per 32"};

#define PROBE_REP8(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7)

// One loop iteration = kUnroll (32) instructions of the kind on 8 independent destination registers.
template <int KIND>
__device__ inline void issue_body(float (&f)[8], int (&n)[8], float a, float b, v16i (&acc)[4], v4i ma, v4i mb) {
#define FMA(i) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(f[i]) : "v"(a), "v"(b));
#define ADD(i) asm volatile("v_add_f32 %0, %0, %1" : "+v"(f[i]) : "v"(a));
#define MUL(i) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(f[i]) : "v"(a));
#define MAX3(i) asm volatile("v_max3_i32 %0, %0, %1, %2" : "+v"(n[i]) : "v"(n[(i + 1) & 7]), "v"(n[(i + 2) & 7]));
#define PKN(i) asm volatile("v_cvt_pknorm_u16_f32 %0, %1, %2" : "=v"(n[i]) : "v"(f[i]), "v"(f[(i + 1) & 7]));
#define PERM(i) asm volatile("v_perm_b32 %0, %0, %1, %2" : "+v"(n[i]) : "v"(n[(i + 1) & 7]), "v"(n[(i + 2) & 7]));
#define EXP(i) asm volatile("v_exp_f32 %0, %0" : "+v"(f[i]));
#define CVTI(i) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(f[i]) : "v"(n[i]));
#define PKFMA(i) asm volatile("v_pk_fma_f16 %0, %0, %1, %2" : "+v"(f[i]) : "v"(a), "v"(b));
#define PKADD(i) asm volatile("v_pk_add_f16 %0, %0, %1" : "+v"(f[i]) : "v"(a));
#define EXP16(i) asm volatile("v_exp_f16 %0, %0" : "+v"(f[i]));
#define MIXLO(i) asm volatile("v_fma_mixlo_f16 %0, %1, %2, %3" : "+v"(f[i]) : "v"(f[(i + 1) & 7]), "v"(a), "v"(b));
#define DOT2(i) asm volatile("v_dot2_f32_f16 %0, %1, %2, %0" : "+v"(f[i]) : "v"(a), "v"(b));
#define PKRTZ(i) asm volatile("v_cvt_pkrtz_f16_f32 %0, %1, %2" : "=v"(n[i]) : "v"(f[i]), "v"(f[(i + 1) & 7]));
#define DPP(i) asm volatile("v_mov_b32_dpp %0, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "+v"(n[i]) : "v"(n[(i + 1) & 7]));
#define SWAP(i) asm volatile("v_permlane32_swap_b32 %0, %1" : "+v"(n[i]), "+v"(n[(i + 1) & 7]));
#define CNDM(i) asm volatile("v_cndmask_b32 %0, %0, %1, vcc" : "+v"(n[i]) : "v"(n[(i + 1) & 7]) : "vcc");
#define ADDU(i) asm volatile("v_add_u32 %0, %0, %1" : "+v"(n[i]) : "v"(n[(i + 1) & 7]));
#define LSHLOR(i) asm volatile("v_lshl_or_b32 %0, %0, 8, %1" : "+v"(n[i]) : "v"(n[(i + 1) & 7]));
#define FOUR(M) PROBE_REP8(M) PROBE_REP8(M) PROBE_REP8(M) PROBE_REP8(M)
    if constexpr (KIND == K_FMA_F32) { FOUR(FMA) }
    else if constexpr (KIND == K_ADD_F32) { FOUR(ADD) }
    else if constexpr (KIND == K_MUL_F32) { FOUR(MUL) }
    else if constexpr (KIND == K_MAX3_I32) { FOUR(MAX3) }
    else if constexpr (KIND == K_CVT_PKNORM_U16) { FOUR(PKN) }
    else if constexpr (KIND == K_PERM_B32) { FOUR(PERM) }
    else if constexpr (KIND == K_EXP_F32) { FOUR(EXP) }
    else if constexpr (KIND == K_CVT_F32_I32) { FOUR(CVTI) }
    else if constexpr (KIND == K_PK_FMA_F16) { FOUR(PKFMA) }
    else if constexpr (KIND == K_PK_ADD_F16) { FOUR(PKADD) }
    else if constexpr (KIND == K_EXP_F16) { FOUR(EXP16) }
    else if constexpr (KIND == K_FMA_MIXLO_F16) { FOUR(MIXLO) }
    else if constexpr (KIND == K_DOT2_F32_F16) { FOUR(DOT2) }
    else if constexpr (KIND == K_CVT_PKRTZ_F16) { FOUR(PKRTZ) }
    else if constexpr (KIND == K_MOV_DPP) { FOUR(DPP) }
    else if constexpr (KIND == K_PERMLANE32_SWAP) { FOUR(SWAP) }
    else if constexpr (KIND == K_CNDMASK) { FOUR(CNDM) }
    else if constexpr (KIND == K_ADD_U32) { FOUR(ADDU) }
    else if constexpr (KIND == K_LSHL_OR) { FOUR(LSHLOR) }
    else if constexpr (KIND == K_MFMA_I8_32) {
        // 32 matrix instructions on four independent accumulators
#pragma unroll
        for (int r = 0; r < kUnroll; ++r) acc[r & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ma, mb, acc[r & 3], 0, 0, 0);
    } else if constexpr (KIND == K_MFMA_I8_16) {
        typedef int v4acc __attribute__((ext_vector_type(4)));
        v4acc c[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) c[r] = v4acc{acc[r][0], acc[r][1], acc[r][2], acc[r][3]};
#pragma unroll
        for (int r = 0; r < kUnroll; ++r) c[r & 3] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ma, mb, c[r & 3], 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) { acc[r][0] = c[r][0]; acc[r][1] = c[r][1]; acc[r][2] = c[r][2]; acc[r][3] = c[r][3]; }
    } else if constexpr (KIND == K_MFMA_WITH_ADD || KIND == K_MFMA_WITH_FMA || KIND == K_MFMA_WITH_EXP || KIND == K_MFMA_WITH_MIX) {
        // a wavefront's own matrix instructions among its own, independent vector instructions:
        // four groups of one matrix instruction (its own accumulator) and about 30 cycles of vector work
#define GROUP(r)                                                                                           \
        acc[r] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ma, mb, acc[r], 0, 0, 0);                               \
        if constexpr (KIND == K_MFMA_WITH_ADD) { PROBE_REP8(ADD) ADD(0) ADD(1) ADD(2) ADD(3) }                 \
        else if constexpr (KIND == K_MFMA_WITH_FMA) { PROBE_REP8(FMA) FMA(0) FMA(1) FMA(2) FMA(3) }            \
        else if constexpr (KIND == K_MFMA_WITH_EXP) { EXP(2 * r) EXP(2 * r + 1) EXP((2 * r + 4) & 7) EXP((2 * r + 5) & 7) } \
        else { FMA(2 * r) FMA(2 * r + 1) EXP(2 * r) EXP(2 * r + 1) ADD(2 * r) ADD(2 * r + 1) MAX3(r) }
        GROUP(0) GROUP(1) GROUP(2) GROUP(3)
#undef GROUP
    } else {
        // the per-logit sequence of the attention kernel, 8 logits per round, 32 instructions:
        // 8 x (fma, exp, add) + 4 cvt_pknorm + 2 perm + 2 max3  (the last two instructions pad to 32 with max3)
#define LOGIT(i) FMA(i) EXP(i) asm volatile("v_add_f32 %0, %0, %1" : "+v"(a) : "v"(f[i]));
        PROBE_REP8(LOGIT)
        PKN(0) PKN(2) PKN(4) PKN(6)
        PERM(0) PERM(4)
        MAX3(1) MAX3(5)
#undef LOGIT
    }
#undef FOUR
}

struct WaveTimes {
    long long cycles;  // s_memtime difference: shader-clock cycles
    long long ticks;   // constant 100 MHz counter difference
    long long start;   // s_memtime at the start of the timed loop
    long long where;   // HW_ID register (SIMD, compute unit, shader engine) | XCC_ID << 32
};

__device__ inline long long where_am_i() {
    const unsigned hw = __builtin_amdgcn_s_getreg(4 | (31 << 11));    // HW_REG_HW_ID, all 32 bits
    const unsigned xcc = __builtin_amdgcn_s_getreg(20 | (31 << 11));  // HW_REG_XCC_ID
    return (long long)hw | ((long long)xcc << 32);
}

// role of a wavefront in a launch with a matrix companion: with 4 W wavefronts per workgroup, wavefront w
// runs on SIMD w % 4; the wavefronts with w / 4 == W - 1 (one per SIMD) issue matrix instructions only
// and keep going until every timed wavefront of the workgroup has finished.
template <int KIND>
__global__ __launch_bounds__(1024) void issue_kernel(int iters, int with_mfma, WaveTimes* __restrict__ out, int* __restrict__ sink) {
    extern __shared__ int lds_flags[];
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    float f[8];
    int n[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        f[i] = 0.001f * (float)(lane + i) - 0.5f;
        n[i] = lane * 7 + i;
    }
    v16i acc[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[r][e] = 0;
    const v4i ma = {lane, 1, 2, 3}, mb = {4, 5, 6, lane};
    if (threadIdx.x == 0) lds_flags[0] = 0;
    __syncthreads();
    const bool companion = with_mfma && wave >= waves - 4;
    long long c0 = 0, c1 = 0, t0 = 0, t1 = 0;
    if (companion) {
        // matrix instructions until the timed wavefronts are done (they count themselves off in LDS);
        // the bound on the rounds makes the loop end whatever happens
        const int done_at = waves - 4;
        for (int round = 0; round < (1 << 22); ++round) {
            t1 = round + 1;  // rounds of 8 matrix instructions completed by this companion
#pragma unroll
            for (int r = 0; r < 8; ++r) acc[r & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ma, mb, acc[r & 3], 0, 0, 0);
            if (__hip_atomic_load(&lds_flags[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) >= done_at) break;
        }
    } else {
        c0 = __builtin_readcyclecounter();
        t0 = wall_clock64();
        for (int i = 0; i < iters; ++i) issue_body<KIND>(f, n, 1.0001f, 0.0003f, acc, ma, mb);
        c1 = __builtin_readcyclecounter();
        t1 = wall_clock64();
        if (lane == 0) __hip_atomic_fetch_add(&lds_flags[0], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    int keep = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) keep += n[i] + (int)f[i];
#pragma unroll
    for (int r = 0; r < 4; ++r) keep += acc[r][0] + acc[r][5];
    if (lane == 0) {
        out[blockIdx.x * waves + wave] = companion ? WaveTimes{0, t1, 0, where_am_i()} : WaveTimes{c1 - c0, t1 - t0, c0, where_am_i()};
        sink[blockIdx.x * waves + wave] = keep;
    }
}

// ---- replica of one live block of the INT8 attention kernel (d = 64, 32 queries x 64 keys per wavefront) ------
// Same instruction sequence per block as the product kernel's loop body minus everything that touches memory:
// 4 + 4 matrix instructions, the integer row maximum, the logit fma + exp2 + row sum, the code conversion and
// packing, and the accumulator update.  `parts` switches groups of it off to price them in place:
// bit 0 matrix instructions, bit 1 exp2, bit 2 conversion + packing, bit 3 row maximum, bit 4 accumulator update,
// bit 5 row sum.
template <int PARTS>
__global__ __launch_bounds__(1024) void block_kernel(int iters, WaveTimes* __restrict__ out, int* __restrict__ sink) {
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    // distinct, compiler-opaque operands per key tile / channel tile, so that no product or exponential of one
    // tile can be reused for the other
    v4i kf[2] = {{lane, 2, 3, 4}, {lane + 1, 5, 3, 4}}, qf = {5, 6, 7, lane}, vf[2] = {{lane, 9, 1, 2}, {lane + 3, 9, 7, 2}};
    asm volatile("" : "+v"(kf[0]), "+v"(kf[1]), "+v"(vf[0]), "+v"(vf[1]), "+v"(qf));
    v16i init;
#pragma unroll
    for (int r = 0; r < 16; ++r) init[r] = 0x4B400000;
    asm volatile("" : "+v"(init));
    float acc[2][16];
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[d][r] = 0.0f;
    float m = -1e30f, l = 0.0f;
    const float c = 3.0e-4f;
    const long long c0 = __builtin_readcyclecounter();
    const long long t0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        v16i s[2];
#pragma unroll
        for (int T = 0; T < 2; ++T) {
            s[T] = init;
            if constexpr (PARTS & 1) {
                s[T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[T], qf, s[T], 0, 0, 0);
                s[T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[1 - T], qf, s[T], 0, 0, 0);
            } else {
                s[T][0] += kf[T][0] + it;
                s[T][7] += kf[T][1] - it;
            }
        }
        int part[4] = {0, 0, 0, 0};
        if constexpr (PARTS & 8) {
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) part[r & 3] = max(part[r & 3], s[T][r]);
        } else {
            part[0] = s[0][0];
        }
        const int mx = max(max(part[0], part[1]), max(part[2], part[3]));
        const float ymax = c * (__int_as_float(mx) - 12582912.0f);
        m = fmaxf(m, ymax);
        const float off = -9.0f - m - c * 12582912.0f;
        // as in the product kernel: all exponentials first, the row sum as four chains, then the conversions
        float ev[2][16];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                ev[T][r] = fmaf(__int_as_float(s[T][r]), c, off);
                if constexpr (PARTS & 2) ev[T][r] = __builtin_amdgcn_exp2f(ev[T][r]);
            }
        float part_sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if constexpr (PARTS & 32) {
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) part_sum[r & 3] += ev[T][r];
        } else {
            part_sum[0] = ev[0][0];
        }
        const float rs = (part_sum[0] + part_sum[1]) + (part_sum[2] + part_sum[3]);
        v4i pf[2];
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                if constexpr (PARTS & 4) {
                    const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd], ev[T][4 * qd + 1]));
                    const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd + 2], ev[T][4 * qd + 3]));
                    pf[T][qd] = (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u);
                } else {
                    pf[T][qd] = __float_as_int(ev[T][4 * qd]) ^ __float_as_int(ev[T][4 * qd + 1]) ^ __float_as_int(ev[T][4 * qd + 2]) ^
                                __float_as_int(ev[T][4 * qd + 3]);
                }
            }
        l = fmaf(rs, 0.5f, l);
        const float w = 1.0f / (1.0f + l);
#pragma unroll
        for (int d = 0; d < 2; ++d) {
            v16i o = init;
            if constexpr (PARTS & 1) {
                o = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[d], pf[0], o, 0, 0, 0);
                o = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[1 - d], pf[1], o, 0, 0, 0);
            } else {
                o[0] += pf[0][d] ^ pf[1][d + 2];
                o[5] += pf[0][d + 2] ^ pf[1][d];
            }
#pragma unroll
            for (int r = 0; r < ((PARTS & 16) ? 16 : 1); ++r) acc[d][r] = fmaf(__int_as_float(o[r]) - 12582912.0f, w, acc[d][r]);
        }
        kf[0][1] ^= it;
        kf[1][2] += it;
    }
    const long long c1 = __builtin_readcyclecounter();
    const long long t1 = wall_clock64();
    float keep = l + m;
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) keep += acc[d][r];
    if (lane == 0) {
        out[blockIdx.x * waves + wave] = WaveTimes{c1 - c0, t1 - t0, c0, where_am_i()};
        sink[blockIdx.x * waves + wave] = (int)keep;
    }
}

// ---- two independent halves of a block per wavefront, matrix instructions of one half issued among the vector
// work of the other (MODE 1) or everything in program order (MODE 0) -----------------------------------------------
// One iteration = one 64-query x 64-key visit = two half-blocks of the replica above.  MODE 1 orders the work as
//   QK(0) | QK(1) among softmax(0) | PV(0) among softmax(1) | PV(1) among update(0) | update(1)
// and pins that order with scheduling barriers, to measure whether a wavefront's own matrix instructions run in
// the shadow of its own vector instructions.  MODE 2 additionally moves QK(0) of the next visit among update(1).
template <int MODE>
__global__ __launch_bounds__(256) void pair_kernel(int iters, WaveTimes* __restrict__ out, int* __restrict__ sink) {
    const int wave = threadIdx.x >> 6;
    const int waves = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    v4i kf[2] = {{lane, 2, 3, 4}, {lane + 1, 5, 3, 4}}, vf[2] = {{lane, 9, 1, 2}, {lane + 3, 9, 7, 2}};
    v4i qf[2] = {{5, 6, 7, lane}, {lane, 1, 7, 3}};
    asm volatile("" : "+v"(kf[0]), "+v"(kf[1]), "+v"(vf[0]), "+v"(vf[1]), "+v"(qf[0]), "+v"(qf[1]));
    v16i init;
#pragma unroll
    for (int r = 0; r < 16; ++r) init[r] = 0x4B400000;
    asm volatile("" : "+v"(init));
    float acc[2][2][16];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[h][d][r] = 0.0f;
    float m[2] = {-1e30f, -1e30f}, l[2] = {0.0f, 0.0f}, w[2] = {0.0f, 0.0f};
    const float c = 3.0e-4f;
    v16i s[2][2], o[2][2];
    v4i pf[2][2];

#define PAIR_QK(h)                                                                      \
    _Pragma("unroll") for (int T = 0; T < 2; ++T) {                                     \
        s[h][T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[T], qf[h], init, 0, 0, 0);    \
        s[h][T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[1 - T], qf[h], s[h][T], 0, 0, 0); \
    }
#define PAIR_PV(h)                                                                      \
    _Pragma("unroll") for (int d = 0; d < 2; ++d) {                                     \
        o[h][d] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[d], pf[h][0], init, 0, 0, 0); \
        o[h][d] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[1 - d], pf[h][1], o[h][d], 0, 0, 0); \
    }
#define PAIR_SOFTMAX(h)                                                                 \
    {                                                                                   \
        int part[4] = {0, 0, 0, 0};                                                     \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) part[r & 3] = max(part[r & 3], s[h][T][r]); \
        const int mx = max(max(part[0], part[1]), max(part[2], part[3]));               \
        const float ymax = c * (__int_as_float(mx) - 12582912.0f);                      \
        m[h] = fmaxf(m[h], ymax);                                                       \
        const float off = -9.0f - m[h] - c * 12582912.0f;                               \
        float ev[2][16];                                                                \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int r = 0; r < 16; ++r)                                  \
            ev[T][r] = __builtin_amdgcn_exp2f(fmaf(__int_as_float(s[h][T][r]), c, off)); \
        float part_sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};                                   \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) part_sum[r & 3] += ev[T][r];     \
        const float rs = (part_sum[0] + part_sum[1]) + (part_sum[2] + part_sum[3]);     \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int qd = 0; qd < 4; ++qd) {                              \
            const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd], ev[T][4 * qd + 1])); \
            const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd + 2], ev[T][4 * qd + 3])); \
            pf[h][T][qd] = (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u);             \
        }                                                                               \
        l[h] = fmaf(rs, 0.5f, l[h]);                                                    \
        w[h] = 1.0f / (1.0f + l[h]);                                                    \
    }
#define PAIR_UPDATE(h)                                                                  \
    _Pragma("unroll") for (int d = 0; d < 2; ++d)                                       \
    _Pragma("unroll") for (int r = 0; r < 16; ++r)                                      \
        acc[h][d][r] = fmaf(__int_as_float(o[h][d][r]) - 12582912.0f, w[h], acc[h][d][r]);
// the region since the last full barrier is scheduled as `groups` x (1 matrix instruction, `valu` vector instructions)
#define PAIR_INTERLEAVE(valu)                                                           \
    _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                     \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                              \
        __builtin_amdgcn_sched_group_barrier(0x002, valu, 0);                           \
    }
#define PAIR_FENCE() __builtin_amdgcn_sched_barrier(0)

// the same work in pieces, for MODE 3: one matrix instruction in front of each run of 8 x (logit fma, exp2)
#define PAIR_QK1(h, i)                                                                  \
    s[h][(i) >> 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[((i) >> 1) ^ ((i) & 1)], qf[h], ((i) & 1) ? s[h][(i) >> 1] : init, 0, 0, 0);
#define PAIR_PV1(h, i)                                                                  \
    o[h][(i) >> 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[((i) >> 1) ^ ((i) & 1)], pf[h][(i) & 1], ((i) & 1) ? o[h][(i) >> 1] : init, 0, 0, 0);
#define PAIR_SM_HEAD(h)                                                                 \
    {                                                                                   \
        int part[4] = {0, 0, 0, 0};                                                     \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) part[r & 3] = max(part[r & 3], s[h][T][r]); \
        const int mx = max(max(part[0], part[1]), max(part[2], part[3]));               \
        const float ymax = c * (__int_as_float(mx) - 12582912.0f);                      \
        m[h] = fmaxf(m[h], ymax);                                                       \
        off = -9.0f - m[h] - c * 12582912.0f;                                           \
    }
#define PAIR_SM_EXP(h, g)                                                               \
    _Pragma("unroll") for (int r = 0; r < 8; ++r)                                       \
        ev[(g) >> 1][8 * ((g) & 1) + r] = __builtin_amdgcn_exp2f(fmaf(__int_as_float(s[h][(g) >> 1][8 * ((g) & 1) + r]), c, off));
#define PAIR_SM_TAIL(h)                                                                 \
    {                                                                                   \
        float part_sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};                                   \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) part_sum[r & 3] += ev[T][r];     \
        const float rs = (part_sum[0] + part_sum[1]) + (part_sum[2] + part_sum[3]);     \
        _Pragma("unroll") for (int T = 0; T < 2; ++T)                                   \
        _Pragma("unroll") for (int qd = 0; qd < 4; ++qd) {                              \
            const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd], ev[T][4 * qd + 1])); \
            const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd + 2], ev[T][4 * qd + 3])); \
            pf[h][T][qd] = (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u);             \
        }                                                                               \
        l[h] = fmaf(rs, 0.5f, l[h]);                                                    \
        w[h] = 1.0f / (1.0f + l[h]);                                                    \
    }
// the logit fma and the exp2 of a run of 8 as separate pieces (MODE 5: the exponentials directly behind a matrix
// instruction, the next run's fma in front of the next matrix instruction)
#define PAIR_SM_FMA(h, g)                                                               \
    _Pragma("unroll") for (int r = 0; r < 8; ++r)                                       \
        ev[(g) >> 1][8 * ((g) & 1) + r] = fmaf(__int_as_float(s[h][(g) >> 1][8 * ((g) & 1) + r]), c, off);
#define PAIR_SM_EXPONLY(g)                                                              \
    _Pragma("unroll") for (int r = 0; r < 8; ++r)                                       \
        ev[(g) >> 1][8 * ((g) & 1) + r] = __builtin_amdgcn_exp2f(ev[(g) >> 1][8 * ((g) & 1) + r]);
// matrix instruction first, then the piece's vector instructions
#define PAIR_MFMA_FIRST()                                                               \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                  \
    __builtin_amdgcn_sched_group_barrier(0x002, 16, 0);                                 \
    PAIR_FENCE();
    float off = 0.0f;
    float ev[2][16];

    const long long c0 = __builtin_readcyclecounter();
    const long long t0 = wall_clock64();
    if constexpr (MODE == 2) { PAIR_QK(0) PAIR_FENCE(); }
    for (int it = 0; it < iters; ++it) {
        if constexpr (MODE == 5) {
            PAIR_QK(0) PAIR_FENCE();
            PAIR_SM_HEAD(0) PAIR_SM_FMA(0, 0) PAIR_FENCE();
            PAIR_QK1(1, 0) PAIR_FENCE(); PAIR_SM_EXPONLY(0) PAIR_SM_FMA(0, 1) PAIR_FENCE();
            PAIR_QK1(1, 1) PAIR_FENCE(); PAIR_SM_EXPONLY(1) PAIR_SM_FMA(0, 2) PAIR_FENCE();
            PAIR_QK1(1, 2) PAIR_FENCE(); PAIR_SM_EXPONLY(2) PAIR_SM_FMA(0, 3) PAIR_FENCE();
            PAIR_QK1(1, 3) PAIR_FENCE(); PAIR_SM_EXPONLY(3) PAIR_FENCE();
            PAIR_SM_TAIL(0) PAIR_FENCE();
            PAIR_SM_HEAD(1) PAIR_SM_FMA(1, 0) PAIR_FENCE();
            PAIR_PV1(0, 0) PAIR_FENCE(); PAIR_SM_EXPONLY(0) PAIR_SM_FMA(1, 1) PAIR_FENCE();
            PAIR_PV1(0, 1) PAIR_FENCE(); PAIR_SM_EXPONLY(1) PAIR_SM_FMA(1, 2) PAIR_FENCE();
            PAIR_PV1(0, 2) PAIR_FENCE(); PAIR_SM_EXPONLY(2) PAIR_SM_FMA(1, 3) PAIR_FENCE();
            PAIR_PV1(0, 3) PAIR_FENCE(); PAIR_SM_EXPONLY(3) PAIR_FENCE();
            PAIR_SM_TAIL(1) PAIR_FENCE();
            PAIR_UPDATE(0) PAIR_FENCE();
            PAIR_PV(1) PAIR_FENCE();
            PAIR_UPDATE(1) PAIR_FENCE();
        } else if constexpr (MODE == 3 || MODE == 4) {
            // MODE 4: the same pieces in the same order without the matrix instructions moved in (they run as two
            // groups of four in front of each softmax), as the reference for MODE 3
            PAIR_QK(0) PAIR_FENCE();
            if constexpr (MODE == 4) { PAIR_QK(1) PAIR_FENCE(); }
            PAIR_SM_HEAD(0) PAIR_FENCE();
            if constexpr (MODE == 3) {
                PAIR_QK1(1, 0) PAIR_SM_EXP(0, 0) PAIR_MFMA_FIRST() PAIR_QK1(1, 1) PAIR_SM_EXP(0, 1) PAIR_MFMA_FIRST()
                PAIR_QK1(1, 2) PAIR_SM_EXP(0, 2) PAIR_MFMA_FIRST() PAIR_QK1(1, 3) PAIR_SM_EXP(0, 3) PAIR_MFMA_FIRST()
            } else {
                PAIR_SM_EXP(0, 0) PAIR_FENCE(); PAIR_SM_EXP(0, 1) PAIR_FENCE(); PAIR_SM_EXP(0, 2) PAIR_FENCE(); PAIR_SM_EXP(0, 3) PAIR_FENCE();
            }
            PAIR_SM_TAIL(0) PAIR_FENCE();
            if constexpr (MODE == 4) { PAIR_PV(0) PAIR_FENCE(); }
            PAIR_SM_HEAD(1) PAIR_FENCE();
            if constexpr (MODE == 3) {
                PAIR_PV1(0, 0) PAIR_SM_EXP(1, 0) PAIR_MFMA_FIRST() PAIR_PV1(0, 1) PAIR_SM_EXP(1, 1) PAIR_MFMA_FIRST()
                PAIR_PV1(0, 2) PAIR_SM_EXP(1, 2) PAIR_MFMA_FIRST() PAIR_PV1(0, 3) PAIR_SM_EXP(1, 3) PAIR_MFMA_FIRST()
            } else {
                PAIR_SM_EXP(1, 0) PAIR_FENCE(); PAIR_SM_EXP(1, 1) PAIR_FENCE(); PAIR_SM_EXP(1, 2) PAIR_FENCE(); PAIR_SM_EXP(1, 3) PAIR_FENCE();
            }
            PAIR_SM_TAIL(1) PAIR_FENCE();
            PAIR_UPDATE(0) PAIR_FENCE();
            PAIR_PV(1) PAIR_FENCE();
            PAIR_UPDATE(1) PAIR_FENCE();
        } else if constexpr (MODE == 0) {
            PAIR_QK(0) PAIR_FENCE();
            PAIR_SOFTMAX(0) PAIR_FENCE();
            PAIR_PV(0) PAIR_FENCE();
            PAIR_UPDATE(0) PAIR_FENCE();
            PAIR_QK(1) PAIR_FENCE();
            PAIR_SOFTMAX(1) PAIR_FENCE();
            PAIR_PV(1) PAIR_FENCE();
            PAIR_UPDATE(1) PAIR_FENCE();
        } else {
            if constexpr (MODE == 1) { PAIR_QK(0) PAIR_FENCE(); }
            PAIR_QK(1) PAIR_SOFTMAX(0) PAIR_INTERLEAVE(48) PAIR_FENCE();
            PAIR_PV(0) PAIR_SOFTMAX(1) PAIR_INTERLEAVE(48) PAIR_FENCE();
            PAIR_PV(1) PAIR_UPDATE(0) PAIR_INTERLEAVE(16) PAIR_FENCE();
            if constexpr (MODE == 1) {
                PAIR_UPDATE(1) PAIR_FENCE();
            }
        }
        kf[0][1] ^= it;
        kf[1][2] += it;
        if constexpr (MODE == 2) {
            // QK(0) of the next visit among update(1) of this one (one visit too many at the end; its result is unused)
            PAIR_FENCE();
            PAIR_QK(0) PAIR_UPDATE(1) PAIR_INTERLEAVE(16) PAIR_FENCE();
        }
    }
    const long long c1 = __builtin_readcyclecounter();
    const long long t1 = wall_clock64();
    float keep = l[0] + m[0] + l[1] + m[1];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
            for (int r = 0; r < 16; ++r) keep += acc[h][d][r];
    if constexpr (MODE == 2) keep += (float)s[0][0][3];
    if (lane == 0) {
        out[blockIdx.x * waves + wave] = WaveTimes{c1 - c0, t1 - t0, c0, where_am_i()};
        sink[blockIdx.x * waves + wave] = (int)keep;
    }
#undef PAIR_QK
#undef PAIR_QK1
#undef PAIR_PV1
#undef PAIR_SM_HEAD
#undef PAIR_SM_EXP
#undef PAIR_SM_TAIL
#undef PAIR_SM_FMA
#undef PAIR_SM_EXPONLY
#undef PAIR_MFMA_FIRST
#undef PAIR_PV
#undef PAIR_SOFTMAX
#undef PAIR_UPDATE
#undef PAIR_INTERLEAVE
#undef PAIR_FENCE
}

// ---- plain streaming copy: what HBM sustains for the byte mix of the path's bandwidth-bound kernels --------------
// Every thread reads 16 bytes per step, grid-stride, and writes 16 bytes for every WRITE_EVERY-th read (1: a copy,
// 2: the quantizer's mix of two bytes read per byte written; the value written folds the reads in between).
template <int WRITE_EVERY>
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, long long n_read) {
    const long long stride = (long long)gridDim.x * blockDim.x * WRITE_EVERY;
    for (long long i = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * WRITE_EVERY; i + WRITE_EVERY <= n_read; i += stride) {
        uint4 v = src[i];
#pragma unroll
        for (int u = 1; u < WRITE_EVERY; ++u) {
            const uint4 t = src[i + u];
            v.x ^= t.x; v.y += t.y; v.z ^= t.z; v.w += t.w;
        }
        dst[i / WRITE_EVERY] = v;
    }
}

template <int KIND>
int launch_issue(int cus, int w, int iters, int with_mfma, WaveTimes* out, int* sink, hipStream_t st) {
    if (with_mfma)
        hipLaunchKernelGGL(issue_kernel<KIND>, dim3(cus), dim3(1024), lds_for(2), st, iters, 1, out, sink);
    else
        hipLaunchKernelGGL(issue_kernel<KIND>, dim3(cus * w), dim3(256), lds_for(w), st, iters, 0, out, sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? 0 : hip_failed("launch of issue_kernel", e);
}

template <int PARTS>
int launch_block(int cus, int w, int iters, WaveTimes* out, int* sink, hipStream_t st) {
    hipLaunchKernelGGL(block_kernel<PARTS>, dim3(cus * w), dim3(256), lds_for(w), st, iters, out, sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? 0 : hip_failed("launch of block_kernel", e);
}

template <int MODE>
int launch_pair(int cus, int iters, WaveTimes* out, int* sink, hipStream_t st) {
    hipLaunchKernelGGL(pair_kernel<MODE>, dim3(cus * 2), dim3(256), lds_for(2), st, iters, out, sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? 0 : hip_failed("launch of pair_kernel", e);
}

}  // namespace

extern "C" {

// Matrix-rate probe: `iters` rounds of four independent v_mfma_i32_32x32x32_i8 (bits 8) or
// v_mfma_f32_32x32x16_bf16 (bits 16) per wavefront, four wavefronts per SIMD on 256 compute units.
// Returns the number of operations performed (2 per multiply-add), or a negative status.
//   out  int32 [out_len] (device), out_len >= 4096
int64_t paro_probe_mfma(int bits, int iters, int32_t* out, int64_t out_len, void* stream) {
    if ((bits != 8 && bits != 16) || iters < 1 || iters > (1 << 20) || !out || out_len < kProbeGroups * 4) return kErrInval;
    if (bits == 8)
        hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(kProbeGroups), dim3(256), 0, (hipStream_t)stream, iters, 1, out);
    else
        hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(kProbeGroups), dim3(256), 0, (hipStream_t)stream, iters, 1, out);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return hip_failed("launch of probe_mfma_kernel", e);
    const int64_t per_instr = bits == 8 ? 2LL * 32 * 32 * 32 : 2LL * 32 * 32 * 16;
    return (int64_t)kProbeGroups * 4 * iters * 4 * per_instr;
}

// Streaming-copy probe: reads n_read 16-byte words of src and writes n_read / write_every of them to dst
// (write_every 1 or 2), `groups` workgroups of 256 threads.  Returns bytes moved (read + written) or a negative status.
//   src  [n_read * 16 bytes] (device);  dst  [n_read / write_every * 16 bytes] (device)
int64_t paro_probe_copy(const void* src, void* dst, int64_t n_read, int write_every, int groups, void* stream) {
    if (!src || !dst || n_read < 2 || (write_every != 1 && write_every != 2) || groups < 1 || groups > (1 << 20)) return kErrInval;
    if (write_every == 1)
        hipLaunchKernelGGL(copy_kernel<1>, dim3(groups), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, (long long)n_read);
    else
        hipLaunchKernelGGL(copy_kernel<2>, dim3(groups), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, (long long)n_read);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return hip_failed("launch of copy_kernel", e);
    const int64_t reads = n_read / write_every * write_every;
    return 16 * (reads + reads / write_every);
}

const char* paro_probe_last_error(void) { return g_error; }

int paro_probe_issue_kinds(void) { return K_COUNT; }

const char* paro_probe_issue_name(int kind) { return kind >= 0 && kind < K_COUNT ? kKindNames[kind] : ""; }

// Enqueues the stream of instruction `kind` with `waves_per_simd` (2..4) wavefronts per SIMD on `cus` compute
// units (pass the device's count).  with_mfma != 0: waves_per_simd must be 4; three wavefronts per SIMD are
// timed and the fourth is a companion that issues v_mfma_i32_32x32x32_i8 back to back for as long as they run.
// Every timed wavefront issues iters * 32 instructions and writes its elapsed {shader cycles, 100 MHz ticks}
// to times[workgroup * wavefronts per workgroup + wavefront]; a companion writes 0 cycles and, as its ticks, the
// number of rounds of 8 matrix instructions it got through meanwhile.
// Returns the number of entries of `times` written, or a negative status.
//   times  int64 [4 * entries] (device: cycles, ticks, start cycle, placement per wavefront);  sink  int32 [entries] (device, keeps the work alive)
int paro_probe_issue(int kind, int cus, int waves_per_simd, int iters, int with_mfma, int64_t* times, int32_t* sink, int64_t capacity, void* stream) {
    if (kind < 0 || kind >= K_COUNT || cus < 1 || cus > 4096 || waves_per_simd < 2 || waves_per_simd > 4 || iters < 1 || iters > (1 << 20) || !times || !sink)
        return kErrInval;
    if (with_mfma && waves_per_simd != 4) return kErrInval;
    const int entries = cus * 4 * waves_per_simd;
    if (capacity < entries) return kErrInval;
    hipStream_t st = (hipStream_t)stream;
    WaveTimes* out = (WaveTimes*)times;
    int rc = kErrInval;
    switch (kind) {
#define CASE(K) case K: rc = launch_issue<K>(cus, waves_per_simd, iters, with_mfma, out, sink, st); break;
        CASE(K_FMA_F32) CASE(K_ADD_F32) CASE(K_MUL_F32) CASE(K_MAX3_I32) CASE(K_CVT_PKNORM_U16) CASE(K_PERM_B32) CASE(K_EXP_F32)
        CASE(K_CVT_F32_I32) CASE(K_PK_FMA_F16) CASE(K_PK_ADD_F16) CASE(K_EXP_F16) CASE(K_FMA_MIXLO_F16) CASE(K_DOT2_F32_F16)
        CASE(K_CVT_PKRTZ_F16) CASE(K_MOV_DPP) CASE(K_PERMLANE32_SWAP) CASE(K_CNDMASK) CASE(K_ADD_U32) CASE(K_LSHL_OR)
        CASE(K_MFMA_I8_32) CASE(K_MFMA_I8_16) CASE(K_SOFTMAX_MIX)
        CASE(K_MFMA_WITH_ADD) CASE(K_MFMA_WITH_FMA) CASE(K_MFMA_WITH_EXP) CASE(K_MFMA_WITH_MIX)
#undef CASE
    }
    return rc < 0 ? rc : entries;
}

// Enqueues the register-only replica of one live block of the INT8 attention kernel (see block_kernel),
// `iters` blocks per wavefront, waves_per_simd (2..4) wavefronts per SIMD on `cus` compute units.
// parts: 63 = everything; clearing a bit leaves that group of instructions out (bit 0 the 8 matrix
// instructions, 1 the 32 exp2, 2 conversion + packing, 3 the row maximum, 4 the accumulator update, 5 the row sum).
// Supported values of parts: 63, 62, 61, 59, 55, 47, 31, 0.  Output as paro_probe_issue.
int paro_probe_block(int parts, int cus, int waves_per_simd, int iters, int64_t* times, int32_t* sink, int64_t capacity, void* stream) {
    if (cus < 1 || cus > 4096 || waves_per_simd < 2 || waves_per_simd > 4 || iters < 1 || iters > (1 << 20) || !times || !sink) return kErrInval;
    const int entries = cus * 4 * waves_per_simd;
    if (capacity < entries) return kErrInval;
    hipStream_t st = (hipStream_t)stream;
    WaveTimes* out = (WaveTimes*)times;
    int rc = kErrInval;
    switch (parts) {
#define CASE(P) case P: rc = launch_block<P>(cus, waves_per_simd, iters, out, sink, st); break;
        CASE(63) CASE(62) CASE(61) CASE(59) CASE(55) CASE(47) CASE(31) CASE(0)
#undef CASE
    }
    return rc < 0 ? rc : entries;
}

// Enqueues the two-halves replica (see pair_kernel) with two wavefronts per SIMD on `cus` compute units:
// mode 0 program order, 1 matrix instructions of one half among the vector work of the other, 2 as 1 plus the
// next visit's first products among the last update, 3 one matrix instruction in front of each run of 8 logit fma +
// 8 exp2, 4 the pieces of 3 with the matrix instructions not moved in, 5 as 3 with the exp2 directly behind the
// matrix instruction.  Every wavefront runs `iters` visits = 2 * iters half-blocks.
// Output as paro_probe_issue.
int paro_probe_pair(int mode, int cus, int iters, int64_t* times, int32_t* sink, int64_t capacity, void* stream) {
    if (mode < 0 || mode > 5 || cus < 1 || cus > 4096 || iters < 1 || iters > (1 << 20) || !times || !sink) return kErrInval;
    const int entries = cus * 4 * 2;
    if (capacity < entries) return kErrInval;
    hipStream_t st = (hipStream_t)stream;
    WaveTimes* out = (WaveTimes*)times;
    const int rc = mode == 0   ? launch_pair<0>(cus, iters, out, sink, st)
                   : mode == 1 ? launch_pair<1>(cus, iters, out, sink, st)
                   : mode == 2 ? launch_pair<2>(cus, iters, out, sink, st)
                   : mode == 3 ? launch_pair<3>(cus, iters, out, sink, st)
                   : mode == 4 ? launch_pair<4>(cus, iters, out, sink, st)
                               : launch_pair<5>(cus, iters, out, sink, st);
    return rc < 0 ? rc : entries;
}

}  // extern "C"
