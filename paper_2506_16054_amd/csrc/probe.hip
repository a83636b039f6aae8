// Measurement aid: the matrix-instruction rate this GPU sustains, to put next to the published
// peak when the attention kernels' roofline fraction is reported.  Every wavefront issues
// `iters` rounds of four independent matrix instructions on register operands (no memory
// traffic), four wavefronts per SIMD on every compute unit.
#include "common.h"

namespace paro {

typedef int p_v4i __attribute__((ext_vector_type(4)));
typedef int p_v16i __attribute__((ext_vector_type(16)));
typedef __bf16 p_v8bf __attribute__((ext_vector_type(8)));
typedef float p_v16f __attribute__((ext_vector_type(16)));

constexpr int kProbeGroups = 1024;  // workgroups of 256 threads: 4096 wavefronts = 4 per SIMD on 256 CUs

template <int KIND>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int seed, int* __restrict__ out) {
    int result = 0;
    if constexpr (KIND == 0) {
        p_v4i a = {seed, 1, 2, 3}, b = {4, 5, 6, seed};
        p_v16i c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
        for (int i = 0; i < iters; ++i) {
            c0 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c3, 0, 0, 0);
        }
        for (int r = 0; r < 16; ++r) result += c0[r] + c1[r] + c2[r] + c3[r];
    } else {
        p_v8bf a, b;
        for (int r = 0; r < 8; ++r) {
            a[r] = (__bf16)(float)(seed + r);
            b[r] = (__bf16)(float)(r - seed);
        }
        p_v16f c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
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

}  // namespace paro

extern "C" int64_t paro_probe_mfma(int bits, int iters, int32_t* out, int64_t out_len, void* stream) {
    using namespace paro;
    if (bits != 8 && bits != 16) return fail(PARO_EINVAL, "bits=%d: 8 (INT8) or 16 (bf16)", bits);
    if (iters < 1 || iters > (1 << 20)) return fail(PARO_EINVAL, "iters=%d out of range [1, 2^20]", iters);
    if (!out || out_len < kProbeGroups * 4) return fail(PARO_EINVAL, "out must hold at least %d entries", kProbeGroups * 4);
    if (bits == 8)
        hipLaunchKernelGGL(probe_mfma_kernel<0>, dim3(kProbeGroups), dim3(256), 0, (hipStream_t)stream, iters, 1, out);
    else
        hipLaunchKernelGGL(probe_mfma_kernel<1>, dim3(kProbeGroups), dim3(256), 0, (hipStream_t)stream, iters, 1, out);
    if (int st = check_launch("paro_probe_mfma")) return st;
    const int64_t per_instr = bits == 8 ? 2LL * 32 * 32 * 32 : 2LL * 32 * 32 * 16;
    return (int64_t)kProbeGroups * 4 * iters * 4 * per_instr;
}
