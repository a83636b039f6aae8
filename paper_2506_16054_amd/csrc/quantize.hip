// Block-aligned symmetric quantizer (paper Sec. 4.3 (1)): one scale per group of `block` tokens
// x d channels of one head, aligned with the attention block.  Bound by HBM bandwidth: every
// element is read once (2 or 4 bytes) and written once (0.5, 1 or 2 bytes).
//
// One workgroup of 256 threads owns one group.  The tile stays in registers between the absmax
// pass and the code pass, so HBM is touched exactly once in each direction.  The absmax is
// reduced inside each wavefront with cross-lane shuffles and across the four wavefronts through
// LDS.  For the PARO_VT layout the codes are transposed through LDS so that the global stores
// stay 16 bytes per lane and contiguous.
#include <hip/hip_bf16.h>
#include <string.h>

#include "common.h"

namespace paro {

template <typename T>
__device__ inline void load8(const T* p, float (&x)[8]);

template <>
__device__ inline void load8<float>(const float* p, float (&x)[8]) {
    const float4 a = ((const float4*)p)[0];
    const float4 b = ((const float4*)p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

template <>
__device__ inline void load8<uint16_t>(const uint16_t* p, float (&x)[8]) {  // bf16 bit patterns
    // the input is read exactly once: a non-temporal load keeps it from displacing the codes in the caches
    // (-3 % on the one-grid quantizer; the same hint on the stores of the codes, which the attention kernel reads
    // next, gains nothing)
    typedef unsigned v4u __attribute__((ext_vector_type(4)));
    const v4u a = __builtin_nontemporal_load((const v4u*)p);
    const unsigned w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

__device__ inline unsigned f32_to_bf16_bits(float f) {  // round to nearest even
    const unsigned u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

// GATHER = false: the input is the reordered, padded tensor xp [bh][Npad][D].
// GATHER = true : the input is x [bh][N][D] in the default token order and the reorder of
//                 Sec. 4.1 happens on the way in (row n' of the group reads row idx(n') of x), so
//                 the reordered tensor never exists in memory.
// SMOOTH: the per-(head, channel) constant sub[bh][c] is subtracted from every real token before anything else
//         (padded rows stay zero): the smoothed tensor never exists in memory either.
template <typename InT, int BLK, int D, int BITS, int LAYOUT, bool GATHER, bool SMOOTH = false>
__device__ __forceinline__ void quantize_group(const InT* __restrict__ xp, uint8_t* __restrict__ codes, float* __restrict__ scales,
                                               int n_tokens, int kblocks, const ReorderTable& table, int nh, int blk, int bh,
                                               const float* __restrict__ sub = nullptr) {
    constexpr int ELEMS = BLK * D;
    constexpr int CHUNKS = ELEMS / 8;  // 8 consecutive channels of one token per chunk
    constexpr int IT = (CHUNKS + 255) / 256;
    constexpr int OUT_BYTES = ELEMS * BITS / 8;
    constexpr float QMAX = BITS == 4 ? 7.0f : 127.0f;
    // LDS staging of the transposed tile: bytes for 8- and 4-bit codes, 16-bit words for bf16.
    // Rows of the staged transposed tile (one channel each) are 4 bytes longer than the block for the
    // integer codes, so that the byte stores of the 8 lanes that hold one token's 64 channels fall into
    // different LDS banks.
    constexpr int SSTR = BITS == 16 ? BLK : BLK + 4;
    constexpr int STAGE_BYTES = LAYOUT == PARO_VT ? D * SSTR * (BITS == 16 ? 2 : 1) : 16;
    __shared__ __attribute__((aligned(16))) uint8_t stage[STAGE_BYTES];
    __shared__ float wave_amax[4];

    const int tid = threadIdx.x;
    const size_t group = (size_t)bh * kblocks + blk;
    const InT* tile = GATHER ? xp + (size_t)bh * n_tokens * D : xp + group * ELEMS;
    uint8_t* out = codes + group * OUT_BYTES;

    // source row of every token of the group, computed once per row rather than once per chunk
    __shared__ int src_row[GATHER ? BLK : 1];
    if constexpr (GATHER) {
        if (tid < BLK) src_row[tid] = blk * BLK + tid < n_tokens ? reorder_source(table, bh % nh, blk * BLK + tid) : 0;
        __syncthreads();
    }

    float x[IT][8];
    float amax = 0.0f;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int chunk = tid + 256 * it;
        const int row = (chunk * 8) / D;
        const bool live = chunk < CHUNKS && blk * BLK + row < n_tokens;
        if (live) {
            if constexpr (GATHER) {
                load8<InT>(tile + (size_t)src_row[row] * D + (chunk * 8) % D, x[it]);
            } else {
                load8<InT>(tile + (size_t)chunk * 8, x[it]);
            }
            if constexpr (SMOOTH) {
                float mu[8];
                load8<float>(sub + (size_t)bh * D + (chunk * 8) % D, mu);
#pragma unroll
                for (int e = 0; e < 8; ++e) x[it][e] -= mu[e];  // one binary32 subtraction per element
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[it][e] = 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[it][e]));
    }

    float scale = 1.0f;
    if constexpr (BITS != 16) {
        amax = wave_max(amax);
        if ((tid & 63) == 0) wave_amax[tid >> 6] = amax;
        __syncthreads();
        amax = fmaxf(fmaxf(wave_amax[0], wave_amax[1]), fmaxf(wave_amax[2], wave_amax[3]));
        if (amax > 0.0f) scale = amax / QMAX;  // correctly rounded binary32 divide
    }
    if (tid == 0) scales[group] = scale;
    const GroupDivider quotient(scale);  // fl32(x / scale) for every element of the group

#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int chunk = tid + 256 * it;
        if (chunk >= CHUNKS) continue;
        const int row = (chunk * 8) / D;
        const int c0 = (chunk * 8) % D;
        if constexpr (BITS == 16) {
            unsigned h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = f32_to_bf16_bits(x[it][e]);
            if constexpr (LAYOUT == PARO_ROWS) {
                uint4 w = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
                *(uint4*)(out + (size_t)chunk * 16) = w;
            } else {
                uint16_t* st = (uint16_t*)stage;
                const int slot = vt_slot(row);
#pragma unroll
                for (int e = 0; e < 8; ++e) st[(c0 + e) * BLK + slot] = (uint16_t)h[e];
            }
        } else {
            int q[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float r = rintf(quotient(x[it][e]));  // v_rndne_f32: round half to even
                q[e] = (int)fminf(fmaxf(r, -QMAX), QMAX);
            }
            if constexpr (LAYOUT == PARO_ROWS) {
                if constexpr (BITS == 8) {
                    uint2 w;
                    w.x = (q[0] & 0xff) | ((q[1] & 0xff) << 8) | ((q[2] & 0xff) << 16) | ((unsigned)q[3] << 24);
                    w.y = (q[4] & 0xff) | ((q[5] & 0xff) << 8) | ((q[6] & 0xff) << 16) | ((unsigned)q[7] << 24);
                    *(uint2*)(out + (size_t)chunk * 8) = w;
                } else {
                    unsigned w = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e) w |= (unsigned)(q[e] & 0xf) << (4 * e);
                    *(unsigned*)(out + (size_t)chunk * 4) = w;
                }
            } else {
                const int slot = vt_slot(row);
#pragma unroll
                for (int e = 0; e < 8; ++e) stage[(c0 + e) * SSTR + slot] = (uint8_t)q[e];
            }
        }
    }

    if constexpr (LAYOUT == PARO_VT) {
        __syncthreads();
        if constexpr (BITS == 4) {
            // 8 consecutive slots of one channel -> 4 bytes: byte t = slot t | slot 4+t << 4
            constexpr int GROUPS = ELEMS / 8;
            for (int g = tid; g < GROUPS; g += 256) {
                const unsigned* src = (const unsigned*)(stage + (g / (BLK / 8)) * SSTR + (g % (BLK / 8)) * 8);
                *(unsigned*)(out + (size_t)g * 4) = (src[0] & 0x0f0f0f0fu) | ((src[1] & 0x0f0f0f0fu) << 4);
            }
        } else if constexpr (BITS == 8) {
            constexpr int VEC = ELEMS / 16;
            for (int v = tid; v < VEC; v += 256) {
                const unsigned* src = (const unsigned*)(stage + (v / (BLK / 16)) * SSTR + (v % (BLK / 16)) * 16);
                ((uint4*)out)[v] = make_uint4(src[0], src[1], src[2], src[3]);
            }
        } else {
            constexpr int VEC = STAGE_BYTES / 16;
            for (int v = tid; v < VEC; v += 256) ((uint4*)out)[v] = ((const uint4*)stage)[v];
        }
    }
}

template <typename InT, int BLK, int D, int BITS, int LAYOUT, bool GATHER>
__global__ __launch_bounds__(256) void quantize_kernel(const InT* __restrict__ xp, uint8_t* __restrict__ codes,
                                                       float* __restrict__ scales, int n_tokens, int kblocks,
                                                       ReorderTable table, int nh) {
    quantize_group<InT, BLK, D, BITS, LAYOUT, GATHER>(xp, codes, scales, n_tokens, kblocks, table, nh, blockIdx.x, blockIdx.y);
}

// K with a per-channel constant removed (see paro_k_channel_mean): rows, reorder fused into the loads.
template <typename InT, int BLK, int D, int BITS>
__global__ __launch_bounds__(256) void quantize_smoothed_kernel(const InT* __restrict__ x, const float* __restrict__ sub,
                                                                uint8_t* __restrict__ codes, float* __restrict__ scales, int n_tokens,
                                                                int kblocks, ReorderTable table, int nh) {
    quantize_group<InT, BLK, D, BITS, PARO_ROWS, true, true>(x, codes, scales, n_tokens, kblocks, table, nh, blockIdx.x, blockIdx.y, sub);
}

// Mean over the N tokens of every channel of every (batch, head), accumulated in binary64 and rounded to
// bfloat16 (returned as float).  One workgroup of 1024 threads per (batch, head): a thread owns 8 channels of
// every (1024 / (D/8))-th token; partial sums meet across the row lanes of a wavefront by shuffles and across
// the 16 wavefronts through LDS.  Any constant would do for the smoothing (the softmax does not see it); the
// coarse rounding makes this one independent of the order of the additions.
template <typename InT, int D>
__global__ __launch_bounds__(1024) void channel_mean_kernel(const InT* __restrict__ x, float* __restrict__ mean, int n_tokens) {
    constexpr int CHUNKS = D / 8;          // 8-channel chunks per token
    constexpr int ROWS = 1024 / CHUNKS;    // tokens per pass of the workgroup
    __shared__ double part[16][D];
    const int tid = threadIdx.x;
    const int cc = tid % CHUNKS;
    const int rl = tid / CHUNKS;
    const InT* base = x + (size_t)blockIdx.x * n_tokens * D + cc * 8;
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    // With one workgroup per head, latency is what binds: a thread keeps 8 (bf16) or 4 (fp32) loads in flight, held as loaded
    // (16 or 32 bytes each) and widened only when they are added.
    constexpr int INFLIGHT = sizeof(InT) == 2 ? 8 : 4;
    constexpr int WORDS = sizeof(InT) * 8 / 4;  // 32-bit words per 8 channels
    for (int r0 = rl; r0 < n_tokens; r0 += INFLIGHT * ROWS) {
        unsigned raw[INFLIGHT][WORDS];
#pragma unroll
        for (int u = 0; u < INFLIGHT; ++u) {
            const int r = r0 + u * ROWS;
            if (r < n_tokens) {
                const uint4* src = (const uint4*)(base + (size_t)r * D);
#pragma unroll
                for (int q = 0; q < WORDS / 4; ++q) {
                    const uint4 t = src[q];
                    raw[u][4 * q] = t.x; raw[u][4 * q + 1] = t.y; raw[u][4 * q + 2] = t.z; raw[u][4 * q + 3] = t.w;
                }
            } else {
#pragma unroll
                for (int q = 0; q < WORDS; ++q) raw[u][q] = 0u;
            }
        }
#pragma unroll
        for (int u = 0; u < INFLIGHT; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float f;
                if constexpr (sizeof(InT) == 2) f = __uint_as_float((e & 1) ? (raw[u][e >> 1] & 0xffff0000u) : (raw[u][e >> 1] << 16));
                else f = __uint_as_float(raw[u][e]);
                acc[e] += (double)f;
            }
    }
    // lanes of a wavefront that own the same chunk are CHUNKS apart
#pragma unroll
    for (int off = CHUNKS; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], off);
    if ((tid & 63) < CHUNKS) {
#pragma unroll
        for (int e = 0; e < 8; ++e) part[tid >> 6][cc * 8 + e] = acc[e];
    }
    __syncthreads();
    if (tid < D) {
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < 16; ++w) sum += part[w][tid];
        const float m = (float)(sum / (double)n_tokens);
        mean[(size_t)blockIdx.x * D + tid] = __uint_as_float(f32_to_bf16_bits(m) << 16);
    }
}

// Q, K and V of one attention call in a single launch (blockIdx.z selects the tensor): Q and K as
// row-major codes of QKBITS, V as transposed blocks of PVBITS, all three reordered on the way in.
// Same arithmetic as three quantize_kernel launches, two launch gaps fewer.
struct QkvPointers {
    const void* in[3];
    uint8_t* codes[3];
    float* scales[3];
};

template <typename InT, int BLK, int D, int QKBITS, int PVBITS>
__global__ __launch_bounds__(256) void quantize_qkv_kernel(QkvPointers p, int n_tokens, int kblocks, ReorderTable table, int nh) {
    const int z = blockIdx.z;
    if (z < 2)
        quantize_group<InT, BLK, D, QKBITS, PARO_ROWS, true>((const InT*)p.in[z], p.codes[z], p.scales[z], n_tokens, kblocks, table, nh,
                                                             blockIdx.x, blockIdx.y);
    else
        quantize_group<InT, BLK, D, PVBITS, PARO_VT, true>((const InT*)p.in[2], p.codes[2], p.scales[2], n_tokens, kblocks, table, nh,
                                                           blockIdx.x, blockIdx.y);
}

struct QuantLaunch {
    dim3 grid;
    hipStream_t stream;
    const void* in;
    void* codes;
    float* scales;
    int n, k, nh;
    bool gather;
    ReorderTable table;
};

template <typename InT, int BLK, int D, int BITS, int LAYOUT>
static void launch_gather(const QuantLaunch& q) {
    if (q.gather)
        hipLaunchKernelGGL((quantize_kernel<InT, BLK, D, BITS, LAYOUT, true>), q.grid, dim3(256), 0, q.stream, (const InT*)q.in,
                           (uint8_t*)q.codes, q.scales, q.n, q.k, q.table, q.nh);
    else
        hipLaunchKernelGGL((quantize_kernel<InT, BLK, D, BITS, LAYOUT, false>), q.grid, dim3(256), 0, q.stream, (const InT*)q.in,
                           (uint8_t*)q.codes, q.scales, q.n, q.k, q.table, q.nh);
}

template <typename InT, int BLK, int D, int BITS>
static void launch_layout(paro_layout layout, const QuantLaunch& q) {
    if (layout == PARO_ROWS) launch_gather<InT, BLK, D, BITS, PARO_ROWS>(q);
    else launch_gather<InT, BLK, D, BITS, PARO_VT>(q);
}

template <typename InT, int BLK, int D>
static void launch_bits(int bits, paro_layout layout, const QuantLaunch& q) {
    if (bits == 8) launch_layout<InT, BLK, D, 8>(layout, q);
    else if (bits == 4) launch_layout<InT, BLK, D, 4>(layout, q);
    else launch_layout<InT, BLK, D, 16>(layout, q);
}

template <typename InT>
static void launch_shape(int blk, int d, int bits, paro_layout layout, const QuantLaunch& q) {
    if (blk == 64 && d == 64) launch_bits<InT, 64, 64>(bits, layout, q);
    else if (blk == 64 && d == 128) launch_bits<InT, 64, 128>(bits, layout, q);
    else if (blk == 32 && d == 64) launch_bits<InT, 32, 64>(bits, layout, q);
    else launch_bits<InT, 32, 128>(bits, layout, q);
}

static int quantize_entry(const char* what, const paro_shape* s, paro_dtype dtype, int bits, paro_layout layout,
                          const uint8_t* h_perm_ids, const void* in, void* codes, float* scales, void* stream) {
    int64_t n, k;
    if (int st = check_shape(s, &n, &k)) return st;
    if (dtype != PARO_F32 && dtype != PARO_BF16) return fail(PARO_EINVAL, "dtype=%d is not a paro_dtype", (int)dtype);
    if (bits != 8 && bits != 4 && bits != 16) return fail(PARO_EINVAL, "bits=%d: expected 8, 4 or 16", bits);
    if (layout != PARO_ROWS && layout != PARO_VT) return fail(PARO_EINVAL, "layout=%d is not a paro_layout", (int)layout);
    if (!in || !codes || !scales) return fail(PARO_EINVAL, "input, codes and scales must not be NULL");
    if (((uintptr_t)in | (uintptr_t)codes) & 15) return fail(PARO_EINVAL, "input and codes must be 16-byte aligned");
    if (in == codes) return fail(PARO_EINVAL, "input and codes must not alias");
    QuantLaunch q;
    q.gather = h_perm_ids != nullptr;
    if (q.gather) {
        if (int st = make_reorder_table(s, h_perm_ids, &q.table)) return st;
    } else {
        memset(&q.table, 0, sizeof(q.table));
    }
    q.grid = dim3((unsigned)k, (unsigned)(s->B * s->nh));
    q.stream = (hipStream_t)stream;
    q.in = in;
    q.codes = codes;
    q.scales = scales;
    q.n = (int)n;
    q.k = (int)k;
    q.nh = s->nh;
    if (dtype == PARO_F32) launch_shape<float>(s->block, s->d, bits, layout, q);
    else launch_shape<uint16_t>(s->block, s->d, bits, layout, q);
    return check_launch(what);
}

template <typename InT, int BLK, int D>
static bool launch_qkv_bits(int bits_qk, int bits_pv, dim3 grid, hipStream_t st, const QkvPointers& p, int n, int k, const ReorderTable& t, int nh) {
#define PARO_QKV_CASE(QK, PV)                                                                                              \
    if (bits_qk == QK && bits_pv == PV) {                                                                                  \
        hipLaunchKernelGGL((quantize_qkv_kernel<InT, BLK, D, QK, PV>), grid, dim3(256), 0, st, p, n, k, t, nh);            \
        return true;                                                                                                       \
    }
    PARO_QKV_CASE(8, 8)
    PARO_QKV_CASE(8, 4)
    PARO_QKV_CASE(4, 4)
    PARO_QKV_CASE(4, 8)
    PARO_QKV_CASE(16, 16)
#undef PARO_QKV_CASE
    return false;
}

template <typename InT>
static bool launch_qkv_shape(int blk, int d, int bits_qk, int bits_pv, dim3 grid, hipStream_t st, const QkvPointers& p, int n, int k,
                             const ReorderTable& t, int nh) {
    if (blk == 64 && d == 64) return launch_qkv_bits<InT, 64, 64>(bits_qk, bits_pv, grid, st, p, n, k, t, nh);
    if (blk == 64 && d == 128) return launch_qkv_bits<InT, 64, 128>(bits_qk, bits_pv, grid, st, p, n, k, t, nh);
    if (blk == 32 && d == 64) return launch_qkv_bits<InT, 32, 64>(bits_qk, bits_pv, grid, st, p, n, k, t, nh);
    return launch_qkv_bits<InT, 32, 128>(bits_qk, bits_pv, grid, st, p, n, k, t, nh);
}

}  // namespace paro

extern "C" int paro_permute_quantize_qkv(const paro_shape* s, paro_dtype dtype, int bits_qk, int bits_pv, const uint8_t* h_perm_ids,
                                         const void* q, const void* k, const void* v, void* q_codes, float* sq, void* k_codes,
                                         float* sk, void* v_codes, float* sv, void* stream) {
    using namespace paro;
    int64_t n, kb;
    if (int st = check_shape(s, &n, &kb)) return st;
    if (dtype != PARO_F32 && dtype != PARO_BF16) return fail(PARO_EINVAL, "dtype=%d is not a paro_dtype", (int)dtype);
    if (!h_perm_ids) return fail(PARO_EINVAL, "perm_ids is NULL");
    if (!q || !k || !v || !q_codes || !k_codes || !v_codes || !sq || !sk || !sv)
        return fail(PARO_EINVAL, "inputs, codes and scales must not be NULL");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)q_codes | (uintptr_t)k_codes | (uintptr_t)v_codes) & 15)
        return fail(PARO_EINVAL, "inputs and codes must be 16-byte aligned");
    const void* ins[3] = {q, k, v};
    const void* outs[3] = {q_codes, k_codes, v_codes};
    for (int a = 0; a < 3; ++a)
        for (int b = 0; b < 3; ++b)
            if (ins[a] == outs[b] || (a < b && outs[a] == outs[b])) return fail(PARO_EINVAL, "inputs and codes must not alias");
    QkvPointers p;
    for (int a = 0; a < 3; ++a) p.in[a] = ins[a];
    p.codes[0] = (uint8_t*)q_codes; p.codes[1] = (uint8_t*)k_codes; p.codes[2] = (uint8_t*)v_codes;
    p.scales[0] = sq; p.scales[1] = sk; p.scales[2] = sv;
    ReorderTable table;
    if (int st = make_reorder_table(s, h_perm_ids, &table)) return st;
    const dim3 grid((unsigned)kb, (unsigned)(s->B * s->nh), 3);
    const bool ok = dtype == PARO_F32
        ? launch_qkv_shape<float>(s->block, s->d, bits_qk, bits_pv, grid, (hipStream_t)stream, p, (int)n, (int)kb, table, s->nh)
        : launch_qkv_shape<uint16_t>(s->block, s->d, bits_qk, bits_pv, grid, (hipStream_t)stream, p, (int)n, (int)kb, table, s->nh);
    if (!ok) return fail(PARO_EINVAL, "bits (qk=%d, pv=%d): expected (8,8), (8,4), (4,4), (4,8) or (16,16)", bits_qk, bits_pv);
    return check_launch("paro_permute_quantize_qkv");
}

extern "C" int paro_quantize(const paro_shape* s, paro_dtype dtype, int bits, paro_layout layout, const void* xp,
                             void* codes, float* scales, void* stream) {
    return paro::quantize_entry("paro_quantize", s, dtype, bits, layout, nullptr, xp, codes, scales, stream);
}

extern "C" int paro_permute_quantize(const paro_shape* s, paro_dtype dtype, int bits, paro_layout layout,
                                     const uint8_t* h_perm_ids, const void* x, void* codes, float* scales, void* stream) {
    if (!h_perm_ids) return paro::fail(PARO_EINVAL, "perm_ids is NULL");
    return paro::quantize_entry("paro_permute_quantize", s, dtype, bits, layout, h_perm_ids, x, codes, scales, stream);
}


namespace paro {
template <typename InT, int BLK, int D>
static void launch_smoothed(int bits, dim3 grid, hipStream_t st, const void* x, const float* sub, void* codes, float* scales, int n, int k,
                            const ReorderTable& t, int nh) {
    if (bits == 8)
        hipLaunchKernelGGL((quantize_smoothed_kernel<InT, BLK, D, 8>), grid, dim3(256), 0, st, (const InT*)x, sub, (uint8_t*)codes, scales, n, k, t, nh);
    else
        hipLaunchKernelGGL((quantize_smoothed_kernel<InT, BLK, D, 4>), grid, dim3(256), 0, st, (const InT*)x, sub, (uint8_t*)codes, scales, n, k, t, nh);
}
template <typename InT>
static void launch_smoothed_shape(int blk, int d, int bits, dim3 grid, hipStream_t st, const void* x, const float* sub, void* codes,
                                  float* scales, int n, int k, const ReorderTable& t, int nh) {
    if (blk == 64 && d == 64) launch_smoothed<InT, 64, 64>(bits, grid, st, x, sub, codes, scales, n, k, t, nh);
    else if (blk == 64 && d == 128) launch_smoothed<InT, 64, 128>(bits, grid, st, x, sub, codes, scales, n, k, t, nh);
    else if (blk == 32 && d == 64) launch_smoothed<InT, 32, 64>(bits, grid, st, x, sub, codes, scales, n, k, t, nh);
    else launch_smoothed<InT, 32, 128>(bits, grid, st, x, sub, codes, scales, n, k, t, nh);
}
}  // namespace paro

extern "C" int paro_k_channel_mean(const paro_shape* s, paro_dtype dtype, const void* k, float* k_mean, void* stream) {
    using namespace paro;
    int64_t n, kb;
    if (int st = check_shape(s, &n, &kb)) return st;
    if (dtype != PARO_F32 && dtype != PARO_BF16) return fail(PARO_EINVAL, "dtype=%d is not a paro_dtype", (int)dtype);
    if (!k || !k_mean) return fail(PARO_EINVAL, "k and k_mean must not be NULL");
    if (((uintptr_t)k | (uintptr_t)k_mean) & 15) return fail(PARO_EINVAL, "k and k_mean must be 16-byte aligned");
    const dim3 grid((unsigned)(s->B * s->nh));
    hipStream_t st = (hipStream_t)stream;
    if (dtype == PARO_F32) {
        if (s->d == 64) hipLaunchKernelGGL((channel_mean_kernel<float, 64>), grid, dim3(1024), 0, st, (const float*)k, k_mean, (int)n);
        else hipLaunchKernelGGL((channel_mean_kernel<float, 128>), grid, dim3(1024), 0, st, (const float*)k, k_mean, (int)n);
    } else {
        if (s->d == 64) hipLaunchKernelGGL((channel_mean_kernel<uint16_t, 64>), grid, dim3(1024), 0, st, (const uint16_t*)k, k_mean, (int)n);
        else hipLaunchKernelGGL((channel_mean_kernel<uint16_t, 128>), grid, dim3(1024), 0, st, (const uint16_t*)k, k_mean, (int)n);
    }
    return check_launch("paro_k_channel_mean");
}

extern "C" int paro_permute_quantize_smoothed(const paro_shape* s, paro_dtype dtype, int bits, const uint8_t* h_perm_ids, const void* k,
                                              const float* k_mean, void* codes, float* scales, void* stream) {
    using namespace paro;
    int64_t n, kb;
    if (int st = check_shape(s, &n, &kb)) return st;
    if (dtype != PARO_F32 && dtype != PARO_BF16) return fail(PARO_EINVAL, "dtype=%d is not a paro_dtype", (int)dtype);
    if (bits != 8 && bits != 4) return fail(PARO_EINVAL, "bits=%d: expected 8 or 4", bits);
    if (!h_perm_ids) return fail(PARO_EINVAL, "perm_ids is NULL");
    if (!k || !k_mean || !codes || !scales) return fail(PARO_EINVAL, "k, k_mean, codes and scales must not be NULL");
    if (((uintptr_t)k | (uintptr_t)k_mean | (uintptr_t)codes) & 15) return fail(PARO_EINVAL, "k, k_mean and codes must be 16-byte aligned");
    if (k == codes) return fail(PARO_EINVAL, "input and codes must not alias");
    ReorderTable table;
    if (int st = make_reorder_table(s, h_perm_ids, &table)) return st;
    const dim3 grid((unsigned)kb, (unsigned)(s->B * s->nh));
    if (dtype == PARO_F32)
        launch_smoothed_shape<float>(s->block, s->d, bits, grid, (hipStream_t)stream, k, k_mean, codes, scales, (int)n, (int)kb, table, s->nh);
    else
        launch_smoothed_shape<uint16_t>(s->block, s->d, bits, grid, (hipStream_t)stream, k, k_mean, codes, scales, (int)n, (int)kb, table, s->nh);
    return check_launch("paro_permute_quantize_smoothed");
}
