// Block-sparse attention over the live blocks of a static per-head mask with INT8 QK^T and
// INT8 / INT4 PV under block-wise scales (paper Sec. 4.2 (2) and Sec. 4.3), for gfx950.
//
// Work split.  One workgroup owns one row block (BLK queries) of one head and walks that row's
// compacted live-block list in ascending order.  A wavefront owns 32 queries; BLK = 64 uses two
// wavefronts, BLK = 32 one.  Both products run on v_mfma_i32_32x32x32_i8 in the transposed
// orientation
//        S^T (keys x queries)   = K_j (A operand, from LDS)   x Q_i^T (B operand, registers)
//        O^T (channels x queries) = V_j^T (A operand, from LDS) x P^T   (B operand, registers)
// because the accumulator layout of a 32x32 result tile gives every lane 16 values of ONE
// query (keys 8q + 4g + p of the tile, q,p = 0..3, g = lane / 32): row reductions of the
// softmax are in-lane plus one cross-lane step, and the 16 quantized probabilities pack into
// exactly the four registers the next matrix instruction wants as its B operand.  The key
// order this imposes on the contraction is matched by the PARO_VT storage order of V, so V
// fragments are plain 16-byte LDS reads.
//
// Pipeline.  K_j and V_j^T tiles travel HBM/L2 -> registers -> LDS through a ring of two LDS
// stages, with the global loads issued two blocks ahead of the math and ONE workgroup barrier
// per live block; the barrier also carries the cross-wavefront exchange of the P-tile maximum
// (the P quantization group is the whole BLK x BLK tile).  Cross-lane reductions use DPP,
// v_permlane32_swap and scalar reads, never LDS.
//
// Arithmetic per live block (X in log2 units, c = sq_i * sk_j * log2(e) / sqrt(d)):
//   m' = max(m, c * rowmax S)  (the row maximum is taken on the integers, c > 0);  e = max over valid rows of (c * rowmax S - m')   (<= 0)
//   E  = qmaxP * 2^(c*S - m' - e)  in (0, qmaxP]  ->  Pc = round-half-even(E), two codes per
//        v_cvt_pknorm_u16_f32 (E is formed pre-divided by 65535), four codes packed by one v_perm_b32.
//        The exponent is ONE fma on the raw accumulator register: the register read as a float is B + S
//        (B = 1.5 * 2^23, see int_result), so c*S + off = c*(B + S) + (off - c*B); the offset off - c*B is
//        rounded to binary32 once per row and block, and that rounding (at most half an ulp of c*B, about
//        1e-4 relative in E) is computed exactly and returned to the block's weight, so the sums see the
//        scale the codes were really formed with,
//   l  = l * 2^(m - m') + sP * rowsum(E),  sP = 2^e / qmaxP   (the P tile maximum over qmaxP)
//   acc = acc * 2^(m - m') + (sP * sv_j) * float(Pc V_j)
// The two running sums are held divided by 2^(m' - m_ref), m_ref being the row's maximum after its
// first block: then the factor 2^(m - m') never has to be applied to them (the new term is
// multiplied by 2^(m' - m_ref) instead, one scalar per row), and since the output is acc / l the
// common factor cancels.  If a row's maximum climbs more than 64 octaves above its reference the
// sums are brought back to the current maximum (a rare, wavefront-uniform branch).
#include <string.h>

#include <type_traits>

#include "common.h"

namespace paro {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Measurement build only (lib/libparo_timeline.so, read by `python -m paper_2506_16054_amd.probe --timeline`; the
// product library is compiled without it): every wavefront of the two main integer kernels records the constant-rate
// clock when it starts and when it has stored its rows, and the number of column blocks it visited, at slot
// (launch item) x (wavefronts per workgroup) + wavefront.  paro_timeline_read copies the records to the host.
#ifndef PARO_TIMELINE
#define PARO_TIMELINE 0
#endif
#if PARO_TIMELINE
constexpr int kTimelineSlots = 1 << 16;
constexpr int kTimelineFields = 8;  // start, end (constant-rate clock), column blocks, shader cycles of phases 0..4
__device__ long long timeline_records[kTimelineSlots][kTimelineFields];
#define PARO_TIMELINE_BEGIN                                \
    const long long timeline_start = wall_clock64();       \
    long long timeline_last = clock64(), timeline_phase[5] = {0, 0, 0, 0, 0};
// closes phase i of the block loop (shader clock at issue, not at completion, of the instructions in front of it)
#define PARO_TIMELINE_PHASE(i)                             \
    {                                                      \
        const long long now_ = clock64();                  \
        timeline_phase[i] += now_ - timeline_last;         \
        timeline_last = now_;                              \
    }
#define PARO_TIMELINE_END(slot, lane, blocks)                                         \
    if ((lane) == 0 && (slot) < kTimelineSlots) {                                     \
        timeline_records[slot][0] = timeline_start;                                   \
        timeline_records[slot][1] = wall_clock64();                                   \
        timeline_records[slot][2] = (blocks);                                         \
        for (int f_ = 0; f_ < 5; ++f_) timeline_records[slot][3 + f_] = timeline_phase[f_]; \
    }
#else
#define PARO_TIMELINE_BEGIN
#define PARO_TIMELINE_PHASE(i)
#define PARO_TIMELINE_END(slot, lane, blocks)
#endif

struct AttnArgs {
    const uint8_t* q;
    const uint8_t* k;
    const uint8_t* v;
    const float* sq;
    const float* sk;
    const float* sv;
    const int* row_ptr;
    const int* col_idx;
    void* op;
    int nnz;
    int nh;
    int kblocks;
    int n_tokens;
    int total_wg;  // B * nh * kblocks
    int per_xcd;   // ceil(total_wg / 8)
    const int* row_order;  // optional [total_wg]: (b*nh + h)*k + i of the row block that runs at each launch position
    float qk_scale;  // log2(e) / sqrt(d)
    int scatter;     // 1: store row n' of the result at row idx(n') of o [B,nh,N,d] (Sec. 4.1 inverse reorder
                     //    done by adjusting the write-back address); 0: store op [B,nh,Npad,d]
    ReorderTable table;
};

// Where this lane's query row goes: element offset of the row in the output tensor, or -1 if the
// row is not stored (a padded row when the output is the unpadded, default-order tensor).
template <int D>
__device__ inline long long out_row_offset(const AttnArgs& a, int bh, int h, size_t head_rows, int row, bool row_valid) {
    if (!a.scatter) return (long long)((head_rows + row) * D);
    if (!row_valid) return -1;
    return (long long)(((size_t)bh * a.n_tokens + reorder_source(a.table, h, row)) * D);
}

__device__ inline unsigned bf16_rne(float f) {
    const unsigned u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ inline void store4(float* p, float a, float b, float c, float d) { *(float4*)p = make_float4(a, b, c, d); }
__device__ inline void store4(uint16_t* p, float a, float b, float c, float d) {
    *(uint2*)p = make_uint2(bf16_rne(a) | (bf16_rne(b) << 16), bf16_rne(c) | (bf16_rne(d) << 16));
}

// ---- cross-lane helpers (no LDS traffic) ---------------------------------------------------
template <int CTRL>
__device__ inline int dpp_mov(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}

// max over lanes n and n + 32 (the two lanes that share a query), returned in both
__device__ inline int xor32_max(int x) {
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return max((int)r[0], (int)r[1]);
}

// Minimum over the wavefront of unsigned values that are equal in lanes l and l + 32 (the two
// lanes of a query), as a wave-uniform value.  Rows of 16 lanes are reduced with DPP (xor 1, xor 2,
// half mirror, mirror); rows 0 and 1 then cover the wave and are combined through scalar registers.
// Used on the bit patterns of floats that are all <= 0 (or -inf): for those a larger value has the
// smaller bit pattern, so this is their maximum.
__device__ inline unsigned wave_umin(unsigned x) {
    x = min(x, (unsigned)dpp_mov<0xB1>((int)x));   // quad_perm [1,0,3,2]
    x = min(x, (unsigned)dpp_mov<0x4E>((int)x));   // quad_perm [2,3,0,1]
    x = min(x, (unsigned)dpp_mov<0x141>((int)x));  // row_half_mirror
    x = min(x, (unsigned)dpp_mov<0x140>((int)x));  // row_mirror
    const unsigned r0 = __builtin_amdgcn_readlane(x, 0), r1 = __builtin_amdgcn_readlane(x, 16);
    return min(r0, r1);
}

// Integer matrix results become floats without a convert instruction: every accumulator chain
// starts at the bit pattern of 1.5 * 2^23, so the register read as a float is 1.5 * 2^23 + result
// exactly (|result| <= 127*127*128 < 2^22) and one subtraction on the full-rate fp32 pipe
// recovers the result, bit-identical to v_cvt_f32_i32.
constexpr int kAccBiasI = 0x4B400000;
constexpr float kAccBiasF = 12582912.0f;
__device__ inline float int_result(int raw) { return __int_as_float(raw) - kAccBiasF; }

// The scale of a column block is the same for every lane and is written by the quantizer before this kernel
// starts: read through the constant address space it becomes a scalar load, needs no vector register while it is
// carried from one block to the next, and enters its one multiplication as a scalar operand.  Used by the kernel
// with four wavefronts per row block (-1.4 % there); the one-wavefront kernel measures the same either way and
// keeps its vector loads.
__device__ inline float uniform_load(const float* p) { return *(const __attribute__((address_space(4))) float*)(unsigned long long)p; }

// 1: with 8-bit P codes the accumulator bias of the logits is folded into the offset of the exponent's
// fma (one vector instruction per logit less); 0: the bias is always subtracted first and the exponent is
// exact to fp32 rounding.  With 4-bit P codes a code that flips at a rounding tie moves an output element
// by up to a seventh of its largest term, so that mode always keeps the exact exponent.
#ifndef PARO_FOLD_LOGIT_BIAS
#define PARO_FOLD_LOGIT_BIAS 1
#endif
#ifndef PARO_ATTN_WAVES_D64
#define PARO_ATTN_WAVES_D64 3  // wavefronts per SIMD the register allocation must allow, d = 64
#endif

// 16 bytes of packed 4-bit codes -> 32 signed bytes holding the codes times 16: a nibble moved to
// the top of its byte is the two's-complement code scaled by 16; the factor is undone in the
// scale.  Of every 8 codes the four even ones come first, then the four odd ones - a fixed
// permutation of the contraction index that Q and K (or P and V) share.
__device__ inline void unpack_nibbles(const v4i x, v4i& first, v4i& second) {
    const v4i lo = (x << 4) & (int)0xF0F0F0F0;
    const v4i hi = x & (int)0xF0F0F0F0;
    first = v4i{lo.x, hi.x, lo.y, hi.y};
    second = v4i{lo.z, hi.z, lo.w, hi.w};
}

// QSRC selects where this row block's Q operand comes from: 0 = codes and scale written by the
// quantizer; 1 (bf16) / 2 (fp32) = the unquantized Q tensor in the default token order, in which case
// the workgroup reorders and quantizes its own 64 x d block on the way in - the quantization group of
// Q is exactly the row block a workgroup owns (Sec. 4.3 (1)), so no other workgroup needs the result.
template <int BLK, int D, int QKBITS, int PVBITS, typename OutT, int QSRC = 0>
__global__ __launch_bounds__(BLK * 2, (D == 64 ? PARO_ATTN_WAVES_D64 : 2)) void attn_i8_kernel(AttnArgs a) {
    static_assert(QSRC == 0 || QKBITS == 8, "in-kernel quantization of Q produces 8-bit codes");
    constexpr int NW = BLK / 32;
    constexpr int NT = 64 * NW;
    constexpr int KSTR = D + 16;    // padded LDS row strides: rows 16 B apart in bank space
    constexpr int VSTR = BLK + 16;
    constexpr int KBYTES = BLK * KSTR;
    constexpr int VBYTES = D * VSTR;
    constexpr int STAGE = KBYTES + VBYTES;
    constexpr int VPACK = PVBITS == 4 ? 2 : 1;
    constexpr int KPACK = QKBITS == 4 ? 2 : 1;
    constexpr int NKC = BLK * D / KPACK / 16 / NT;  // 16-byte pieces of a K tile per thread
    constexpr int NVC = BLK * D / VPACK / 16 / NT;  // 16-byte pieces of a V tile per thread
    constexpr int KS = D / 32;    // contraction steps of QK^T
    constexpr int KT = BLK / 32;  // 32-key tiles per block
    constexpr int DT = D / 32;    // 32-channel tiles of the output
    constexpr float QMAXP = PVBITS == 4 ? 7.0f : 127.0f;
    constexpr float LOG2_QMAXP = PVBITS == 4 ? 2.807354922057604f : 6.988684686772166f;
    static_assert(NKC >= 1 && NVC >= 1, "tile too small for the workgroup");

    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE];
    __shared__ unsigned tile_e[2][NW];
    __shared__ float q_amax[NW];

    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of
    // (head, row block) so the K/V of the heads it works on stay in its own L2.
    const int wg = blockIdx.x;
    const int logical = (wg & 7) * a.per_xcd + (wg >> 3);
    if (logical >= a.total_wg) return;
    const int item = a.row_order ? min(max(a.row_order[logical], 0), a.total_wg - 1) : logical;
    const int bh = item / a.kblocks;
    const int i = item - bh * a.kblocks;
    const int h = bh % a.nh;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int n = lane & 31;
    const int g = lane >> 5;

    const int* rp = a.row_ptr + (size_t)h * (a.kblocks + 1) + i;
    // (the same for every lane: kept in scalar registers, so the loop control costs no vector work)
    const int beg = __builtin_amdgcn_readfirstlane(min(max(rp[0], 0), a.nnz));
    const int end = __builtin_amdgcn_readfirstlane(min(max(rp[1], beg), a.nnz));
    const int cnt = end - beg;
    const int* cols = a.col_idx + beg;
    // A row block that attends more than half of all column blocks (text rows of an image model,
    // Sec. 4.2 (1)) is on the critical path of the launch: its blocks are visited one after the other,
    // so its wavefronts get issue priority over the short rows they share a SIMD with.
    if (2 * cnt > a.kblocks) __builtin_amdgcn_s_setprio(2);

    const size_t head_rows = (size_t)bh * a.kblocks * BLK;
    const int row = i * BLK + 32 * w + n;  // this lane's query, in the reordered sequence
    const bool row_valid = row < a.n_tokens;
    const uint8_t* kbase = a.k + head_rows * D / KPACK;
    const uint8_t* vbase = a.v + head_rows * D / VPACK;
    const float* skp = a.sk + (size_t)bh * a.kblocks;
    const float* svp = a.sv + (size_t)bh * a.kblocks;
    v4i qf[KS];
    float sq_i = 0.0f;
    float x[QSRC != 0 ? KS : 1][16];  // this lane's slice of the unquantized row (QSRC != 0)
    if constexpr (QSRC != 0) {
        // ---- reorder + quantize this row block of Q here (same arithmetic as the quantizer:
        // absmax over real rows, scale = absmax / 127 in binary32, code = rint(fl32(x / scale))).
        // The loads are issued now; the reduction finishes behind the first K/V tile loads.
        using RawT = std::conditional_t<QSRC == 1, uint16_t, float>;
        const RawT* qsrc = (const RawT*)a.q + ((size_t)bh * a.n_tokens + (row_valid ? reorder_source(a.table, h, row) : 0)) * D + 16 * g;
        float amax = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            if (row_valid) {
                if constexpr (QSRC == 1) {
                    const uint4 lo = *(const uint4*)(qsrc + 32 * s), hi = *(const uint4*)(qsrc + 32 * s + 8);
                    const unsigned wv[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        x[s][2 * e] = __uint_as_float(wv[e] << 16);
                        x[s][2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float4 f = *(const float4*)(qsrc + 32 * s + 4 * e);
                        x[s][4 * e] = f.x;
                        x[s][4 * e + 1] = f.y;
                        x[s][4 * e + 2] = f.z;
                        x[s][4 * e + 3] = f.w;
                    }
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) x[s][e] = 0.0f;
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) amax = fmaxf(amax, fabsf(x[s][e]));
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
        if (lane == 0) q_amax[w] = amax;  // exchanged across the barrier that opens the block loop
    } else if constexpr (QKBITS == 4) {
        // 4-bit Q and K codes both enter the product times 16
        sq_i = a.sq[(size_t)bh * a.kblocks + i] * a.qk_scale * (1.0f / 256.0f);
        const uint8_t* qrow = a.q + ((head_rows + row) * D + 16 * g) / 2;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const uint2 x = *(const uint2*)(qrow + 16 * s);  // 16 codes of this lane's contraction slice
            v4i unused;
            unpack_nibbles(v4i{(int)x.x, (int)x.y, 0, 0}, qf[s], unused);
        }
    } else {
        sq_i = a.sq[(size_t)bh * a.kblocks + i] * a.qk_scale;
        const uint8_t* qrow = a.q + (head_rows + row) * D + 16 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *(const v4i*)(qrow + 32 * s);
    }

    // Column indices of the live list are fetched 64 at a time, one per lane, one chunk ahead;
    // the column of block t is then a lane read, not a memory access on the per-block path.
    auto load_cols = [&](int chunk) {
        const int idx = min(chunk * 64 + lane, cnt - 1);
        return cnt > 0 && chunk * 64 < cnt ? min(max(cols[idx], 0), a.kblocks - 1) : 0;
    };
    int cols_cur = load_cols(0), cols_nxt = load_cols(1);
    int cur_chunk = 0;
    auto col_of = [&](int t) {  // valid for t in chunk cur_chunk or cur_chunk + 1
        return (t >> 6) == cur_chunk ? __builtin_amdgcn_readlane(cols_cur, t & 63) : __builtin_amdgcn_readlane(cols_nxt, t & 63);
    };

    v4i kreg[NKC], vreg[NVC];
    int j_reg = 0;  // column block whose tiles sit in kreg / vreg (wave-uniform)
    auto gload = [&](int t) {
        const int j = col_of(t);
        j_reg = j;
        const uint8_t* kp = kbase + (size_t)j * (BLK * D / KPACK);
        const uint8_t* vp = vbase + (size_t)j * (BLK * D / VPACK);
#pragma unroll
        for (int c = 0; c < NKC; ++c) kreg[c] = *(const v4i*)(kp + 16 * (tid + NT * c));
#pragma unroll
        for (int c = 0; c < NVC; ++c) vreg[c] = *(const v4i*)(vp + 16 * (tid + NT * c));
    };
    // LDS store offsets of this thread's 16-byte pieces: piece c lies a whole number of rows below
    // piece 0, so one address per tile and stage serves all pieces through immediate offsets.
    constexpr int KROWB = D / KPACK, VROWB = BLK / VPACK;  // bytes of one stored row in global memory
    static_assert((16 * NT) % KROWB == 0 && (16 * NT) % VROWB == 0, "pieces must be whole rows apart");
    const int k_off = ((16 * tid) / KROWB) * KSTR + KPACK * ((16 * tid) % KROWB);
    const int v_off = KBYTES + ((16 * tid) / VROWB) * VSTR + VPACK * ((16 * tid) % VROWB);
    auto lstore_k = [&](int stage) {
        uint8_t* dst0 = lds + stage * STAGE + k_off;
#pragma unroll
        for (int c = 0; c < NKC; ++c) {
            uint8_t* dst = dst0 + c * (16 * NT / KROWB) * KSTR;
            if constexpr (QKBITS == 4) {  // 16 packed bytes = 32 channels of one key
                v4i first, second;
                unpack_nibbles(kreg[c], first, second);
                *(v4i*)dst = first;
                *(v4i*)(dst + 16) = second;
            } else {
                *(v4i*)dst = kreg[c];
            }
        }
    };
    auto lstore_v = [&](int stage) {
        uint8_t* dst0 = lds + stage * STAGE + v_off;
#pragma unroll
        for (int c = 0; c < NVC; ++c) {
            uint8_t* dst = dst0 + c * (16 * NT / VROWB) * VSTR;
            if constexpr (PVBITS == 4) {
                // 16 packed bytes = 32 slots of one channel (the PARO_VT nibble order makes the
                // unpacked bytes land in slot order)
                v4i first, second;
                unpack_nibbles(vreg[c], first, second);
                *(v4i*)dst = first;
                *(v4i*)(dst + 16) = second;
            } else {
                *(v4i*)dst = vreg[c];
            }
        }
    };

    float m = -INFINITY;  // running row maximum, log2 units
    float m_ref = -INFINITY;  // the maximum the stored sums are expressed against (set by the first block)
    constexpr float kLog2_65535 = 15.999977986052736f;
    float w_base = INFINITY;  // -log2(65535) - m_ref
    float l = 0.0f;       // this lane's share of the running denominator, divided by 65535 * 2^(m - m_ref)
    float acc[DT][16];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;

    // Start value of every integer accumulator chain, held in registers for the whole loop.
    v16i acc_init;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_init[r] = kAccBiasI;
    asm volatile("" : "+v"(acc_init));  // opaque to the optimizer: not re-created per block

    // LDS ring of two stages, one barrier per live block (placed after the row maxima):
    //   K_{t+1} is stored at the top of iteration t  - every wavefront finished reading K_{t-1}
    //                                                  before barrier t-1;
    //   V_{t+1} is stored right after barrier t      - every wavefront finished reading V_{t-1}
    //                                                  before it arrived at barrier t;
    //   the registers are refilled from global memory (block t+2) after both stores.
    // The scales of a block are fetched one block ahead of their use (behind the barrier of the block
    // before), straight into the registers the next iteration reads: its column index is carried in a
    // scalar register from the tile prefetch, so nothing per lane rotates from block to block.
    float sk_cur = 0.0f, sv_cur = 0.0f;  // scales of block t
    if (cnt > 0) {
        gload(0);
        lstore_k(0);
        lstore_v(0);
        sk_cur = skp[j_reg];
        sv_cur = svp[j_reg];
    }
    if (cnt > 1) gload(1);
    __syncthreads();
    if constexpr (QSRC != 0) {
        float amax = q_amax[0];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) amax = fmaxf(amax, q_amax[ww]);
        const float scale = amax > 0.0f ? amax / 127.0f : 1.0f;
        const GroupDivider quotient(scale);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                unsigned word = 0;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float r = fminf(fmaxf(rintf(quotient(x[s][4 * e4 + e])), -127.0f), 127.0f);
                    word |= ((unsigned)(int)r & 0xffu) << (8 * e);
                }
                qf[s][e4] = (int)word;
            }
        }
        sq_i = scale * a.qk_scale;
    }

    int stage = 0;
    // One live block.  TAIL selects the variant that masks keys past N (only the last column
    // block of a ragged sequence needs it; keeping it out of the common path saves two
    // instructions per logit).
    auto step = [&](auto tail_tag, auto fold_tag, int t) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        constexpr bool FOLD = decltype(fold_tag)::value;
        const int next = stage ^ 1;
        if (t + 1 < cnt) lstore_k(next);

        const float c = sq_i * sk_cur;
        const uint8_t* ks = lds + stage * STAGE;
        const uint8_t* vs = ks + KBYTES;

        // ---- S^T = K_j Q_i^T (i32, biased)
        v16i sacc[KT];
#pragma unroll
        for (int T = 0; T < KT; ++T) {
            sacc[T] = acc_init;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const v4i kf = *(const v4i*)(ks + (32 * T + n) * KSTR + 32 * s + 16 * g);
                sacc[T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf, qf[s], sacc[T], 0, 0, 0);
            }
        }
        // Raw accumulator value of a masked logit: it loses every maximum (real values carry the
        // accumulator bias); its exponential is forced to zero below.
        constexpr int kMaskedS = 0;
        if constexpr (TAIL) {  // keys past N never receive probability mass
            const int nkeys = a.n_tokens - (a.kblocks - 1) * BLK;
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * T + 8 * (r >> 2) + 4 * g + (r & 3) >= nkeys) sacc[T][r] = kMaskedS;
        }

        // ---- running maximum (on the raw integers: c > 0) and the tile's quantization scale
        int part[4] = {kMaskedS, kMaskedS, kMaskedS, kMaskedS};
#pragma unroll
        for (int T = 0; T < KT; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) part[r & 3] = max(part[r & 3], sacc[T][r]);
        const float ymax = c * int_result(xor32_max(max(max(part[0], part[1]), max(part[2], part[3]))));
        const float m_new = fmaxf(m, ymax);
        // e = log2 of the largest entry of the Pt tile = max over valid rows of (row maximum of
        // the block - running maximum), always <= 0; reduced as an unsigned minimum of bit patterns
        unsigned eb = wave_umin(row_valid ? __float_as_uint(ymax - m_new) : 0xFF800000u);
        if constexpr (NW > 1) {
            if (lane == 0) tile_e[t & 1][w] = eb;
        }
        __syncthreads();
        // scales of block t+1 (j_reg still names it: the prefetch of block t+2 comes below)
        // (behind the last block it names that block again: a harmless reload)
        const float sk_next = skp[j_reg], sv_next = svp[j_reg];
        if (t + 1 < cnt) lstore_v(next);
        if (((t + 2) & 63) == 0) {  // block t+2 opens a new chunk of 64 column indices
            cols_cur = cols_nxt;
            ++cur_chunk;
            cols_nxt = load_cols(cur_chunk + 1);
        }
        if (t + 2 < cnt) gload(t + 2);
        if constexpr (NW > 1) {
#pragma unroll
            for (int ww = 0; ww < NW; ++ww) eb = min(eb, tile_e[t & 1][ww]);
        }
        const float e = __uint_as_float(eb);
        // The first block of a row finds m_ref = -inf: growth = +inf takes the branch below, which
        // scales the (zero) sums by 2^-inf = 0 and makes the block's maximum the reference.
        const float growth = m_new - m_ref;
        if (__builtin_amdgcn_ballot_w64(growth > 64.0f) != 0) {  // keep the stored sums far from overflow
            const float down = __builtin_amdgcn_exp2f(-growth);
            l *= down;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[dt][r] *= down;
            m_ref = m_new;
            w_base = -kLog2_65535 - m_new;
        }
        m = m_new;

        // ---- E = qmaxP * 2^(X - m' - e); row sum; round half to even and pack as B operand
        float rs = 0.0f;
        v4i pf[KT];
        // E is formed divided by 65535, so that v_cvt_pknorm_u16_f32 (which rounds x * 65535 to the
        // nearest 16-bit integer, two values per instruction) yields the codes; one byte permute
        // packs four of them.  The row sum carries the same factor, undone once per row.
        // Exponent offset: X - m' - e + log2(qmaxP) - log2(65535): the tile maximum maps to qmaxP / 65535.
        const float off_n = (LOG2_QMAXP - kLog2_65535) - m_new - e;
        // weight of this block's terms in the stored sums, sP * 2^(m' - m_ref) = 2^(e + m' - m_ref - log2(qmaxP)),
        // written against the offset above: the part that depends on m_ref alone changes only with m_ref
        float off_f = off_n, w_blk;
        if constexpr (FOLD) {
            // c * (B + S) + off_f with off_f = fl(off_n - c*B).  c*B = cb_hi + cb_lo exactly (fma residual) and
            // off_n - cb_hi = off_f + terr exactly (two-sum), so E comes out as E_exact * 2^delta with
            // delta = cb_lo - terr known exactly; the block's weight takes the factor 2^-delta.
            const float cb_hi = c * kAccBiasF;
            const float cb_lo = fmaf(c, kAccBiasF, -cb_hi);
            off_f = off_n - cb_hi;
            const float bb = off_f - off_n;
            const float terr = (off_n - (off_f - bb)) + (-cb_hi - bb);
            w_blk = __builtin_amdgcn_exp2f((w_base - off_n) - (cb_lo - terr));
        } else {
            w_blk = __builtin_amdgcn_exp2f(w_base - off_n);
        }
        // All exponentials of the block first (in place of the raw logits), then the row sum as four independent
        // chains and the conversions: neighbouring instructions do not wait for each other's results.
        float ev[KT][16];
#pragma unroll
        for (int T = 0; T < KT; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                ev[T][r] = __builtin_amdgcn_exp2f(fmaf(FOLD ? __int_as_float(sacc[T][r]) : int_result(sacc[T][r]), c, off_f));
                if constexpr (TAIL) {
                    if (32 * T + 8 * (r >> 2) + 4 * g + (r & 3) >= a.n_tokens - (a.kblocks - 1) * BLK) ev[T][r] = 0.0f;
                }
            }
        float part_sum[4];
#pragma unroll
        for (int T = 0; T < KT; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) part_sum[r & 3] = (T == 0 && r < 4) ? ev[T][r] : part_sum[r & 3] + ev[T][r];
        rs = (part_sum[0] + part_sum[1]) + (part_sum[2] + part_sum[3]);
#pragma unroll
        for (int T = 0; T < KT; ++T)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                // (the builtin, not inline assembly: the instruction consumes results of the
                // transcendental unit, and only instructions the compiler can see get the wait state
                // that this needs when they follow the exponential directly)
                const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd], ev[T][4 * qd + 1]));
                const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd + 2], ev[T][4 * qd + 3]));
                pf[T][qd] = (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u);
            }
        l = fmaf(rs, w_blk, l);  // rs carries the factor 1/65535; it is undone once, at the end

        // ---- O^T += (sP sv_j 2^(m' - m_ref)) V_j^T P^T
        const float sv_eff = w_blk * sv_cur * (PVBITS == 4 ? 0.0625f : 1.0f);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            v16i o = acc_init;
#pragma unroll
            for (int T = 0; T < KT; ++T) {
                const v4i vf = *(const v4i*)(vs + (32 * dt + n) * VSTR + 32 * T + 16 * g);
                o = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf[T], o, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[dt][r] = fmaf(int_result(o[r]), sv_eff, acc[dt][r]);
        }
        sk_cur = sk_next;
        sv_cur = sv_next;
        stage = next;
    };

    // col_of(cnt - 1) is only addressable while its chunk is current, so the ragged-tail test
    // reads the list directly (once per workgroup).
    const bool has_tail = (a.n_tokens % BLK) != 0 && cnt > 0 && min(max(cols[cnt - 1], 0), a.kblocks - 1) == a.kblocks - 1;
    const int cnt_main = has_tail ? cnt - 1 : cnt;
    // The folded form of the exponent is taken where the logit scales of the row block's tiles keep the
    // rounding of its offset small: c * B < 2^13 for the largest K scale among the live column blocks, i.e.
    // at most 2^-12 in the exponent.  Row blocks whose inputs have an unusual magnitude take the exact
    // form.  The decision is the same in every lane of the workgroup (one row block, one list).
    constexpr bool FOLDABLE = PARO_FOLD_LOGIT_BIAS && PVBITS == 8;
    bool fold = false;
    if constexpr (FOLDABLE) {
        float sk_max = 0.0f;
        for (int base = 0; base < cnt; base += 64)
            if (base + lane < cnt) sk_max = fmaxf(sk_max, skp[min(max(cols[base + lane], 0), a.kblocks - 1)]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sk_max = fmaxf(sk_max, __shfl_xor(sk_max, off));
        fold = sq_i * sk_max * kAccBiasF < 8192.0f;
    }
    auto visit_all = [&](auto fold_tag) {
        for (int t = 0; t < cnt_main; ++t) step(std::false_type{}, fold_tag, t);
        if (has_tail) step(std::true_type{}, fold_tag, cnt - 1);
    };
    if (fold) visit_all(std::bool_constant<FOLDABLE>{});
    else visit_all(std::false_type{});

    // ---- finalize: divide by the denominator, store the row (zeros for padded rows)
    const float l_tot = (l + __shfl_xor(l, 32)) * 65535.0f;
    const float inv = (row_valid && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
    const long long ooff = out_row_offset<D>(a, bh, h, head_rows, row, row_valid);
    if (ooff >= 0) {
        OutT* orow = (OutT*)a.op + ooff + 4 * g;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                store4(orow + 32 * dt + 8 * qd, acc[dt][4 * qd] * inv, acc[dt][4 * qd + 1] * inv, acc[dt][4 * qd + 2] * inv,
                       acc[dt][4 * qd + 3] * inv);
    }
}

// -------------------------------------------------------------------------------------------
// d = 64, block 64, 8-bit Q and K codes (P and V 8-bit or 4-bit): ONE wavefront per row block, no barrier.
//
// The wavefront owns all 64 queries of the row block as two halves of 32 (H = 0, 1; a lane holds query
// n of each half).  The P quantization group - the whole 64 x 64 tile - then lives in one wavefront: its
// maximum is an in-wave reduction, nothing is exchanged between wavefronts and nothing has to be
// synchronised.  K_j and V_j^T travel from global memory (L2) straight into LDS with
// global_load_lds_dwordx4, which bypasses the vector registers: every lane fetches exactly the 16-byte
// fragments the matrix instructions will take from it as A operand (K rows and PARO_VT rows are 64 bytes;
// a lane pair reads 32 contiguous bytes), so a tile arrives in LDS as eight 1 KB fragments in lane order
// and is read back with conflict-free 16-byte LDS reads just before use.  The LDS is a private two-slot
// ring per wavefront: block t+1 is requested at the top of block t and has all of block t to arrive; the
// only wait is one vmcnt(0) per block.  Each fragment feeds two matrix instructions (one per half).
// Per block and half the arithmetic is that of attn_i8_kernel.
// -------------------------------------------------------------------------------------------
#ifndef PARO_ATTN_SINGLE_WAVE
#define PARO_ATTN_SINGLE_WAVE 1
#endif

// Lane L's 16 bytes at base + lane_off + OFFSET land at lds_dst + 16 L (lds_dst wave-uniform, lds_dst >= OFFSET
// bytes into its array).  The instruction's immediate offset moves the global AND the LDS address, so the LDS
// base is handed over OFFSET bytes low; the four or two requests of a tile then share one address register pair
// instead of costing a per-lane 64-bit addition each.
template <int OFFSET>
__device__ inline void lds_dma16(const uint8_t* base, unsigned lane_off, uint8_t* lds_dst) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + lane_off),
                                     (__attribute__((address_space(3))) void*)(lds_dst - OFFSET), 16, OFFSET, 0);
}

// QSRC as in attn_i8_kernel: 0 = Q codes and scale from the quantizer; 1 (bf16) / 2 (fp32) = the unquantized Q in the
// default token order, reordered and quantized here - the quantization group is the row block this wavefront owns,
// so its absmax is one in-wave reduction.
// QKBITS 4: Q and K rows are 32 bytes of packed 4-bit codes; a lane fetches the 16 bytes that hold its 32 channels
// (32 g .. 32 g + 31) of a K row - one fragment per key tile instead of two - and widens them to two 16-byte operands
// (codes times 16, undone in the scale) right after the LDS read; Q is widened the same way once.
template <int QKBITS, int PVBITS, typename OutT, int QSRC>
__device__ __forceinline__ void attn_i8_w64_body(const AttnArgs& a) {
    static_assert(QSRC == 0 || QKBITS == 8, "in-kernel quantization of Q produces 8-bit codes");
    constexpr int BLK = 64, D = 64;
    constexpr int KPACK = QKBITS == 4 ? 2 : 1;
    constexpr int VPACK = PVBITS == 4 ? 2 : 1;
    constexpr float LOG2_QMAXP = PVBITS == 4 ? 2.807354922057604f : 6.988684686772166f;
    constexpr float kLog2_65535 = 15.999977986052736f;
    // [slot][fragment][16 B per lane]; fragments 0-3: K (T,s) - with 4-bit K only 0-1: (T); 4-7: V^T (dt,T) - with 4-bit V only 4-5: (dt), where
    // lane (n, g) holds bytes 16g .. 16g+15 of packed channel row 32 dt + n, i.e. the 32 slots of key tile g
    __shared__ __attribute__((aligned(16))) uint8_t ring[2][8][1024];

    const int wg = blockIdx.x;
    const int logical = (wg & 7) * a.per_xcd + (wg >> 3);
    if (logical >= a.total_wg) return;
    const int item = a.row_order ? min(max(a.row_order[logical], 0), a.total_wg - 1) : logical;
    const int bh = item / a.kblocks;
    const int i = item - bh * a.kblocks;
    const int h = bh % a.nh;
    const int lane = threadIdx.x;
    const int n = lane & 31;
    const int g = lane >> 5;
    PARO_TIMELINE_BEGIN

    const int* rp = a.row_ptr + (size_t)h * (a.kblocks + 1) + i;
    const int beg = __builtin_amdgcn_readfirstlane(min(max(rp[0], 0), a.nnz));
    const int end = __builtin_amdgcn_readfirstlane(min(max(rp[1], beg), a.nnz));
    const int cnt = end - beg;
    const int* cols = a.col_idx + beg;
    if (2 * cnt > a.kblocks) __builtin_amdgcn_s_setprio(2);

    const size_t head_rows = (size_t)bh * a.kblocks * BLK;
    const uint8_t* kbase = a.k + head_rows * D / KPACK;  // the head's K codes (wave-uniform)
    const uint8_t* vbase = a.v + head_rows * D / VPACK;  // the head's V^T codes (wave-uniform)
    const unsigned klane = n * (D / KPACK) + 16 * g;     // this lane's K fragment of key tile 0, step 0, inside a block
    const unsigned vlane = n * (BLK / VPACK) + 16 * g;   // this lane's V^T piece of channel tile 0, inside a block
    const float* skp = a.sk + (size_t)bh * a.kblocks;
    const float* svp = a.sv + (size_t)bh * a.kblocks;
    float sq_i;
    int row[2];
    bool row_valid[2];
    unsigned invalid_row[2];
    v4i qf[2][2];  // [half][contraction step]
#pragma unroll
    for (int H = 0; H < 2; ++H) {
        row[H] = i * BLK + 32 * H + n;
        row_valid[H] = row[H] < a.n_tokens;
        // or-ed into the bit pattern of a value <= 0 it gives a pattern at or above that of -inf: larger, as an
        // unsigned number, than the pattern of every value a real row can have
        invalid_row[H] = row_valid[H] ? 0u : 0xFF800000u;
    }
    if constexpr (QSRC == 0 && QKBITS == 4) {
        sq_i = a.sq[(size_t)bh * a.kblocks + i] * a.qk_scale * (1.0f / 256.0f);  // Q and K codes both enter times 16
#pragma unroll
        for (int H = 0; H < 2; ++H) unpack_nibbles(*(const v4i*)(a.q + (head_rows + row[H]) * (D / 2) + 16 * g), qf[H][0], qf[H][1]);
    } else if constexpr (QSRC == 0) {
        sq_i = a.sq[(size_t)bh * a.kblocks + i] * a.qk_scale;
#pragma unroll
        for (int H = 0; H < 2; ++H) {
            const uint8_t* qrow = a.q + (head_rows + row[H]) * D + 16 * g;
#pragma unroll
            for (int s = 0; s < 2; ++s) qf[H][s] = *(const v4i*)(qrow + 32 * s);
        }
    } else {
        // same arithmetic as the quantizer: absmax over the real rows of the block, scale = absmax / 127 in
        // binary32, code = rint(fl32(x / scale))
        using RawT = std::conditional_t<QSRC == 1, uint16_t, float>;
        float x[2][2][16];  // this lane's slices of its two unquantized rows
        float amax = 0.0f;
#pragma unroll
        for (int H = 0; H < 2; ++H) {
            const RawT* qsrc = (const RawT*)a.q + ((size_t)bh * a.n_tokens + (row_valid[H] ? reorder_source(a.table, h, row[H]) : 0)) * D + 16 * g;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                if (row_valid[H]) {
                    if constexpr (QSRC == 1) {
                        const uint4 lo = *(const uint4*)(qsrc + 32 * s), hi = *(const uint4*)(qsrc + 32 * s + 8);
                        const unsigned wv[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            x[H][s][2 * e] = __uint_as_float(wv[e] << 16);
                            x[H][s][2 * e + 1] = __uint_as_float(wv[e] & 0xffff0000u);
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float4 f = *(const float4*)(qsrc + 32 * s + 4 * e);
                            x[H][s][4 * e] = f.x;
                            x[H][s][4 * e + 1] = f.y;
                            x[H][s][4 * e + 2] = f.z;
                            x[H][s][4 * e + 3] = f.w;
                        }
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 16; ++e) x[H][s][e] = 0.0f;
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) amax = fmaxf(amax, fabsf(x[H][s][e]));
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
        const float scale = amax > 0.0f ? amax / 127.0f : 1.0f;
        const GroupDivider quotient(scale);
#pragma unroll
        for (int H = 0; H < 2; ++H)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    unsigned word = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float r = fminf(fmaxf(rintf(quotient(x[H][s][4 * e4 + e])), -127.0f), 127.0f);
                        word |= ((unsigned)(int)r & 0xffu) << (8 * e);
                    }
                    qf[H][s][e4] = (int)word;
                }
        sq_i = scale * a.qk_scale;
    }

    // column indices: 64 per fetch, one per lane, one chunk ahead
    auto load_cols = [&](int chunk) {
        const int idx = min(chunk * 64 + lane, cnt - 1);
        return cnt > 0 && chunk * 64 < cnt ? min(max(cols[idx], 0), a.kblocks - 1) : 0;
    };
    int cols_cur = load_cols(0), cols_nxt = load_cols(1);
    int cur_chunk = 0;  // chunk held by cols_cur

    // request the tiles of column block j into ring slot `slot`
    auto request = [&](int j, int slot) {
        const uint8_t* kp = kbase + (size_t)j * (BLK * D / KPACK);  // j comes from a scalar register: kp, vp are wave-uniform
        const uint8_t* vp = vbase + (size_t)j * (BLK * D / VPACK);
        if constexpr (QKBITS == 4) {
            lds_dma16<0>(kp, klane, &ring[slot][0][0]);
            lds_dma16<32 * D / 2>(kp, klane, &ring[slot][1][0]);
        } else {
            lds_dma16<0>(kp, klane, &ring[slot][0][0]);
            lds_dma16<32>(kp, klane, &ring[slot][1][0]);
            lds_dma16<32 * D>(kp, klane, &ring[slot][2][0]);
            lds_dma16<32 * D + 32>(kp, klane, &ring[slot][3][0]);
        }
        if constexpr (PVBITS == 4) {
            lds_dma16<0>(vp, vlane, &ring[slot][4][0]);
            lds_dma16<32 * BLK / 2>(vp, vlane, &ring[slot][5][0]);
        } else {
            lds_dma16<0>(vp, vlane, &ring[slot][4][0]);
            lds_dma16<32>(vp, vlane, &ring[slot][5][0]);
            lds_dma16<32 * BLK>(vp, vlane, &ring[slot][6][0]);
            lds_dma16<32 * BLK + 32>(vp, vlane, &ring[slot][7][0]);
        }
    };

    float m[2] = {-INFINITY, -INFINITY};
    float m_ref[2] = {-INFINITY, -INFINITY};
    float w_base[2] = {INFINITY, INFINITY};
    float l[2] = {0.0f, 0.0f};
    float acc[2][2][16];  // [half][channel tile][register]
#pragma unroll
    for (int H = 0; H < 2; ++H)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[H][dt][r] = 0.0f;
    v16i acc_init;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_init[r] = kAccBiasI;
    asm volatile("" : "+v"(acc_init));

    float sk_cur = 0.0f, sv_cur = 0.0f;
    int j_cur = 0;
    if (cnt > 0) {
        j_cur = __builtin_amdgcn_readlane(cols_cur, 0);
        request(j_cur, 0);
        sk_cur = skp[j_cur];
        sv_cur = svp[j_cur];
    }
    const int tail_block = (a.n_tokens % BLK) != 0 ? a.kblocks - 1 : -1;  // the column block with padded keys, if any

    auto step = [&](auto fold_tag, int t) {
        constexpr bool FOLD = decltype(fold_tag)::value;
        const float c = sq_i * sk_cur;
        const float sv_now = sv_cur;
        const int j_now = j_cur;
        const uint8_t* slot = &ring[t & 1][0][0] + 16 * lane;

        // ---- the tiles of this block have arrived (everything this wavefront has in flight is theirs)
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0); the other counters untouched
        v4i kf[2][2];
#pragma unroll
        for (int T = 0; T < 2; ++T) {
            if constexpr (QKBITS == 4) {
                unpack_nibbles(*(const v4i*)(slot + T * 1024), kf[T][0], kf[T][1]);
            } else {
#pragma unroll
                for (int s = 0; s < 2; ++s) kf[T][s] = *(const v4i*)(slot + (2 * T + s) * 1024);
            }
        }
        // ---- request the next block's tiles into the other slot (its previous content, block t-1, is consumed)
        if (t + 1 < cnt) {
            if (((t + 1) & 63) == 0) {
                cols_cur = cols_nxt;
                ++cur_chunk;
                cols_nxt = load_cols(cur_chunk + 1);
            }
            j_cur = __builtin_amdgcn_readlane(cols_cur, (t + 1) & 63);
            request(j_cur, (t + 1) & 1);
            sk_cur = skp[j_cur];
            sv_cur = svp[j_cur];
        }

        // ---- S^T = K_j Q_i^T for both halves (i32, biased); every K fragment feeds two products
        v16i sacc[2][2];  // [half][key tile]
#pragma unroll
        for (int T = 0; T < 2; ++T)
#pragma unroll
            for (int H = 0; H < 2; ++H) {
                sacc[H][T] = acc_init;
#pragma unroll
                for (int s = 0; s < 2; ++s) sacc[H][T] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[T][s], qf[H][s], sacc[H][T], 0, 0, 0);
            }
        // Keys past N (ragged last column block) never receive probability mass: their raw logits become the
        // bit pattern of -inf, which as an integer loses every maximum and as a float sends the exponent's fma
        // (c > 0) to -inf, i.e. E = 0.  A wave-uniform branch, taken for that one column block only.
        if (j_now == tail_block) {
            const int nkeys = a.n_tokens - (a.kblocks - 1) * BLK;
#pragma unroll
            for (int H = 0; H < 2; ++H)
#pragma unroll
                for (int T = 0; T < 2; ++T)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * T + 8 * (r >> 2) + 4 * g + (r & 3) >= nkeys) sacc[H][T][r] = (int)0xFF800000;
        }

        // ---- running maxima of both halves and the tile's quantization scale (one in-wave reduction)
        float m_new[2];
        unsigned eb = 0xFF800000u;
#pragma unroll
        for (int H = 0; H < 2; ++H) {
            int part[4] = {0, 0, 0, 0};  // below every real value (those carry the accumulator bias)
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) part[r & 3] = max(part[r & 3], sacc[H][T][r]);
            const float ymax = c * int_result(xor32_max(max(max(part[0], part[1]), max(part[2], part[3]))));
            m_new[H] = fmaxf(m[H], ymax);
            eb = min(eb, __float_as_uint(ymax - m_new[H]) | invalid_row[H]);  // a padded row loses the minimum
        }
        const float e = __uint_as_float(wave_umin(eb));
        if (__builtin_amdgcn_ballot_w64(m_new[0] - m_ref[0] > 64.0f || m_new[1] - m_ref[1] > 64.0f) != 0) {
#pragma unroll
            for (int H = 0; H < 2; ++H) {
                const float down = __builtin_amdgcn_exp2f(m_ref[H] - m_new[H]);  // first block: 2^-inf = 0 on zero sums
                l[H] *= down;
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[H][dt][r] *= down;
                m_ref[H] = m_new[H];
                w_base[H] = -kLog2_65535 - m_new[H];
            }
        }
        v4i vf[2][2];  // V_j^T fragments [channel tile][key tile]
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int T = 0; T < 2; ++T) {
                if constexpr (PVBITS == 4) {
                    // this lane's 16 slots of key tile T: 8 packed bytes inside the piece that lane (n, T) fetched;
                    // a nibble moved to the top of its byte is the code times 16 (undone in the scale), and the
                    // PARO_VT nibble order makes the bytes come out in slot order
                    const uint2 x = *(const uint2*)(&ring[t & 1][4 + dt][0] + (n + 32 * T) * 16 + 8 * g);
                    vf[dt][T] = v4i{(int)((x.x << 4) & 0xF0F0F0F0u), (int)(x.x & 0xF0F0F0F0u), (int)((x.y << 4) & 0xF0F0F0F0u),
                                    (int)(x.y & 0xF0F0F0F0u)};
                } else {
                    vf[dt][T] = *(const v4i*)(slot + (4 + 2 * dt + T) * 1024);
                }
            }

        float cb_hi = 0.0f, cb_lo = 0.0f;
        if constexpr (FOLD) {
            cb_hi = c * kAccBiasF;
            cb_lo = fmaf(c, kAccBiasF, -cb_hi);
        }
#pragma unroll
        for (int H = 0; H < 2; ++H) {
            m[H] = m_new[H];
            const float off_n = (LOG2_QMAXP - kLog2_65535) - m_new[H] - e;
            float off_f = off_n, w_blk;
            if constexpr (FOLD) {
                off_f = off_n - cb_hi;
                const float bb = off_f - off_n;
                const float terr = (off_n - (off_f - bb)) + (-cb_hi - bb);
                w_blk = __builtin_amdgcn_exp2f((w_base[H] - off_n) - (cb_lo - terr));
            } else {
                w_blk = __builtin_amdgcn_exp2f(w_base[H] - off_n);
            }
            // ---- E (all of the half first, in place of the raw logits), row sum as four independent chains,
            // codes packed as B operand
            float ev[2][16];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    ev[T][r] = __builtin_amdgcn_exp2f(fmaf(FOLD ? __int_as_float(sacc[H][T][r]) : int_result(sacc[H][T][r]), c, off_f));
            float part_sum[4];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) part_sum[r & 3] = (T == 0 && r < 4) ? ev[T][r] : part_sum[r & 3] + ev[T][r];
            const float rs = (part_sum[0] + part_sum[1]) + (part_sum[2] + part_sum[3]);
            v4i pf[2];
#pragma unroll
            for (int T = 0; T < 2; ++T)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd], ev[T][4 * qd + 1]));
                    const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][4 * qd + 2], ev[T][4 * qd + 3]));
                    pf[T][qd] = (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u);
                }
            l[H] = fmaf(rs, w_blk, l[H]);
            // ---- O^T += (sP sv_j 2^(m' - m_ref)) V_j^T P^T for this half
            const float sv_eff = w_blk * sv_now * (PVBITS == 4 ? 0.0625f : 1.0f);
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                v16i o = acc_init;
#pragma unroll
                for (int T = 0; T < 2; ++T) o = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf[dt][T], pf[T], o, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[H][dt][r] = fmaf(int_result(o[r]), sv_eff, acc[H][dt][r]);
            }
        }
    };

    constexpr bool FOLDABLE = PARO_FOLD_LOGIT_BIAS && PVBITS == 8;
    bool fold = false;
    if constexpr (FOLDABLE) {  // same rule as attn_i8_kernel
        // the first two chunks of column indices are in registers already (a lane past the end holds the row's last column)
        float sk_max = cnt > 0 ? skp[cols_cur] : 0.0f;
        if (cnt > 64) sk_max = fmaxf(sk_max, skp[cols_nxt]);
        for (int base = 128; base < cnt; base += 64)
            if (base + lane < cnt) sk_max = fmaxf(sk_max, skp[min(max(cols[base + lane], 0), a.kblocks - 1)]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sk_max = fmaxf(sk_max, __shfl_xor(sk_max, off));
        fold = sq_i * sk_max * kAccBiasF < 8192.0f;
    }
    if (fold) {
        for (int t = 0; t < cnt; ++t) step(std::bool_constant<FOLDABLE>{}, t);
    } else {
        for (int t = 0; t < cnt; ++t) step(std::false_type{}, t);
    }

#pragma unroll
    for (int H = 0; H < 2; ++H) {
        const float l_tot = (l[H] + __shfl_xor(l[H], 32)) * 65535.0f;
        const float inv = (row_valid[H] && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
        const long long ooff = out_row_offset<D>(a, bh, h, head_rows, row[H], row_valid[H]);
        if (ooff >= 0) {
            OutT* orow = (OutT*)a.op + ooff + 4 * g;
#pragma unroll
            for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    store4(orow + 32 * dt + 8 * qd, acc[H][dt][4 * qd] * inv, acc[H][dt][4 * qd + 1] * inv, acc[H][dt][4 * qd + 2] * inv,
                           acc[H][dt][4 * qd + 3] * inv);
        }
    }
    PARO_TIMELINE_END(item, lane, cnt)
}

template <int PVBITS, typename OutT, int QSRC = 0>
__global__ __launch_bounds__(64, 2) void attn_i8_w64_kernel(AttnArgs a) {
    attn_i8_w64_body<8, PVBITS, OutT, QSRC>(a);
}

// the same wavefront program on 4-bit Q and K codes (Tab. 1, "QK (INT4)")
template <int PVBITS, typename OutT>
__global__ __launch_bounds__(64, 2) void attn_i8_w64_qk4_kernel(AttnArgs a) {
    attn_i8_w64_body<4, PVBITS, OutT, 0>(a);
}

// -------------------------------------------------------------------------------------------
// d = 128, block 64, 8-bit Q, K, P and V codes: FOUR wavefronts per row block, 16 queries each, on
// v_mfma_i32_16x16x64_i8.
//
// At d = 128 a wavefront of 32 queries carries 64 accumulator registers and needs ~200 in all: two
// wavefronts per SIMD, each alone for long stretches, and a row block that attends every column block (the
// text rows of an image model, Sec. 4.2 (1)) is a chain of 72 such block visits that the whole launch
// waits for.  With 16 queries per wavefront the visit is half as long, the registers allow three
// wavefronts per SIMD, and the matrix work is unchanged (a 16x16x64 instruction takes half the time of a
// 32x32x32 one).
//
// Layouts.  S^T tile T (16 keys x 16 queries): lane (n = lane % 16, G = lane / 16) holds query n, keys
// 4 G + r (r = 0..3) of the tile.  Which key sits in which row of a tile is free - K rows are fetched from
// LDS by address - and is chosen so that the four codes of a lane's tile T land, packed into register T
// of the B operand, on the contraction slots 16 G + 4 T + r that lane group G of the PV instruction
// covers: row 4 G + r of tile T is the key whose PARO_VT slot is 16 G + 4 T + r, i.e. token
// 32 (G >> 1) + 8 T + 4 (G & 1) + r of the block.  V^T fragments are then plain 16-byte reads of PARO_VT rows.
//
// Tiles.  K_j (64 x 128 B) and V_j^T (128 x 64 B) are contiguous 8 KB in global memory and go to LDS as
// they are with global_load_lds_dwordx4, each wavefront moving a quarter, except that inside every 128-byte
// line the eight 16-byte pieces are stored at position (piece ^ line % 8): the reads of 16 lanes that walk
// down a column of pieces then spread over all banks.  Two K slots and two V slots; ONE barrier per block,
// after the wavefront has written its share of the tile exponent and waited for its own requests: behind
// it K_{t+2} may overwrite K_t (all K_t reads precede the barrier) and V_{t+1} may overwrite V_{t-1}.  K_{t+2}
// is requested right behind the barrier; V_{t+1} only after the V_t fragments have been read, because the
// compiler makes every read of the V ring wait for all requests into that ring issued before it.
// Arithmetic per block as in attn_i8_kernel.
// -------------------------------------------------------------------------------------------
#ifndef PARO_ATTN_Q16
#define PARO_ATTN_Q16 1
#endif

typedef int v4acc __attribute__((ext_vector_type(4)));

// max over the four lanes n, n + 16, n + 32, n + 48 (the lanes that share a query), returned in all four
__device__ inline int quad_rows_max(int x) {
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    return xor32_max(max((int)r[0], (int)r[1]));
}
__device__ inline float quad_rows_sum(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(x), __float_as_int(x), false, false);
    const float y = __int_as_float((int)r[0]) + __int_as_float((int)r[1]);
    return y + __shfl_xor(y, 32);
}

template <typename OutT>
__global__ __launch_bounds__(256, 3) void attn_i8_q16_kernel(AttnArgs a) {
    constexpr int BLK = 64, D = 128;
    constexpr int KS = D / 64;     // contraction steps of QK^T (64 channels each)
    constexpr int CT = D / 16;     // 16-channel tiles of the output
    constexpr int TILE = BLK * D;  // bytes of a K tile and of a V^T tile
    constexpr float LOG2_QMAXP = 6.988684686772166f;
    constexpr float kLog2_65535 = 15.999977986052736f;
    __shared__ __attribute__((aligned(16))) uint8_t kring[2][TILE];
    __shared__ __attribute__((aligned(16))) uint8_t vring[2][TILE];
    __shared__ unsigned tile_e[2][4];

    const int wg = blockIdx.x;
    const int logical = (wg & 7) * a.per_xcd + (wg >> 3);
    if (logical >= a.total_wg) return;
    const int item = a.row_order ? min(max(a.row_order[logical], 0), a.total_wg - 1) : logical;
    const int bh = item / a.kblocks;
    const int i = item - bh * a.kblocks;
    const int h = bh % a.nh;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;
    const int G = lane >> 4;
    PARO_TIMELINE_BEGIN

    const int* rp = a.row_ptr + (size_t)h * (a.kblocks + 1) + i;
    const int beg = __builtin_amdgcn_readfirstlane(min(max(rp[0], 0), a.nnz));
    const int end = __builtin_amdgcn_readfirstlane(min(max(rp[1], beg), a.nnz));
    const int cnt = end - beg;
    const int* cols = a.col_idx + beg;
    if (2 * cnt > a.kblocks) __builtin_amdgcn_s_setprio(2);

    const size_t head_rows = (size_t)bh * a.kblocks * BLK;
    const uint8_t* kbase = a.k + head_rows * D;
    const uint8_t* vbase = a.v + head_rows * D;
    const float* skp = a.sk + (size_t)bh * a.kblocks;
    const float* svp = a.sv + (size_t)bh * a.kblocks;
    const float sq_i = a.sq[(size_t)bh * a.kblocks + i] * a.qk_scale;
    const int row = i * BLK + 16 * w + n;  // this lane's query, in the reordered sequence
    const bool row_valid = row < a.n_tokens;
    // or-ed into the bit pattern of a value <= 0 it gives a pattern at or above that of -inf: larger, as an unsigned
    // number, than the pattern of every value a real row can have
    const unsigned invalid_row = row_valid ? 0u : 0xFF800000u;
    v4i qf[KS];
    {
        const uint8_t* qrow = a.q + (head_rows + row) * D + 16 * G;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *(const v4i*)(qrow + 64 * s);
    }
    // a wavefront moves two of the eight 1 KB pieces of a tile: lane L fills LDS bytes 16 L of the piece, which is
    // position L % 8 of line L / 8 and holds the line's global piece (L % 8) ^ (L / 8)
    const unsigned fill_lane = 2048u * w + 128u * (lane >> 3) + 16u * ((lane & 7) ^ (lane >> 3));
    // K fragment of tile T, step s: row 32 (n >> 3) + 8 T + (n & 7) of the tile, piece 4 s + G
    unsigned kread[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) kread[s] = 128u * (32 * (n >> 3) + (n & 7)) + 16u * ((4 * s + G) ^ (n & 7));
    // V^T fragment of channel tile ct: PARO_VT row 16 ct + n = line 8 ct + n / 2, piece 4 (n % 2) + G
    const unsigned vread = 128u * (n >> 1) + 16u * ((4 * (n & 1) + G) ^ (n >> 1));

    // column indices: 64 per fetch, one per lane; `cols_cur` holds the chunk of the newest step looked up
    auto load_cols = [&](int chunk) {
        const int idx = min(chunk * 64 + lane, cnt - 1);
        return cnt > 0 && chunk * 64 < cnt ? min(max(cols[idx], 0), a.kblocks - 1) : 0;
    };
    int cols_cur = load_cols(0), cols_nxt = load_cols(1);
    int cur_chunk = 0;
    auto col_at = [&](int u) {  // u advances by one per call
        if ((u & 63) == 0 && u > 0) {
            cols_cur = cols_nxt;
            ++cur_chunk;
            cols_nxt = load_cols(cur_chunk + 1);
        }
        return __builtin_amdgcn_readlane(cols_cur, u & 63);
    };
    auto request_k = [&](int j, int slot) {
        const uint8_t* kp = kbase + (size_t)j * TILE;
        lds_dma16<0>(kp, fill_lane, &kring[slot][2048 * w]);
        lds_dma16<1024>(kp, fill_lane, &kring[slot][2048 * w + 1024]);
    };
    auto request_v = [&](int j, int slot) {
        const uint8_t* vp = vbase + (size_t)j * TILE;
        lds_dma16<0>(vp, fill_lane, &vring[slot][2048 * w]);
        lds_dma16<1024>(vp, fill_lane, &vring[slot][2048 * w + 1024]);
    };

    float m = -INFINITY, m_ref = -INFINITY, w_base = INFINITY, l = 0.0f;
    float acc[CT][4];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[ct][r] = 0.0f;
    v4acc acc_init = {kAccBiasI, kAccBiasI, kAccBiasI, kAccBiasI};
    asm volatile("" : "+v"(acc_init));

    // columns of the steps t, t + 1, t + 2 and the scales of t, t + 1
    int j0 = 0, j1 = 0, j2 = 0;
    float sk0 = 0.0f, sv0 = 0.0f, sk1 = 0.0f, sv1 = 0.0f;
    if (cnt > 0) {
        j0 = col_at(0);
        request_k(j0, 0);
        request_v(j0, 0);
        sk0 = uniform_load(skp + j0);
        sv0 = uniform_load(svp + j0);
        if (cnt > 1) {
            j1 = col_at(1);
            request_k(j1, 1);
            sk1 = uniform_load(skp + j1);
            sv1 = uniform_load(svp + j1);
        }
        if (cnt > 2) j2 = col_at(2);
    }
    constexpr bool FOLDABLE = PARO_FOLD_LOGIT_BIAS;
    bool fold = false;
    if constexpr (FOLDABLE) {  // same rule as attn_i8_kernel; its loads travel while the first tiles do
        // the first two chunks of column indices are in registers already (a lane past the end holds the row's last column)
        float sk_max = cnt > 0 ? skp[cols_cur] : 0.0f;
        if (cnt > 64) sk_max = fmaxf(sk_max, skp[cols_nxt]);
        for (int base = 128; base < cnt; base += 64)
            if (base + lane < cnt) sk_max = fmaxf(sk_max, skp[min(max(cols[base + lane], 0), a.kblocks - 1)]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sk_max = fmaxf(sk_max, __shfl_xor(sk_max, off));
        fold = sq_i * sk_max * kAccBiasF < 8192.0f;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    const int tail_block = (a.n_tokens % BLK) != 0 ? a.kblocks - 1 : -1;  // the column block with padded keys, if any

    auto step = [&](auto fold_tag, int t) {
        constexpr bool FOLD = decltype(fold_tag)::value;
        const float c = sq_i * sk0;
        const float sv_now = sv0;
        const uint8_t* kslot = &kring[t & 1][0];
        const uint8_t* vslot = &vring[t & 1][0];
        PARO_TIMELINE_PHASE(3)  // behind the previous block's accumulator update (and the loop's own overhead)

        // ---- S^T = K_j Q_i^T (i32, biased): four 16-key tiles
        v4acc sacc[4];
#pragma unroll
        for (int T = 0; T < 4; ++T) {
            sacc[T] = acc_init;
#pragma unroll
            for (int s = 0; s < KS; ++s)
                sacc[T] = __builtin_amdgcn_mfma_i32_16x16x64_i8(*(const v4i*)(kslot + 1024 * T + kread[s]), qf[s], sacc[T], 0, 0, 0);
        }
        if (j0 == tail_block) {  // keys past N: the bit pattern of -inf loses every maximum and gives E = 0
            const int nkeys = a.n_tokens - (a.kblocks - 1) * BLK;
#pragma unroll
            for (int T = 0; T < 4; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (32 * (G >> 1) + 8 * T + 4 * (G & 1) + r >= nkeys) sacc[T][r] = (int)0xFF800000;
        }
        // ---- running maximum and this wavefront's share of the tile's quantization scale
        int part[4] = {0, 0, 0, 0};  // below every real value (those carry the accumulator bias)
#pragma unroll
        for (int T = 0; T < 4; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[r] = max(part[r], sacc[T][r]);
        const float ymax = c * int_result(quad_rows_max(max(max(part[0], part[1]), max(part[2], part[3]))));
        const float m_new = fmaxf(m, ymax);
        unsigned eb = __float_as_uint(ymax - m_new) | invalid_row;  // a padded row loses the minimum
        eb = min(eb, (unsigned)dpp_mov<0xB1>((int)eb));  // the four rows of 16 lanes hold the same 16 queries:
        eb = min(eb, (unsigned)dpp_mov<0x4E>((int)eb));  // one row is reduced
        eb = min(eb, (unsigned)dpp_mov<0x141>((int)eb));
        eb = min(eb, (unsigned)dpp_mov<0x140>((int)eb));
        if (lane == 0) tile_e[t & 1][w] = eb;
        // ---- everything this wavefront has in flight (its share of K_{t+1} and V_t) has landed; behind the
        // barrier both tiles and all four exponents are whole, K_t has been read by all and V_{t-1} is consumed
        PARO_TIMELINE_PHASE(0)  // K reads, products, row maximum, share of the tile exponent
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        PARO_TIMELINE_PHASE(1)  // wait for the tiles and for the other wavefronts
        if (t + 2 < cnt) request_k(j2, t & 1);
        const int j_v = j1;
        const float e = __uint_as_float(min(min(tile_e[t & 1][0], tile_e[t & 1][1]), min(tile_e[t & 1][2], tile_e[t & 1][3])));
        // the next step's column, scales and the column after it (scalar work, hidden behind the vector work below)
        j0 = j1;
        j1 = j2;
        sk0 = sk1;
        sv0 = sv1;
        if (t + 2 < cnt) {
            sk1 = uniform_load(skp + j1);
            sv1 = uniform_load(svp + j1);
        }
        if (t + 3 < cnt) j2 = col_at(t + 3);

        if (__builtin_amdgcn_ballot_w64(m_new - m_ref > 64.0f) != 0) {
            const float down = __builtin_amdgcn_exp2f(m_ref - m_new);  // first block: 2^-inf = 0 on zero sums
            l *= down;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[ct][r] *= down;
            m_ref = m_new;
            w_base = -kLog2_65535 - m_new;
        }
        m = m_new;
        const float off_n = (LOG2_QMAXP - kLog2_65535) - m_new - e;
        float off_f = off_n, w_blk;
        if constexpr (FOLD) {
            const float cb_hi = c * kAccBiasF;
            const float cb_lo = fmaf(c, kAccBiasF, -cb_hi);
            off_f = off_n - cb_hi;
            const float bb = off_f - off_n;
            const float terr = (off_n - (off_f - bb)) + (-cb_hi - bb);
            w_blk = __builtin_amdgcn_exp2f((w_base - off_n) - (cb_lo - terr));
        } else {
            w_blk = __builtin_amdgcn_exp2f(w_base - off_n);
        }
        // ---- E (in place of the raw logits), row sum, codes packed as B operand: register T = tile T
        float ev[4][4];
#pragma unroll
        for (int T = 0; T < 4; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                ev[T][r] = __builtin_amdgcn_exp2f(fmaf(FOLD ? __int_as_float(sacc[T][r]) : int_result(sacc[T][r]), c, off_f));
        const float rs = ((ev[0][0] + ev[0][1]) + (ev[0][2] + ev[0][3])) + ((ev[1][0] + ev[1][1]) + (ev[1][2] + ev[1][3])) +
                         (((ev[2][0] + ev[2][1]) + (ev[2][2] + ev[2][3])) + ((ev[3][0] + ev[3][1]) + (ev[3][2] + ev[3][3])));
        v4i pf;
#pragma unroll
        for (int T = 0; T < 4; ++T) {
            const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][0], ev[T][1]));
            const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pknorm_u16(ev[T][2], ev[T][3]));
            pf[T] = (int)__builtin_amdgcn_perm(hi, lo, 0x06040200u);
        }
        l = fmaf(rs, w_blk, l);
        PARO_TIMELINE_PHASE(2)  // exponentials, row sum, codes
        // ---- O^T += (sP sv_j 2^(m' - m_ref)) V_j^T P^T: eight 16-channel tiles, one instruction each
        const float sv_eff = w_blk * sv_now;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const v4acc o = __builtin_amdgcn_mfma_i32_16x16x64_i8(*(const v4i*)(vslot + 1024 * ct + vread), pf, acc_init, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[ct][r] = fmaf(int_result(o[r]), sv_eff, acc[ct][r]);
        }
        if (t + 1 < cnt) request_v(j_v, (t + 1) & 1);
    };

    PARO_TIMELINE_PHASE(4)  // everything in front of the block loop
    if (fold) {
        for (int t = 0; t < cnt; ++t) step(std::bool_constant<FOLDABLE>{}, t);
    } else {
        for (int t = 0; t < cnt; ++t) step(std::false_type{}, t);
    }
    PARO_TIMELINE_PHASE(3)

    const float l_tot = quad_rows_sum(l) * 65535.0f;
    const float inv = (row_valid && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
    const long long ooff = out_row_offset<D>(a, bh, h, head_rows, row, row_valid);
    if (ooff >= 0) {
        OutT* orow = (OutT*)a.op + ooff + 4 * G;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) store4(orow + 16 * ct, acc[ct][0] * inv, acc[ct][1] * inv, acc[ct][2] * inv, acc[ct][3] * inv);
    }
    PARO_TIMELINE_END(4 * item + w, lane, cnt)
}

// -------------------------------------------------------------------------------------------
// bf16 unquantized block-sparse mode (the sparse-only rows of the paper's tables): same work
// split, transposed orientation and block list, on v_mfma_f32_32x32x16_bf16.  P is not quantized,
// so there is no tile-wide scale and no cross-wavefront exchange; P enters the PV product rounded
// to bf16 while the denominator accumulates it in fp32.  The 16-bit tiles are twice as large as
// the 8-bit ones, so this kernel keeps ONE LDS stage and pays a second barrier per block instead
// of a second stage: the smaller footprint admits a third wavefront per SIMD (d = 64), which is
// worth more here than the barrier costs.
// -------------------------------------------------------------------------------------------
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));

template <int BLK, int D>
struct Bf16Cfg {
    static constexpr int KSTR = 2 * D + 16;    // bytes per K row in LDS (bf16 + 16 B pad)
    static constexpr int VSTR = 2 * BLK + 16;  // bytes per V^T row in LDS
    static constexpr int KBYTES = BLK * KSTR;
    static constexpr int VBYTES = D * VSTR;
    static constexpr int STAGE = KBYTES + VBYTES;
    static constexpr int LDS_BYTES = STAGE;
};

template <int BLK, int D, typename OutT>
__global__ __launch_bounds__(BLK * 2, (D == 64 ? 3 : 2)) void attn_bf16_kernel(AttnArgs a) {
    using C = Bf16Cfg<BLK, D>;
    constexpr int NW = BLK / 32;
    constexpr int NT = 64 * NW;
    constexpr int KSTR = C::KSTR, VSTR = C::VSTR, KBYTES = C::KBYTES, STAGE = C::STAGE;
    constexpr int NKC = BLK * D * 2 / 16 / NT;  // 16-byte pieces of a K tile per thread
    constexpr int NVC = NKC;
    constexpr int KS = D / 16;    // contraction steps of QK^T (16 channels each)
    constexpr int KT = BLK / 32;  // 32-key tiles per block
    constexpr int DT = D / 32;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int wg = blockIdx.x;
    const int logical = (wg & 7) * a.per_xcd + (wg >> 3);
    if (logical >= a.total_wg) return;
    const int item = a.row_order ? min(max(a.row_order[logical], 0), a.total_wg - 1) : logical;
    const int bh = item / a.kblocks;
    const int i = item - bh * a.kblocks;
    const int h = bh % a.nh;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int n = lane & 31;
    const int g = lane >> 5;

    const int* rp = a.row_ptr + (size_t)h * (a.kblocks + 1) + i;
    const int beg = __builtin_amdgcn_readfirstlane(min(max(rp[0], 0), a.nnz));  // uniform: scalar loop control
    const int end = __builtin_amdgcn_readfirstlane(min(max(rp[1], beg), a.nnz));
    const int cnt = end - beg;
    const int* cols = a.col_idx + beg;

    const size_t head_rows = (size_t)bh * a.kblocks * BLK;
    const int row = i * BLK + 32 * w + n;
    const bool row_valid = row < a.n_tokens;
    const uint8_t* kbase = a.k + head_rows * D * 2;
    const uint8_t* vbase = a.v + head_rows * D * 2;
    const float c = a.qk_scale;

    v8bf qf[KS];
    {
        const uint8_t* qrow = a.q + (head_rows + row) * D * 2 + 16 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *(const v8bf*)(qrow + 32 * s);
    }

    // column indices: 64 per fetch, one per lane, read back with v_readlane (as in the INT8 kernel)
    auto load_cols = [&](int chunk) {
        const int idx = min(chunk * 64 + lane, cnt - 1);
        return cnt > 0 && chunk * 64 < cnt ? min(max(cols[idx], 0), a.kblocks - 1) : 0;
    };
    int cols_cur = load_cols(0), cols_nxt = load_cols(1);
    int cur_chunk = 0;
    auto col_of = [&](int t) {
        return (t >> 6) == cur_chunk ? __builtin_amdgcn_readlane(cols_cur, t & 63) : __builtin_amdgcn_readlane(cols_nxt, t & 63);
    };

    v4i kreg[NKC], vreg[NVC];
    // LDS store offsets: piece cc of a thread lies a whole number of rows below its piece 0, so one
    // address per tile serves all pieces through immediate offsets
    static_assert((16 * NT) % (2 * D) == 0 && (16 * NT) % (2 * BLK) == 0, "pieces must be whole rows apart");
    const int k_off = ((16 * tid) / (2 * D)) * KSTR + (16 * tid) % (2 * D);
    const int v_off = KBYTES + ((16 * tid) / (2 * BLK)) * VSTR + (16 * tid) % (2 * BLK);
    auto lstore_k = [&](int stage) {
        uint8_t* dst0 = lds + stage * STAGE + k_off;
#pragma unroll
        for (int cc = 0; cc < NKC; ++cc) *(v4i*)(dst0 + cc * (16 * NT / (2 * D)) * KSTR) = kreg[cc];
    };
    auto lstore_v = [&](int stage) {
        uint8_t* dst0 = lds + stage * STAGE + v_off;
#pragma unroll
        for (int cc = 0; cc < NVC; ++cc) *(v4i*)(dst0 + cc * (16 * NT / (2 * BLK)) * VSTR) = vreg[cc];
    };

    // The exponentials are taken against a fixed reference per row (its maximum after the first
    // block) instead of the running maximum: P is not quantized here, so the common factor
    // 2^(m - m_ref) of numerator and denominator cancels in acc / l and no rescaling pass is needed.
    // A row whose maximum climbs more than 64 octaves above the reference is re-referenced.
    float m_ref = -INFINITY;
    float l = 0.0f;
    v16f acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.0f;

    // One LDS stage and two barriers per live block: K_t is read before the first barrier; behind it
    // K_{t+1} and V_t replace K_t and V_{t-1} (every wavefront is past their last reads), the second
    // barrier publishes them.  Half the LDS footprint, which lets a third wavefront per SIMD in.
    auto gload_k = [&](int t) {
        const uint8_t* kp = kbase + (size_t)col_of(t) * (BLK * D * 2);
#pragma unroll
        for (int cc = 0; cc < NKC; ++cc) kreg[cc] = *(const v4i*)(kp + 16 * (tid + NT * cc));
    };
    auto gload_v = [&](int t) {
        const uint8_t* vp = vbase + (size_t)col_of(t) * (BLK * D * 2);
#pragma unroll
        for (int cc = 0; cc < NVC; ++cc) vreg[cc] = *(const v4i*)(vp + 16 * (tid + NT * cc));
    };
    if (cnt > 0) {
        gload_k(0);
        gload_v(0);
        lstore_k(0);
        if (cnt > 1) gload_k(1);
    }
    __syncthreads();

    constexpr int stage = 0;
    auto step = [&](auto tail_tag, int t) {
        constexpr bool TAIL = decltype(tail_tag)::value;
        const uint8_t* ks = lds + stage * STAGE;
        const uint8_t* vs = ks + KBYTES;

        v16f sacc[KT];
#pragma unroll
        for (int T = 0; T < KT; ++T) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[T][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const v8bf kf = *(const v8bf*)(ks + (32 * T + n) * KSTR + 32 * s + 16 * g);
                sacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[T], 0, 0, 0);
            }
        }
        if constexpr (TAIL) {
            const int nkeys = a.n_tokens - (a.kblocks - 1) * BLK;
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * T + 8 * (r >> 2) + 4 * g + (r & 3) >= nkeys) sacc[T][r] = -INFINITY;
        }
        auto row_max = [&]() {  // maximum over the block's keys of this lane's query, in both of its lanes
            float part[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) part[r & 3] = fmaxf(part[r & 3], sacc[T][r]);
            const float mx = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_int(mx), __float_as_int(mx), false, false);
            return fmaxf(__int_as_float((int)sw[0]), __int_as_float((int)sw[1]));
        };
        // a row without a reference yet (first block, or nothing but masked keys so far) takes its block maximum
        if (__builtin_amdgcn_ballot_w64(m_ref == -INFINITY) != 0) {
            const float ymax = c * row_max();
            if (m_ref == -INFINITY) m_ref = ymax;
        }
        // y = c S - m_ref, the exponent of P, FIRST, in place of S: its maximum tells whether the row has climbed past
        // its reference (results of an fma need no NaN quieting before a maximum, raw matrix results would)
#pragma unroll
        for (int T = 0; T < KT; ++T)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[T][r] = fmaf(sacc[T][r], c, -m_ref);
        const float climb = row_max();  // row maximum - reference
        __syncthreads();
        lstore_v(0);                      // V_t (loaded one block ago)
        if (t + 1 < cnt) lstore_k(0);     // K_{t+1}
        if (t + 1 < cnt) gload_v(t + 1);  // before the column chunk moves on: t+1 may be its last entry
        if (((t + 2) & 63) == 0) {
            cols_cur = cols_nxt;
            ++cur_chunk;
            cols_nxt = load_cols(cur_chunk + 1);
        }
        if (t + 2 < cnt) gload_k(t + 2);
        if (__builtin_amdgcn_ballot_w64(climb > 64.0f) != 0) {
            const float up = fmaxf(climb, 0.0f);  // rows that have not climbed keep their reference
            const float down = __builtin_amdgcn_exp2f(-up);
            l *= down;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[dt][r] *= down;
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[T][r] -= up;
            m_ref += up;
        }

        float rs = 0.0f;
        v8bf pf[KT][2];
#pragma unroll
        for (int T = 0; T < KT; ++T)
#pragma unroll
            for (int u = 0; u < 2; ++u)
#pragma unroll
                for (int e2 = 0; e2 < 4; ++e2) {
                    const float p0 = __builtin_amdgcn_exp2f(sacc[T][8 * u + 2 * e2]);
                    const float p1 = __builtin_amdgcn_exp2f(sacc[T][8 * u + 2 * e2 + 1]);
                    rs += p0 + p1;
                    const v2bf pb = __builtin_convertvector(v2f{p0, p1}, v2bf);
                    pf[T][u][2 * e2] = pb[0];
                    pf[T][u][2 * e2 + 1] = pb[1];
                }
        l += rs;

        __syncthreads();  // K_{t+1} and V_t are in place
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const v8bf vf = *(const v8bf*)(vs + (32 * dt + n) * VSTR + 2 * (32 * T + 16 * g + 8 * u));
                    acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[T][u], acc[dt], 0, 0, 0);
                }
    };

    const bool has_tail = (a.n_tokens % BLK) != 0 && cnt > 0 && min(max(cols[cnt - 1], 0), a.kblocks - 1) == a.kblocks - 1;
    const int cnt_main = has_tail ? cnt - 1 : cnt;
    for (int t = 0; t < cnt_main; ++t) step(std::false_type{}, t);
    if (has_tail) step(std::true_type{}, cnt - 1);

    const float l_tot = l + __shfl_xor(l, 32);
    const float inv = (row_valid && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
    const long long ooff = out_row_offset<D>(a, bh, h, head_rows, row, row_valid);
    if (ooff >= 0) {
        OutT* orow = (OutT*)a.op + ooff + 4 * g;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                store4(orow + 32 * dt + 8 * qd, acc[dt][4 * qd] * inv, acc[dt][4 * qd + 1] * inv, acc[dt][4 * qd + 2] * inv,
                       acc[dt][4 * qd + 3] * inv);
    }
}

// -------------------------------------------------------------------------------------------
// bf16 mode at d = 64, block 64: FOUR wavefronts of 16 queries per row block on v_mfma_f32_16x16x32_bf16, built like
// attn_i8_q16_kernel.  A bf16 K tile at d = 64 (64 rows of 128 bytes) and a bf16 V^T tile (64 channel rows of 128
// bytes) have the geometry of the 8-bit tiles at d = 128, so the tiles go to LDS the same way (global_load_lds,
// a quarter per wavefront, pieces of a line at position piece ^ line % 8, two K and two V slots, one barrier per
// block).  P is not quantized: nothing is exchanged between the wavefronts, the exponentials are taken against the
// row's fixed reference and O^T accumulates in the matrix accumulators themselves (16 registers), so the vector
// work per block is the logits' alone.
// Row 4 G + r of S^T tile T is the key whose PARO_VT slot is 32 (T >> 1) + 8 G + 4 (T & 1) + r - the slot that
// element 4 (T & 1) + r of lane group G covers in contraction step T >> 1 of the PV product - i.e. token
// 32 (T >> 1) + 8 (T & 1) + 16 (G & 1) + 4 (G >> 1) + r of the block.
// -------------------------------------------------------------------------------------------
#ifndef PARO_BF16_Q16
#define PARO_BF16_Q16 1
#endif
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ inline float quad_rows_fmax(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(x), __float_as_int(x), false, false);
    const float y = fmaxf(__int_as_float((int)r[0]), __int_as_float((int)r[1]));
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_int(y), __float_as_int(y), false, false);
    return fmaxf(__int_as_float((int)q[0]), __int_as_float((int)q[1]));
}

template <typename OutT>
__global__ __launch_bounds__(256, 4) void attn_bf16_q16_kernel(AttnArgs a) {
    constexpr int BLK = 64, D = 64;
    constexpr int KS = D / 32;     // contraction steps of QK^T (32 channels each)
    constexpr int US = BLK / 32;   // contraction steps of PV (32 slots each)
    constexpr int CT = D / 16;     // 16-channel tiles of the output
    constexpr int TILE = BLK * D * 2;  // bytes of a K tile and of a V^T tile
    static_assert(TILE == 8192, "the tile transfer below moves eight 1 KB pieces");
    __shared__ __attribute__((aligned(16))) uint8_t kring[2][TILE];
    __shared__ __attribute__((aligned(16))) uint8_t vring[2][TILE];

    const int wg = blockIdx.x;
    const int logical = (wg & 7) * a.per_xcd + (wg >> 3);
    if (logical >= a.total_wg) return;
    const int item = a.row_order ? min(max(a.row_order[logical], 0), a.total_wg - 1) : logical;
    const int bh = item / a.kblocks;
    const int i = item - bh * a.kblocks;
    const int h = bh % a.nh;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15;
    const int G = lane >> 4;

    const int* rp = a.row_ptr + (size_t)h * (a.kblocks + 1) + i;
    const int beg = __builtin_amdgcn_readfirstlane(min(max(rp[0], 0), a.nnz));
    const int end = __builtin_amdgcn_readfirstlane(min(max(rp[1], beg), a.nnz));
    const int cnt = end - beg;
    const int* cols = a.col_idx + beg;
    if (2 * cnt > a.kblocks) __builtin_amdgcn_s_setprio(2);

    const size_t head_rows = (size_t)bh * a.kblocks * BLK;
    const uint8_t* kbase = a.k + head_rows * D * 2;
    const uint8_t* vbase = a.v + head_rows * D * 2;
    const float c = a.qk_scale;
    const int row = i * BLK + 16 * w + n;  // this lane's query, in the reordered sequence
    const bool row_valid = row < a.n_tokens;
    v8bf qf[KS];
    {
        const uint8_t* qrow = a.q + (head_rows + row) * D * 2 + 16 * G;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *(const v8bf*)(qrow + 64 * s);
    }
    // tile transfer as in attn_i8_q16_kernel
    const unsigned fill_lane = 2048u * w + 128u * (lane >> 3) + 16u * ((lane & 7) ^ (lane >> 3));
    // K fragment of tile T, step s: row 32 (T >> 1) + 8 (T & 1) + 16 ((n >> 2) & 1) + 4 (n >> 3) + (n & 3), piece 4 s + G
    const unsigned krow = 16 * ((n >> 2) & 1) + 4 * (n >> 3) + (n & 3);
    unsigned kread[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) kread[s] = 128u * krow + 16u * ((4 * s + G) ^ (krow & 7));
    // V^T fragment of channel tile ct, step u: PARO_VT row 16 ct + n, piece 4 u + G
    unsigned vread[US];
#pragma unroll
    for (int u = 0; u < US; ++u) vread[u] = 128u * n + 16u * ((4 * u + G) ^ (n & 7));

    auto load_cols = [&](int chunk) {
        const int idx = min(chunk * 64 + lane, cnt - 1);
        return cnt > 0 && chunk * 64 < cnt ? min(max(cols[idx], 0), a.kblocks - 1) : 0;
    };
    int cols_cur = load_cols(0), cols_nxt = load_cols(1);
    int cur_chunk = 0;
    auto col_at = [&](int u) {  // u advances by one per call
        if ((u & 63) == 0 && u > 0) {
            cols_cur = cols_nxt;
            ++cur_chunk;
            cols_nxt = load_cols(cur_chunk + 1);
        }
        return __builtin_amdgcn_readlane(cols_cur, u & 63);
    };
    auto request_k = [&](int j, int slot) {
        const uint8_t* kp = kbase + (size_t)j * TILE;
        lds_dma16<0>(kp, fill_lane, &kring[slot][2048 * w]);
        lds_dma16<1024>(kp, fill_lane, &kring[slot][2048 * w + 1024]);
    };
    auto request_v = [&](int j, int slot) {
        const uint8_t* vp = vbase + (size_t)j * TILE;
        lds_dma16<0>(vp, fill_lane, &vring[slot][2048 * w]);
        lds_dma16<1024>(vp, fill_lane, &vring[slot][2048 * w + 1024]);
    };

    float m_ref = -INFINITY, l = 0.0f;
    v4f acc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc[ct] = v4f{0.0f, 0.0f, 0.0f, 0.0f};

    int j0 = 0, j1 = 0, j2 = 0;  // columns of the steps t, t + 1, t + 2
    if (cnt > 0) {
        j0 = col_at(0);
        request_k(j0, 0);
        request_v(j0, 0);
        if (cnt > 1) {
            j1 = col_at(1);
            request_k(j1, 1);
        }
        if (cnt > 2) j2 = col_at(2);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();
    const int tail_block = (a.n_tokens % BLK) != 0 ? a.kblocks - 1 : -1;  // the column block with padded keys, if any

    for (int t = 0; t < cnt; ++t) {
        const uint8_t* kslot = &kring[t & 1][0];
        const uint8_t* vslot = &vring[t & 1][0];
        // ---- S^T = K_j Q_i^T: four 16-key tiles
        v4f sacc[4];
#pragma unroll
        for (int T = 0; T < 4; ++T) {
            sacc[T] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int s = 0; s < KS; ++s)
                sacc[T] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const v8bf*)(kslot + 4096 * (T >> 1) + 1024 * (T & 1) + kread[s]), qf[s],
                                                                  sacc[T], 0, 0, 0);
        }
        if (j0 == tail_block) {  // keys past N never receive probability mass
            const int nkeys = a.n_tokens - (a.kblocks - 1) * BLK;
#pragma unroll
            for (int T = 0; T < 4; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (32 * (T >> 1) + 8 * (T & 1) + 16 * (G & 1) + 4 * (G >> 1) + r >= nkeys) sacc[T][r] = -INFINITY;
        }
        // a row without a reference yet (first block, or nothing but masked keys so far) takes its block maximum
        if (__builtin_amdgcn_ballot_w64(m_ref == -INFINITY) != 0) {
            float part[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) part[r] = fmaxf(fmaxf(sacc[0][r], sacc[1][r]), fmaxf(sacc[2][r], sacc[3][r]));
            const float ymax = c * quad_rows_fmax(fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3])));
            if (m_ref == -INFINITY) m_ref = ymax;
        }
        // ---- y = c S - m_ref, the exponent of P, FIRST: its maximum tells whether the row has climbed past its
        // reference (results of an fma need no NaN quieting before a maximum, raw matrix results would)
        float p[4][4];
#pragma unroll
        for (int T = 0; T < 4; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) p[T][r] = fmaf(sacc[T][r], c, -m_ref);
        float part[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) part[r] = fmaxf(fmaxf(p[0][r], p[1][r]), fmaxf(p[2][r], p[3][r]));
        const float climb = quad_rows_fmax(fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3])));  // row maximum - reference
        // ---- this wavefront's requests have landed; behind the barrier both tiles are whole, K_t has been read by
        // all and V_{t-1} is consumed
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        if (t + 2 < cnt) request_k(j2, t & 1);
        const int j_v = j1;
        j0 = j1;
        j1 = j2;
        if (t + 3 < cnt) j2 = col_at(t + 3);

        if (__builtin_amdgcn_ballot_w64(climb > 64.0f) != 0) {
            const float up = fmaxf(climb, 0.0f);  // rows that have not climbed keep their reference
            const float down = __builtin_amdgcn_exp2f(-up);
            l *= down;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[ct][r] *= down;
#pragma unroll
            for (int T = 0; T < 4; ++T)
#pragma unroll
                for (int r = 0; r < 4; ++r) p[T][r] -= up;
            m_ref += up;
        }
        // ---- P = 2^y, its row sum in fp32, and P rounded to bf16 as B operand: element 4 (T & 1) + r of step T >> 1
#pragma unroll
        for (int T = 0; T < 4; ++T)
#pragma unroll
            for (int r = 0; r < 4; ++r) p[T][r] = __builtin_amdgcn_exp2f(p[T][r]);
        l += ((p[0][0] + p[0][1]) + (p[0][2] + p[0][3])) + ((p[1][0] + p[1][1]) + (p[1][2] + p[1][3])) +
             (((p[2][0] + p[2][1]) + (p[2][2] + p[2][3])) + ((p[3][0] + p[3][1]) + (p[3][2] + p[3][3])));
        v8bf pf[US];
#pragma unroll
        for (int u = 0; u < US; ++u)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh)
#pragma unroll
                for (int e2 = 0; e2 < 2; ++e2) {
                    const v2bf pb = __builtin_convertvector(v2f{p[2 * u + hh][2 * e2], p[2 * u + hh][2 * e2 + 1]}, v2bf);
                    pf[u][4 * hh + 2 * e2] = pb[0];
                    pf[u][4 * hh + 2 * e2 + 1] = pb[1];
                }
        // ---- O^T += V_j^T P^T, accumulated in the matrix accumulators
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int u = 0; u < US; ++u)
                acc[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*(const v8bf*)(vslot + 2048 * ct + vread[u]), pf[u], acc[ct], 0, 0, 0);
        if (t + 1 < cnt) request_v(j_v, (t + 1) & 1);
    }

    const float l_tot = quad_rows_sum(l);
    const float inv = (row_valid && l_tot > 0.0f) ? 1.0f / l_tot : 0.0f;
    const long long ooff = out_row_offset<D>(a, bh, h, head_rows, row, row_valid);
    if (ooff >= 0) {
        OutT* orow = (OutT*)a.op + ooff + 4 * G;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) store4(orow + 16 * ct, acc[ct][0] * inv, acc[ct][1] * inv, acc[ct][2] * inv, acc[ct][3] * inv);
    }
}

template <int BLK, int D, typename OutT>
static int launch_bf16_t(const AttnArgs& a, hipStream_t st) {
    constexpr int bytes = Bf16Cfg<BLK, D>::LDS_BYTES;
    static_assert(bytes <= 48 * 1024, "beyond 48 KB the launch would have to raise the function's dynamic LDS limit first");
    hipLaunchKernelGGL((attn_bf16_kernel<BLK, D, OutT>), dim3((unsigned)(a.per_xcd * 8)), dim3(BLK * 2), bytes, st, a);
    return PARO_OK;
}

template <typename OutT>
static int launch_bf16(int blk, int d, const AttnArgs& a, hipStream_t st) {
    if constexpr (PARO_BF16_Q16) {
        if (blk == 64 && d == 64) {  // four wavefronts of 16 queries per row block
            hipLaunchKernelGGL((attn_bf16_q16_kernel<OutT>), dim3((unsigned)(a.per_xcd * 8)), dim3(256), 0, st, a);
            return PARO_OK;
        }
    }
    if (blk == 64 && d == 64) return launch_bf16_t<64, 64, OutT>(a, st);
    if (blk == 64 && d == 128) return launch_bf16_t<64, 128, OutT>(a, st);
    if (blk == 32 && d == 64) return launch_bf16_t<32, 64, OutT>(a, st);
    return launch_bf16_t<32, 128, OutT>(a, st);
}

template <int BLK, int D, int QKBITS, int PVBITS>
static void launch_out(paro_dtype out_dtype, const AttnArgs& a, hipStream_t st) {
    dim3 grid((unsigned)(a.per_xcd * 8));
    if (out_dtype == PARO_F32)
        hipLaunchKernelGGL((attn_i8_kernel<BLK, D, QKBITS, PVBITS, float>), grid, dim3(BLK * 2), 0, st, a);
    else
        hipLaunchKernelGGL((attn_i8_kernel<BLK, D, QKBITS, PVBITS, uint16_t>), grid, dim3(BLK * 2), 0, st, a);
}

// Q taken from the unquantized tensor (block 64 only): QSRC 1 = bf16, 2 = fp32
template <int D, int PVBITS, int QSRC>
static void launch_rawq(paro_dtype out_dtype, const AttnArgs& a, hipStream_t st) {
    dim3 grid((unsigned)(a.per_xcd * 8));
    if (out_dtype == PARO_F32)
        hipLaunchKernelGGL((attn_i8_kernel<64, D, 8, PVBITS, float, QSRC>), grid, dim3(128), 0, st, a);
    else
        hipLaunchKernelGGL((attn_i8_kernel<64, D, 8, PVBITS, uint16_t, QSRC>), grid, dim3(128), 0, st, a);
}

template <int PVBITS, int QSRC>
static void launch_rawq_w64(paro_dtype out_dtype, const AttnArgs& a, hipStream_t st) {
    dim3 grid((unsigned)(a.per_xcd * 8));
    if (out_dtype == PARO_F32) hipLaunchKernelGGL((attn_i8_w64_kernel<PVBITS, float, QSRC>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((attn_i8_w64_kernel<PVBITS, uint16_t, QSRC>), grid, dim3(64), 0, st, a);
}

template <int QSRC>
static void launch_rawq_shape(int d, int bits_pv, paro_dtype out_dtype, const AttnArgs& a, hipStream_t st) {
    if constexpr (PARO_ATTN_SINGLE_WAVE) {
        if (d == 64) {  // block 64 is a precondition of this entry point: the one-wavefront kernel applies
            if (bits_pv == 8) launch_rawq_w64<8, QSRC>(out_dtype, a, st);
            else launch_rawq_w64<4, QSRC>(out_dtype, a, st);
            return;
        }
    }
    if (d == 64 && bits_pv == 8) launch_rawq<64, 8, QSRC>(out_dtype, a, st);
    else if (d == 64) launch_rawq<64, 4, QSRC>(out_dtype, a, st);
    else if (bits_pv == 8) launch_rawq<128, 8, QSRC>(out_dtype, a, st);
    else launch_rawq<128, 4, QSRC>(out_dtype, a, st);
}

template <int QKBITS, int PVBITS>
static void launch_i8(int blk, int d, paro_dtype out_dtype, const AttnArgs& a, hipStream_t st) {
    if constexpr (PARO_ATTN_SINGLE_WAVE) {
        if (blk == 64 && d == 64) {  // one wavefront per row block
            dim3 grid((unsigned)(a.per_xcd * 8));
            if constexpr (QKBITS == 8) {
                if (out_dtype == PARO_F32) hipLaunchKernelGGL((attn_i8_w64_kernel<PVBITS, float>), grid, dim3(64), 0, st, a);
                else hipLaunchKernelGGL((attn_i8_w64_kernel<PVBITS, uint16_t>), grid, dim3(64), 0, st, a);
            } else {
                if (out_dtype == PARO_F32) hipLaunchKernelGGL((attn_i8_w64_qk4_kernel<PVBITS, float>), grid, dim3(64), 0, st, a);
                else hipLaunchKernelGGL((attn_i8_w64_qk4_kernel<PVBITS, uint16_t>), grid, dim3(64), 0, st, a);
            }
            return;
        }
    }
    if constexpr (PARO_ATTN_Q16 && QKBITS == 8 && PVBITS == 8) {
        if (blk == 64 && d == 128) {  // four wavefronts of 16 queries per row block
            dim3 grid((unsigned)(a.per_xcd * 8));
            if (out_dtype == PARO_F32) hipLaunchKernelGGL((attn_i8_q16_kernel<float>), grid, dim3(256), 0, st, a);
            else hipLaunchKernelGGL((attn_i8_q16_kernel<uint16_t>), grid, dim3(256), 0, st, a);
            return;
        }
    }
    if (blk == 64 && d == 64) launch_out<64, 64, QKBITS, PVBITS>(out_dtype, a, st);
    else if (blk == 64 && d == 128) launch_out<64, 128, QKBITS, PVBITS>(out_dtype, a, st);
    else if (blk == 32 && d == 64) launch_out<32, 64, QKBITS, PVBITS>(out_dtype, a, st);
    else launch_out<32, 128, QKBITS, PVBITS>(out_dtype, a, st);
}

}  // namespace paro

namespace paro {
static int attn_entry(const char* what, const paro_shape* s, int bits_qk, int bits_pv, const void* q, const float* sq, const void* k,
                      const float* sk, const void* v, const float* sv, const int32_t* row_ptr, const int32_t* col_idx,
                      int64_t nnz, const int32_t* row_order, const uint8_t* h_perm_ids, paro_dtype out_dtype, void* op,
                      void* stream, int q_raw = 0) {
    int64_t n, kb;
    if (int st = check_shape(s, &n, &kb)) return st;
    if (q_raw) {
        if (bits_qk != 8 || (bits_pv != 8 && bits_pv != 4))
            return fail(PARO_EUNSUPPORTED, "in-kernel quantization of Q: bits (qk=%d, pv=%d), supported qk 8 with pv 8 or 4", bits_qk, bits_pv);
        if (s->block != 64) return fail(PARO_EUNSUPPORTED, "in-kernel quantization of Q needs block 64, got %d", s->block);
    }
    const bool i8 = (bits_qk == 8 || bits_qk == 4) && (bits_pv == 8 || bits_pv == 4);
    const bool b16 = bits_qk == 16 && bits_pv == 16;
    if (!i8 && !b16) {
        const bool known = (bits_qk == 8 || bits_qk == 4 || bits_qk == 16) && (bits_pv == 8 || bits_pv == 4 || bits_pv == 16);
        return fail(known ? PARO_EUNSUPPORTED : PARO_EINVAL,
                    "bits (qk=%d, pv=%d): supported pairs are qk in {8,4} with pv in {8,4}, and (16,16)", bits_qk, bits_pv);
    }
    if (out_dtype != PARO_F32 && out_dtype != PARO_BF16) return fail(PARO_EINVAL, "out_dtype=%d is not a paro_dtype", (int)out_dtype);
    if (!q || !k || !v || !op || !row_ptr) return fail(PARO_EINVAL, "q, k, v, op and row_ptr must not be NULL");
    if (i8 && ((!sq && !q_raw) || !sk || !sv)) return fail(PARO_EINVAL, "sq, sk and sv are required for integer operands");
    if (nnz < 0 || nnz > 0x7fffffffLL) return fail(PARO_EINVAL, "nnz=%lld out of range", (long long)nnz);
    if (nnz > 0 && !col_idx) return fail(PARO_EINVAL, "col_idx is NULL but nnz=%lld", (long long)nnz);
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)op) & 15) return fail(PARO_EINVAL, "q, k, v and op must be 16-byte aligned");

    AttnArgs a;
    a.q = (const uint8_t*)q;
    a.k = (const uint8_t*)k;
    a.v = (const uint8_t*)v;
    a.sq = sq;
    a.sk = sk;
    a.sv = sv;
    a.row_ptr = row_ptr;
    a.col_idx = col_idx;
    a.op = op;
    a.nnz = (int)nnz;
    a.nh = s->nh;
    a.kblocks = (int)kb;
    a.n_tokens = (int)n;
    a.total_wg = (int)((int64_t)s->B * s->nh * kb);
    a.per_xcd = (a.total_wg + 7) / 8;
    a.row_order = row_order;
    a.qk_scale = (float)(1.4426950408889634 / sqrt((double)s->d));
    a.scatter = h_perm_ids != nullptr;
    if (a.scatter) {
        if (int st = make_reorder_table(s, h_perm_ids, &a.table)) return st;
    } else {
        memset(&a.table, 0, sizeof(a.table));
    }
    if (b16) {
        const int st = out_dtype == PARO_F32 ? launch_bf16<float>(s->block, s->d, a, (hipStream_t)stream)
                                             : launch_bf16<uint16_t>(s->block, s->d, a, (hipStream_t)stream);
        if (st) return st;
    } else if (q_raw) {
        if (q_raw == 1) launch_rawq_shape<1>(s->d, bits_pv, out_dtype, a, (hipStream_t)stream);
        else launch_rawq_shape<2>(s->d, bits_pv, out_dtype, a, (hipStream_t)stream);
    } else if (bits_qk == 8) {
        if (bits_pv == 8) launch_i8<8, 8>(s->block, s->d, out_dtype, a, (hipStream_t)stream);
        else launch_i8<8, 4>(s->block, s->d, out_dtype, a, (hipStream_t)stream);
    } else {
        if (bits_pv == 8) launch_i8<4, 8>(s->block, s->d, out_dtype, a, (hipStream_t)stream);
        else launch_i8<4, 4>(s->block, s->d, out_dtype, a, (hipStream_t)stream);
    }
    return check_launch(what);
}
}  // namespace paro

extern "C" int paro_sparse_attn(const paro_shape* s, int bits_qk, int bits_pv, const void* q, const float* sq, const void* k,
                                const float* sk, const void* v, const float* sv, const int32_t* row_ptr,
                                const int32_t* col_idx, int64_t nnz, const int32_t* row_order, paro_dtype out_dtype, void* op,
                                void* stream) {
    return paro::attn_entry("paro_sparse_attn", s, bits_qk, bits_pv, q, sq, k, sk, v, sv, row_ptr, col_idx, nnz, row_order, nullptr,
                            out_dtype, op, stream);
}

extern "C" int paro_sparse_attn_unpermuted(const paro_shape* s, int bits_qk, int bits_pv, const void* q, const float* sq,
                                           const void* k, const float* sk, const void* v, const float* sv,
                                           const int32_t* row_ptr, const int32_t* col_idx, int64_t nnz,
                                           const int32_t* row_order, const uint8_t* h_perm_ids, paro_dtype out_dtype,
                                           void* o, void* stream) {
    if (!h_perm_ids) return paro::fail(PARO_EINVAL, "perm_ids is NULL");
    return paro::attn_entry("paro_sparse_attn_unpermuted", s, bits_qk, bits_pv, q, sq, k, sk, v, sv, row_ptr, col_idx, nnz,
                            row_order, h_perm_ids, out_dtype, o, stream);
}

extern "C" int paro_sparse_attn_unpermuted_rawq(const paro_shape* s, paro_dtype q_dtype, int bits_pv, const void* q, const void* k,
                                                const float* sk, const void* v, const float* sv, const int32_t* row_ptr,
                                                const int32_t* col_idx, int64_t nnz, const int32_t* row_order,
                                                const uint8_t* h_perm_ids, paro_dtype out_dtype, void* o, void* stream) {
    if (!h_perm_ids) return paro::fail(PARO_EINVAL, "perm_ids is NULL");
    if (q_dtype != PARO_F32 && q_dtype != PARO_BF16) return paro::fail(PARO_EINVAL, "q_dtype=%d is not a paro_dtype", (int)q_dtype);
    return paro::attn_entry("paro_sparse_attn_unpermuted_rawq", s, 8, bits_pv, q, nullptr, k, sk, v, sv, row_ptr, col_idx, nnz, row_order,
                            h_perm_ids, out_dtype, o, stream, q_dtype == PARO_BF16 ? 1 : 2);
}

#if PARO_TIMELINE
// h_records: int64 [slots][8] (HOST; start clock, end clock, column blocks visited, shader cycles of the block loop's
// phases 0..3 and of the part in front of the loop); returns the rate of the start/end clock in kHz (> 0)
// or a negative status.  Synchronises the device.
extern "C" int64_t paro_timeline_read(int64_t* h_records, int64_t slots) {
    if (!h_records || slots < 0 || slots > paro::kTimelineSlots) return PARO_EINVAL;
    if (hipMemcpyFromSymbol(h_records, HIP_SYMBOL(paro::timeline_records), sizeof(long long) * paro::kTimelineFields * (size_t)slots) != hipSuccess) return PARO_EHIP;
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return PARO_EHIP;
    return khz;
}
#endif
