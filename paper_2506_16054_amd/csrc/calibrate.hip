// Offline calibration of PAROAttention on the GPU (paper Sec. 4.1 "Metric for Permutation Order",
// Sec. 4.2 (3) "Efficient Offline Mask Generation"), for gfx950.
//
//   paro_calib_block_stats   per b x b block of the post-softmax map P = softmax(Q K^T / sqrt(d)) of
//                            already reordered 16-bit operands: sum, maximum, and the number of
//                            entries below eps (the n_ij of Eq. (M_sparse)).  The map is never
//                            stored: one workgroup owns a row block, sweeps all column blocks once
//                            for the row maxima and denominators and a second time for the block
//                            statistics, both on v_mfma_f32_32x32x16_bf16 in the transposed
//                            orientation (a lane holds 16 keys of ONE query, so the row statistics
//                            are in-lane plus one cross-lane step).
//   paro_calib_metrics       M_sparse and M_quant of Eq. (M_sparse) / (M_quant) per head.
//   paro_calib_choose        the combined metric over the six orders and the order that minimises it.
//   paro_calib_mask          block-sum thresholding with explicit density control: the n_live
//                            largest block sums of a head stay live (exact radix selection on the
//                            bit patterns, equal sums resolved by position), written as the bitmask
//                            the attention path consumes.
//
// This is an offline step (the paper runs it once per model on one or two prompts); it is written
// for exactness of the integer decisions first and is not on the measured hot path.
#include <math.h>

#include <type_traits>

#include "common.h"

namespace paro {

typedef int c_v4i __attribute__((ext_vector_type(4)));
typedef __bf16 c_v8bf __attribute__((ext_vector_type(8)));
typedef float c_v16f __attribute__((ext_vector_type(16)));

struct CalibArgs {
    const uint8_t* q;  // bf16 [B, nh, Npad, d], reordered, padded rows zero
    const uint8_t* k;
    float* bsum;       // [B, nh, k, k]
    float* bmax;
    int* bcnt;
    int nh;
    int kblocks;
    int n_tokens;
    int total_wg;  // B * nh * kblocks
    int per_xcd;
    float qk_scale;  // log2(e) / sqrt(d)
    float eps;
};

template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2, 2) void calib_stats_kernel(CalibArgs a) {
    constexpr int NW = BLK / 32;
    constexpr int NT = 64 * NW;
    constexpr int KSTR = 2 * D + 16;  // bytes per K row in LDS (bf16 + 16 B pad)
    constexpr int KBYTES = BLK * KSTR;
    constexpr int NKC = BLK * D * 2 / 16 / NT;  // 16-byte pieces of a K tile per thread
    constexpr int KS = D / 16;                  // contraction steps of 16 channels
    constexpr int KT = BLK / 32;                // 32-key tiles per block
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * KBYTES];
    __shared__ float red_sum[2][NW], red_max[2][NW];
    __shared__ int red_cnt[2][NW];

    // each XCD takes a contiguous range of (head, row block): a head's K stays in its L2
    const int wg = blockIdx.x;
    const int item = (wg & 7) * a.per_xcd + (wg >> 3);
    if (item >= a.total_wg) return;
    const int bh = item / a.kblocks;
    const int i = item - bh * a.kblocks;
    const int kb = a.kblocks;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int n = lane & 31;
    const int g = lane >> 5;
    const size_t head_rows = (size_t)bh * kb * BLK;
    const int row = i * BLK + 32 * w + n;
    const bool row_valid = row < a.n_tokens;
    const uint8_t* kbase = a.k + head_rows * D * 2;
    const float c = a.qk_scale;
    const bool ragged = (a.n_tokens % BLK) != 0;
    const int nkeys_tail = a.n_tokens - (kb - 1) * BLK;

    c_v8bf qf[KS];
    {
        const uint8_t* qrow = a.q + (head_rows + row) * D * 2 + 16 * g;
#pragma unroll
        for (int s = 0; s < KS; ++s) qf[s] = *(const c_v8bf*)(qrow + 32 * s);
    }

    c_v4i kreg[NKC];
    auto gload = [&](int t) {
        const uint8_t* kp = kbase + (size_t)t * (BLK * D * 2);
#pragma unroll
        for (int cc = 0; cc < NKC; ++cc) kreg[cc] = *(const c_v4i*)(kp + 16 * (tid + NT * cc));
    };
    auto lstore = [&](int stage) {
        uint8_t* ks = lds + stage * KBYTES;
#pragma unroll
        for (int cc = 0; cc < NKC; ++cc) {
            const int o = 16 * (tid + NT * cc);
            *(c_v4i*)(ks + (o / (2 * D)) * KSTR + (o % (2 * D))) = kreg[cc];
        }
    };

    float m = -INFINITY;  // running row maximum (log2 units), then the final one
    float l = 0.0f;       // this lane's share of the denominator, then 1 / denominator
    float* out_sum = a.bsum + ((size_t)bh * kb + i) * kb;
    float* out_max = a.bmax + ((size_t)bh * kb + i) * kb;
    int* out_cnt = a.bcnt + ((size_t)bh * kb + i) * kb;

    // One column block.  PASS 0 updates the running maximum and denominator; PASS 1 forms the
    // probabilities with the final maximum and denominator and reduces them over the block.
    // The LDS ring is the one of the attention kernels: tile t+1 is stored at the top of
    // iteration t (every wavefront finished reading tile t-1 before the previous barrier), one
    // barrier per column block, registers refilled (tile t+2) after it.
    int stage = 0;
    auto step = [&](auto pass_tag, auto tail_tag, int t) {
        constexpr int PASS = decltype(pass_tag)::value;
        constexpr bool TAIL = decltype(tail_tag)::value;
        const int next = stage ^ 1;
        if (t + 1 < kb) lstore(next);
        const uint8_t* ks = lds + stage * KBYTES;

        c_v16f sacc[KT];
#pragma unroll
        for (int T = 0; T < KT; ++T) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[T][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const c_v8bf kf = *(const c_v8bf*)(ks + (32 * T + n) * KSTR + 32 * s + 16 * g);
                sacc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[T], 0, 0, 0);
            }
        }
        if constexpr (TAIL) {  // keys past N do not exist
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * T + 8 * (r >> 2) + 4 * g + (r & 3) >= nkeys_tail) sacc[T][r] = -INFINITY;
        }
        if constexpr (PASS == 0) {
            float mx = -INFINITY;
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[T][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m, c * mx);
            float rs = 0.0f;
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) rs += __builtin_amdgcn_exp2f(fmaf(sacc[T][r], c, -m_new));
            l = fmaf(l, __builtin_amdgcn_exp2f(m - m_new), rs);
            m = m_new;
        } else {
            float ps = 0.0f, pm = 0.0f;
            int pc = 0;
#pragma unroll
            for (int T = 0; T < KT; ++T)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[T][r], c, -m)) * l;
                    ps += p;
                    pm = fmaxf(pm, p);
                    const bool real = !TAIL || (32 * T + 8 * (r >> 2) + 4 * g + (r & 3) < nkeys_tail);
                    pc += (real && p < a.eps) ? 1 : 0;
                }
            if (!row_valid) {  // rows past N do not exist
                ps = 0.0f;
                pm = 0.0f;
                pc = 0;
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                ps += __shfl_xor(ps, off);
                pm = fmaxf(pm, __shfl_xor(pm, off));
                pc += __shfl_xor(pc, off);
            }
            if (lane == 0) {
                red_sum[t & 1][w] = ps;
                red_max[t & 1][w] = pm;
                red_cnt[t & 1][w] = pc;
            }
        }
        __syncthreads();
        if (t + 2 < kb) gload(t + 2);
        if constexpr (PASS == 1) {
            if (tid == 0) {
                float ps = red_sum[t & 1][0], pm = red_max[t & 1][0];
                int pc = red_cnt[t & 1][0];
#pragma unroll
                for (int ww = 1; ww < NW; ++ww) {
                    ps += red_sum[t & 1][ww];
                    pm = fmaxf(pm, red_max[t & 1][ww]);
                    pc += red_cnt[t & 1][ww];
                }
                out_sum[t] = ps;
                out_max[t] = pm;
                out_cnt[t] = pc;
            }
        }
        stage = next;
    };
    auto sweep = [&](auto pass_tag) {
        gload(0);
        lstore(0);
        if (kb > 1) gload(1);
        __syncthreads();
        stage = 0;
        const int main_blocks = ragged ? kb - 1 : kb;
        for (int t = 0; t < main_blocks; ++t) step(pass_tag, std::false_type{}, t);
        if (ragged) step(pass_tag, std::true_type{}, kb - 1);
        __syncthreads();  // every wavefront is done with both stages before the next sweep refills them
    };

    sweep(std::integral_constant<int, 0>{});
    l = 1.0f / (l + __shfl_xor(l, 32));
    sweep(std::integral_constant<int, 1>{});
}

// -------------------------------------------------------------------------------------------
// M_sparse and M_quant of one head: a reduction over its B * k * k blocks.
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void calib_metrics_kernel(int B, int nh, int kb, int n_tokens, int blk, const float* __restrict__ bsum,
                                                            const float* __restrict__ bmax, const int* __restrict__ bcnt, float sigma,
                                                            float* __restrict__ m_sparse, float* __restrict__ m_quant) {
    __shared__ double s_psi[256];
    __shared__ int s_sparse[256];
    const int h = blockIdx.x;
    const int t = threadIdx.x;
    const int per_head = kb * kb;
    double psi = 0.0;
    int sparse = 0;
    for (int b = 0; b < B; ++b) {
        const size_t base = ((size_t)b * nh + h) * per_head;
        for (int e = t; e < per_head; e += 256) {
            const int i = e / kb, j = e - i * kb;
            const int rows = min(blk, n_tokens - i * blk), cols = min(blk, n_tokens - j * blk);
            const float entries = (float)(rows * cols);
            sparse += ((float)bcnt[base + e] >= sigma * entries) ? 1 : 0;
            const float s = bsum[base + e];
            if (s > 0.0f) psi += (double)bmax[base + e] / ((double)s / (double)entries);
        }
    }
    s_psi[t] = psi;
    s_sparse[t] = sparse;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (t < off) {
            s_psi[t] += s_psi[t + off];
            s_sparse[t] += s_sparse[t + off];
        }
        __syncthreads();
    }
    if (t == 0) {
        const double total = (double)B * per_head;
        m_sparse[h] = (float)((double)s_sparse[0] / total);
        m_quant[h] = (float)(s_psi[0] / total);
    }
}

__global__ __launch_bounds__(256) void calib_choose_kernel(int nh, const float* __restrict__ ms, const float* __restrict__ mq, float alpha,
                                                           float* __restrict__ m_out, uint8_t* __restrict__ perm_ids) {
    const int h = blockIdx.x * 256 + threadIdx.x;
    if (h >= nh) return;
    double dense[6], quant[6], sd = 0.0, sq = 0.0;
    for (int t = 0; t < 6; ++t) {
        dense[t] = 1.0 - (double)ms[t * nh + h];  // share of blocks that are not sparse: lower is better
        quant[t] = (double)mq[t * nh + h];
        sd += dense[t];
        sq += quant[t];
    }
    int best = 0;
    double best_m = 0.0;
    for (int t = 0; t < 6; ++t) {
        const double mt = (double)alpha * (sd > 0.0 ? dense[t] / sd : 0.0) + (1.0 - (double)alpha) * (sq > 0.0 ? quant[t] / sq : 0.0);
        m_out[t * nh + h] = (float)mt;
        if (t == 0 || mt < best_m) {
            best = t;
            best_m = mt;
        }
    }
    perm_ids[h] = (uint8_t)best;
}

// -------------------------------------------------------------------------------------------
// Block-sum thresholding with density control, one workgroup per head.
// -------------------------------------------------------------------------------------------
constexpr int kMaskThreads = 1024;
constexpr int kMaskMaxWords = 12288;  // k*k <= 393216 mask bits held in LDS

__global__ __launch_bounds__(kMaskThreads) void calib_mask_kernel(int B, int nh, int kb, int k_img, int n_live, const float* __restrict__ bsum,
                                                                  uint8_t* __restrict__ bitmask) {
    __shared__ unsigned words[kMaskMaxWords];
    __shared__ int hist[256];
    __shared__ int part[kMaskThreads];
    __shared__ int sel_bin, sel_remaining;
    const int h = blockIdx.x;
    const int t = threadIdx.x;
    const int per_head = kb * kb;
    const int nwords = (per_head + 31) / 32;
    const int nbytes = (per_head + 7) / 8;
    // the sum over the calibration samples, in sample order; non-negative, so the bit pattern orders it
    auto key_of = [&](int e) {
        float s = 0.0f;
        for (int b = 0; b < B; ++b) s += bsum[((size_t)b * nh + h) * per_head + e];
        return __float_as_uint(s);
    };
    auto is_img = [&](int e) { return e / kb < k_img && e % kb < k_img; };

    for (int wd = t; wd < nwords; wd += kMaskThreads) words[wd] = 0u;

    // ---- exact n_live-th largest key among the image x image blocks: radix selection, 8 bits a pass
    unsigned prefix = 0u, decided = 0u;
    int remaining = n_live;  // afterwards: how many blocks equal to the threshold stay live
    const bool select = n_live > 0 && n_live < k_img * k_img;
    if (select) {
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (t < 256) hist[t] = 0;
            __syncthreads();
            for (int e = t; e < per_head; e += kMaskThreads) {
                if (!is_img(e)) continue;
                const unsigned key = key_of(e);
                if ((key & decided) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
            }
            __syncthreads();
            if (t == 0) {
                int above = 0, bin = 255;
                for (; bin > 0; --bin) {
                    if (above + hist[bin] >= remaining) break;
                    above += hist[bin];
                }
                sel_bin = bin;
                sel_remaining = remaining - above;
            }
            __syncthreads();
            prefix |= (unsigned)sel_bin << shift;
            decided |= 255u << shift;
            remaining = sel_remaining;
            __syncthreads();
        }
    }
    const unsigned thr = prefix;

    // ---- live bits; blocks equal to the threshold are taken in ascending position until `remaining`
    const int per = (per_head + kMaskThreads - 1) / kMaskThreads;
    const int lo = min(t * per, per_head), hi = min(lo + per, per_head);
    int equal = 0;
    if (select)
        for (int e = lo; e < hi; ++e) equal += (is_img(e) && key_of(e) == thr) ? 1 : 0;
    part[t] = equal;
    __syncthreads();
    for (int off = 1; off < kMaskThreads; off <<= 1) {
        const int add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    int rank = part[t] - equal;
    for (int e = lo; e < hi; ++e) {
        bool live;
        if (!is_img(e)) {
            live = true;  // rows and columns of text blocks are never sparsified
        } else if (!select) {
            live = n_live > 0;
        } else {
            const unsigned key = key_of(e);
            live = key > thr || (key == thr && rank < remaining);
            rank += key == thr ? 1 : 0;
        }
        if (live) atomicOr(&words[e >> 5], 1u << (e & 31));
    }
    __syncthreads();
    uint8_t* out = bitmask + (size_t)h * nbytes;
    for (int b = t; b < nbytes; b += kMaskThreads) out[b] = (uint8_t)((words[b >> 2] >> (8 * (b & 3))) & 255u);
}

static int calib_shape(const paro_shape* s, int64_t* n, int64_t* kb) {
    if (int st = check_shape(s, n, kb)) return st;
    if (s->T_text > 0 && ((int64_t)s->F * s->Hg * s->Wg) % s->block != 0)
        return fail(PARO_EUNSUPPORTED, "with text tokens the image tokens must fill whole blocks (F*Hg*Wg=%lld, block=%d)",
                    (long long)s->F * s->Hg * s->Wg, s->block);
    return PARO_OK;
}

}  // namespace paro

extern "C" int paro_calib_block_stats(const paro_shape* s, const void* q16, const void* k16, float eps, float* block_sum,
                                      float* block_max, int32_t* block_cnt, void* stream) {
    using namespace paro;
    int64_t n, kb;
    if (int st = calib_shape(s, &n, &kb)) return st;
    if (!q16 || !k16 || !block_sum || !block_max || !block_cnt) return fail(PARO_EINVAL, "q16, k16, block_sum, block_max and block_cnt must not be NULL");
    if (((uintptr_t)q16 | (uintptr_t)k16) & 15) return fail(PARO_EINVAL, "q16 and k16 must be 16-byte aligned");
    if (!(eps > 0.0f)) return fail(PARO_EINVAL, "eps=%g must be positive", (double)eps);
    CalibArgs a;
    a.q = (const uint8_t*)q16;
    a.k = (const uint8_t*)k16;
    a.bsum = block_sum;
    a.bmax = block_max;
    a.bcnt = block_cnt;
    a.nh = s->nh;
    a.kblocks = (int)kb;
    a.n_tokens = (int)n;
    a.total_wg = (int)((int64_t)s->B * s->nh * kb);
    a.per_xcd = (a.total_wg + 7) / 8;
    a.qk_scale = (float)(1.4426950408889634 / sqrt((double)s->d));
    a.eps = eps;
    const dim3 grid((unsigned)(a.per_xcd * 8));
    hipStream_t st = (hipStream_t)stream;
    if (s->block == 64 && s->d == 64) hipLaunchKernelGGL((calib_stats_kernel<64, 64>), grid, dim3(128), 0, st, a);
    else if (s->block == 64 && s->d == 128) hipLaunchKernelGGL((calib_stats_kernel<64, 128>), grid, dim3(128), 0, st, a);
    else if (s->block == 32 && s->d == 64) hipLaunchKernelGGL((calib_stats_kernel<32, 64>), grid, dim3(64), 0, st, a);
    else hipLaunchKernelGGL((calib_stats_kernel<32, 128>), grid, dim3(64), 0, st, a);
    return check_launch("paro_calib_block_stats");
}

extern "C" int paro_calib_metrics(const paro_shape* s, const float* block_sum, const float* block_max, const int32_t* block_cnt,
                                  float sigma, float* m_sparse, float* m_quant, void* stream) {
    using namespace paro;
    int64_t n, kb;
    if (int st = calib_shape(s, &n, &kb)) return st;
    if (!block_sum || !block_max || !block_cnt || !m_sparse || !m_quant)
        return fail(PARO_EINVAL, "block_sum, block_max, block_cnt, m_sparse and m_quant must not be NULL");
    if (!(sigma >= 0.0f && sigma <= 1.0f)) return fail(PARO_EINVAL, "sigma=%g must lie in [0, 1]", (double)sigma);
    hipLaunchKernelGGL(calib_metrics_kernel, dim3((unsigned)s->nh), dim3(256), 0, (hipStream_t)stream, s->B, s->nh, (int)kb, (int)n, s->block,
                       block_sum, block_max, block_cnt, sigma, m_sparse, m_quant);
    return check_launch("paro_calib_metrics");
}

extern "C" int paro_calib_choose(int nh, const float* m_sparse6, const float* m_quant6, float alpha, float* m_combined6,
                                 uint8_t* perm_ids, void* stream) {
    using namespace paro;
    if (nh < 1 || nh > kMaxHeads) return fail(PARO_EINVAL, "nh=%d out of range [1, %d]", nh, kMaxHeads);
    if (!m_sparse6 || !m_quant6 || !m_combined6 || !perm_ids) return fail(PARO_EINVAL, "m_sparse6, m_quant6, m_combined6 and perm_ids must not be NULL");
    if (!(alpha >= 0.0f && alpha <= 1.0f)) return fail(PARO_EINVAL, "alpha=%g must lie in [0, 1]", (double)alpha);
    hipLaunchKernelGGL(calib_choose_kernel, dim3((unsigned)((nh + 255) / 256)), dim3(256), 0, (hipStream_t)stream, nh, m_sparse6, m_quant6,
                       alpha, m_combined6, perm_ids);
    return check_launch("paro_calib_choose");
}

extern "C" int paro_calib_mask(const paro_shape* s, const float* block_sum, float density, uint8_t* bitmask, void* stream) {
    using namespace paro;
    int64_t n, kb;
    if (int st = calib_shape(s, &n, &kb)) return st;
    if (!block_sum || !bitmask) return fail(PARO_EINVAL, "block_sum and bitmask must not be NULL");
    if (!(density >= 0.0f && density <= 1.0f)) return fail(PARO_EINVAL, "density=%g must lie in [0, 1]", (double)density);
    if (kb * kb > (int64_t)kMaskMaxWords * 32)
        return fail(PARO_EUNSUPPORTED, "k=%lld: masks of more than %d blocks per head are not supported", (long long)kb, kMaskMaxWords * 32);
    const int64_t k_img = ((int64_t)s->F * s->Hg * s->Wg + s->block - 1) / s->block;
    const int64_t n_live = (int64_t)nearbyint((double)density * (double)(k_img * k_img));  // ties to even
    hipLaunchKernelGGL(calib_mask_kernel, dim3((unsigned)s->nh), dim3(kMaskThreads), 0, (hipStream_t)stream, s->B, s->nh, (int)kb, (int)k_img,
                       (int)n_live, block_sum, bitmask);
    return check_launch("paro_calib_mask");
}
