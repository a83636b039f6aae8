// Token reorder and its inverse (paper Sec. 4.1): pure data movement, bound by HBM bandwidth.
//
// Both directions are written as a gather with sequential, fully coalesced 16-byte stores; the
// source row of every destination row is computed arithmetically from the head's axis order,
// so no index array is read.  A token row is d*sizeof(T) = 128..512 contiguous bytes (one to
// four whole 128-byte lines), so the gathered reads are line-granular as well.
#include "common.h"

namespace paro {

struct PermArgs {
    int n_tokens;   // N
    int n_img;      // F*Hg*Wg
    int npad;       // rows of the padded side
    int chunks;     // 16-byte chunks per row
    int Hg, Wg;
    int fwd[6][5];  // per axis order: extents of the middle and fastest axis, then the default-order
                    // stride of the slowest, middle and fastest axis
    int inv[6][3];  // per axis order: multiplier of the f, h and w coordinate in the reordered position
    uint8_t perm[kMaxHeads];
};

// Position in the default [F,H,W] order of the token at position n_new of the reordered sequence.
__device__ inline int source_of(int n_new, int d1, int d2, int s0, int s1, int s2) {
    const int c2 = n_new % d2;
    const int t = n_new / d2;
    const int c1 = t % d1;
    const int c0 = t / d1;
    return c0 * s0 + c1 * s1 + c2 * s2;
}

// forward: dst = xp [bh][npad][row], src = x [bh][N][row];   dst row n' <- src row idx(n')
__global__ __launch_bounds__(256) void permute_kernel(PermArgs a, const uint4* __restrict__ src, uint4* __restrict__ dst, int nh) {
    const int bh = blockIdx.y;
    const unsigned gid = blockIdx.x * 256u + threadIdx.x;
    const int row = gid / a.chunks;
    const int c = gid % a.chunks;
    if (row >= a.npad) return;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (row < a.n_tokens) {
        int from = row;
        if (row < a.n_img) {
            const int* t = a.fwd[a.perm[bh % nh]];
            from = source_of(row, t[0], t[1], t[2], t[3], t[4]);
        }
        val = src[((size_t)bh * a.n_tokens + from) * a.chunks + c];
    }
    dst[((size_t)bh * a.npad + row) * a.chunks + c] = val;
}

// inverse: dst = o [bh][N][row], src = op [bh][npad][row];   dst row n <- src row n' with idx(n') = n
__global__ __launch_bounds__(256) void unpermute_kernel(PermArgs a, const uint4* __restrict__ src, uint4* __restrict__ dst, int nh) {
    const int bh = blockIdx.y;
    const unsigned gid = blockIdx.x * 256u + threadIdx.x;
    const int row = gid / a.chunks;
    const int c = gid % a.chunks;
    if (row >= a.n_tokens) return;
    int from = row;
    if (row < a.n_img) {
        const int* mul = a.inv[a.perm[bh % nh]];
        const int w = row % a.Wg;
        const int t = row / a.Wg;
        const int h = t % a.Hg;
        const int f = t / a.Hg;
        from = f * mul[0] + h * mul[1] + w * mul[2];
    }
    dst[((size_t)bh * a.n_tokens + row) * a.chunks + c] = src[((size_t)bh * a.npad + from) * a.chunks + c];
}

static int launch(bool forward, const paro_shape* s, paro_dtype dtype, const uint8_t* h_perm_ids, const void* src,
                  void* dst, void* stream) {
    int64_t n, k;
    if (int st = check_shape(s, &n, &k)) return st;
    if (dtype != PARO_F32 && dtype != PARO_BF16) return fail(PARO_EINVAL, "dtype=%d is not a paro_dtype", (int)dtype);
    if (!h_perm_ids || !src || !dst) return fail(PARO_EINVAL, "perm_ids, source and destination must not be NULL");
    if (src == dst) return fail(PARO_EINVAL, "source and destination must not alias");
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return fail(PARO_EINVAL, "tensors must be 16-byte aligned");
    PermArgs a;
    for (int h = 0; h < s->nh; ++h) {
        if (h_perm_ids[h] > 5) return fail(PARO_EINVAL, "perm_ids[%d]=%d not in 0..5", h, (int)h_perm_ids[h]);
        a.perm[h] = h_perm_ids[h];
    }
    a.n_tokens = (int)n;
    a.n_img = s->F * s->Hg * s->Wg;
    a.npad = (int)(k * s->block);
    a.chunks = s->d * (dtype == PARO_F32 ? 4 : 2) / 16;
    a.Hg = s->Hg;
    a.Wg = s->Wg;
    const int dims[3] = {s->F, s->Hg, s->Wg};
    const int stride[3] = {s->Hg * s->Wg, s->Wg, 1};
    for (int p = 0; p < 6; ++p) {
        const AxisOrder o = axis_order(p);
        a.fwd[p][0] = dims[o.a[1]];
        a.fwd[p][1] = dims[o.a[2]];
        for (int i = 0; i < 3; ++i) a.fwd[p][2 + i] = stride[o.a[i]];
        a.inv[p][o.a[0]] = dims[o.a[1]] * dims[o.a[2]];
        a.inv[p][o.a[1]] = dims[o.a[2]];
        a.inv[p][o.a[2]] = 1;
    }
    const int64_t rows = forward ? a.npad : a.n_tokens;
    dim3 grid((unsigned)((rows * a.chunks + 255) / 256), (unsigned)(s->B * s->nh));
    if (forward)
        hipLaunchKernelGGL(permute_kernel, grid, dim3(256), 0, (hipStream_t)stream, a, (const uint4*)src, (uint4*)dst, s->nh);
    else
        hipLaunchKernelGGL(unpermute_kernel, grid, dim3(256), 0, (hipStream_t)stream, a, (const uint4*)src, (uint4*)dst, s->nh);
    return check_launch(forward ? "paro_permute" : "paro_unpermute");
}

}  // namespace paro

extern "C" int paro_permute(const paro_shape* s, paro_dtype dtype, const uint8_t* h_perm_ids, const void* x, void* xp,
                            void* stream) {
    return paro::launch(true, s, dtype, h_perm_ids, x, xp, stream);
}

extern "C" int paro_unpermute(const paro_shape* s, paro_dtype dtype, const uint8_t* h_perm_ids, const void* op, void* o,
                              void* stream) {
    return paro::launch(false, s, dtype, h_perm_ids, op, o, stream);
}
