// Token reorder and its inverse (paper Sec. 4.1): pure data movement, bound by HBM bandwidth.
//
// Both directions are written as a gather with sequential, fully coalesced 16-byte stores; the
// source row of every destination row is computed arithmetically from the head's axis order,
// so no index array is read.  A token row is d*sizeof(T) = 128..512 contiguous bytes (one to
// four whole 128-byte lines), so the gathered reads are line-granular as well.
#include "common.h"

namespace paro {

// forward: dst = xp [bh][npad][row], src = x [bh][N][row];   dst row n' <- src row idx(n')
__global__ __launch_bounds__(256) void permute_kernel(ReorderTable t, int npad, int chunks, const uint4* __restrict__ src,
                                                      uint4* __restrict__ dst, int nh) {
    const int bh = blockIdx.y;
    const unsigned gid = blockIdx.x * 256u + threadIdx.x;
    const int row = gid / chunks;
    const int c = gid % chunks;
    if (row >= npad) return;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (row < t.n_tokens) val = src[((size_t)bh * t.n_tokens + reorder_source(t, bh % nh, row)) * chunks + c];
    dst[((size_t)bh * npad + row) * chunks + c] = val;
}

// inverse: dst = o [bh][N][row], src = op [bh][npad][row];   dst row n <- src row n' with idx(n') = n
__global__ __launch_bounds__(256) void unpermute_kernel(ReorderTable t, int npad, int chunks, const uint4* __restrict__ src,
                                                        uint4* __restrict__ dst, int nh) {
    const int bh = blockIdx.y;
    const unsigned gid = blockIdx.x * 256u + threadIdx.x;
    const int row = gid / chunks;
    const int c = gid % chunks;
    if (row >= t.n_tokens) return;
    dst[((size_t)bh * t.n_tokens + row) * chunks + c] = src[((size_t)bh * npad + reorder_dest(t, bh % nh, row)) * chunks + c];
}

static int launch(bool forward, const paro_shape* s, paro_dtype dtype, const uint8_t* h_perm_ids, const void* src,
                  void* dst, void* stream) {
    int64_t n, k;
    if (int st = check_shape(s, &n, &k)) return st;
    if (dtype != PARO_F32 && dtype != PARO_BF16) return fail(PARO_EINVAL, "dtype=%d is not a paro_dtype", (int)dtype);
    if (!h_perm_ids || !src || !dst) return fail(PARO_EINVAL, "perm_ids, source and destination must not be NULL");
    if (src == dst) return fail(PARO_EINVAL, "source and destination must not alias");
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return fail(PARO_EINVAL, "tensors must be 16-byte aligned");
    ReorderTable t;
    if (int st = make_reorder_table(s, h_perm_ids, &t)) return st;
    const int npad = (int)(k * s->block);
    const int chunks = s->d * (dtype == PARO_F32 ? 4 : 2) / 16;
    const int64_t rows = forward ? npad : n;
    dim3 grid((unsigned)((rows * chunks + 255) / 256), (unsigned)(s->B * s->nh));
    if (forward)
        hipLaunchKernelGGL(permute_kernel, grid, dim3(256), 0, (hipStream_t)stream, t, npad, chunks, (const uint4*)src, (uint4*)dst, s->nh);
    else
        hipLaunchKernelGGL(unpermute_kernel, grid, dim3(256), 0, (hipStream_t)stream, t, npad, chunks, (const uint4*)src, (uint4*)dst, s->nh);
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
