// Device-side expansion of per-head block bitmasks into the compacted live-block list that
// paro_sparse_attn walks (paper Sec. 4.2 (1): masks are kept as bitmasks, 9.2 KB per head, and
// prefetched per transformer block and timestep; App. C "Overhead of Prefetch": the load of the
// next mask overlaps the attention of the current one through two buffers).  The caller copies the
// next bitmask to the GPU on a side stream and enqueues this expansion behind the copy; nothing
// here touches the host.
//
// Three small launches on the caller's stream:
//   1. count:  c[h][i] = live blocks of row block i of head h, c[h][k] = 0, stored in row_ptr;
//   2. scan:   in-place exclusive prefix sum over the flat [nh][k+1] array by one workgroup, which
//              yields exactly the offsets of the list (row_ptr[h][k] = end of head h = start of
//              head h+1), and the total;
//   3. fill:   one wavefront per row block writes its live columns in ascending order (ballot +
//              prefix popcount keeps the order without atomics).
#include "common.h"

namespace paro {

// Number of set bits among bits [bit0, bit0 + nbits) of a little-endian bit string.
__device__ inline int count_bits(const uint8_t* bm, int bit0, int nbits) {
    int cnt = 0;
    int pos = bit0;
    const int end = bit0 + nbits;
    while (pos < end) {
        const int lo = pos & 7;
        const int take = min(8 - lo, end - pos);
        cnt += __popc(((unsigned)bm[pos >> 3] >> lo) & ((1u << take) - 1u));
        pos += take;
    }
    return cnt;
}

__global__ __launch_bounds__(256) void blocklist_count_kernel(int nh, int k, int nbytes, const uint8_t* __restrict__ bitmask,
                                                              int* __restrict__ row_ptr) {
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e >= nh * (k + 1)) return;
    const int h = e / (k + 1);
    const int i = e - h * (k + 1);
    row_ptr[e] = i < k ? count_bits(bitmask + (size_t)h * nbytes, i * k, k) : 0;
}

constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void blocklist_scan_kernel(int n, int* __restrict__ row_ptr, int* __restrict__ nnz_out) {
    __shared__ int part[kScanThreads];
    const int t = threadIdx.x;
    const int per = (n + kScanThreads - 1) / kScanThreads;
    const int lo = min(t * per, n), hi = min(lo + per, n);
    int sum = 0;
    for (int e = lo; e < hi; ++e) sum += row_ptr[e];
    part[t] = sum;
    __syncthreads();
    // inclusive Hillis-Steele scan over the 1024 partial sums
    for (int off = 1; off < kScanThreads; off <<= 1) {
        const int add = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    int run = part[t] - sum;  // exclusive prefix of this thread's chunk
    for (int e = lo; e < hi; ++e) {
        const int c = row_ptr[e];
        row_ptr[e] = run;
        run += c;
    }
    if (nnz_out && t == kScanThreads - 1) *nnz_out = part[t];
}

__global__ __launch_bounds__(256) void blocklist_fill_kernel(int nh, int k, int nbytes, const uint8_t* __restrict__ bitmask,
                                                             const int* __restrict__ row_ptr, int* __restrict__ col_idx, int cap) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nh * k) return;
    const int lane = threadIdx.x & 63;
    const int h = row / k;
    const int i = row - h * k;
    const uint8_t* bm = bitmask + (size_t)h * nbytes;
    int base = row_ptr[h * (k + 1) + i];
    for (int j0 = 0; j0 < k; j0 += 64) {
        const int j = j0 + lane;
        const int bit = i * k + j;
        const bool live = j < k && ((bm[bit >> 3] >> (bit & 7)) & 1);
        const unsigned long long b = __ballot(live);
        const int pos = base + __popcll(b & ((1ull << lane) - 1ull));
        if (live && (unsigned)pos < (unsigned)cap) col_idx[pos] = j;  // entries outside [0, cap) are dropped, never written
        base += __popcll(b);
    }
}

}  // namespace paro

extern "C" int paro_mask_to_blocklist_device(int nh, int k, const uint8_t* bitmask, int32_t* row_ptr, int32_t* col_idx,
                                             int64_t cap, int32_t* nnz_out, void* stream) {
    using namespace paro;
    if (nh < 1 || nh > kMaxHeads) return fail(PARO_EINVAL, "nh=%d out of range [1, %d]", nh, kMaxHeads);
    if (k < 1 || k > 32768) return fail(PARO_EINVAL, "k=%d out of range [1, 32768]", k);
    if (!bitmask || !row_ptr) return fail(PARO_EINVAL, "bitmask and row_ptr must not be NULL");
    if (cap < 0 || cap > 0x7fffffffLL) return fail(PARO_EINVAL, "cap=%lld out of range", (long long)cap);
    if (cap > 0 && !col_idx) return fail(PARO_EINVAL, "col_idx is NULL but cap=%lld", (long long)cap);
    if ((int64_t)nh * k * k > 0x7fffffffLL) return fail(PARO_EINVAL, "nh*k*k = %lld live blocks cannot be indexed with int32", (long long)nh * k * k);
    const int nbytes = (int)(((int64_t)k * k + 7) / 8);
    const int n = nh * (k + 1);
    hipStream_t st = (hipStream_t)stream;
    hipLaunchKernelGGL(blocklist_count_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, nh, k, nbytes, bitmask, row_ptr);
    hipLaunchKernelGGL(blocklist_scan_kernel, dim3(1), dim3(kScanThreads), 0, st, n, row_ptr, nnz_out);
    if (cap > 0)
        hipLaunchKernelGGL(blocklist_fill_kernel, dim3((unsigned)((nh * k + 3) / 4)), dim3(256), 0, st, nh, k, nbytes, bitmask, row_ptr,
                           col_idx, (int)cap);
    return check_launch("paro_mask_to_blocklist_device");
}

extern "C" int paro_blocklist_cols_device(int nh, int k, const uint8_t* bitmask, const int32_t* row_ptr, int32_t* col_idx,
                                          int64_t cap, void* stream) {
    using namespace paro;
    if (nh < 1 || nh > kMaxHeads) return fail(PARO_EINVAL, "nh=%d out of range [1, %d]", nh, kMaxHeads);
    if (k < 1 || k > 32768) return fail(PARO_EINVAL, "k=%d out of range [1, 32768]", k);
    if (!bitmask || !row_ptr || !col_idx) return fail(PARO_EINVAL, "bitmask, row_ptr and col_idx must not be NULL");
    if (cap < 1 || cap > 0x7fffffffLL) return fail(PARO_EINVAL, "cap=%lld out of range", (long long)cap);
    if ((int64_t)nh * k * k > 0x7fffffffLL) return fail(PARO_EINVAL, "nh*k*k = %lld live blocks cannot be indexed with int32", (long long)nh * k * k);
    const int nbytes = (int)(((int64_t)k * k + 7) / 8);
    hipLaunchKernelGGL(blocklist_fill_kernel, dim3((unsigned)((nh * k + 3) / 4)), dim3(256), 0, (hipStream_t)stream, nh, k, nbytes, bitmask,
                       row_ptr, col_idx, (int)cap);
    return check_launch("paro_blocklist_cols_device");
}
