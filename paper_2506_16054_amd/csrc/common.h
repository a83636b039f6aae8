// Internal helpers shared by the translation units of libparo (not part of the public ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "paro.h"

namespace paro {

// Records the text returned by paro_last_error() for the calling thread; returns `status`.
int fail(int status, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Shape check shared by every entry point; fills N, k on success.
int check_shape(const paro_shape* s, int64_t* n_tokens, int64_t* k_blocks);

int check_launch(const char* what);

constexpr int kMaxHeads = 256;

// The six orders of (F,H,W), slowest axis first, numbered lexicographically over "FHW".
struct AxisOrder {
    int a[3];
};
__host__ __device__ inline AxisOrder axis_order(int perm_id) {
    switch (perm_id) {
        case 0: return {{0, 1, 2}};
        case 1: return {{0, 2, 1}};
        case 2: return {{1, 0, 2}};
        case 3: return {{1, 2, 0}};
        case 4: return {{2, 0, 1}};
        default: return {{2, 1, 0}};
    }
}

// Slot of token i of a block in the PARO_VT layout: inside every run of 32 tokens the index
// bits [q1 q0 g p1 p0] are stored as [g q1 q0 p1 p0].  A lane of the 32x32 matrix instruction
// that produced S^T holds, for one query, the keys 8q + 4g + p (q, p = 0..3) of each 32-key
// tile; with this order those 16 keys are 16 consecutive bytes of a V^T row.
__host__ __device__ inline int vt_slot(int i) {
    return (i & ~31) | ((i & 4) << 2) | ((i & 24) >> 1) | (i & 3);
}

}  // namespace paro
