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

// Everything a kernel needs to map a position of a head's reordered sequence to the position of
// the same token in the default [F,H,W] order (and back), for all six axis orders at once.
struct ReorderTable {
    int n_tokens;   // N
    int n_img;      // F*Hg*Wg; tokens at or beyond it are text and keep their place
    int Hg, Wg;
    int fwd[6][5];  // per axis order: extents of the middle and fastest axis, then the default-order
                    // stride of the slowest, middle and fastest axis
    int inv[6][3];  // per axis order: multiplier of the f, h and w coordinate in the reordered position
    uint8_t perm[kMaxHeads];
};

// Fills `t` from the shape and the per-head order ids (host pointer); rejects ids above 5.
int make_reorder_table(const paro_shape* s, const uint8_t* h_perm_ids, ReorderTable* t);

// Default-order position of the token that sits at position n_new of head `head`'s sequence.
__device__ inline int reorder_source(const ReorderTable& t, int head, int n_new) {
    if (n_new >= t.n_img) return n_new;
    const int* f = t.fwd[t.perm[head]];
    const int c2 = n_new % f[1];
    const int q = n_new / f[1];
    const int c1 = q % f[0];
    const int c0 = q / f[0];
    return c0 * f[2] + c1 * f[3] + c2 * f[4];
}

// Position in head `head`'s reordered sequence of the token at default-order position n.
__device__ inline int reorder_dest(const ReorderTable& t, int head, int n) {
    if (n >= t.n_img) return n;
    const int* mul = t.inv[t.perm[head]];
    const int w = n % t.Wg;
    const int q = n / t.Wg;
    return (q / t.Hg) * mul[0] + (q % t.Hg) * mul[1] + w * mul[2];
}

// x / scale, correctly rounded, for the many elements of a quantization group that share one divisor
// (Sec. 4.3 (1): one scale per block).  With y the correctly rounded reciprocal of the divisor,
// q0 = RN(x y) and r = x - q0 scale (one fma), RN(q0 + r y) is the correctly rounded quotient
// (Markstein's division theorem).  The theorem excludes divisors whose significand is all ones, and
// the reciprocal must be a normal number: those groups take the generic divide.  Either way the
// result equals fl32(x / scale) bit for bit.  Compile with correctly rounded fp32 division.
struct GroupDivider {
    float scale, inv;
    bool generic;
    __device__ explicit GroupDivider(float s)
        : scale(s), inv(1.0f / s), generic((__float_as_uint(s) & 0x7fffffu) == 0x7fffffu || !(s > 1e-20f && s < 1e20f)) {}
    __device__ float operator()(float v) const {
        if (generic) return v / scale;
        const float q0 = v * inv;
        const float rem = fmaf(-q0, scale, v);
        return fmaf(rem, inv, q0);
    }
};

// Slot of token i of a block in the PARO_VT layout: inside every run of 32 tokens the index
// bits [q1 q0 g p1 p0] are stored as [g q1 q0 p1 p0].  A lane of the 32x32 matrix instruction
// that produced S^T holds, for one query, the keys 8q + 4g + p (q, p = 0..3) of each 32-key
// tile; with this order those 16 keys are 16 consecutive bytes of a V^T row.
__host__ __device__ inline int vt_slot(int i) {
    return (i & ~31) | ((i & 4) << 2) | ((i & 24) >> 1) | (i & 3);
}

}  // namespace paro
