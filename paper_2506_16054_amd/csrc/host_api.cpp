// Host-only part of libparo: status text, shape arithmetic, the gather index of an axis order
// (paper Sec. 4.1), the PARO_VT slot map and the bitmask -> block-list conversion (Sec. 4.2).
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "common.h"

namespace paro {

static thread_local char g_last_error[512] = "";

int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_last_error, sizeof(g_last_error), fmt, ap);
    va_end(ap);
    return status;
}

int check_shape(const paro_shape* s, int64_t* n_tokens, int64_t* k_blocks) {
    if (!s) return fail(PARO_EINVAL, "shape is NULL");
    if (s->B < 1 || s->nh < 1) return fail(PARO_EINVAL, "B=%d nh=%d must be >= 1", s->B, s->nh);
    if ((int64_t)s->B * s->nh > 65535) return fail(PARO_EUNSUPPORTED, "B*nh=%lld exceeds 65535", (long long)s->B * s->nh);
    if (s->nh > kMaxHeads) return fail(PARO_EUNSUPPORTED, "nh=%d exceeds %d", s->nh, kMaxHeads);
    if (s->d != 64 && s->d != 128) return fail(PARO_EUNSUPPORTED, "d=%d: only 64 and 128 are built", s->d);
    if (s->block != 32 && s->block != 64)
        return fail(PARO_EUNSUPPORTED, "block=%d: only 32 and 64 are built", s->block);
    if (s->F < 1 || s->Hg < 1 || s->Wg < 1 || s->T_text < 0)
        return fail(PARO_EINVAL, "grid %dx%dx%d (+%d text) is not a valid token grid", s->F, s->Hg, s->Wg, s->T_text);
    const int64_t n = (int64_t)s->F * s->Hg * s->Wg + s->T_text;
    const int64_t k = (n + s->block - 1) / s->block;
    if (n > (1 << 24)) return fail(PARO_EUNSUPPORTED, "N=%lld exceeds 2^24 tokens", (long long)n);
    if ((int64_t)s->B * s->nh * k > (int64_t)1 << 30)
        return fail(PARO_EUNSUPPORTED, "B*nh*k=%lld exceeds the launch limit", (long long)((int64_t)s->B * s->nh * k));
    if (n_tokens) *n_tokens = n;
    if (k_blocks) *k_blocks = k;
    return PARO_OK;
}

int make_reorder_table(const paro_shape* s, const uint8_t* h_perm_ids, ReorderTable* t) {
    if (!h_perm_ids) return fail(PARO_EINVAL, "perm_ids is NULL");
    for (int h = 0; h < s->nh; ++h) {
        if (h_perm_ids[h] > 5) return fail(PARO_EINVAL, "perm_ids[%d]=%d not in 0..5", h, (int)h_perm_ids[h]);
        t->perm[h] = h_perm_ids[h];
    }
    t->n_img = s->F * s->Hg * s->Wg;
    t->n_tokens = t->n_img + s->T_text;
    t->Hg = s->Hg;
    t->Wg = s->Wg;
    const int dims[3] = {s->F, s->Hg, s->Wg};
    const int stride[3] = {s->Hg * s->Wg, s->Wg, 1};
    for (int p = 0; p < 6; ++p) {
        const AxisOrder o = axis_order(p);
        t->fwd[p][0] = dims[o.a[1]];
        t->fwd[p][1] = dims[o.a[2]];
        for (int i = 0; i < 3; ++i) t->fwd[p][2 + i] = stride[o.a[i]];
        t->inv[p][o.a[0]] = dims[o.a[1]] * dims[o.a[2]];
        t->inv[p][o.a[1]] = dims[o.a[2]];
        t->inv[p][o.a[2]] = 1;
    }
    return PARO_OK;
}

int check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(PARO_EHIP, "%s: %s", what, hipGetErrorString(e));
    return PARO_OK;
}

}  // namespace paro

using namespace paro;

extern "C" {

int paro_version(void) { return 1; }

const char* paro_strerror(int status) {
    switch (status) {
        case PARO_OK: return "ok";
        case PARO_EINVAL: return "invalid argument";
        case PARO_EUNSUPPORTED: return "unsupported configuration";
        case PARO_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

const char* paro_last_error(void) { return g_last_error; }

int64_t paro_ntokens(const paro_shape* s) {
    int64_t n, k;
    int st = check_shape(s, &n, &k);
    return st ? st : n;
}

int64_t paro_nblocks(const paro_shape* s) {
    int64_t n, k;
    int st = check_shape(s, &n, &k);
    return st ? st : k;
}

int64_t paro_npad(const paro_shape* s) {
    int64_t n, k;
    int st = check_shape(s, &n, &k);
    return st ? st : k * s->block;
}

int paro_perm_index(const paro_shape* s, int perm_id, int32_t* h_idx) {
    int64_t n, k;
    if (int st = check_shape(s, &n, &k)) return st;
    if (perm_id < 0 || perm_id > 5) return fail(PARO_EINVAL, "perm_id=%d not in 0..5", perm_id);
    if (!h_idx) return fail(PARO_EINVAL, "h_idx is NULL");
    const AxisOrder o = axis_order(perm_id);
    const int dims[3] = {s->F, s->Hg, s->Wg};
    const int stride[3] = {s->Hg * s->Wg, s->Wg, 1};
    // Walk the reordered sequence: the three loop counters are the coordinates along the
    // slowest, middle and fastest axis of the chosen order.
    int64_t pos = 0;
    for (int c0 = 0; c0 < dims[o.a[0]]; ++c0)
        for (int c1 = 0; c1 < dims[o.a[1]]; ++c1)
            for (int c2 = 0; c2 < dims[o.a[2]]; ++c2)
                h_idx[pos++] = c0 * stride[o.a[0]] + c1 * stride[o.a[1]] + c2 * stride[o.a[2]];
    for (; pos < n; ++pos) h_idx[pos] = (int32_t)pos;  // text tokens keep their place
    return PARO_OK;
}

int paro_vt_slot(int block, int i) {
    if (block != 32 && block != 64) return fail(PARO_EUNSUPPORTED, "block=%d: only 32 and 64 are built", block);
    if (i < 0 || i >= block) return fail(PARO_EINVAL, "token %d outside a block of %d", i, block);
    return vt_slot(i);
}

int paro_mask_to_blocklist(int nh, int k, const uint8_t* h_bitmask, int32_t* h_row_ptr, int32_t* h_col_idx,
                           int64_t cap, int64_t* nnz_out) {
    if (nh < 1 || k < 1) return fail(PARO_EINVAL, "nh=%d k=%d must be >= 1", nh, k);
    if (!h_bitmask || !h_row_ptr || !nnz_out) return fail(PARO_EINVAL, "h_bitmask, h_row_ptr and nnz_out must not be NULL");
    if (cap < 0 || (cap > 0 && !h_col_idx)) return fail(PARO_EINVAL, "h_col_idx is NULL but cap=%lld", (long long)cap);
    const int64_t bits = (int64_t)k * k;
    const int64_t bytes_per_head = (bits + 7) / 8;
    if ((int64_t)nh * bits >= ((int64_t)1 << 31)) return fail(PARO_EUNSUPPORTED, "block list offsets would overflow int32");
    int64_t nnz = 0;
    for (int h = 0; h < nh; ++h) {
        const uint8_t* m = h_bitmask + (int64_t)h * bytes_per_head;
        for (int i = 0; i < k; ++i) {
            h_row_ptr[(int64_t)h * (k + 1) + i] = (int32_t)nnz;
            for (int j = 0; j < k; ++j) {
                const int64_t bit = (int64_t)i * k + j;
                if ((m[bit >> 3] >> (bit & 7)) & 1) {
                    if (nnz < cap) h_col_idx[nnz] = j;
                    ++nnz;
                }
            }
        }
        h_row_ptr[(int64_t)h * (k + 1) + k] = (int32_t)nnz;
    }
    *nnz_out = nnz;
    if (nnz > cap) return fail(PARO_EINVAL, "h_col_idx holds %lld entries but the mask has %lld live blocks", (long long)cap, (long long)nnz);
    return PARO_OK;
}

int paro_check_blocklist(int nh, int k, const int32_t* h_row_ptr, const int32_t* h_col_idx, int64_t nnz) {
    if (nh < 1 || k < 1) return fail(PARO_EINVAL, "nh=%d k=%d must be >= 1", nh, k);
    if (!h_row_ptr) return fail(PARO_EINVAL, "h_row_ptr is NULL");
    if (nnz < 0 || nnz > 0x7fffffffLL) return fail(PARO_EINVAL, "nnz=%lld out of range", (long long)nnz);
    if (nnz > 0 && !h_col_idx) return fail(PARO_EINVAL, "h_col_idx is NULL but nnz=%lld", (long long)nnz);
    for (int h = 0; h < nh; ++h) {
        const int32_t* rp = h_row_ptr + (int64_t)h * (k + 1);
        for (int i = 0; i < k; ++i) {
            const int64_t beg = rp[i], end = rp[i + 1];
            if (beg < 0 || end < beg || end > nnz)
                return fail(PARO_EINVAL, "head %d row block %d: offsets [%lld, %lld) are not an ascending range inside [0, %lld]", h, i,
                            (long long)beg, (long long)end, (long long)nnz);
            if (end - beg > k) return fail(PARO_EINVAL, "head %d row block %d lists %lld blocks, more than k=%d", h, i, (long long)(end - beg), k);
            for (int64_t t = beg; t < end; ++t) {
                const int32_t j = h_col_idx[t];
                if (j < 0 || j >= k) return fail(PARO_EINVAL, "head %d row block %d: column block %d outside [0, %d)", h, i, j, k);
                if (t > beg && j <= h_col_idx[t - 1])
                    return fail(PARO_EINVAL, "head %d row block %d: column blocks %d, %d are not strictly ascending", h, i, h_col_idx[t - 1], j);
            }
        }
    }
    return PARO_OK;
}

int paro_check_row_order(const paro_shape* s, const int32_t* h_order) {
    int64_t n, k;
    if (int st = check_shape(s, &n, &k)) return st;
    if (!h_order) return fail(PARO_EINVAL, "h_order is NULL");
    const int64_t total = (int64_t)s->B * s->nh * k;
    std::vector<uint8_t> seen((size_t)total, 0);
    for (int64_t p = 0; p < total; ++p) {
        const int64_t id = h_order[p];
        if (id < 0 || id >= total) return fail(PARO_EINVAL, "launch position %lld names row block %lld outside [0, %lld)", (long long)p, (long long)id, (long long)total);
        if (seen[(size_t)id]) return fail(PARO_EINVAL, "row block %lld appears twice in the launch order (second time at position %lld)", (long long)id, (long long)p);
        seen[(size_t)id] = 1;
    }
    return PARO_OK;
}

int paro_schedule_rows(const paro_shape* s, int bits_qk, int bits_pv, const int32_t* h_row_ptr, int32_t* h_order) {
    int64_t n, k;
    if (int st = check_shape(s, &n, &k)) return st;
    if (!h_row_ptr || !h_order) return fail(PARO_EINVAL, "h_row_ptr and h_order must not be NULL");
    if ((bits_qk != 8 && bits_qk != 4 && bits_qk != 16) || (bits_pv != 8 && bits_pv != 4 && bits_pv != 16))
        return fail(PARO_EINVAL, "bits (qk=%d, pv=%d): expected 4, 8 or 16", bits_qk, bits_pv);
    const int64_t total = (int64_t)s->B * s->nh * k;
    const int64_t per_xcd = (total + 7) / 8;  // the kernels give launch positions [x*per_xcd, (x+1)*per_xcd) to XCD x
    // Heads whose K and V operands fit one XCD's L2 (4 MB) together are scheduled as one group, so
    // that starting the heaviest rows first never costs the L2 residency of K/V.  Groups are
    // aligned to whole heads; an XCD whose entire range fits the budget is a single group, so a
    // small problem gets a plain heaviest-first order and no late start of a long row.
    const int64_t kv_bytes = k * s->block * (int64_t)s->d * (bits_qk + bits_pv) / 8;
    const int64_t l2_budget = 4 << 20;
    const int64_t window = std::max<int64_t>(1, l2_budget / std::max<int64_t>(kv_bytes, 1));
    // Workgroups one XCD holds at a time (32 compute units x 8 one-wavefront workgroups of the d = 64 / block 64 / 8-bit
    // kernel, x 4 workgroups of the others).  A wavefront that has its SIMD to itself runs no faster than one that shares
    // it, so when the last group of an XCD runs out of row blocks the launch drains for as long as the last-started
    // rows take.  With several groups per XCD the lightest rows of the whole range - half as many as the XCD holds
    // workgroups - are therefore kept back and started last, heaviest first: they are the shortest filler there is,
    // and being few and short they cost the L2 little.
    const int64_t resident = (s->d == 64 && s->block == 64 && bits_qk == 8) ? 256 : 128;
    // Which (batch, head) an XCD works on.  Positions are in units of whole (batch, head) "slots" of k row blocks; slot
    // v holds head_at[v].  Masks made with one threshold per head (Sec. 4.2 (3)) can differ in live blocks from head to
    // head; when every XCD's range is a whole number of heads and the heads in their natural order would load some XCD
    // more than 2 % above the mean, heads are dealt heaviest first to the XCD with the least work that still has room.
    const int64_t n_heads = (int64_t)s->B * s->nh;
    std::vector<int64_t> head_at(n_heads);
    for (int64_t v = 0; v < n_heads; ++v) head_at[v] = v;
    if (per_xcd % k == 0 && total == 8 * per_xcd) {
        const int64_t hpx = per_xcd / k;
        std::vector<int64_t> work(n_heads), load(8, 0);
        int64_t sum = 0;
        for (int64_t v = 0; v < n_heads; ++v) {
            const int64_t h = v % s->nh;
            work[v] = (int64_t)h_row_ptr[h * (k + 1) + k] - h_row_ptr[h * (k + 1)];
            load[v / hpx] += work[v];
            sum += work[v];
        }
        if (*std::max_element(load.begin(), load.end()) * 8 * 100 > sum * 102) {
            std::vector<int64_t> by_work(n_heads);
            for (int64_t v = 0; v < n_heads; ++v) by_work[v] = v;
            std::stable_sort(by_work.begin(), by_work.end(), [&](int64_t a, int64_t b) { return work[a] > work[b]; });
            std::vector<std::vector<int64_t>> dealt(8);
            std::fill(load.begin(), load.end(), 0);
            for (int64_t v : by_work) {
                int best = -1;
                for (int x = 0; x < 8; ++x)
                    if ((int64_t)dealt[x].size() < hpx && (best < 0 || load[x] < load[best])) best = x;
                dealt[best].push_back(v);
                load[best] += work[v];
            }
            int64_t v = 0;
            for (int x = 0; x < 8; ++x) {
                std::sort(dealt[x].begin(), dealt[x].end());
                for (int64_t hd : dealt[x]) head_at[v++] = hd;
            }
        }
    }
    // ids below are positions in slot order: id -> row block head_at[id / k] * k + id % k
    auto item = [&](int32_t id) { return (int32_t)(head_at[id / k] * k + id % k); };
    auto live = [&](int32_t id) {
        const int64_t h = head_at[id / k] % s->nh, i = id % k;
        return h_row_ptr[h * (k + 1) + i + 1] - h_row_ptr[h * (k + 1) + i];
    };
    auto heavier = [&](int32_t a, int32_t b) { return live(a) > live(b); };
    std::vector<int32_t> ids, kept_back;
    std::vector<char> held;
    for (int x = 0; x < 8; ++x) {
        const int64_t lo = x * per_xcd, hi = std::min(total, (x + 1) * per_xcd);
        if (lo >= hi) continue;
        const bool one_group = ((hi - 1) / k - lo / k + 1) * kv_bytes <= l2_budget;
        const bool several_groups = !one_group && ((hi - 1) / k) / window != (lo / k) / window;
        held.assign(hi - lo, 0);
        kept_back.clear();
        if (several_groups) {
            ids.resize(hi - lo);
            for (int64_t t = lo; t < hi; ++t) ids[t - lo] = (int32_t)t;
            std::stable_sort(ids.begin(), ids.end(), [&](int32_t a, int32_t b) { return live(a) < live(b); });
            kept_back.assign(ids.begin(), ids.begin() + std::min<int64_t>(resident / 2, (hi - lo) / 4));
            for (int32_t id : kept_back) held[id - lo] = 1;
            std::stable_sort(kept_back.begin(), kept_back.end(), heavier);
        }
        int64_t pos = lo, out = lo;
        while (pos < hi) {
            const int64_t group = (pos / k) / window;
            int64_t end = pos;
            while (end < hi && (one_group || (end / k) / window == group)) ++end;
            ids.clear();
            for (int64_t t = pos; t < end; ++t)
                if (!held[t - lo]) ids.push_back((int32_t)t);
            std::stable_sort(ids.begin(), ids.end(), heavier);
            for (int32_t id : ids) h_order[out++] = item(id);
            pos = end;
        }
        for (int32_t id : kept_back) h_order[out++] = item(id);
    }
    return PARO_OK;
}

}  // extern "C"
