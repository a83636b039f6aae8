// Exercises the host-only entry points of the library (shape arithmetic, reorder index, bitmask ->
// block list, launch schedule, slot map, argument rejection); tests/test_host_sanitizers.py builds it
// together with csrc/host_api.cpp under AddressSanitizer and UndefinedBehaviorSanitizer and runs it.
#include <stdio.h>
#include <stdlib.h>
#include <vector>
#include "paro.h"
int main() {
    paro_shape s = {1, 3, 64, 5, 12, 13, 0, 64};
    int64_t n = paro_ntokens(&s), k = paro_nblocks(&s);
    std::vector<int32_t> idx(n);
    for (int p = 0; p < 6; ++p) if (paro_perm_index(&s, p, idx.data())) return 1;
    const int64_t nbytes = (k * k + 7) / 8;
    std::vector<uint8_t> bm(3 * nbytes);
    srand(1);
    for (auto& b : bm) b = (uint8_t)rand();
    std::vector<int32_t> rp(3 * (k + 1));
    int64_t nnz = 0;
    paro_mask_to_blocklist(3, (int)k, bm.data(), rp.data(), nullptr, 0, &nnz);
    std::vector<int32_t> ci(nnz);
    if (paro_mask_to_blocklist(3, (int)k, bm.data(), rp.data(), ci.data(), nnz, &nnz)) return 2;
    std::vector<int32_t> order(3 * k);
    if (paro_schedule_rows(&s, 8, 8, rp.data(), order.data())) return 3;
    for (int i = 0; i < 64; ++i) if (paro_vt_slot(64, i) < 0) return 4;
    paro_shape bad = {0, 3, 64, 5, 12, 13, 0, 64};
    if (paro_ntokens(&bad) >= 0) return 5;
    printf("host api under sanitizers: ok (N=%lld k=%lld nnz=%lld) %s\n", (long long)n, (long long)k, (long long)nnz, paro_last_error());
    return 0;
}
