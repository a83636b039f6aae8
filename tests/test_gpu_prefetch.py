"""GPU parity of the mask-prefetch path (paper Sec. 4.2 (1), App. C "Overhead of Prefetch"): the
device-side bitmask expansion against the oracle's block list, bit for bit, and the double-buffered
sequence of attention calls against the same calls with host-built block lists."""
import numpy as np
import pytest

from oracle import paro_oracle as po
from paper_2506_16054_amd import workloads as wl
from tests.helpers import gather_fn

pytestmark = pytest.mark.gpu


def _mods():
    import torch

    from paper_2506_16054_amd import binding as pb

    return torch, pb


def random_bitmask(rng, nh, k, density, garbage_tail=False):
    masks = rng.random((nh, k, k)) < density
    bits = wl.pack_bitmask(masks)
    if garbage_tail and (k * k) % 8:
        bits = bits.copy()
        bits[:, -1] |= np.uint8((0xFF << ((k * k) % 8)) & 0xFF)  # bits at or above k*k must be ignored
    return bits


def expand_on_device(nh, k, bits, cap=None):
    torch, pb = _mods()
    dev = "cuda:0"
    cap = nh * k * k if cap is None else cap
    d_bits = torch.from_numpy(bits).to(dev)
    row_ptr = torch.full((nh, k + 1), -7, dtype=torch.int32, device=dev)
    col_idx = torch.full((cap + 16,), -7, dtype=torch.int32, device=dev)  # 16 guard entries behind the capacity
    nnz = torch.full((1,), -7, dtype=torch.int32, device=dev)
    pb.paro_mask_to_blocklist_device(nh, k, d_bits, row_ptr, col_idx[:cap] if cap else None, nnz)
    torch.cuda.synchronize()
    return row_ptr.cpu().numpy(), col_idx.cpu().numpy(), int(nnz.item())


@pytest.mark.parametrize("nh,k,density", [(1, 1, 1.0), (1, 1, 0.0), (2, 7, 0.5), (3, 64, 0.3), (2, 65, 0.3), (5, 130, 0.1),
                                          (4, 33, 0.0), (2, 40, 1.0), (48, 275, 0.3)])
def test_device_blocklist_equals_oracle(nh, k, density):
    rng = np.random.default_rng([91, nh, k])
    bits = random_bitmask(rng, nh, k, density, garbage_tail=True)
    ref_ptr, ref_cols = po.mask_to_blocklist(bits, nh, k)
    row_ptr, col_idx, nnz = expand_on_device(nh, k, bits)
    assert nnz == ref_cols.size
    assert np.array_equal(row_ptr, ref_ptr)
    assert np.array_equal(col_idx[:nnz], ref_cols)
    assert np.all(col_idx[nnz:] == -7)  # nothing written past the list


def test_device_blocklist_truncates_at_capacity_without_overrun():
    nh, k = 3, 50
    rng = np.random.default_rng(92)
    bits = random_bitmask(rng, nh, k, 0.4)
    ref_ptr, ref_cols = po.mask_to_blocklist(bits, nh, k)
    cap = ref_cols.size // 2
    row_ptr, col_idx, nnz = expand_on_device(nh, k, bits, cap=cap)
    assert nnz == ref_cols.size and np.array_equal(row_ptr, ref_ptr)  # offsets and total still complete
    assert np.array_equal(col_idx[:cap], ref_cols[:cap])
    assert np.all(col_idx[cap:] == -7)
    row_ptr0, _, nnz0 = expand_on_device(nh, k, bits, cap=0)  # offsets only
    assert nnz0 == ref_cols.size and np.array_equal(row_ptr0, ref_ptr)


@pytest.mark.parametrize("nh,k,density", [(1, 1, 1.0), (3, 64, 0.3), (2, 65, 0.5), (48, 275, 0.3)])
def test_columns_from_precomputed_offsets_equal_oracle(nh, k, density):
    """paro_blocklist_cols_device: offsets computed offline (here by the oracle), columns written on the device."""
    torch, pb = _mods()
    rng = np.random.default_rng([93, nh, k])
    bits = random_bitmask(rng, nh, k, density, garbage_tail=True)
    ref_ptr, ref_cols = po.mask_to_blocklist(bits, nh, k)
    cap = max(int(ref_cols.size), 1)
    col_idx = torch.full((cap + 16,), -7, dtype=torch.int32, device="cuda:0")
    pb.paro_blocklist_cols_device(nh, k, torch.from_numpy(bits).to("cuda:0"), torch.from_numpy(ref_ptr).to("cuda:0"), col_idx[:cap])
    torch.cuda.synchronize()
    got = col_idx.cpu().numpy()
    assert np.array_equal(got[: ref_cols.size], ref_cols)
    assert np.all(got[cap:] == -7)


def test_columns_with_corrupt_offsets_stay_inside_the_list():
    torch, pb = _mods()
    nh, k = 2, 40
    rng = np.random.default_rng(94)
    bits = random_bitmask(rng, nh, k, 0.5)
    ref_ptr, ref_cols = po.mask_to_blocklist(bits, nh, k)
    bad = ref_ptr.copy()
    bad[0, 3] = -1000          # would land before the array
    bad[1, 7] = 2 ** 30        # would land far behind it
    cap = int(ref_cols.size)
    buf = torch.full((cap + 64,), -7, dtype=torch.int32, device="cuda:0")
    pb.paro_blocklist_cols_device(nh, k, torch.from_numpy(bits).to("cuda:0"), torch.from_numpy(bad).to("cuda:0"), buf[32: 32 + cap])
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    assert np.all(got[:32] == -7) and np.all(got[32 + cap:] == -7)  # guard zones on both sides untouched


@pytest.mark.parametrize("lists_on_host", [False, True])
def test_prefetched_sequence_is_bit_identical_to_host_built_lists(lists_on_host):
    """Five 'timesteps' with different masks through the two slots, two rounds without any host
    synchronisation in between: every output equals the one obtained with that mask's host-built
    block list - with the masks expanded on the device, and with the expanded lists kept on the host."""
    torch, pb = _mods()
    from paper_2506_16054_amd.pipeline import MaskPrefetcher, ParoAttention

    w = wl.Workload("video64_steps", 1, 3, 64, 5, 12, 13, 0, 64, 0.4, 8, 8, "bf16", 31, perm_choice=(3, 0, 5))
    s = pb.shape_of(w)
    perm_ids = wl.make_perm_ids(w)
    densities = (0.2, 0.5, 0.35, 1.0, 0.1)
    bitmasks = [wl.pack_bitmask(wl.make_block_masks(w.replace(density=rho), gather_fn(w), perm_ids)) for rho in densities]
    q, k, v = (torch.from_numpy(x).to("cuda:0").to(torch.bfloat16) for x in wl.make_qkv(w))

    # reference: one ParoAttention per mask, block list built on the host
    want = []
    for bm in bitmasks:
        pa = ParoAttention(s, perm_ids, bm, w.bits_qk, w.bits_pv, torch.bfloat16)
        want.append(pa.run_fused(q, k, v).clone())
    orders = np.stack([pb.paro_schedule_rows(s, w.bits_qk, w.bits_pv, pb.paro_mask_to_blocklist(w.nh, w.k, bm)[0]) for bm in bitmasks])

    pa = ParoAttention(s, perm_ids, bitmasks[0], w.bits_qk, w.bits_pv, torch.bfloat16)
    pf = MaskPrefetcher(s, np.stack(bitmasks), orders, lists_on_host=lists_on_host)
    T = len(bitmasks)
    steps = 2 * T
    got = []
    pf.prefetch(0, 0)
    for i in range(steps):
        slot = i & 1
        if i + 1 < steps:
            pf.prefetch(slot ^ 1, (i + 1) % T)  # load the next mask while this step computes
        pa.prepare_fused(q, k, v)
        pa.use_blocklist(*pf.acquire(slot))
        got.append(pa.attend_fused().clone())
        pf.release(slot)
    torch.cuda.synchronize()
    for i, o in enumerate(got):
        assert torch.equal(o, want[i % T]), "step %d (mask %d) differs from the host-built block list" % (i, i % T)
    # and at least two of the masks give different outputs, so the comparison can tell them apart
    assert not torch.equal(want[0], want[3])

