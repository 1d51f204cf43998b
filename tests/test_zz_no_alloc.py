"""The entry point that allocates nothing (coop_bucket_by_owner_static: its workspace is a device array of the library)
against the entry point it is a variant of (coop_bucket_by_owner, workspace passed in), through the C ABI: two calls in
a row, the second with a smaller input, every output bit-equal; then the oracle's grouping as well."""
import gc

import numpy as np
import pytest
import torch

from oracle import coopref as R

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2310_12403_amd as P
    return P


def test_static_entry_equals_workspace_entry_twice_second_smaller(P):
    rng = np.random.default_rng(5)
    nv = 2_000_003
    big = torch.from_numpy(rng.integers(0, nv, size=3_000_017).astype(np.int32)).cuda()
    small = torch.from_numpy(rng.integers(0, nv, size=70_001).astype(np.int32)).cuda()
    # outputs preallocated once: the calls below allocate nothing, on either side of the boundary
    out = torch.empty_like(big)
    origin = torch.empty_like(big)
    offsets = torch.empty(65, dtype=torch.int64, device="cuda")
    for ids, n_parts, scheme in ((big, 64, P.COOP_OWNER_HASH), (small, 8, P.COOP_OWNER_RANGE), (small[:0], 3, P.COOP_OWNER_RANGE)):
        n = ids.numel()
        want = P.coop_bucket_by_owner(ids, nv, n_parts, scheme, seed=7)
        out.fill_(-1)
        origin.fill_(-1)
        offsets.fill_(-1)
        gc.collect()                 # (garbage of earlier tests goes now, not while the two readings below are apart)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        free_before = torch.cuda.mem_get_info()[0]
        got = P.coop_bucket_by_owner_static(ids, nv, n_parts, scheme, seed=7, out=out, origin=origin, offsets=offsets)
        torch.cuda.synchronize()
        # nothing new from torch's allocator and nothing new from the driver (a collection in between can only lower the first)
        assert torch.cuda.memory_allocated() <= before and torch.cuda.mem_get_info()[0] >= free_before
        P.coop_gather_status()
        assert torch.equal(got[0][:n], want[0]) and torch.equal(got[1][:n], want[1])
        assert torch.equal(got[2][: n_parts + 1], want[2])
        ref = R.bucket_by_owner(ids.cpu().numpy(), nv, n_parts, scheme, seed=7)
        assert np.array_equal(got[0][:n].cpu().numpy(), ref[0]) and np.array_equal(got[2][: n_parts + 1].cpu().numpy(), ref[2])


def test_static_entry_rejects_what_the_other_rejects(P):
    ids = torch.arange(100, dtype=torch.int32, device="cuda")
    for nv, n_parts in ((1000, 0), (1000, 65), (0, 4)):
        with pytest.raises(P.CoopError) as e:
            P.coop_bucket_by_owner_static(ids, nv, n_parts)
        assert e.value.code == -4
