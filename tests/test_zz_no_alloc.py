"""The allocation-free changeset entry point (ginex_changeset_noalloc) against
ginex_changeset, through the C ABI, list by list with tolerance zero: two calls in a row on
one GPU, the second on a smaller input, so that whatever the first call left in the
library's built-in scratch array must not leak into the second."""
import numpy as np
import pytest
import torch

import oracle
from workload import make_workload

pytestmark = pytest.mark.gpu

FIELDS = ("init_ids", "in_ids", "out_ids", "in_positions")


def compare(a, b):
    for k in FIELDS:
        assert torch.equal(getattr(a, k), getattr(b, k)), k
    assert np.array_equal(a.cs_offsets, b.cs_offsets)
    assert np.array_equal(a.miss_count, b.miss_count)
    assert np.array_equal(a.init_ready, b.init_ready)


def test_noalloc_changeset_equals_the_workspace_one_on_two_calls_in_a_row():
    import paper_2208_09151_amd as ginex
    assert torch.cuda.is_available()
    w = make_workload(1, device="cuda", features=False)
    cfg = w.cfg
    samp = ginex.sample_superbatch(w.offsets, w.indices, w.seeds.cuda(), w.seed_offsets.numpy(),
                                   cfg.fanout, rng_seed=0, with_adj=False)
    io = samp.ids_offsets
    print(f"[noalloc] first call: {int(io[-1])} ids, S={cfg.S}, cap={cfg.cap}", flush=True)
    want = ginex.changeset(cfg.num_nodes, samp.ids, io, cfg.cap)
    got = ginex.changeset(cfg.num_nodes, samp.ids, io, cfg.cap, builtin_scratch=True)
    compare(got, want)
    assert int(want.cs_offsets[-1]) > 0          # the recurrence really ran
    ref = oracle.changeset(cfg.num_nodes, samp.ids.cpu().numpy(), io, cfg.cap)
    for k in FIELDS:
        assert np.array_equal(getattr(got, k).cpu().numpy(), ref[k]), k
    assert np.array_equal(got.miss_count, ref["miss_count"])

    # second call, smaller: fewer nodes, fewer iterations, a smaller cache
    rng = np.random.default_rng(3)
    n2, S2, cap2 = 700, 5, 60
    tr = [rng.choice(n2, size=int(rng.integers(20, 200)), replace=False) for _ in range(S2)]
    ids2 = torch.as_tensor(np.concatenate(tr).astype(np.int32)).cuda()
    io2 = np.cumsum([0] + [len(x) for x in tr]).astype(np.int64)
    print(f"[noalloc] second call: {int(io2[-1])} ids, S={S2}, cap={cap2}", flush=True)
    got2 = ginex.changeset(n2, ids2, io2, cap2, builtin_scratch=True)
    want2 = ginex.changeset(n2, ids2, io2, cap2)
    compare(got2, want2)
    ref2 = oracle.changeset(n2, ids2.cpu().numpy(), io2, cap2)
    for k in FIELDS:
        assert np.array_equal(getattr(got2, k).cpu().numpy(), ref2[k]), k
    assert np.array_equal(got2.miss_count, ref2["miss_count"])
    # and the first input once more: the smaller call left nothing behind that matters
    compare(ginex.changeset(cfg.num_nodes, samp.ids, io, cfg.cap, builtin_scratch=True), want)


def test_noalloc_changeset_rejects_shapes_beyond_its_scratch_array():
    import paper_2208_09151_amd as ginex
    io = np.array([0, 1 << 22, 1 << 23], dtype=np.int64)     # 8 M ids: 128 MiB of sort buffers
    ids = torch.zeros(1, dtype=torch.int32, device="cuda")   # never read: rejected on the host
    with pytest.raises(ginex.GinexError) as err:
        ginex.changeset(1 << 24, ids, io, 1000, builtin_scratch=True)
    assert err.value.code == -3 and "scratch" in str(err.value)
