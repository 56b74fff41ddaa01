"""The entry point that allocates nothing (ptq4vm_validate_scales_static) against the entry point it is a variant
of (ptq4vm_validate_scales with a caller-provided workspace): same counts, on two calls in a row that share the
library's static device array, the second with a smaller input.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import paper_2412_20386_amd as ptq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BAD = [0.0, -1.0, float("nan"), float("inf"), float("-inf"), -0.0]


def _vectors(seed, sizes, plant):
    g = torch.Generator().manual_seed(seed)
    vecs = [torch.rand(n, generator=g) + 0.01 for n in sizes]
    if plant:
        for vi, v in enumerate(vecs):
            for j, b in enumerate(BAD):
                if j < v.numel():
                    v[(j * 2741 + 13 * vi) % v.numel()] = b
    want = [int(np.count_nonzero(~((a > 0) & np.isfinite(a)))) for a in (v.numpy() for v in vecs)]
    return [v.to(DEV) for v in vecs], want


def _both(vecs):
    rc, counts = ptq.validate_scales(*vecs)
    static_counts = torch.full((3,), -7, dtype=torch.int32, device=DEV)
    ptq.validate_scales_static(*vecs, static_counts)
    torch.cuda.synchronize()
    return rc, counts.cpu().tolist(), static_counts.cpu().tolist()


def test_static_scratch_variant_matches_workspace_variant():
    # large first (73 partial-count slots of the static array are written), then small (4 slots): stale slots of the
    # first call must not leak into the second
    for seed, sizes, plant in [(1, (150000, 90000, 57000), True), (2, (197, 768, 3072), True),
                               (3, (50000, 4096, 12288), False), (4, (5, 1, 3), True)]:
        vecs, want = _vectors(seed, sizes, plant)
        rc, counts, static_counts = _both(vecs)
        assert counts == want and static_counts == counts, (sizes, want, counts, static_counts)
        assert rc == (-6 if any(want) else 0)


def test_static_scratch_variant_limits_and_absent_vectors():
    counts = torch.zeros(3, dtype=torch.int32, device=DEV)
    ok = torch.ones(8, device=DEV)
    ptq.validate_scales_static(ok, None, None, counts)
    torch.cuda.synchronize()
    assert counts.cpu().tolist() == [0, 0, 0]
    lib = ptq.binding.load()
    too_many = (1 << 24) - 7  # + 8 entries of the other vector: one more than the array covers; rejected before any launch
    assert lib.ptq4vm_validate_scales_static(ok.data_ptr(), too_many, ok.data_ptr(), 8, None, 0, counts.data_ptr(), None) == -2
