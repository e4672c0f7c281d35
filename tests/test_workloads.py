"""The seeded input generators: determinism, exact counts, storage rounding."""
import numpy as np

import workloads as wl


def test_configs_have_the_stated_shapes_and_counts():
    want = {1: (128, 256, 256, 16, 16, None), 2: (128, 3072, 3072, 32, 32, 922),
            3: (4096, 768, 3072, 16, 16, 1843), 4: (256, 4096, 4096, 16, 1, 52429)}
    for cid, (m, k, n, br, bc, nnzb) in want.items():
        p = wl.config(cid)
        assert (p.m, p.k, p.n, p.bs_r, p.bs_c) == (m, k, n, br, bc)
        assert p.X.shape == (m, k) and p.block_data.shape == (p.nnzb, br, bc)
        assert p.index_pointer[0] == 0 and p.index_pointer[-1] == p.nnzb
        if nnzb is not None:
            assert p.nnzb == nnzb
        for r in range(n // br):                     # sorted, unique, in range
            seg = p.block_indices[p.index_pointer[r]:p.index_pointer[r + 1]]
            assert np.all(np.diff(seg) > 0) and (seg.size == 0 or (seg[0] >= 0 and seg[-1] < k // bc))


def test_config_is_reproducible():
    a, b = wl.config(2, m=4), wl.config(2, m=4)
    assert np.array_equal(a.X, b.X) and np.array_equal(a.block_data, b.block_data)
    assert np.array_equal(a.block_indices, b.block_indices)


def test_power_law_profile():
    p = wl.config(5, m=1)
    counts = np.diff(p.index_pointer)
    assert counts.sum() == 819 and counts.max() == 128 and counts.min() >= 1
    top = sorted(counts.tolist(), reverse=True)[:6]
    assert top == [128, 111, 69, 49, 37, 30]
    assert int((counts == 1).sum()) == 56


def test_storage_rounding_is_exact_in_the_storage_type():
    import torch
    x = np.random.default_rng(0).normal(size=4096).astype(np.float32)
    for name, tdt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
        r = wl.round_to_storage(x, name)
        t = torch.from_numpy(x).to(tdt).to(torch.float32).numpy()
        assert np.array_equal(r, t)                  # same nearest-even rounding as torch
    assert wl.config(3, m=2).in_dtype == "bf16"


def test_flops_and_bytes():
    p = wl.config(2)
    assert p.flops == 2 * 128 * 922 * 32 * 32
    assert p.algorithmic_bytes() == 128 * 3072 * 4 + 922 * 1024 * 4 + 4 * (922 + 97) + 128 * 3072 * 4
