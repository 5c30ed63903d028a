"""The seeded input generators: counter-based, sliceable, and identical to a scalar reference."""
import numpy as np
import torch

import workloads as wl


def test_splitmix_matches_scalar_reference():
    got = wl.raw_bits(7, 5, 64).numpy().view(np.uint64)
    want = [wl.splitmix64_py(((7 << 40) + i) & ((1 << 64) - 1)) for i in range(5, 69)]
    assert [int(x) for x in got] == want


def test_streams_are_sliceable():
    for cfg in wl.configs():
        whole = cfg.gen_data(0, 3)
        part = cfg.gen_data(1, 2)
        assert torch.equal(wl.bits_view(whole)[cfg.tile_elems:], wl.bits_view(part))
    c5 = wl.config(5)
    assert torch.equal(c5.gen_idx(0, 2)[c5.tile_elems:], c5.gen_idx(1, 1))


def test_value_ranges():
    c1, c2, c3, c5 = wl.config(1), wl.config(2), wl.config(3), wl.config(5)
    x = c1.gen_data(0, 1)
    assert x.dtype == torch.int32 and x.min() < -(1 << 29) and x.max() > (1 << 29)
    y = c2.gen_data(0, 1).float()
    assert y.min() >= -1.0 and y.max() <= 1.0 and abs(float(y.mean())) < 0.05
    z = c3.gen_data(0, 4)
    assert abs(float(z.mean())) < 0.05 and abs(float(z.std()) - 1.0) < 0.05
    i = c5.gen_idx(0, 1)
    assert i.dtype == torch.int32 and int(i.min()) == 0 and int(i.max()) == 63


def test_config_shapes_and_bases():
    sizes = {1: (12, 4, 1), 2: (14, 2, 8192), 3: (12, 4, 32768), 4: (16, 4, 4096), 5: (14, 2, 16384)}
    for cfg in wl.configs():
        d, w, nt = sizes[cfg.cid]
        assert (cfg.d, cfg.elem_bytes, cfg.ntiles) == (d, w, nt)
        assert len(cfg.src_bases) == d and sum(cfg.out_dim_bits) == d
        for bases in (cfg.src_bases, cfg.dst_bases):
            if bases is None:
                continue
            assert len(bases) == d
            if cfg.cid != 4:        # permutation layouts: the columns are the d distinct unit vectors
                assert sorted(bases) == [1 << k for k in range(d)]
    c4 = wl.config(4)
    assert any(bin(c).count("1") >= 2 for c in c4.src_bases)
    assert any(bin(c).count("1") >= 2 for c in c4.dst_bases)
    assert wl.config(2).algorithmic_bytes() == 512 << 20
    assert wl.config(3).algorithmic_bytes() == 1 << 30
    assert wl.config(4).algorithmic_bytes() == 2 << 30
    assert wl.config(5).algorithmic_bytes() == 2 << 30
