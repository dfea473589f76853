"""nixie_place against the placement oracle on seeded random machines: every decision equal."""
import numpy as np
import pytest

from oracle import place_oracle as po


@pytest.mark.parametrize("seed", range(12))
def test_random_instances(seed):
    import paper_2601_11743_amd as nx
    rng = np.random.default_rng(1000 + seed)
    done = errors = 0
    for _ in range(300):
        n_apps = int(rng.integers(2, 6))
        n = int(rng.integers(1, 40))
        gpu_cap = int(rng.integers(1, 200)) << 20
        pin_cap = int(rng.integers(0, 100)) << 20
        chunks, g, p = [], 0, 0
        for i in range(n):
            b = int(rng.integers(0, 24 << 20)) if rng.random() < 0.9 else 0
            t = int(rng.integers(0, 3))
            if t == po.GPU and g + b > gpu_cap:
                t = po.PAGEABLE
            if t == po.PINNED and p + b > pin_cap:
                t = po.PAGEABLE
            g += b if t == po.GPU else 0
            p += b if t == po.PINNED else 0
            chunks.append((b, int(rng.integers(0, n_apps)), t))
        incoming = int(rng.integers(0, n_apps))
        victims = [int(a) for a in rng.permutation(n_apps) if a != incoming][: int(rng.integers(0, n_apps))]
        try:
            want = po.place(gpu_cap, pin_cap, chunks, incoming, victims)
        except po.PlacementError:
            with pytest.raises(nx.NixieError):
                nx.place(gpu_cap, pin_cap, chunks, incoming, victims)
            errors += 1
            continue
        got = nx.place(gpu_cap, pin_cap, chunks, incoming, victims)
        assert got[0] == want[0]
        assert got[1] == want[1]
        assert got[2] == want[2]
        done += 1
    assert done > 100 and errors > 5
