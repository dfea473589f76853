"""Pins for the CPU oracle (no GPU).  Each test fixes the oracle to something
other than itself: a library copy, brute force, a published vector, an
invariant, or a planted mistake that a check must catch."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import OracleError, FAULTS
from tests.helpers import HostSet, AliasedPair, RED

G = 0x9E3779B97F4A7C15
M = (1 << 64) - 1
KiB, MiB = 1 << 10, 1 << 20


def _golden():
    p = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_seed0.txt")
    return [int(l, 16) for l in open(p) if l.strip() and not l.startswith("#")]


# ---- mix64 / hash ----------------------------------------------------------

def py_mix64(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    return z ^ (z >> 31)


def py_hash64(b: bytes) -> int:
    """Independent big-integer evaluation of the per-allocation hash."""
    h = py_mix64(len(b))
    for k in range((len(b) + 7) // 8):
        w = int.from_bytes(b[8 * k:8 * k + 8].ljust(8, b"\0"), "little")
        h = (h + py_mix64((w + G * (k + 1)) & M)) & M
    return h


def test_mix64_published_vectors(oracle):
    gold = _golden()
    assert [oracle.mix64(G * (k + 1)) for k in range(4)] == gold
    assert [int(x) for x in W.splitmix64_stream(0, 4)] == gold
    assert [py_mix64((G * (k + 1)) & M) for k in range(4)] == gold


def test_hash_anchored_on_published_vectors(oracle):
    gold = _golden()
    z16 = np.zeros(16, np.uint8)
    # word 1 changed from 0 to G: its term moves from mix64(2G) to mix64(3G)
    b = z16.copy(); b[8:16] = np.frombuffer(G.to_bytes(8, "little"), np.uint8)
    assert (oracle.hash64(b) - oracle.hash64(z16)) & M == (gold[2] - gold[1]) & M
    # word 0 changed from 0 to G: mix64(G) -> mix64(2G)
    c = z16.copy(); c[0:8] = np.frombuffer(G.to_bytes(8, "little"), np.uint8)
    assert (oracle.hash64(c) - oracle.hash64(z16)) & M == (gold[1] - gold[0]) & M
    # an 8-byte zero buffer is mix64(8) + mix64(G)
    assert oracle.hash64(np.zeros(8, np.uint8)) == (py_mix64(8) + gold[0]) & M
    assert oracle.hash64(np.zeros(0, np.uint8)) == 0  # mix64(0) = 0, no words


@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 15, 16, 17, 63, 64, 65, 1000, 4099])
def test_hash_matches_bigint_python(oracle, n):
    data = W.content_bytes(77, n, n)
    assert oracle.hash64(data) == py_hash64(data.tobytes())


def test_hash_properties(oracle):
    data = W.content_bytes(3, 0, 257).copy()
    h = oracle.hash64(data)
    for pos in (0, 1, 8, 128, 255, 256):   # any one byte matters, also in the padded tail word
        d = data.copy(); d[pos] ^= 1
        assert oracle.hash64(d) != h
    # position keyed: swapping two different words changes the hash
    d = data.copy(); d[0:8], d[8:16] = data[8:16].copy(), data[0:8].copy()
    assert oracle.hash64(d) != h
    # length keyed: trailing zero bytes are not ignored
    z = np.zeros(24, np.uint8)
    assert oracle.hash64(z[:17]) != oracle.hash64(z[:24])


# ---- result definition -----------------------------------------------------

def _sets(sizes_a, sizes_b, seed=11, **kw):
    return (HostSet(sizes_a, seed, "dev", **kw), HostSet(sizes_b, seed + 1, "host", **kw))


def test_direct_equals_library_copy(oracle):
    A, B = _sets([1, 15, 16, 17, 4096, 70001, 0, 3], [5, 0, 65536, 99999])
    dev_before = [d.copy() for d, _ in A.pairs()]
    host_before = [h.copy() for _, h in B.pairs()]
    oracle.switch_direct(A.pairs(), B.pairs())
    for (d, h), ref in zip(A.pairs(), dev_before):
        assert np.array_equal(h, ref)            # numpy slicing copy as the library routine
    for (d, h), ref in zip(B.pairs(), host_before):
        assert np.array_equal(d, ref)
    A.check_moved(); B.check_moved()


def test_direct_brute_force_tiny(oracle):
    """Byte-by-byte Python loops on a tiny input."""
    A, B = _sets([3, 40, 1], [17, 2])
    exp_host = {}
    for i, (d, h) in enumerate(A.pairs()):
        exp_host[i] = [int(d[k]) for k in range(d.size)]
    exp_dev = {}
    for j, (d, h) in enumerate(B.pairs()):
        exp_dev[j] = [int(h[k]) for k in range(h.size)]
    oracle.switch_direct(A.pairs(), B.pairs())
    for i, (d, h) in enumerate(A.pairs()):
        assert [int(x) for x in h] == exp_host[i]
    for j, (d, h) in enumerate(B.pairs()):
        assert [int(x) for x in d] == exp_dev[j]


def test_direct_empty_tables(oracle):
    A, B = _sets([100, 200], [300])
    oracle.switch_direct(A.pairs(), [])
    A.check_moved()
    for d, h in B.pairs():
        assert (d == 0xA5).all()                 # untouched
    oracle.switch_direct([], B.pairs())
    B.check_moved()
    oracle.switch_direct([], [])


# ---- staged form -------------------------------------------------------------

S = 4 * KiB


@pytest.mark.parametrize("pack", [False, True])
@pytest.mark.parametrize("seed", [0, 1, 2, 12345])
def test_staged_equals_direct_and_invariants(oracle, pack, seed):
    sizes_a = [1, 15, 16, 17, S - 1, S, S + 1, 3 * S + 5, 0, 10 * S]
    sizes_b = [S + 1, 2, 7 * S - 3, 0, 31]
    A, B = _sets(sizes_a, sizes_b)
    R = 8 * S
    rep = oracle.switch_staged(A.pairs(), B.pairs(), R, S, pack=pack, seed=seed, check_bytes=True)
    A.check_moved(); B.check_moved()
    assert rep["hwm_staged_bytes"] <= R
    assert rep["final_staged_bytes"] == 0
    assert rep["count_errors"] == 0
    assert rep["bytes_out"] == sum(sizes_a) and rep["bytes_in"] == sum(sizes_b)
    # same final state as the direct definition on a second copy of the inputs
    A2, B2 = _sets(sizes_a, sizes_b)
    oracle.switch_direct(A2.pairs(), B2.pairs())
    assert np.array_equal(A.host, A2.host) and np.array_equal(B.dev, B2.dev)


def test_staged_chunk_counts_closed_form(oracle):
    sizes = [S, 2 * S, S // 2, S // 2, 1]
    A, B = _sets(sizes, [])
    rep = oracle.switch_staged(A.pairs(), [], 4 * S, S, pack=False, seed=3)
    assert rep["n_out_chunks"] == 1 + 2 + 1 + 1 + 1      # ceil(size / S) per allocation
    A, B = _sets(sizes, [])
    rep = oracle.switch_staged(A.pairs(), [], 4 * S, S, pack=True, seed=3)
    assert rep["n_out_chunks"] == -(-sum(sizes) // S)     # ceil(total / S) when packed
    assert rep["n_in_chunks"] == 0


@pytest.mark.parametrize("skew", [(1, 0), (0, 7), (15, 9), (3, 3)])
def test_staged_unaligned_bases(oracle, skew):
    A, B = _sets([100, 1000, S + 3], [999, 16], skew_dev=skew[0], skew_host=skew[1])
    oracle.switch_staged(A.pairs(), B.pairs(), 4 * S, S, seed=5, check_bytes=True)
    A.check_moved(); B.check_moved()


@pytest.mark.parametrize("n_out_slots", [1, 2, 5, 7])
def test_staged_uneven_ring_split(oracle, n_out_slots):
    A, B = _sets([9 * S + 1, 77], [5 * S, 3])
    rep = oracle.switch_staged(A.pairs(), B.pairs(), 8 * S, S, n_out_slots=n_out_slots,
                               seed=9, check_bytes=True)
    A.check_moved(); B.check_moved()
    assert rep["hwm_staged_bytes"] <= 8 * S


def test_staged_order_independence(oracle):
    """Every seed (chunk order, slot choice, interleaving) gives the same bytes."""
    sizes_a, sizes_b = [5 * S + 1, 300, 2 * S], [4 * S, 11, 6 * S + 9]
    ref = None
    for seed in range(12):
        A, B = _sets(sizes_a, sizes_b)
        oracle.switch_staged(A.pairs(), B.pairs(), 6 * S, S, seed=seed, pack=bool(seed & 1))
        state = (A.host.tobytes(), B.dev.tobytes())
        ref = ref or state
        assert state == ref


def test_staged_pure_evict_and_pure_restore(oracle):
    A, B = _sets([3 * S + 1, 5], [2 * S, 9])
    rep = oracle.switch_staged(A.pairs(), [], 2 * S, S, seed=1, check_bytes=True)
    assert rep["n_in_chunks"] == 0
    A.check_moved()
    rep = oracle.switch_staged([], B.pairs(), 2 * S, S, seed=1, check_bytes=True)
    assert rep["n_out_chunks"] == 0
    B.check_moved()
    oracle.switch_staged([], [], 2 * S, S)


def test_staged_rejects_bad_ring(oracle):
    A, B = _sets([10], [10])
    with pytest.raises(OracleError):
        oracle.switch_staged(A.pairs(), B.pairs(), S - 1, S)           # ring below one slot
    with pytest.raises(OracleError):
        oracle.switch_staged(A.pairs(), B.pairs(), 2 * S, S, n_out_slots=2)  # nothing left for B
    with pytest.raises(OracleError):
        oracle.switch_staged(A.pairs(), B.pairs(), 2 * S, S, n_out_slots=0)  # nothing for A
    with pytest.raises(OracleError):
        oracle.switch_staged(A.pairs(), B.pairs(), 2 * S, 0)


@pytest.mark.parametrize("fault", [f for f in FAULTS if f not in ("none", "ignore_alias")])
def test_planted_mistakes_are_caught(oracle, fault):
    """A dropped chunk, a short or long piece, a shifted slot offset, a double copy or a
    wrong source each trip a check: copy counts, content compare or red zones."""
    A, B = _sets([2 * S + 100, 555, S], [3 * S, 64])
    caught = False
    try:
        oracle.switch_staged(A.pairs(), B.pairs(), 4 * S, S, seed=4, check_bytes=True, fault=fault)
    except OracleError:
        caught = True
    for X in (A, B):
        try:
            X.check_moved()
        except AssertionError:
            caught = True
    assert caught, fault


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("fault,code", [("reuse_busy_slot", -3), ("overcommit", -4)])
def test_slot_and_budget_invariants_are_falsifiable(oracle, fault, code, seed):
    """The two staging-tier invariants are recounted from the slot table after every step: a chunk
    staged into a slot that still holds another one is reported as ESLOT_BUSY (the overwritten chunk
    is missing from the table), a direction that uses a slot the ring never gave it as EBUDGET."""
    A, B = _sets([5 * S + 100, 555, S], [6 * S, 64])
    with pytest.raises(OracleError) as e:
        oracle.switch_staged(A.pairs(), B.pairs(), 4 * S, S, seed=seed, fault=fault)
    assert e.value.code == code
    # the same inputs without the planted mistake pass, and really use the whole budget at some point
    A, B = _sets([5 * S + 100, 555, S], [6 * S, 64])
    rep = oracle.switch_staged(A.pairs(), B.pairs(), 4 * S, S, seed=seed)
    assert 0 < rep["hwm_staged_bytes"] <= 4 * S


# ---- in-place switch: B reuses the GPU memory A gives up ---------------------

ALIAS_CASES = [
    # sizes_a, sizes_b, shift of B's layout inside the shared arena
    ([5 * S + 1, 300, 2 * S], [4 * S, 11, 3 * S + 9], 0),        # same start, different cuts
    ([3 * S, 3 * S, 3 * S], [3 * S, 3 * S, 3 * S], 0),            # identical layouts: exact reuse
    ([2 * S + 7, 900], [S, S, 500], 1000),                        # shifted: partial overlaps
    ([4 * S], [100, 200, 6 * S], 3 * S),                          # B extends past the end of A
]


@pytest.mark.parametrize("case", range(len(ALIAS_CASES)))
def test_in_place_direct_is_evict_then_restore(oracle, case):
    """Library pin: numpy slicing in the order the definition fixes (all of A out, then B in)."""
    sa, sb, shift = ALIAS_CASES[case]
    P = AliasedPair(sa, sb, 21, shift_b=shift)
    oracle.switch_direct(P.pairs_a(), P.pairs_b())
    P.check()


@pytest.mark.parametrize("case", range(len(ALIAS_CASES)))
@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5])
def test_in_place_staged_equals_direct(oracle, case, seed):
    sa, sb, shift = ALIAS_CASES[case]
    P = AliasedPair(sa, sb, 21, shift_b=shift, skew_a=seed % 3, skew_b=(seed * 5) % 7)
    rep = oracle.switch_staged(P.pairs_a(), P.pairs_b(), 4 * S, S, seed=seed, pack=bool(seed & 1),
                               check_bytes=True, in_place=True)
    assert rep["hwm_staged_bytes"] <= 4 * S and rep["final_staged_bytes"] == 0
    P.check()


def test_in_place_rule_is_needed(oracle):
    """Scattering without waiting for the eviction of the bytes underneath loses A's data for at
    least some step orders; with the rule no order does."""
    sa, sb, shift = ALIAS_CASES[1]
    lost = 0
    for seed in range(12):
        P = AliasedPair(sa, sb, 21)
        oracle.switch_staged(P.pairs_a(), P.pairs_b(), 4 * S, S, seed=seed, in_place=True, fault="ignore_alias")
        try:
            P.check()
        except AssertionError:
            lost += 1
    assert lost > 0


def test_staged_mt_equals_direct(oracle):
    sizes_a = [S * 9 + 3, 17, 0, 5 * S]
    sizes_b = [S * 4, 1, 12 * S + 7]
    A, B = _sets(sizes_a, sizes_b)
    sec = oracle.switch_staged_mt(A.pairs(), B.pairs(), 8 * S, S, threads_per_dir=3)
    assert sec >= 0
    A.check_moved(); B.check_moved()
    with pytest.raises(OracleError):
        oracle.switch_staged_mt(A.pairs(), B.pairs(), 4 * S, S, threads_per_dir=3)  # 6 slots needed


def test_hash_table_sides(oracle):
    A, B = _sets([100, 0, 4097], [33])
    h_dev = oracle.hash_table(A.pairs(), "dev")
    oracle.switch_direct(A.pairs(), B.pairs())
    h_host = oracle.hash_table(A.pairs(), "host")
    assert (h_dev == h_host).all()
    assert [int(x) for x in h_dev] == [py_hash64(A.expected(i).tobytes()) for i in range(3)]


# ---- the benchmark configs at sizes the CPU finishes quickly ----------------

def test_config1_full_size(oracle):
    cf = W.config(1)
    A = HostSet(cf["A"], cf["seed_A"], "dev")
    B = HostSet(cf["B"], cf["seed_B"], "host")
    rep = oracle.switch_staged(A.pairs(), B.pairs(), cf["ring_bytes"][0], cf["slot_bytes"],
                               seed=1, check_bytes=True)
    assert rep["hwm_staged_bytes"] <= 4 * MiB
    A.check_moved(); B.check_moved()


@pytest.mark.parametrize("cfg,scale", [(2, 1 / 2048), (3, 1 / 2048), (5, 1 / 2048)])
def test_config_shapes_scaled(oracle, cfg, scale):
    cf = W.config(cfg, scale=scale)
    A = HostSet(cf["A"], cf["seed_A"], "dev")
    B = HostSet(cf["B"], cf["seed_B"], "host")
    slot = max(4096, int((cf["slot_bytes"] or 2 * MiB) * scale))
    ring = max(4 * slot, int(cf["ring_bytes"][0] * scale) // slot * slot)
    oracle.switch_staged(A.pairs(), B.pairs(), ring, slot, seed=cfg)
    A.check_moved(); B.check_moved()


def test_workload_generators():
    cf = W.config(2)
    assert len(cf["A"]) == 355 and len([n for n, _ in cf["A"] if not n.startswith("kv")]) == 291
    assert sum(b for _, b in cf["A"]) == 18_208_006_144       # 16.06 GB weights + 2 GiB KV
    cf4 = W.config(4, scale=1 / 64)
    assert len(cf4["A"]) == 100_016
    small = [b for _, b in cf4["A"][:100_000]]
    assert min(small) >= 256 and max(small) <= 64 * KiB
    s = W.log_uniform_sizes(1, 20000, 4 * KiB, 1 * MiB, 1)
    # log-uniform: the median sits near the geometric mean of the range
    assert 0.8 < np.median(s) / (4 * KiB * 1 * MiB) ** 0.5 < 1.25
    lay = W.make_layout([10, 20, 30], skew=3)
    assert all(o % 256 == 3 for o in lay.offsets)
    assert lay.offsets[1] >= lay.offsets[0] + 10 + 256


def test_staged_form_on_random_inputs(oracle):
    """Property test (hypothesis): whatever the sizes, the slot size, the ring split, the packing mode and
    the seeded order of steps, the staged form ends in the state of the direct definition (generated content
    at the destination, red zones intact), moves every byte exactly once each way, leaves the ring empty and
    never holds more than the ring; and any of the planted mistakes is noticed somewhere."""
    from hypothesis import given, settings, strategies as st, HealthCheck

    sizes = st.lists(st.one_of(st.integers(0, 40), st.integers(1, 3000), st.integers(3000, 40000)), min_size=0, max_size=10)

    @settings(max_examples=80, deadline=None, suppress_health_check=[HealthCheck.too_slow])
    @given(sizes, sizes, st.sampled_from([64, 1024, 4096]), st.integers(2, 9), st.integers(1, 8), st.booleans(),
           st.integers(0, 2**32), st.integers(0, 15), st.integers(0, 15))
    def run(sa, sb, slot, n_slots, n_out, pack, seed, skew_d, skew_h):
        A, B = _sets(sa, sb, skew_dev=skew_d, skew_host=skew_h)
        n_out = min(max(n_out, 1), n_slots - 1)
        rep = oracle.switch_staged(A.pairs(), B.pairs(), n_slots * slot, slot, n_out_slots=n_out, pack=pack, seed=seed,
                                   check_bytes=True)
        A.check_moved(); B.check_moved()
        assert rep["count_errors"] == 0 and rep["final_staged_bytes"] == 0
        assert rep["hwm_staged_bytes"] <= n_slots * slot
        assert rep["bytes_out"] == sum(sa) and rep["bytes_in"] == sum(sb)
        if sum(sa) + sum(sb) > 4 * slot:                       # enough chunks for a planted mistake to matter
            fault = ["drop_chunk", "double_copy", "reuse_busy_slot", "overcommit"][seed % 4]
            A2, B2 = _sets(sa, sb, skew_dev=skew_d, skew_host=skew_h)
            caught = False
            try:
                oracle.switch_staged(A2.pairs(), B2.pairs(), n_slots * slot, slot, n_out_slots=n_out, pack=pack, seed=seed,
                                     check_bytes=True, fault=fault)
            except OracleError:
                caught = True
            for X in (A2, B2):
                try:
                    X.check_moved()
                except AssertionError:
                    caught = True
            # reuse_busy_slot needs a busy slot at the moment the mistake is armed; with very few chunks
            # per direction that may never happen, and then the run is simply correct
            assert caught or fault == "reuse_busy_slot", fault

    run()
