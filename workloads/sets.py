"""Size lists, arena layouts and byte contents for the five benchmark configs.

The sets stand in for the applications the paper switches between (quantised
LLMs under Ollama / SGLang, diffusion pipelines under ComfyUI; paper,
"Evaluation", Setup): same shapes, size mixes and value distributions, all
synthetic and seeded.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

GOLDEN = 0x9E3779B97F4A7C15
_M64 = (1 << 64) - 1
KiB, MiB, GiB = 1 << 10, 1 << 20, 1 << 30


def mix64(x):
    """splitmix64 output function on numpy uint64 (array or scalar)."""
    with np.errstate(over="ignore"):
        z = np.asarray(x, dtype=np.uint64)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def splitmix64_stream(seed: int, n: int) -> np.ndarray:
    """The first n outputs of splitmix64 started from state ``seed``."""
    with np.errstate(over="ignore"):
        k = np.arange(1, n + 1, dtype=np.uint64)
        return mix64(np.uint64(seed & _M64) + np.uint64(GOLDEN) * k)


def _alloc_state(seed: int, index: int) -> int:
    return int(mix64(np.uint64((seed + GOLDEN * (index + 1)) & _M64)))


def content_bytes(seed: int, index: int, nbytes: int, offset: int = 0) -> np.ndarray:
    """Bytes [offset, offset+nbytes) of allocation ``index`` of the set ``seed``.

    Counter based: word k of the allocation is the (k+1)-th splitmix64 output
    from a per-allocation state, little endian, so any piece can be regenerated
    without the rest.
    """
    if nbytes == 0:
        return np.zeros(0, dtype=np.uint8)
    w0 = offset // 8
    w1 = (offset + nbytes + 7) // 8
    words = np.empty(w1 - w0, dtype="<u8")
    s = _alloc_state(seed, index)
    step = 1 << 20
    with np.errstate(over="ignore"):
        for a in range(w0, w1, step):
            b = min(w1, a + step)
            k = np.arange(a + 1, b + 1, dtype=np.uint64)
            words[a - w0:b - w0] = mix64(np.uint64(s) + np.uint64(GOLDEN) * k)
    raw = words.view(np.uint8)
    lo = offset - 8 * w0
    return raw[lo:lo + nbytes]


def log_uniform_sizes(seed: int, n: int, lo: int, hi: int, gran: int = 1) -> list[int]:
    """n sizes, log-uniform on [lo, hi], rounded to a multiple of gran (>= gran)."""
    u = (splitmix64_stream(seed, n) >> np.uint64(11)).astype(np.float64) / float(1 << 53)
    raw = lo * np.power(hi / lo, u)
    sz = np.maximum(gran, (np.round(raw / gran)).astype(np.int64) * gran)
    return [int(min(max(s, lo if gran == 1 else gran), hi)) for s in sz]


def llm_tensor_sizes(layers: int = 32, hidden: int = 4096, kv_dim: int = 1024,
                     mlp: int = 14336, vocab: int = 128256, elt: int = 2,
                     kv_cache_tensors: int = 64, kv_tensor_bytes: int = 32 * MiB):
    """An 8B dense decoder in bf16 plus a KV cache, tensor by tensor."""
    t: list[tuple[str, int]] = [("embed", vocab * hidden * elt)]
    for l in range(layers):
        t += [(f"l{l}.q", hidden * hidden * elt), (f"l{l}.k", kv_dim * hidden * elt),
              (f"l{l}.v", kv_dim * hidden * elt), (f"l{l}.o", hidden * hidden * elt),
              (f"l{l}.gate", mlp * hidden * elt), (f"l{l}.up", mlp * hidden * elt),
              (f"l{l}.down", hidden * mlp * elt), (f"l{l}.norm1", hidden * elt),
              (f"l{l}.norm2", hidden * elt)]
    t += [("final_norm", hidden * elt), ("lm_head", vocab * hidden * elt)]
    t += [(f"kv{j}", kv_tensor_bytes) for j in range(kv_cache_tensors)]
    return t


def _scaled(sizes, scale: float, gran: int):
    if scale == 1.0:
        return list(sizes)
    return [(n, max(gran, int(b * scale) // gran * gran)) for n, b in sizes]


def _named(prefix, sizes):
    return [(f"{prefix}{i}", int(b)) for i, b in enumerate(sizes)]


def _until_total(seed, lo, hi, gran, total):
    """log-uniform sizes until their sum reaches total; the last one is cut to fit."""
    out, acc, block, drawn = [], 0, 256, 0
    while acc < total:
        for s in log_uniform_sizes(seed + drawn, block, lo, hi, gran):
            if acc + s >= total:
                s = total - acc
                s = max(gran, s // gran * gran)
                out.append(s)
                acc = total
                break
            out.append(s)
            acc += s
        drawn += block
    return out


CONFIG_NAMES = {1: "tiny", 2: "llm", 3: "asymmetric", 4: "fragmented", 5: "budget_sweep", 6: "exact16"}


def config(cfg: int, seed: int = 2601, scale: float = 1.0) -> dict:
    """Size lists and ring parameters of benchmark config ``cfg`` (1..5; 6 = exactly 16 GiB each way).

    Returns {"A": [(name, bytes)...], "B": [...], "ring_bytes": [..], "slot_bytes",
    "content": "splitmix"|"bf16_normal", "seed_A", "seed_B"}.  A is GPU resident
    and is evicted; B sits in pageable host memory and is brought in.
    ``scale`` shrinks every size (not the counts) for quick CPU runs.
    """
    sa, sb = seed, seed + 1
    if cfg == 1:
        A = _named("a", log_uniform_sizes(sa, 64, 4 * KiB, 1 * MiB, 1))
        B = _named("b", log_uniform_sizes(sb, 64, 4 * KiB, 1 * MiB, 1))
        return dict(A=_scaled(A, scale, 1), B=_scaled(B, scale, 1), ring_bytes=[4 * MiB],
                    slot_bytes=256 * KiB, content="splitmix", seed_A=sa, seed_B=sb, cfg=1)
    if cfg == 2:
        A = llm_tensor_sizes()
        B = llm_tensor_sizes()
        return dict(A=_scaled(A, scale, 16), B=_scaled(B, scale, 16), ring_bytes=[256 * MiB],
                    slot_bytes=4 * MiB, content="bf16_normal", seed_A=sa, seed_B=sb, cfg=2)
    if cfg == 3:
        A = (_named("dit", log_uniform_sizes(sa, 800, 1 * MiB, 64 * MiB, 16))
             + _named("vae", log_uniform_sizes(sa + 7, 300, 16 * KiB, 8 * MiB, 16))
             + [(f"act{i}", 128 * MiB) for i in range(32)])
        have = sum(b for _, b in A)
        if have < 20 * GiB:  # text-encoder group tops the set up to the stated 20 GiB
            A += _named("txt", _until_total(sa + 13, 1 * MiB, 64 * MiB, 16, 20 * GiB - have))
        B, acc = [], 0
        for n, b in llm_tensor_sizes(kv_cache_tensors=0):
            if acc + b > 6 * GiB:
                continue
            B.append((n, b))
            acc += b
        return dict(A=_scaled(A, scale, 16), B=_scaled(B, scale, 16), ring_bytes=[128 * MiB],
                    slot_bytes=None, content="bf16_normal", seed_A=sa, seed_B=sb, cfg=3)
    if cfg == 4:
        def one(s):
            return (_named("s", log_uniform_sizes(s, 100_000, 256, 64 * KiB, 1))
                    + [(f"big{i}", 512 * MiB) for i in range(16)])
        A, B = one(sa), one(sb)
        if scale != 1.0:  # keep the small allocations literal, shrink only the big ones
            A = A[:100_000] + _scaled(A[100_000:], scale, 1)
            B = B[:100_000] + _scaled(B[100_000:], scale, 1)
        return dict(A=A, B=B, ring_bytes=[64 * MiB], slot_bytes=None, content="splitmix",
                    seed_A=sa, seed_B=sb, cfg=4)
    if cfg == 5:
        tot = int(24 * GiB * scale) // 16 * 16
        lo, hi = max(16, int(1 * MiB * scale) // 16 * 16), max(32, int(256 * MiB * scale) // 16 * 16)
        A = _named("t", _until_total(sa, lo, hi, 16, tot))
        B = _named("t", _until_total(sb, lo, hi, 16, tot))
        return dict(A=A, B=B, ring_bytes=[16 * MiB, 64 * MiB, 256 * MiB, 1024 * MiB],
                    slot_bytes=None, content="bf16_normal", seed_A=sa, seed_B=sb, cfg=5)
    if cfg == 6:   # the metric's wording taken literally: exactly 16 GiB out and 16 GiB in, 256 MiB ring
        A = [(f"t{i}", 256 * MiB) for i in range(64)]
        B = [(f"t{i}", 256 * MiB) for i in range(64)]
        return dict(A=_scaled(A, scale, 16), B=_scaled(B, scale, 16), ring_bytes=[256 * MiB],
                    slot_bytes=4 * MiB, content="bf16_normal", seed_A=sa, seed_B=sb, cfg=6)
    raise ValueError(f"no config {cfg}")


@dataclass
class Layout:
    """Where each allocation sits inside one arena, with red zones between."""
    offsets: list[int]
    sizes: list[int]
    total: int
    redzone: int
    names: list[str] = field(default_factory=list)


def make_layout(sizes, align: int = 256, redzone: int = 256, skew: int = 0) -> Layout:
    """Place allocations one after another: [redzone][alloc, base % align == skew]..."""
    offs, pos = [], redzone
    names = []
    for item in sizes:
        name, b = item if isinstance(item, tuple) else ("", item)
        pos = (pos + align - 1) // align * align + skew
        offs.append(pos)
        names.append(name)
        pos += int(b) + redzone
    total = (pos + align - 1) // align * align + align
    return Layout(offs, [int(s[1]) if isinstance(s, tuple) else int(s) for s in sizes],
                  total, redzone, names)


def fill_content(arena: np.ndarray, layout: Layout, seed: int) -> None:
    """Write the splitmix content of every allocation of set ``seed`` into arena."""
    for i, (o, b) in enumerate(zip(layout.offsets, layout.sizes)):
        arena[o:o + b] = content_bytes(seed, i, b)
