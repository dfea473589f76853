"""Seeded synthetic working sets shaped like the paper's consumer workloads.

Input generation only: sizes, layouts and contents.  Holds none of the swap's
own arithmetic (no chunking, no hashing, no copying of working sets), so both
the CPU oracle's tests and the GPU library's tests may draw inputs from here.
"""
from .sets import (  # noqa: F401
    GOLDEN, mix64, splitmix64_stream, content_bytes, log_uniform_sizes,
    config, CONFIG_NAMES, Layout, make_layout, fill_content, llm_tensor_sizes,
)
