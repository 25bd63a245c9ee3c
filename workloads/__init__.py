"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package only *makes inputs*: a counter-based 64-bit generator, the
pseudo-word text stream, the piece splitter and the registry of benchmark
workloads.  It contains no part of the BPE merge loop itself, and imports
neither the oracle nor the HIP binding.
"""
from .textgen import (  # noqa: F401
    splitmix64,
    make_wordlist,
    gen_text_stream,
    gen_stress_stream,
    pretokenize,
)
from .configs import (  # noqa: F401
    CONFIGS,
    load_merges,
    make_eval,
    make_train_corpus,
    table_path,
    manifest,
)
