"""Seeded synthetic workloads: parameter-list shapes and input generators.

Shared by the oracle-side tests and the HIP-side tests/benchmark so that both receive the same
bytes.  Nothing in this package performs any arithmetic of the optimizer: it draws random
numbers and lays out tensors, nothing else.
"""
from .shapes import CONFIGS, ParamList, bert_shaped, gpt_shaped, make_config, padded_len, tiny  # noqa: F401
from .gen import Streams, gradient, init_state, foreign_worker_chunks, foreign_server_chunks  # noqa: F401
from .schedule import lr_seqlen128, PAPER_SEQLEN128, PAPER_SEQLEN512  # noqa: F401
