"""Parameter lists shaped like the models the paper trains (Section 6: BERT-Large) and the
neighbouring sizes the benchmark configurations name.  A parameter list is the ordered list of
tensors whose concatenation is the flat fp32 buffer ("momentum fusion", Appendix A.5.1): it is
described by `offsets` (L+1 entries, offsets[0] = 0, offsets[L] = N), tightly packed in list
order with no alignment padding between tensors.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np


def padded_len(n: int, num_workers: int) -> int:
    """Smallest multiple of 256*W that holds n elements (every chunk is then 256-aligned)."""
    q = 256 * num_workers
    return ((n + q - 1) // q) * q


@dataclass
class ParamList:
    name: str
    tensors: List[Tuple[str, int]]
    offsets: np.ndarray = field(init=False)

    def __post_init__(self):
        sizes = np.array([n for _, n in self.tensors], dtype=np.int64)
        self.offsets = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)

    @property
    def L(self) -> int:
        return len(self.tensors)

    @property
    def N(self) -> int:
        return int(self.offsets[-1])


def tiny() -> ParamList:
    return ParamList("tiny", [(f"w{i}", 512 * 512) for i in range(4)])


def bert_shaped(hidden: int, ffn: int, layers: int, vocab: int, max_pos: int = 512,
                fused_qkv: bool = True, name: str = "bert") -> ParamList:
    H = hidden
    t: List[Tuple[str, int]] = [
        ("emb.word", vocab * H), ("emb.pos", max_pos * H), ("emb.type", 2 * H),
        ("emb.ln.w", H), ("emb.ln.b", H)]
    for i in range(layers):
        p = f"l{i}."
        if fused_qkv:
            t += [(p + "qkv.w", H * 3 * H), (p + "qkv.b", 3 * H)]
        else:
            for q in "qkv":
                t += [(p + q + ".w", H * H), (p + q + ".b", H)]
        t += [(p + "out.w", H * H), (p + "out.b", H), (p + "ln1.w", H), (p + "ln1.b", H),
              (p + "ffn1.w", H * ffn), (p + "ffn1.b", ffn), (p + "ffn2.w", ffn * H),
              (p + "ffn2.b", H), (p + "ln2.w", H), (p + "ln2.b", H)]
    t += [("pooler.w", H * H), ("pooler.b", H),
          ("mlm.transform.w", H * H), ("mlm.transform.b", H), ("mlm.ln.w", H), ("mlm.ln.b", H),
          ("mlm.decoder.b", vocab), ("nsp.w", 2 * H), ("nsp.b", 2)]
    return ParamList(name, t)


def gpt_shaped(hidden: int, ffn: int, layers: int, vocab: int, max_pos: int,
               name: str = "gpt") -> ParamList:
    H = hidden
    t: List[Tuple[str, int]] = [("emb.word", vocab * H), ("emb.pos", max_pos * H)]
    for i in range(layers):
        p = f"l{i}."
        t += [(p + "qkv.w", H * 3 * H), (p + "qkv.b", 3 * H), (p + "out.w", H * H),
              (p + "out.b", H), (p + "ln1.w", H), (p + "ln1.b", H), (p + "ffn1.w", H * ffn),
              (p + "ffn1.b", ffn), (p + "ffn2.w", ffn * H), (p + "ffn2.b", H), (p + "ln2.w", H),
              (p + "ln2.b", H)]
    t += [("lnf.w", H), ("lnf.b", H)]
    return ParamList(name, t)


# name -> (parameter list factory, W, gradient recipe, steps)
CONFIGS = {
    "tiny": dict(plist=tiny, W=4, grad="normal", steps=10),
    "bert_base": dict(plist=lambda: bert_shaped(768, 3072, 12, 30522, name="bert_base"),
                      W=16, grad="normal_layer_scaled", steps=100),
    "bert_large": dict(plist=lambda: bert_shaped(1024, 4096, 24, 30528, fused_qkv=False,
                                                 name="bert_large"),
                       W=64, grad="student_t3", steps=100),
    "bert_large_w256": dict(plist=lambda: bert_shaped(1024, 4096, 24, 30528, fused_qkv=False,
                                                      name="bert_large"),
                            W=256, grad="student_t3", steps=100),
    # the same model with Q, K and V in one tensor per block: 302 tensors, the count Appendix A.5.1 gives
    "bert_large_fused_qkv": dict(plist=lambda: bert_shaped(1024, 4096, 24, 30528, fused_qkv=True,
                                                           name="bert_large_fused_qkv"),
                                 W=64, grad="student_t3", steps=100),
    "gpt_1p3b": dict(plist=lambda: gpt_shaped(2048, 8192, 24, 50304, 2048, name="gpt_1p3b"),
                     W=128, grad="normal_sparse_layers", steps=50),
    # not a benchmark configuration: the GPT-1.3B block repeated until the flat buffer is longer than
    # 2^32 elements (4.54e9; 18 GB per fp32 array), for the tests of 64-bit indexing
    "gpt_beyond_2p32": dict(plist=lambda: gpt_shaped(2048, 8192, 88, 50304, 2048, name="gpt_beyond_2p32"),
                            W=256, grad="normal", steps=4),
    # not a benchmark configuration: a BERT-patterned list small enough for the CPU oracle to run
    # 100-step trajectories in seconds, with the same odd tensor sizes (2-element bias, etc.)
    "bert_mini": dict(plist=lambda: bert_shaped(64, 256, 2, 1000, max_pos=32, fused_qkv=False,
                                                name="bert_mini"),
                      W=8, grad="student_t3", steps=100),
}


def make_config(name: str):
    c = dict(CONFIGS[name])
    c["plist"] = c["plist"]()
    c["name"] = name
    c["n_pad"] = padded_len(c["plist"].N, c["W"])
    c["n_c"] = c["n_pad"] // c["W"]
    return c
