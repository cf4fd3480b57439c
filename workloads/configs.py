"""The five benchmark workloads (populations per subgraph, k, verify settings).

0  one fp32 GEMM 512^3, 4,096 candidates, draft top-64
1  one fp32 conv2d N1 C64 56x56 K64 3x3, 65,536 candidates, draft top-128
2  20 GEMM / batched-GEMM subgraphs of a BERT-base-shaped encoder (Table 4:
   hidden 768, 12 heads, intermediate 3072; batch 1, sequence 128),
   50,000 candidates each, draft top-512 per subgraph
3  workload 2 followed by the verify stage on the 20 x 512 drafted candidates,
   final top-32 per subgraph
4  16M candidates of an fp16 GEMM 4096^3 with 16x16x16 fragments (Sec. 6.4) plus
   4M candidates of a depthwise conv, draft top-4096, then verify, final top-32

`scale` shrinks every population (and k with it) for quick tests; scale=1 is
the full size.
"""
from dataclasses import dataclass
from typing import Tuple

import numpy as np

from .schedules import sample_population
from .subgraphs import Subgraph, batched_gemm, conv2d, depthwise_conv2d, gemm, n_slots

CONFIG_NAMES = (
    "cfg0_gemm512_4k",
    "cfg1_conv2d_64k",
    "cfg2_bert_base_20x50k",
    "cfg3_bert_base_draft_verify",
    "cfg4_stress_gemm4096_dwconv_20M",
)


@dataclass
class Workload:
    name: str
    subgraphs: Tuple[Subgraph, ...]
    seg_off: np.ndarray        # int64 [n_sg + 1], candidate ranges per subgraph
    tiles: np.ndarray          # uint16 [max_slots, n]  (pitch = n; unused slots hold 0)
    ann: np.ndarray            # uint16 [n]
    k_draft: int
    verify: bool               # run the learned model on the drafted set
    k_final: int               # final top-k per subgraph after verify (0 if no verify)
    n_stmt: Tuple[int, ...]    # valid statement rows per candidate, per subgraph
    seed: int

    @property
    def n(self):
        return int(self.seg_off[-1])


def bert_base_subgraphs(n_sg=20):
    """GEMM shapes of a BERT-base-shaped encoder layer at batch 1, sequence 128.

    The paper does not list the subgraphs; subgraph t takes shape t mod 6 of
    QKV projection, attention score, attention x value, output projection and
    the two feed-forward GEMMs.
    """
    seq, hid, heads, hd, ffn = 128, 768, 12, 64, 3072
    shapes = (
        lambda: gemm(seq, 3 * hid, hid, name="qkv_proj"),
        lambda: batched_gemm(heads, seq, seq, hd, name="attn_score"),
        lambda: batched_gemm(heads, seq, hd, seq, name="attn_value"),
        lambda: gemm(seq, hid, hid, name="out_proj"),
        lambda: gemm(seq, ffn, hid, name="ffn1"),
        lambda: gemm(seq, hid, ffn, name="ffn2"),
    )
    return tuple(shapes[t % 6]() for t in range(n_sg))


def _assemble(name, subgraphs, counts, seed, k_draft, verify, k_final, n_stmt):
    seg_off = np.zeros(len(subgraphs) + 1, dtype=np.int64)
    seg_off[1:] = np.cumsum(counts)
    n = int(seg_off[-1])
    slots = max(n_slots(sg) for sg in subgraphs)
    tiles = np.zeros((slots, n), dtype=np.uint16)
    ann = np.empty(n, dtype=np.uint16)
    for t, (sg, cnt) in enumerate(zip(subgraphs, counts)):
        lo = int(seg_off[t])
        # generate in pieces to bound temporary memory on the large populations
        step = 1 << 21
        for first in range(0, cnt, step):
            m = min(step, cnt - first)
            tl, an = sample_population(sg, m, seed, stream=t, first=first)
            tiles[: tl.shape[0], lo + first: lo + first + m] = tl
            ann[lo + first: lo + first + m] = an
    return Workload(name, tuple(subgraphs), seg_off, tiles, ann, k_draft, verify, k_final, tuple(n_stmt), seed)


def make_config(idx: int, scale: float = 1.0) -> Workload:
    def sz(x):
        return max(1, int(round(x * scale)))

    if idx == 0:
        return _assemble(CONFIG_NAMES[0], [gemm(512, 512, 512)], [sz(4096)], 0, min(64, sz(4096)), False, 0, (3,))
    if idx == 1:
        sg = conv2d(1, 64, 56, 56, 64, 3, 3, stride=1, pad=1)
        return _assemble(CONFIG_NAMES[1], [sg], [sz(65536)], 0, min(128, sz(65536)), False, 0, (3,))
    if idx in (2, 3):
        sgs = bert_base_subgraphs(20)
        cnt = sz(50000)
        n_stmt = tuple(3 + (t % 6) for t in range(20))
        k = min(512, cnt)
        return _assemble(CONFIG_NAMES[idx], sgs, [cnt] * 20, 0, k, idx == 3, min(32, k) if idx == 3 else 0, n_stmt)
    if idx == 4:
        g = gemm(4096, 4096, 4096, dtype_bytes=2, sp_levels=4, rd_levels=3, frag=(16, 16, 16), name="gemm4096_fp16_frag16")
        d = depthwise_conv2d(1, 512, 28, 28, 3, 3, stride=1, pad=1)
        counts = [sz(16 * 1024 * 1024), sz(4 * 1024 * 1024)]
        k = min(4096, min(counts))
        return _assemble(CONFIG_NAMES[4], [g, d], counts, 0, k, True, min(32, k), (5, 4))
    raise ValueError(f"no config {idx}")
