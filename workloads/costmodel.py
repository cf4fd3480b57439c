"""Synthetic inputs of the verify stage: statement features and model weights.

The learned cost model consumes, per candidate, one 164-wide feature row per
innermost statement (Introduction: the statement features of Ansor/TenSet;
Sec. 4.2 "Pattern-aware Transformer": statement features go through linear
layers and are then summed).  The real rows come from a compiler's feature
extractor, which is not available; rows here have the same shape and the
value profile of log-scaled counters (half zeros, the rest in [0, 24)).
Weights are random-initialised, not trained.
"""
import numpy as np

from .rng import hash_u64, uniform01

FEAT_DIM = 164     # per-statement feature width
MAX_STMT = 8       # statement rows per candidate (zero-padded)
HIDDEN = 256       # width of the two hidden layers
FLOW_DIM = 23      # per-block temporal dataflow feature width (Sec. 4.2)
MAX_BLOCKS = 8     # data-movement blocks per candidate
EMBED = 64         # width of the dataflow branch


def f32_to_bf16_bits(x):
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _uniform_sym(seed, stream, shape, bound):
    n = int(np.prod(shape))
    u = uniform01(hash_u64(seed, stream, np.arange(n, dtype=np.uint64)))
    return ((2.0 * u - 1.0) * bound).astype(np.float32).reshape(shape)


def make_mlp_weights(seed=1, feat_dim=FEAT_DIM, hidden=HIDDEN):
    """164 -> 256 -> 256 -> 1 weights, U(-1/sqrt(fan_in), +1/sqrt(fan_in)).

    Matrices are [out, in] row-major and given as bf16 bit patterns; biases
    stay float32.
    """
    b1 = 1.0 / np.sqrt(feat_dim)
    b2 = 1.0 / np.sqrt(hidden)
    return {
        "W1": f32_to_bf16_bits(_uniform_sym(seed, 1, (hidden, feat_dim), b1)),
        "b1": _uniform_sym(seed, 2, (hidden,), b1),
        "W2": f32_to_bf16_bits(_uniform_sym(seed, 3, (hidden, hidden), b2)),
        "b2": _uniform_sym(seed, 4, (hidden,), b2),
        "w3": f32_to_bf16_bits(_uniform_sym(seed, 5, (hidden,), b2)),
        "b3": float(_uniform_sym(seed, 6, (1,), b2)[0]),
    }


def make_pacm_weights(seed=1):
    """Weights of the whole Pattern-aware Transformer in the dimensions this build takes (statement branch 164-256-256,
    dataflow branch 23-64 with one attention layer, head 320-256-1), U(-1/sqrt(fan_in), +1/sqrt(fan_in)), matrices as
    bf16 bit patterns [out, in], biases float32."""
    m = make_mlp_weights(seed)
    out = {k: m[k] for k in ("W1", "b1", "W2", "b2")}
    be = 1.0 / np.sqrt(FLOW_DIM)
    ba = 1.0 / np.sqrt(EMBED)
    bh = 1.0 / np.sqrt(HIDDEN + EMBED)
    bo = 1.0 / np.sqrt(HIDDEN)
    out["We"] = f32_to_bf16_bits(_uniform_sym(seed, 11, (EMBED, FLOW_DIM), be))
    out["be"] = _uniform_sym(seed, 12, (EMBED,), be)
    for i, name in enumerate(("Wq", "Wk", "Wv", "Wo")):
        out[name] = f32_to_bf16_bits(_uniform_sym(seed, 13 + i, (EMBED, EMBED), ba))
    out["Wh"] = f32_to_bf16_bits(_uniform_sym(seed, 17, (HIDDEN, HIDDEN + EMBED), bh))
    out["bh"] = _uniform_sym(seed, 18, (HIDDEN,), bh)
    out["wo"] = f32_to_bf16_bits(_uniform_sym(seed, 19, (HIDDEN,), bo))
    out["bo"] = float(_uniform_sym(seed, 20, (1,), bo)[0])
    return out


def make_flow_features(cand_ids, n_blk, seed=0, pad_value=0.0):
    """Temporal dataflow rows keyed by global candidate id: float32 [n_d, MAX_BLOCKS, FLOW_DIM], the value profile of the
    statement rows (half zeros, the rest in [0, 24)); rows i >= n_blk[c] hold `pad_value`."""
    cand_ids = np.asarray(cand_ids, dtype=np.uint64)
    n_blk = np.asarray(n_blk, dtype=np.int64)
    per = MAX_BLOCKS * FLOW_DIM
    ctr = cand_ids[:, None] * np.uint64(per) + np.arange(per, dtype=np.uint64)[None, :]
    keep = (hash_u64(seed, 0xF10A, ctr) & np.uint64(1)).astype(bool)
    val = uniform01(hash_u64(seed, 0xF10B, ctr)) * 24.0
    flow = np.where(keep, val, 0.0).astype(np.float32).reshape(len(cand_ids), MAX_BLOCKS, FLOW_DIM)
    flow[np.arange(MAX_BLOCKS)[None, :] >= n_blk[:, None]] = np.float32(pad_value)
    return flow


def make_statement_features(cand_ids, n_stmt, seed=0, pad_value=0.0):
    """Feature rows keyed by global candidate id.

    cand_ids [n_d] integer ids, n_stmt [n_d] valid statement rows (1..MAX_STMT).
    Returns float32 [n_d, MAX_STMT, FEAT_DIM].  Element (c, s, f) is a function
    of (seed, cand_ids[c], s, f) only.  Rows s >= n_stmt[c] hold `pad_value`
    (zero in the workloads; tests set garbage there to check they are ignored).
    """
    cand_ids = np.asarray(cand_ids, dtype=np.uint64)
    n_stmt = np.asarray(n_stmt, dtype=np.int64)
    n_d = len(cand_ids)
    per = MAX_STMT * FEAT_DIM
    ctr = cand_ids[:, None] * np.uint64(per) + np.arange(per, dtype=np.uint64)[None, :]
    bits = hash_u64(seed, 0x5EA7, ctr)
    keep = (bits & np.uint64(1)).astype(bool)
    val = uniform01(hash_u64(seed, 0x5EA8, ctr)) * 24.0
    feat = np.where(keep, val, 0.0).astype(np.float32).reshape(n_d, MAX_STMT, FEAT_DIM)
    pad = np.arange(MAX_STMT)[None, :] >= n_stmt[:, None]
    feat[pad] = np.float32(pad_value)
    return feat
