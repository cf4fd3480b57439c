#!/usr/bin/env python3
"""Writes tests/golden/lse_trace.json: hand-traceable cases of the explorer loop's SchMutation and PriorFilter order
(Alg. 2), worked out in plain Python integers from the published SplitMix64 definition.

This script imports nothing from the repository: neither the oracle nor the HIP library.  It restates the reading of
Alg. 2 that both follow, in the most literal integer arithmetic (// and %), so that the stored children, parents and
hashes pin the oracle from outside:

  draw c                  the c-th output of SplitMix64 started from the seed (Steele, Lea, Flood 2014; splitmix64.c)
  child j of step t       draws u1 = draw((t << 41) + 2 j + 1), u2 = draw((t << 41) + 2 j + 2)
  parent                  member floor(low32(u1) * spec_count / 2^32) of the subgraph's S_spec
  mutates                 iff bits 32..47 of u1, as a number, are below mutate_q16
  axis                    floor(bits 0..7 of u2 * n_axes / 256)          (spatial axes first)
  src level               floor(bits 8..15 of u2 * levels / 256)
  dst level               d = floor(bits 16..23 of u2 * (levels - 1) / 256); d + 1 if d >= src
  prime                   number floor(bits 24..31 of u2 * n_primes / 256) of the distinct primes of the src factor, ascending
  move                    src factor / prime, dst factor * prime; none if the src factor is 1, none if the src level is
                          the innermost one of a fragment axis and the quotient is no multiple of the fragment
  schedule hash           h = n_slots; for every slot in order: h = draw c = factor + 1 of SplitMix64 started from h
  S_spec order            score descending, then hash ascending, then age; a copy of its predecessor is dropped

The scenarios are built so that the expected S_spec is known without evaluating the draft model: every schedule of a
scenario has the same symbols (virtual-thread and inner factors of an axis swapped: only their product enters Table 2's
symbols outside fragment mode), hence the same score, and the hash alone orders them.

Run:  python tests/golden/make_lse_trace.py     (rewrites lse_trace.json next to it)
"""
import json
import os

M64 = (1 << 64) - 1


def draw(seed, c):
    z = (seed + c * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


# published outputs of splitmix64.c: the generator above is the published one
assert [draw(0, c) for c in (1, 2, 3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
assert [draw(1234567, c) for c in (1, 2, 3)] == [6457827717110365317, 3203168211198807973, 9817491932198370423]


def schedule_hash(f):
    h = len(f)
    for v in f:
        h = draw(h, v + 1)
    return h


def distinct_primes(v):
    out, p = [], 2
    while v > 1:
        if v % p == 0:
            out.append(p)
            while v % p == 0:
                v //= p
        p += 1
    return out


def trace_child(seed, t, j, spec, mutate_q16, n_sp, n_rd, rd_levels, frag):
    """One child, every intermediate value written out."""
    c = (t << 41) + 2 * j
    u1, u2 = draw(seed, c + 1), draw(seed, c + 2)
    low32 = u1 & 0xFFFFFFFF
    parent = low32 * len(spec) // (1 << 32)
    gate = (u1 >> 32) & 0xFFFF
    child = list(spec[parent])
    rec = {"j": j, "t": t, "u1": f"0x{u1:016X}", "u2": f"0x{u2:016X}", "low32_u1": low32, "parent": parent,
           "gate": gate, "mutates": gate < mutate_q16}
    if gate < mutate_q16:
        n_axes = n_sp + n_rd
        f_axis, f_src, f_dst, f_prime = u2 & 0xFF, (u2 >> 8) & 0xFF, (u2 >> 16) & 0xFF, (u2 >> 24) & 0xFF
        axis = f_axis * n_axes // 256
        levels = 4 if axis < n_sp else rd_levels
        base = axis * 4 if axis < n_sp else n_sp * 4 + (axis - n_sp) * rd_levels
        src = f_src * levels // 256
        dst = f_dst * (levels - 1) // 256
        if dst >= src:
            dst += 1
        v = child[base + src]
        primes = distinct_primes(v)
        rec.update({"fields": [f_axis, f_src, f_dst, f_prime], "axis": axis, "src": src, "dst": dst, "v": v, "primes": primes})
        if not primes:
            rec["outcome"] = "factor is 1: plain copy"
        else:
            p = primes[f_prime * len(primes) // 256]
            rec["p"] = p
            g = 0
            if frag[0] and src == levels - 1:
                if axis == n_sp - 2:
                    g = frag[0]
                if axis == n_sp - 1:
                    g = frag[1]
                if axis == n_axes - 1:
                    g = frag[2]
            if g and (v // p) % g != 0:
                rec["outcome"] = "would break the fragment multiple: plain copy"
            else:
                child[base + src] = v // p
                child[base + dst] = child[base + dst] * p
                rec["outcome"] = "moved"
    else:
        rec["outcome"] = "gate not below mutate_q16: plain copy"
    rec["child"] = child
    return rec


def tie_gemm():
    """GEMM 96 x 120 x 36 (fp32, 4 + 4 + 2 levels).  i = (6, V, 2, I) with V I = 8, j = (15, V, 1, I) with V I = 8,
    k = (6, 6); the 16 combinations of (V, I) in {(1,8), (2,4), (4,2), (8,1)}^2 have the same symbols, hence the same
    score.  The population is 64 candidates, candidate c holding combination c mod 16."""
    vi = [(1, 8), (2, 4), (4, 2), (8, 1)]
    variants = [[6, a[0], 2, a[1], 15, b[0], 1, b[1], 6, 6] for b in vi for a in vi]
    # S_spec after the first PriorFilter: the 16 schedules (the k = 16 best of S_x are candidates 0..15, all tied), by hash
    spec = sorted(variants, key=schedule_hash)
    out = {"subgraph": {"kind": "gemm", "M": 96, "N": 120, "K": 36, "rd_levels": 2, "frag": [0, 0, 0]},
           "variants": variants, "population": "64 candidates, candidate c = variants[c mod 16]", "n": 64, "k": 16, "seed": 0,
           "spec": spec, "spec_hash": [f"0x{schedule_hash(s):016X}" for s in spec]}
    # child 0 of step 0 with seed 0 uses the two first published outputs; its gate is 0xA839 = 43065:
    assert (0xE220A8397B1DCDAF >> 32) & 0xFFFF == 43065
    runs = []
    for q16, count in ((43066, 64), (43065, 8)):
        kids = [trace_child(0, 0, j, spec, q16, 2, 1, 2, (0, 0, 0)) for j in range(count)]
        runs.append({"mutate_q16": q16, "n_steps": 1, "children": kids})
    assert runs[0]["children"][0]["mutates"] and not runs[1]["children"][0]["mutates"]      # either side of the threshold
    seen = {k["outcome"] for k in runs[0]["children"]}
    assert {"moved", "factor is 1: plain copy", "gate not below mutate_q16: plain copy"} <= seen
    assert any(len(k.get("primes", ())) > 1 and k["p"] != k["primes"][0] for k in runs[0]["children"])   # a later prime is picked
    # two steps without mutation: step 1 copies members of S_spec, which then stays as it is; the children of the second
    # step (t = 1) show the step's place in the counter
    kids = [trace_child(0, 1, j, spec, 0, 2, 1, 2, (0, 0, 0)) for j in range(24)]
    runs.append({"mutate_q16": 0, "n_steps": 2, "children": kids})
    out["runs"] = runs
    return out


def fragment_gemm():
    """fp16 GEMM 256 x 256 x 128 in fragment mode (16 x 16 x 16), 4 + 4 + 3 levels; the population is 256 copies of one
    schedule, so S_spec is that schedule alone and every child mutates it."""
    base = [2, 2, 2, 32, 4, 2, 2, 16, 2, 2, 32]
    kids = [trace_child(1234567, 0, j, [base], 65536, 2, 1, 3, (16, 16, 16)) for j in range(96)]
    seen = {k["outcome"] for k in kids}
    assert "would break the fragment multiple: plain copy" in seen
    assert any(k["outcome"] == "moved" and k["src"] == (3 if k["axis"] < 2 else 2) for k in kids)   # a legal move out of an innermost tile
    return {"subgraph": {"kind": "gemm", "M": 256, "N": 256, "K": 128, "rd_levels": 3, "frag": [16, 16, 16], "dtype_bytes": 2},
            "variants": [base], "population": "256 copies of variants[0]", "n": 256, "k": 1, "seed": 1234567, "spec": [base], "spec_hash": [f"0x{schedule_hash(base):016X}"],
            "runs": [{"mutate_q16": 65536, "n_steps": 1, "children": kids}]}


def main():
    doc = {"what": "explorer-loop cases traced in plain integer arithmetic from the published SplitMix64; written by make_lse_trace.py",
           "scenarios": {"tie_gemm": tie_gemm(), "fragment_gemm": fragment_gemm()}}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lse_trace.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=None, separators=(",", ":"))
        f.write("\n")
    print(path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
