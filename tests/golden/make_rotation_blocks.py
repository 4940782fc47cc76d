#!/usr/bin/env python3
"""Writes tests/golden/rotation_sensitive_blocks.txt: INPUT blocks (32 bf16 bit patterns each) on which the
rounding order of the 32-point rotation of App. A.2 is observable in the FP4 codes.

The rotation is evaluated in fp32: butterflies h = 1, 2, 4, 8, 16, each add/sub rounded, then one multiply by
fl32(2^-2.5).  Moving the multiply in front, a constant one ulp off or another stage order change the rotated
values by an ulp or so, which shows in a code only when a value sits next to a rounding threshold (about one
element in a million), so such blocks are searched for here once, with numpy alone (no oracle, no GPU code),
and only the inputs are stored: tests/test_oracle_quantize.py recomputes every variant stage by stage.

Usage: python tests/golden/make_rotation_blocks.py   (a few minutes; seeded, reproducible)
"""
import os

import numpy as np

VARIANTS = ("scale_first", "ulp_down", "ulp_up", "stages_reversed")
WANT = 4  # blocks per variant
THR = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])


def rotate(X, variant):
    c_bits = {"ulp_down": 0x3E3504F2, "ulp_up": 0x3E3504F4}.get(variant, 0x3E3504F3)
    c = np.array([c_bits], dtype=np.uint32).view(np.float32)[0]
    V = X.copy()
    if variant == "scale_first":
        V = V * c
    idx = np.arange(32)
    for h in ((16, 8, 4, 2, 1) if variant == "stages_reversed" else (1, 2, 4, 8, 16)):
        lo = idx[(idx & h) == 0]
        a, b = V[:, lo].copy(), V[:, lo + h].copy()
        V[:, lo] = a + b
        V[:, lo + h] = a - b
    if variant != "scale_first":
        V = V * c
    return V


def codes(V):
    eb = (np.abs(V).view(np.uint32).max(axis=1) >> 23).astype(np.int64)
    sb = np.clip(eb - 2, 0, 254)
    t = np.abs(V.astype(np.float64)) * 2.0 ** (127 - sb)[:, None]
    code = np.zeros(t.shape, dtype=np.int64)
    for k, th in enumerate(THR):
        code += (t > th) | ((t == th) & (k % 2 == 1))
    return sb, code + 8 * np.signbit(V)


def to_bf16(X):
    u = X.view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32).view(np.float32)


def main():
    rng = np.random.default_rng(2605)
    found = {v: [] for v in VARIANTS}
    N = 200000
    while any(len(found[v]) < WANT for v in VARIANTS):
        if rng.integers(0, 2):   # one scale per block
            X = rng.standard_normal((N, 32)).astype(np.float32) * rng.choice(
                np.array([1e-3, 1.0, 37.0], dtype=np.float32), size=(N, 1))
        else:                    # exponents spread inside the block: the butterflies themselves round
            X = rng.standard_normal((N, 32)).astype(np.float32) * np.exp2(rng.uniform(-9, 9, size=(N, 32))).astype(np.float32)
        X = to_bf16(np.ascontiguousarray(X))
        sb0, c0 = codes(rotate(X, "ref"))
        for v in VARIANTS:
            if len(found[v]) >= WANT:
                continue
            sb1, c1 = codes(rotate(X, v))
            hit = np.flatnonzero((sb1 != sb0) | (c1 != c0).any(axis=1))
            for i in hit[: WANT - len(found[v])]:
                found[v].append(X[i].view(np.uint32) >> 16)
        print({v: len(found[v]) for v in VARIANTS}, flush=True)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "rotation_sensitive_blocks.txt")
    with open(path, "w") as f:
        f.write("# Input blocks (32 bf16 bit patterns, hex) whose FP4 codes after the 32-point rotation of App. A.2 depend on\n"
                "# the rounding order; first column: the variant that was seen to differ from the reference order.\n"
                "# Written by tests/golden/make_rotation_blocks.py (numpy only); holds inputs, no expected values.\n")
        for v in VARIANTS:
            for blk in found[v]:
                f.write(v + " " + " ".join(f"{int(b):04x}" for b in blk) + "\n")
    print("wrote", path)


if __name__ == "__main__":
    main()
