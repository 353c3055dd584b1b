"""Brute force on tiny inputs: an independent model of the data path written in plain Python
(a dict of applied sequence numbers, numpy scalar arithmetic per element) must agree with
the C oracle on random record streams that mix every feature."""
import numpy as np
import pytest

import oracle
from synth.layout import NO_FORWARD, FORWARD_ONLY, F32, BF16, F16, I32, SUM, MAX, MIN, COPY, PROD, ELEM_SIZE

from randstream import random_stream
from test_oracle_pins import nearest_even_bf16


def model_element(a, r, dtype, op):
    """One element, by the definition, using numpy scalars (never the oracle)."""
    if op == COPY:
        return r
    if dtype == I32:
        with np.errstate(over="ignore"):
            return {SUM: np.int32(a) + np.int32(r), PROD: np.int32(a) * np.int32(r),
                    MAX: r if r > a else a, MIN: r if r < a else a}[op]
    if dtype == F32:
        with np.errstate(over="ignore", invalid="ignore"):
            return {SUM: np.float32(a) + np.float32(r), PROD: np.float32(a) * np.float32(r),
                    MAX: r if r > a else a, MIN: r if r < a else a}[op]
    wide = (lambda h: np.array([h], np.uint16).view(np.float16).astype(np.float32)[0]) if dtype == F16 else \
           (lambda h: (np.array([h], np.uint32) << 16).view(np.float32)[0])
    fa, fr = wide(a), wide(r)
    if op in (MAX, MIN):
        take = fr > fa if op == MAX else fr < fa
        return r if take else a
    with np.errstate(over="ignore", invalid="ignore"):
        f = np.float32(fa + fr) if op == SUM else np.float32(fa * fr)
        if dtype == F16:
            return np.array([f], np.float32).astype(np.float16).view(np.uint16)[0]
        return nearest_even_bf16(np.array([f], np.float32))[0]


def model_apply(s):
    es = ELEM_SIZE[s["dtype"]]
    acc, out, seen = s["acc"].copy(), np.full(s["out_bytes"], 0x3C, np.uint8), {}
    outv = out.view(acc.dtype)
    for d in s["descs"]:
        if int(d["seq"]) in seen:
            continue
        seen[int(d["seq"])] = True
        fwd = d["out_off"] != NO_FORWARD
        keep = not (fwd and (d["out_off"] & FORWARD_ONLY))
        o = int(d["out_off"] & ~FORWARD_ONLY) // es
        for i in range(int(d["len"]) // es):
            t = model_element(acc[int(d["dst_off"]) // es + i], s["recv"][int(d["src_off"]) // es + i], s["dtype"], s["op"])
            if keep:
                acc[int(d["dst_off"]) // es + i] = t
            if fwd:
                outv[o + i] = t
    bits = np.zeros(s["n_bits"], np.uint8)
    bits[list(seen)] = 1
    return acc, out, bits


@pytest.mark.parametrize("dtype", [F32, BF16, F16, I32])
@pytest.mark.parametrize("op", [SUM, MAX, MIN, COPY, PROD])
def test_oracle_equals_python_model_on_random_streams(dtype, op):
    for seed in range(4):
        s = random_stream(1000 * dtype + 10 * op + seed, dtype, op, max_chunks=9, max_len=260)
        macc, mout, mbits = model_apply(s)
        acc, out, seen = s["acc"].copy(), np.full(s["out_bytes"], 0x3C, np.uint8), oracle.new_seen(s["n_bits"])
        half = len(s["descs"]) // 2
        oracle.apply(acc, out, s["recv"], s["descs"][:half], seen, dtype, op)   # in two calls
        oracle.apply(acc, out, s["recv"], s["descs"][half:], seen, dtype, op)
        nan = np.zeros(len(acc), bool)
        if dtype in (F32,):
            nan = np.isnan(macc)
        assert np.array_equal(acc[~nan], macc[~nan]) and np.array_equal(seen, mbits)
        assert np.array_equal(out, mout) or dtype == F32 and np.isnan(mout.view(np.float32)).any()
