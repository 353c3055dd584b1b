"""Multi-sender reduce (one record folds several receive slots into one destination chunk):
oracle pins on the CPU, parity of the GPU path under -m gpu."""
import numpy as np
import pytest

import oracle
from synth import payload as pl
from synth import workloads as wl
from synth.layout import GATHER_DESC, DESC, NO_FORWARD, FORWARD_ONLY, F32, BF16, F16, I32, SUM, MAX, MIN, PROD, ELEM_SIZE

from test_oracle_pins import nearest_even_bf16


def run_oracle(w, op=None):
    acc = w.acc.copy()
    out = np.zeros(max(w.out_bytes, 16), dtype=np.uint8) if w.out_bytes else None
    seen = oracle.new_seen(w.n_bits)
    ph = w.phases[0]
    n = oracle.reduce_gather(acc, out, w.recv_stage, ph.descs, seen, w.dtype, ph.op if op is None else op)
    return acc, out, oracle.pack_bitmap(seen), n


def numpy_fold(w, f, order=None):
    """Third opinion for fp32 / int32: fold each destination chunk with numpy, one
    operation (one rounding) per source, in the record's order."""
    acc = w.acc.copy()
    es = ELEM_SIZE[w.dtype]
    done = set()
    for d in w.phases[0].descs:
        if int(d["seq"]) in done:
            continue
        done.add(int(d["seq"]))
        n, t = d["len"] // es, d["dst_off"] // es
        val = acc[t:t + n]
        srcs = d["src_off"][:d["n_src"]]
        for so in (srcs if order is None else srcs[order]):
            val = f(val, w.recv_stage[so // es: so // es + n])
        acc[t:t + n] = val
    return acc


def make(dtype, dist="uniform", op=SUM, R=8, C=1024, chunks=37, seed=3, **kw):
    es = ELEM_SIZE[dtype]
    M = R * (chunks * C - 3 * 16)  # the last chunk is short
    return wl.direct_reduce_scatter("g", seed, R=R, M=M, C=C, dtype=dtype, paths=5, dup=0.15, dist=dist, op=op,
                                    reissue=0.3, **kw)


def test_fp32_fold_in_listed_order_against_numpy():
    w = make(F32)
    with np.errstate(over="ignore"):
        acc, _, bm, n = run_oracle(w)
        assert n == w.phases[0].n_unique and len(w.phases[0].descs) > n, "stream re-issues some records"
        assert np.array_equal(acc, numpy_fold(w, np.add))
        # the order of sources is part of the result: another order gives another rounding somewhere
        rev = w.phases[0].descs.copy()
        k = int(rev["n_src"][0])
        rev["src_off"][:, :k] = rev["src_off"][:, :k][:, ::-1]
        w.phases[0].descs = rev
        acc_rev = run_oracle(w)[0]
        assert np.array_equal(acc_rev, numpy_fold(w, np.add))
        assert not np.array_equal(acc_rev, acc)
        assert np.allclose(acc_rev, acc, rtol=1e-5, atol=1e-5)


@pytest.mark.parametrize("op,f", [(MAX, np.maximum), (MIN, np.minimum), (PROD, np.multiply)])
def test_fp32_other_ops_against_numpy(op, f):
    w = make(F32, op=op, R=4)
    assert np.array_equal(run_oracle(w)[0], numpy_fold(w, f))


def test_int32_wraps_and_matches_numpy():
    w = make(I32, R=6)
    with np.errstate(over="ignore"):
        assert np.array_equal(run_oracle(w)[0], numpy_fold(w, np.add))
        assert np.array_equal(run_oracle(w, PROD)[0], numpy_fold(w, np.multiply))
    assert np.array_equal(run_oracle(w, MAX)[0], numpy_fold(w, np.maximum))


def test_bf16_accumulates_in_fp32_and_rounds_once():
    w = make(BF16, dist="normal", R=8)
    wide = lambda h: (h.astype(np.uint32) << 16).view(np.float32)
    acc32 = wide(w.acc).copy()
    per_hop = w.acc.copy()
    done = set()
    for d in w.phases[0].descs:
        if int(d["seq"]) in done:
            continue
        done.add(int(d["seq"]))
        n, t = d["len"] // 2, d["dst_off"] // 2
        for so in d["src_off"][:d["n_src"]]:
            r = wide(w.recv_stage[so // 2: so // 2 + n])
            acc32[t:t + n] = acc32[t:t + n] + r                       # numpy fp32 add
            per_hop[t:t + n] = nearest_even_bf16(wide(per_hop[t:t + n]) + r)
    expect = w.acc.copy()
    S = len(expect)
    expect[:] = nearest_even_bf16(acc32)
    got = run_oracle(w)[0]
    assert np.array_equal(got, expect)
    # and that is not the same as rounding after every source (what chained single applies do)
    assert not np.array_equal(got, per_hop)


def _widen16(dtype):
    """uint16 patterns -> float32 values, through numpy's own types (exact for both formats)."""
    if dtype == BF16:
        return lambda h: (h.astype(np.uint32) << 16).view(np.float32)
    return lambda h: h.view(np.float16).astype(np.float32)


def _fold16(w, step):
    """Per destination chunk: fp32 running array seeded from acc, `step(running, source_bits)` per
    source in the record's order.  Returns {chunk start element: (n, running)}."""
    wide = _widen16(w.dtype)
    runs, done = {}, set()
    for d in w.phases[0].descs:
        if int(d["seq"]) in done:
            continue
        done.add(int(d["seq"]))
        n, t = d["len"] // 2, d["dst_off"] // 2
        val = wide(w.acc[t:t + n])
        for so in d["src_off"][:d["n_src"]]:
            val = step(val, w.recv_stage[so // 2: so // 2 + n])
        runs[int(t)] = (int(n), val)
    return runs


@pytest.mark.parametrize("dtype", [BF16, F16])
def test_16bit_product_fold_runs_in_fp32_and_rounds_once(dtype):
    """numpy multiplies fp32 arrays source by source (one rounding each, in fp32); the 16-bit result is
    that running product rounded once: nearest-even by the exact definition for bf16, numpy's own
    binary16 conversion for f16.  A fold that adds, or that rounds after every source, differs."""
    w = make(dtype, dist="normal" if dtype == BF16 else "uniform", op=PROD, R=6)
    wide = _widen16(dtype)
    narrow = nearest_even_bf16 if dtype == BF16 else (lambda f: f.astype(np.float16).view(np.uint16))
    with np.errstate(over="ignore", under="ignore"):
        runs = _fold16(w, lambda val, r: val * wide(r))
        hops = _fold16(w, lambda val, r: wide(narrow(val * wide(r))))
    got = run_oracle(w)[0]
    expect, per_hop = w.acc.copy(), w.acc.copy()
    for t, (n, val) in runs.items():
        expect[t:t + n] = narrow(val)
        per_hop[t:t + n] = narrow(hops[t][1])
    assert np.array_equal(got, expect)
    assert not np.array_equal(got, per_hop), "the inputs must tell one rounding from a rounding per source"
    assert len(np.unique(got)) > 100, "products neither all vanish nor all overflow"


@pytest.mark.parametrize("dtype", [BF16, F16])
@pytest.mark.parametrize("op,npf", [(MAX, np.maximum), (MIN, np.minimum)])
def test_16bit_selection_fold_against_numpy(dtype, op, npf):
    """Selection is exact: the result is numpy's maximum / minimum over the widened values, and it
    is one of the input patterns unchanged."""
    w = make(dtype, dist="normal" if dtype == BF16 else "uniform", op=op, R=7)
    wide = _widen16(dtype)
    runs = _fold16(w, lambda val, r: npf(val, wide(r)))
    got = run_oracle(w)[0]
    expect = w.acc.copy()
    for t, (n, val) in runs.items():
        # val holds exactly representable 16-bit values: narrowing it back loses nothing
        expect[t:t + n] = (val.view(np.uint32) >> 16).astype(np.uint16) if dtype == BF16 else val.astype(np.float16).view(np.uint16)
        assert np.array_equal(wide(expect[t:t + n]), val)
    assert np.array_equal(got, expect)
    assert not np.array_equal(got, w.acc), "some source beats the local value somewhere"
    last = w.acc.copy()   # a fold that merely copies the last source would give this instead
    for d in w.phases[0].descs:
        n, t, so = d["len"] // 2, d["dst_off"] // 2, d["src_off"][d["n_src"] - 1] // 2
        last[t:t + n] = w.recv_stage[so:so + n]
    assert not np.array_equal(got, last)


def test_int32_min_fold_against_numpy():
    w = make(I32, R=5, op=MIN)
    got = run_oracle(w)[0]
    assert np.array_equal(got, numpy_fold(w, np.minimum))
    assert not np.array_equal(got, numpy_fold(w, np.maximum))


@pytest.mark.parametrize("dtype", [F32, BF16, F16, I32])
def test_integer_inputs_give_the_exact_sum(dtype):
    es = ELEM_SIZE[dtype]
    w = make(dtype, dist="smallint", R=9)
    got = run_oracle(w)[0]
    vals = {F32: lambda x: x.astype(np.int64), I32: lambda x: x.astype(np.int64),
            BF16: lambda x: pl.bf16_bits_to_f64(x).astype(np.int64),
            F16: lambda x: x.view(np.float16).astype(np.int64)}[dtype]
    total = vals(w.acc).copy()
    done = set()
    for d in w.phases[0].descs:
        if int(d["seq"]) in done:
            continue
        done.add(int(d["seq"]))
        n, t = d["len"] // es, d["dst_off"] // es
        for so in d["src_off"][:d["n_src"]]:
            total[t:t + n] += vals(w.recv_stage[so // es: so // es + n])
    assert np.array_equal(vals(got), total) and np.abs(total).max() <= 9 * 8


def test_one_source_is_the_plain_apply():
    w = make(F32, R=2)
    g = w.phases[0].descs
    d = np.zeros(len(g), dtype=DESC)
    d["src_off"], d["dst_off"], d["out_off"], d["len"], d["seq"] = g["src_off"][:, 0], g["dst_off"], g["out_off"], g["len"], g["seq"]
    acc = w.acc.copy()
    oracle.apply(acc, None, w.recv_stage, d, oracle.new_seen(w.n_bits), F32, SUM)
    assert np.array_equal(acc, run_oracle(w)[0])


def test_forwarding_and_relay_flags():
    w = make(F32, R=4)
    d = w.phases[0].descs.copy()
    d["out_off"] = d["dst_off"]
    d["out_off"][d["seq"] % 2 == 1] |= FORWARD_ONLY
    w.phases[0].descs = d
    w.out_bytes = w.acc.nbytes
    acc, out, _, _ = run_oracle(w)
    full = numpy_fold(w, np.add)
    S = 1024 // 4
    for c in range(w.n_bits):
        seg = slice(c * S, min((c + 1) * S, len(full)))
        assert np.array_equal(out.view(np.float32)[seg], full[seg])
        assert np.array_equal(acc[seg], w.acc[seg] if c % 2 else full[seg])


def test_rejects_malformed_records():
    acc, recv = np.zeros(64, np.float32), np.zeros(256, np.float32)
    def rec(n_src=2, src=(0, 256), dst=0, ln=64):
        d = np.zeros(1, dtype=GATHER_DESC)
        d["dst_off"], d["out_off"], d["len"], d["seq"], d["n_src"] = dst, NO_FORWARD, ln, 0, n_src
        d["src_off"][0, :len(src)] = src
        return d
    for bad, code in ((rec(n_src=0), -1), (rec(n_src=17), -1), (rec(src=(0, 8)), -3), (rec(src=(0, 1024 - 32)), -4),
                      (rec(dst=256), -4), (rec(ln=62), -3)):
        with pytest.raises(oracle.OraclePrecondition) as e:
            oracle.reduce_gather(acc, None, recv, bad, oracle.new_seen(1), F32, SUM)
        assert e.value.code == code
    with pytest.raises(oracle.OraclePrecondition):
        oracle.reduce_gather(acc, None, recv, rec(), oracle.new_seen(1), F32, 3)  # COPY is not a fold


# ---- GPU parity ----------------------------------------------------------------------------------

def gpu_run(pkg, w, op=None, checked=True, opts=None):
    import torch
    from gpuhelp import to_dev, to_host
    ph = w.phases[0]
    acc, recv = to_dev(w.acc), to_dev(w.recv_stage)
    out = torch.zeros(max(w.out_bytes, 16), dtype=torch.uint8, device="cuda") if w.out_bytes else None
    bm = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
    rej = torch.zeros(1, dtype=torch.int32, device="cuda")
    pkg.uccl_chunk_reduce_gather(acc, out, recv, to_dev(ph.descs), len(ph.descs), bm, w.dtype,
                                 ph.op if op is None else op, n_rejected=rej if checked else None,
                                 n_bits=w.n_bits if checked else None, opts=opts)
    torch.cuda.synchronize()
    return (to_host(acc, w.acc.dtype), None if out is None else out.cpu().numpy(),
            bm.cpu().numpy().view(np.uint32), int(rej.item()))


@pytest.mark.gpu
@pytest.mark.parametrize("hint", [0, 1024, 4096, 65536])
@pytest.mark.parametrize("dtype,op", [(F32, SUM), (BF16, SUM), (F16, SUM), (I32, SUM), (BF16, MAX), (F16, MIN),
                                      (F32, PROD), (BF16, PROD), (I32, MAX)])
def test_gpu_gather_reduce_parity(gpu_lib, dtype, op, hint):
    from gpuhelp import assert_same
    w = make(dtype, dist="normal" if dtype == BF16 else "uniform", op=op, R=8, C=4112, chunks=29)
    for checked in (True, False):
        acc, out, bm, rej = gpu_run(gpu_lib, w, checked=checked, opts=(hint, 0))
        eacc, eout, ebm, _ = run_oracle(w)
        assert rej == 0
        assert_same(bm, ebm, "bitmap")
        wide = {F32: lambda x: x, BF16: lambda x: (x.astype(np.uint32) << 16).view(np.float32),
                F16: lambda x: x.view(np.float16).astype(np.float32), I32: lambda x: x.astype(np.float32)}[dtype]
        with np.errstate(over="ignore", invalid="ignore"):
            nan = np.isnan(wide(eacc))
        assert np.array_equal(np.isnan(wide(acc)), nan)
        assert_same(acc[~nan], eacc[~nan], "acc")


@pytest.mark.gpu
@pytest.mark.parametrize("R", [2, 3, 17])
def test_gpu_gather_source_counts_forward_and_rejects(gpu_lib, R):
    from gpuhelp import assert_same
    w = make(F32, R=R, C=2064, chunks=11)
    d = w.phases[0].descs.copy()
    d["out_off"] = d["dst_off"]
    d["out_off"][d["seq"] % 3 == 1] |= FORWARD_ONLY
    d["out_off"][d["seq"] % 3 == 2] = NO_FORWARD
    bad = d[:3].copy()
    bad["seq"] = [w.n_bits + 5, 0, 1]           # out of range seq; too many / zero sources
    bad["n_src"][1], bad["n_src"][2] = 17, 0
    w.phases[0].descs = np.concatenate([bad, d])
    w.out_bytes = w.acc.nbytes
    acc, out, bm, rej = gpu_run(gpu_lib, w)
    assert rej == 3
    w.phases[0].descs = d
    eacc, eout, ebm, _ = run_oracle(w)
    assert_same(acc, eacc, "acc"); assert_same(out[:w.out_bytes], eout[:w.out_bytes], "out_stage"); assert_same(bm, ebm, "bitmap")


@pytest.mark.gpu
@pytest.mark.parametrize("opts", [None, (8192, 1), (8192, 5), (65536, 16)])
def test_gpu_gather_exactly_once_all_ones(gpu_lib, opts):
    """Every record several times, far apart, also with each record cut into 5 or 16 parts: 15 = each of
    the 15 sources folded exactly once (a double apply shows as 30, a lost part as 0)."""
    w = make(BF16, dist="ones", R=16, C=8192, chunks=64)
    w.acc[:] = pl.ints_as(np.zeros(1, dtype=np.int64), BF16)[0]
    d = w.phases[0].descs
    w.phases[0].descs = np.concatenate([d, d[::2], d[::-1]])  # every record several times, far apart
    acc, _, bm, rej = gpu_run(gpu_lib, w, opts=opts)
    fifteen = pl.ints_as(np.array([15]), BF16)[0]
    assert rej == 0 and np.all(acc == fifteen)
    assert sum(int(x).bit_count() for x in bm) == w.n_bits
    assert gpu_lib.uccl_claim_timeouts() == 0


@pytest.mark.gpu
def test_gpu_gather_cut_records_on_two_streams(gpu_lib):
    """The same multi-source records issued on two streams at once, every record cut into parts: each
    stream has claim words of its own, the bitmap decides between the streams, every part learns the one
    decision taken for its record."""
    import torch
    from gpuhelp import to_dev, to_host
    w = make(F32, dist="ones", R=8, C=48 << 10, chunks=40)
    w.acc[:] = 0
    ph = w.phases[0]
    for trial in range(3):
        acc, recv, descs = to_dev(w.acc), to_dev(w.recv_stage), to_dev(ph.descs)
        bm = torch.zeros((w.n_bits + 31) // 32, dtype=torch.int32, device="cuda")
        s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        for s in (s1, s2, s1):
            gpu_lib.uccl_chunk_reduce_gather(acc, None, recv, descs, len(ph.descs), bm, F32, SUM, opts=(48 << 10, 4), stream=s)
        s1.synchronize(); s2.synchronize()
        got = to_host(acc, np.float32)
        assert np.all(got == 7.0), f"trial {trial}: {np.count_nonzero(got != 7.0)} elements not exactly 7"
        assert sum(int(x).bit_count() for x in bm.cpu().numpy().view(np.uint32)) == w.n_bits
    assert gpu_lib.uccl_claim_timeouts() == 0
