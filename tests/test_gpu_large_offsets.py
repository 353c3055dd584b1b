"""Offsets beyond 4 GiB: every buffer is 5 GiB on the device, the chunks sit around the 2^32
byte boundary (one straddles it) and at the very end, so that any 32-bit offset arithmetic in a
kernel would read or write the wrong place.  The oracle works on compact host copies of the
touched regions with the same records rebased; the device result is compared region by region
and everything outside the regions must stay zero."""
import numpy as np
import pytest
import torch

import oracle
from synth import payload as pl
from synth.layout import DESC, GATHER_DESC, NO_FORWARD, FORWARD_ONLY, F32, BF16, SUM, COPY

from gpuhelp import to_dev

pytestmark = pytest.mark.gpu

BIG = 5 << 30
C = 64 << 10
N = 24


def big_offsets():
    """(src, dst, out) byte offsets of chunk i in the 5 GiB buffers; 16-byte aligned, disjoint."""
    i = np.arange(N, dtype=np.uint64)
    src = np.uint64(BIG) - (i + np.uint64(1)) * np.uint64(C)                       # from the end downwards
    dst = np.uint64((1 << 32) - 2 * C) + i * np.uint64(3 * C)                       # spaced, from just below 4 GiB
    out = np.uint64((1 << 32) - C // 2) + i * np.uint64(C)                          # chunk 0 straddles 2^32
    return src, dst, out


def upload(big, offsets, small, nbytes):
    view = small.view(np.uint8).reshape(N, nbytes)
    for k, off in enumerate(offsets):
        big[int(off):int(off) + nbytes] = torch.from_numpy(view[k].copy()).cuda()


def download_and_clear(big, offsets, nbytes):
    rows = []
    for off in offsets:
        rows.append(big[int(off):int(off) + nbytes].cpu().numpy())
        big[int(off):int(off) + nbytes] = 0
    return np.stack(rows)


@pytest.mark.parametrize("dtype,op,relay", [(F32, SUM, False), (BF16, SUM, True), (F32, COPY, False)])
def test_apply_beyond_4gib(gpu_lib, dtype, op, relay):
    g = pl.rng(77, dtype * 10 + op)
    es = 4 if dtype == F32 else 2
    draw = (lambda s: pl.uniform_f32(77, s, N * C // 4)) if dtype == F32 else (lambda s: pl.uniform_bf16(77, s, N * C // 2))
    recv_s, acc_s = draw(1), draw(2)
    src, dst, out = big_offsets()
    order = g.permutation(N)
    arrivals = np.concatenate([order, order[:5]])                                # five retransmitted copies
    lens = np.full(N, C, dtype=np.uint32)
    lens[3], lens[7] = C - 48, 16 + es                                           # ragged units and a byte tail
    d_big = np.zeros(len(arrivals), dtype=DESC)
    d_small = np.zeros(len(arrivals), dtype=DESC)
    for k, s in enumerate(arrivals):
        flag = FORWARD_ONLY if (relay and s % 2 == 0) else np.uint64(0)
        fwd = s % 5 != 4
        d_big[k] = (src[s], dst[s], (out[s] | flag) if fwd else NO_FORWARD, lens[s], s)
        d_small[k] = (s * C, s * C, (np.uint64(s * C) | flag) if fwd else NO_FORWARD, lens[s], s)
    # oracle on the compact copies
    eacc, eout, seen = acc_s.copy(), np.zeros(N * C, dtype=np.uint8), oracle.new_seen(N)
    assert oracle.apply(eacc, eout, recv_s, d_small, seen, dtype, op) == N
    # device: 5 GiB buffers, regions uploaded at the big offsets
    acc = torch.zeros(BIG, dtype=torch.uint8, device="cuda")
    recv = torch.zeros(BIG, dtype=torch.uint8, device="cuda")
    outb = torch.zeros(BIG, dtype=torch.uint8, device="cuda")
    upload(acc, dst, acc_s, C)
    upload(recv, src, recv_s, C)
    bitmap = torch.zeros(1, dtype=torch.int32, device="cuda")
    rejected = torch.zeros(1, dtype=torch.int32, device="cuda")
    half = len(arrivals) // 2
    dd = to_dev(d_big)
    gpu_lib.uccl_chunk_apply(acc, outb, recv, dd, half, bitmap, dtype, op)
    gpu_lib.uccl_chunk_apply_checked(acc, outb, recv, dd[half * 32:], len(arrivals) - half, bitmap, dtype, op,
                                     n_rejected=rejected, n_bits=N)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0 and int(bitmap.item()) == (1 << N) - 1
    got_acc = download_and_clear(acc, dst, C)
    got_out = download_and_clear(outb, out, C)
    assert np.array_equal(got_acc.reshape(-1), eacc.view(np.uint8)), "accumulator regions"
    assert np.array_equal(got_out.reshape(-1), eout), "staging regions"
    assert not bool(acc.any()) and not bool(outb.any()), "nothing outside the chunks' own regions was written"
    del acc, recv, outb
    torch.cuda.empty_cache()


def test_scatter_and_gather_beyond_4gib(gpu_lib):
    g = pl.rng(78, 1)
    src, dst, out = big_offsets()
    recv_s = pl.uniform_f32(78, 1, 3 * N * C // 4)                                  # three sources per chunk
    acc_s = pl.uniform_f32(78, 2, N * C // 4)
    dst_big = torch.zeros(BIG, dtype=torch.uint8, device="cuda")
    recv = torch.zeros(BIG, dtype=torch.uint8, device="cuda")
    # source j of chunk i lives at src[i] - j * N * C (three bands below the end of the buffer)
    band = np.uint64(N * C)
    for j in range(3):
        upload(recv, src - np.uint64(j) * band, recv_s[j * N * C // 4:(j + 1) * N * C // 4], C)
    # scatter of band 0 with byte-granular lengths
    lens = np.full(N, C, dtype=np.uint32)
    lens[1], lens[2] = 4099, 1
    arrivals = np.concatenate([g.permutation(N), [0, 5]])
    d_big = np.zeros(len(arrivals), dtype=DESC)
    d_small = np.zeros(len(arrivals), dtype=DESC)
    for k, s in enumerate(arrivals):
        d_big[k] = (src[s], dst[s], NO_FORWARD, lens[s], s)
        d_small[k] = (s * C, s * C, NO_FORWARD, lens[s], s)
    edst, seen = np.zeros(N * C, dtype=np.uint8), oracle.new_seen(N)
    assert oracle.scatter(edst, recv_s[:N * C // 4], d_small, seen) == N
    bitmap = torch.zeros(1, dtype=torch.int32, device="cuda")
    gpu_lib.uccl_chunk_scatter(dst_big, recv, to_dev(d_big), len(arrivals), bitmap)
    torch.cuda.synchronize()
    got = download_and_clear(dst_big, dst, C)
    assert np.array_equal(got.reshape(-1), edst) and not bool(dst_big.any())
    # gather-reduce of the three bands into the accumulator at the big destinations
    upload(dst_big, dst, acc_s, C)
    gd_big = np.zeros(N, dtype=GATHER_DESC)
    gd_small = np.zeros(N, dtype=GATHER_DESC)
    for k, s in enumerate(g.permutation(N)):
        gd_big[k]["dst_off"], gd_big[k]["out_off"], gd_big[k]["len"], gd_big[k]["seq"], gd_big[k]["n_src"] = dst[s], NO_FORWARD, C, s, 3
        gd_small[k]["dst_off"], gd_small[k]["out_off"], gd_small[k]["len"], gd_small[k]["seq"], gd_small[k]["n_src"] = s * C, NO_FORWARD, C, s, 3
        for j in range(3):
            gd_big[k]["src_off"][j] = src[s] - np.uint64(j) * band
            gd_small[k]["src_off"][j] = j * N * C + s * C
    eacc, seen = acc_s.copy(), oracle.new_seen(N)
    assert oracle.reduce_gather(eacc, None, recv_s, gd_small, seen, F32, SUM) == N
    bitmap.zero_()
    gpu_lib.uccl_chunk_reduce_gather(dst_big, None, recv, to_dev(gd_big), N, bitmap, F32, SUM)
    torch.cuda.synchronize()
    got = download_and_clear(dst_big, dst, C)
    assert np.array_equal(got.reshape(-1), eacc.view(np.uint8)) and not bool(dst_big.any())
    del dst_big, recv
    torch.cuda.empty_cache()


@pytest.mark.parametrize("length", [0xFFFFFFF0, 0xFFFFFFFC])
def test_one_record_of_almost_4gib(gpu_lib, length):
    """The largest chunk a record can name (len is 32 bits wide): one workgroup walks two million
    units.  Too large for the host oracle to be worth it; the expected value is the device
    library's own IEEE fp32 add, which equals one correctly rounded add per element."""
    n = 1 << 30                                     # fp32 elements in 4 GiB
    g = torch.Generator(device="cuda").manual_seed(5)
    acc = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1, 1, generator=g)
    recv = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1, 1, generator=g)
    out = torch.zeros(n, dtype=torch.float32, device="cuda")
    ref = acc + recv
    k = length // 4
    ref[k:] = acc[k:]                               # beyond the chunk the accumulator is untouched
    d = np.zeros(2, dtype=DESC)
    d[0] = (0, 0, 0, length, 0)
    d[1] = (0, 0, 0, length, 0)                     # and its retransmitted copy
    bitmap = torch.zeros(1, dtype=torch.int32, device="cuda")
    gpu_lib.uccl_chunk_apply(acc, out, recv, to_dev(d), 2, bitmap, F32, SUM)
    torch.cuda.synchronize()
    assert int(bitmap.item()) == 1
    assert torch.equal(acc.view(torch.int32), ref.view(torch.int32))
    assert torch.equal(out[:k].view(torch.int32), ref[:k].view(torch.int32)) and not bool(out[k:].any())
    del acc, recv, out, ref
    torch.cuda.empty_cache()
