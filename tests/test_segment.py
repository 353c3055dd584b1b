"""Sender-side segmentation (tensor buffer -> staged chunks + send records): pins of the oracle on
the CPU, parity of the GPU path under -m gpu."""
import numpy as np
import pytest

import oracle
from synth import header as hd
from synth import payload as pl
from synth.layout import DESC, NO_FORWARD


def tensor_bytes(seed, n):
    return pl.rng(seed, 77).integers(0, 256, n).astype(np.uint8)


# ---- oracle pins ---------------------------------------------------------------------------

@pytest.mark.parametrize("n_chunks,chunk,stride", [(1, 16, 16), (7, 48, 48), (7, 48, 80), (300, 64, 64), (520, 32, 96)])
def test_whole_chunks_are_a_reshape(n_chunks, chunk, stride):
    """With a length that is a whole number of chunks, staging viewed as rows of `stride` bytes holds
    the tensor range viewed as rows of `chunk` bytes; bytes between and around the slots keep theirs."""
    t = tensor_bytes(1, 4096 + n_chunks * chunk)
    off, base = 1024, 32
    stage = np.full(base + n_chunks * stride + 64, 0xEE, dtype=np.uint8)
    d = oracle.segment(stage, t, off, n_chunks * chunk, chunk, base, stride)
    rows = stage[base:base + n_chunks * stride].reshape(n_chunks, stride)
    assert np.array_equal(rows[:, :chunk], t[off:off + n_chunks * chunk].reshape(n_chunks, chunk))
    assert np.all(rows[:, chunk:] == 0xEE) and np.all(stage[:base] == 0xEE) and np.all(stage[base + n_chunks * stride:] == 0xEE)
    assert np.array_equal(d["stage_off"], base + stride * np.arange(n_chunks)) and np.all(d["len"] == chunk)


@pytest.mark.parametrize("nbytes", [1, 15, 16, 17, 47, 49, 100, 4097])
def test_ragged_tail_and_concatenation(nbytes):
    """The staged payloads, read back in record order, are the tensor range; only the last is short."""
    chunk, stride = 48, 64
    t = tensor_bytes(2, 8192)
    stage = np.full(2 * 8192, 0x5A, dtype=np.uint8)
    d = oracle.segment(stage, t, 160, nbytes, chunk, 16, stride)
    assert len(d) == -(-nbytes // chunk) and np.all(d["len"][:-1] == chunk) and d["len"][-1] == nbytes - chunk * (len(d) - 1)
    back = np.concatenate([stage[o:o + n] for o, n in zip(d["stage_off"], d["len"])])
    assert np.array_equal(back, t[160:160 + nbytes])
    used = np.zeros(len(stage), bool)
    for o, n in zip(d["stage_off"], d["len"]):
        used[o:o + n] = True
    assert np.all(stage[~used] == 0x5A), "nothing outside the payloads is written"
    assert len(oracle.segment(stage, t, 0, 0, chunk)) == 0


def test_headers_follow_the_field_widths():
    """Section 3.1: 8-bit connection id, 7-bit message id, 8-bit chunk sequence number, last-chunk mark.
    A run of 600 chunks starting at sequence number 250 of message 126: messages of 256 chunks, ids
    wrapping at 128, the mark on sequence number 255 and on the very last chunk."""
    chunk = 16
    t = tensor_bytes(3, 600 * chunk)
    stage = np.zeros(600 * chunk, dtype=np.uint8)
    d = oracle.segment(stage, t, 0, 600 * chunk - 5, chunk, conn_id=201, msg_id=126, first_csn=250)
    f = hd.unpack(d["header"])      # the field positions are the shared interface; widths are the paper's
    number = 250 + np.arange(600)
    assert np.array_equal(f["csn"], number % 256) and np.array_equal(f["msg"], (126 + number // 256) % 128)
    assert np.all(f["conn"] == 201) and np.all(f["spare"] == 0)
    assert np.array_equal(f["last"], ((number % 256 == 255) | (np.arange(600) == 599)).astype(np.uint32))
    assert np.array_equal(d["header"], hd.pack(201, (126 + number // 256) % 128, number % 256, f["last"]))
    # what the receiver derives from these headers: every message's chunk count
    counts = hd.chunk_counts(d["header"])
    # chunk numbers 250..849: messages 126 (from its sequence number 250), 127, 0 run to 255; message 1 ends at 849 - 768
    assert counts[126] == 256 and counts[127] == 256 and counts[0] == 256 and counts[1] == 82 and counts[2:126].sum() == 0


def test_segment_then_scatter_is_the_identity():
    """The staged chunks, taken as arrivals of an all-to-all scatter whose records point back at the
    tensor's offsets, rebuild the tensor range: segmentation and placement are inverse to each other."""
    chunk, stride, nbytes = 64, 64, 64 * 37 + 40
    t = tensor_bytes(4, 8192)
    stage = np.zeros(40 * stride, dtype=np.uint8)
    d = oracle.segment(stage, t, 512, nbytes, chunk, 0, stride)
    rec = np.zeros(len(d), dtype=DESC)
    rec["src_off"], rec["dst_off"], rec["out_off"] = d["stage_off"], 512 + chunk * np.arange(len(d)), NO_FORWARD
    rec["len"], rec["seq"] = d["len"], np.arange(len(d))
    dst = np.zeros_like(t)
    order = pl.rng(4, 1).permutation(len(d))
    assert oracle.scatter(dst, stage, rec[order], oracle.new_seen(len(d))) == len(d)
    assert np.array_equal(dst[512:512 + nbytes], t[512:512 + nbytes]) and not dst[:512].any() and not dst[512 + nbytes:].any()


def test_rejections():
    t, stage = tensor_bytes(5, 1024), np.zeros(1024, dtype=np.uint8)
    bad = [dict(chunk_bytes=24), dict(chunk_bytes=0), dict(tensor_off=8), dict(stage_off=4), dict(slot_stride=40),
           dict(slot_stride=16), dict(nbytes=2048), dict(stage_off=1008), dict(conn_id=256), dict(msg_id=128)]
    codes = [-3, -3, -3, -3, -3, -4, -4, -4, -1, -1]
    for kw, code in zip(bad, codes):
        args = dict(tensor_off=0, nbytes=512, chunk_bytes=32, stage_off=0, slot_stride=32, conn_id=0, msg_id=0)
        args.update(kw)
        with pytest.raises(oracle.OraclePrecondition) as e:
            oracle.segment(stage, t, args["tensor_off"], args["nbytes"], args["chunk_bytes"], args["stage_off"],
                           args["slot_stride"], args["conn_id"], args["msg_id"])
        assert e.value.code == code, kw
    assert not stage.any(), "a rejected call writes nothing"


# ---- GPU parity ----------------------------------------------------------------------------------

def gpu_segment(pkg, t, off, nbytes, chunk, stage_bytes, stage_off=0, stride=None, pinned_descs=False, **hdr):
    import torch
    from gpuhelp import to_dev
    n = -(-nbytes // chunk)
    stage = torch.full((stage_bytes,), 0xC3, dtype=torch.uint8, device="cuda")
    recs = (torch.zeros(max(n, 1) * 16 + 16, dtype=torch.uint8, pin_memory=True) if pinned_descs else
            torch.full((max(n, 1) * 16 + 16,), 0x99, dtype=torch.uint8, device="cuda"))
    pkg.uccl_chunk_segment(stage, to_dev(t), off, nbytes, chunk, stage_off, stride, recs, **hdr)
    torch.cuda.synchronize()
    raw = recs.cpu().numpy() if not pinned_descs else recs.numpy()
    return stage.cpu().numpy(), raw[:n * 16].view(oracle.SEND_DESC).copy(), raw[n * 16:]


@pytest.mark.gpu
@pytest.mark.parametrize("nbytes,chunk,stride", [(1, 16, 16), (15, 16, 32), (4096, 4096, 4096), (300000, 4096, 4096),
                                                 (300001, 32768, 32768 + 64), (70000 * 16 + 7, 2048 + 16, 4096),
                                                 (5 << 20, 128 << 10, 128 << 10), (600 * 48 - 9, 48, 48)])
def test_gpu_segment_parity(gpu_lib, nbytes, chunk, stride):
    t = tensor_bytes(nbytes % 97, nbytes + 4096)
    off, base = 2048, 64
    n = -(-nbytes // chunk)
    stage_bytes = base + n * stride + 256
    hdr = dict(conn_id=77, msg_id=120, first_csn=200)
    got_stage, got_d, beyond = gpu_segment(gpu_lib, t, off, nbytes, chunk, stage_bytes, base, stride, **hdr)
    exp_stage = np.full(stage_bytes, 0xC3, dtype=np.uint8)
    exp_d = oracle.segment(exp_stage, t, off, nbytes, chunk, base, stride, **hdr)
    assert np.array_equal(got_stage, exp_stage), "staging bytes (payloads, gaps and surroundings)"
    assert np.array_equal(got_d, exp_d), "send records"
    assert np.all(beyond == 0x99), "wrote past the records"


@pytest.mark.gpu
def test_gpu_segment_records_in_pinned_memory_and_copy_only(gpu_lib):
    import torch
    from gpuhelp import to_dev
    t = tensor_bytes(9, 1 << 20)
    stage, d, _ = gpu_segment(gpu_lib, t, 0, 1 << 20, 32 << 10, 1 << 20, pinned_descs=True, conn_id=1, msg_id=2)
    exp = np.zeros(1 << 20, dtype=np.uint8)
    assert np.array_equal(d, oracle.segment(exp, t, 0, 1 << 20, 32 << 10, conn_id=1, msg_id=2)) and np.array_equal(stage, exp)
    st = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    gpu_lib.uccl_chunk_segment(st, to_dev(t), 0, 1 << 20, 32 << 10)   # no records asked for
    gpu_lib.uccl_chunk_segment(st, to_dev(t), 0, 0, 32 << 10)         # nothing to do
    torch.cuda.synchronize()
    assert np.array_equal(st.cpu().numpy(), exp)


@pytest.mark.gpu
def test_gpu_segment_equals_scatter_with_identity_records(gpu_lib):
    """The same staging bytes come out of the all-to-all scatter when it is given one record per
    chunk with the tensor as its source: segmentation needs no kernel of its own to be correct,
    the dedicated one only saves the record list, the bitmap and a host-side loop."""
    import torch
    from gpuhelp import to_dev
    nbytes, chunk, stride = 3 * (1 << 20) + 4000, 32 << 10, (32 << 10) + 256
    t = tensor_bytes(11, nbytes + 512)
    n = -(-nbytes // chunk)
    stage, d, _ = gpu_segment(gpu_lib, t, 256, nbytes, chunk, n * stride, 0, stride)
    rec = np.zeros(n, dtype=DESC)
    rec["src_off"], rec["dst_off"], rec["out_off"] = 256 + chunk * np.arange(n), d["stage_off"], NO_FORWARD
    rec["len"], rec["seq"] = d["len"], np.arange(n)
    other = torch.full((n * stride,), 0xC3, dtype=torch.uint8, device="cuda")
    gpu_lib.uccl_chunk_scatter(other, to_dev(t), to_dev(rec), n, torch.zeros((n + 31) // 32, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert np.array_equal(other.cpu().numpy(), stage)


@pytest.mark.gpu
def test_gpu_closed_loop_ring_with_segmented_first_hop(gpu_lib):
    """All ranks on the GPU path, the first hop's chunks cut by uccl_chunk_segment from each rank's
    accumulator (ragged last chunk): equals the textbook ring."""
    import torch
    from gpuhelp import assert_same, to_host
    from ringloop import closed_loop_allreduce
    from test_gpu_parity import GpuBackend
    from synth.layout import F32, BF16, SUM

    class WithSegment(GpuBackend):
        def segment(self, h, off, nbytes, C):
            n = -(-nbytes // C)
            stage = torch.zeros(n * (C + 64), dtype=torch.uint8, device="cuda")
            recs = torch.zeros(n * 16, dtype=torch.uint8, pin_memory=True)
            self.pkg.uccl_chunk_segment(stage, h["acc"], off, nbytes, C, 0, C + 64, recs)
            torch.cuda.synchronize()
            d = recs.numpy().view(oracle.SEND_DESC)
            host = stage.cpu().numpy()
            return [host[o:o + ln].copy() for o, ln in zip(d["stage_off"], d["len"])]

    for dtype, R, n, C in ((F32, 8, 1 << 20, 64 << 10), (BF16, 3, 3 * 5000, 2048)):
        x = pl.uniform_f32(18, 8, R * n).reshape(R, n) if dtype == F32 else pl.normal_bf16(18, 8, R * n).reshape(R, n)
        got = closed_loop_allreduce(WithSegment(gpu_lib), x, dtype, C, seed=6, paths=4, window=None, dup=0.05)
        assert_same(got, oracle.ring_allreduce(x, dtype, SUM), "closed loop, segmented first hop")
