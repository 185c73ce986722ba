"""Bit-exact parity of ntp_reshard_grad against the oracle's reshard, on a real MI355X."""
import sys

import numpy as np
import pytest

from oracle import ntp_oracle as O

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-case] {msg}", file=sys.stderr, flush=True)


def _run(G, pd, unit, a, b, kind=O.PLAIN, n_q=0, n_kv=0, pad_src=0, pad_dst=0, misalign=0):
    """Cut G into the TP=a layout, reshard a -> b on the GPU, return (got shards, oracle shards, src shards)."""
    import torch
    import paper_2504_06095_amd as N
    Bd = N.binding
    n_units = G.shape[pd] // unit
    src_np = [O.cut_shard(G, pd, unit, kind, a, r, n_q, n_kv) for r in range(a)]
    want = O.reshard(src_np, pd, unit, kind, a, b, n_units, n_q, n_kv)
    tdt = {4: torch.int32, 2: torch.int16}[G.dtype.itemsize]
    sdt = {4: np.int32, 2: np.int16}[G.dtype.itemsize]

    def dev(arr, pad, fill):
        r, c = arr.shape
        # optional misalignment: start `misalign` elements into a larger buffer
        flat = torch.full((r * (c + pad) + misalign + 8,), fill, dtype=tdt, device="cuda")
        view = flat[misalign: misalign + r * (c + pad)].view(r, c + pad)[:, :c]
        if arr.size:
            view.copy_(torch.from_numpy(np.ascontiguousarray(arr).view(sdt)).cuda())
        return view, flat

    src = [dev(s, pad_src, 0x11)[0] for s in src_np]
    dst_pairs = [dev(np.zeros_like(w), pad_dst, 0x22) for w in want]
    dst = [p[0] for p in dst_pairs]
    kind_c = Bd.NTP_KIND_QKV_GQA if kind == O.QKV_GQA else Bd.NTP_KIND_PLAIN
    spec = N.tensor_spec(G.shape[0], G.shape[1], pd, unit, G.dtype.itemsize, kind_c, n_q, n_kv)
    N.ntp_reshard_grad(spec, a, b, src, dst)
    torch.cuda.synchronize()
    got = [d.cpu().numpy().view(G.dtype) for d in dst]
    # padding and guard words of the destination buffers are untouched
    for (view, flat), w in zip(dst_pairs, want):
        r, c = w.shape
        body = flat[misalign: misalign + r * (c + pad_dst)].view(r, c + pad_dst)
        assert (body[:, c:] == 0x22).all() and (flat[:misalign] == 0x22).all()
        assert (flat[misalign + r * (c + pad_dst):] == 0x22).all()
    return got, want, src_np


def _logical(rows, cols, dtype=np.uint32, seed=0):
    g = np.random.default_rng(seed)
    return g.integers(0, np.iinfo(dtype).max, size=(rows, cols), dtype=dtype)


CASES = [
    # rows, cols, pd, unit, a, b, pad_src, pad_dst, misalign
    (4096, 1024, 0, 1, 7, 8, 0, 0, 0),     # config 1 dB: row blocks, dense
    (1024, 4096, 1, 1, 7, 8, 0, 0, 0),     # config 1 dA in the paper's orientation: column blocks, odd widths
    (1024, 4096, 1, 1, 8, 7, 0, 0, 0),
    (333, 1000, 1, 1, 7, 9, 3, 5, 0),      # padded leading dimensions
    (1000, 333, 0, 1, 9, 7, 3, 5, 1),      # padded rows, buffers off 16-byte alignment
    (64, 12000, 1, 1, 30, 32, 0, 0, 3),    # the paper's 375 / 25 sub-shards
    (16 * 24, 40, 0, 16, 5, 7, 0, 0, 0),   # unit > 1 (heads) on rows
    (40, 16 * 24, 1, 16, 7, 5, 0, 1, 0),   # unit > 1 on columns
    (5, 3, 0, 1, 8, 3, 0, 0, 0),           # more ranks than units
    (1, 100000, 1, 1, 3, 4, 0, 0, 0),      # a single long row
    (20000, 1, 0, 1, 4, 3, 0, 0, 0),       # a single column
    (256, 256, 1, 1, 4, 4, 0, 0, 0),       # same degree: plain copy
    (3, 7, 1, 1, 2, 3, 0, 0, 0),           # dense destinations smaller than a 16-byte chunk per row
    (1000, 5, 1, 1, 2, 3, 0, 0, 0),        # one- and two-element rows: a chunk spans several rows
    (17, 1001, 1, 1, 3, 2, 0, 0, 0),       # odd widths, total bytes not a multiple of 16
    (257, 2250, 1, 1, 3, 2, 0, 0, 0),      # several blocks of the flat destination kernel, pieces split mid-chunk
    (4100, 1500, 1, 1, 2, 2, 0, 0, 0),     # same degree on columns, many blocks
]


@pytest.mark.parametrize("rows,cols,pd,unit,a,b,pad_src,pad_dst,misalign", CASES)
def test_reshard_fp32_bit_exact(rows, cols, pd, unit, a, b, pad_src, pad_dst, misalign):
    _say(f"reshard {rows}x{cols} pd={pd} unit={unit} {a}->{b} pads {pad_src},{pad_dst} mis {misalign}")
    G = _logical(rows, cols)
    got, want, _ = _run(G, pd, unit, a, b, pad_src=pad_src, pad_dst=pad_dst, misalign=misalign)
    for s in range(b):
        assert np.array_equal(got[s], want[s]), f"dst rank {s}"


@pytest.mark.parametrize("pd,a,b,misalign", [(1, 7, 8, 0), (1, 7, 8, 1), (0, 8, 7, 0), (1, 5, 3, 3)])
def test_reshard_bf16_elements(pd, a, b, misalign):
    _say(f"reshard 2-byte elements pd={pd} {a}->{b} mis {misalign}")
    G = _logical(301, 515, np.uint16) if pd == 1 else _logical(515, 301, np.uint16)
    got, want, _ = _run(G, pd, 1, a, b, misalign=misalign)
    for s in range(b):
        assert np.array_equal(got[s], want[s])


@pytest.mark.parametrize("pd", [0, 1])
def test_reshard_qkv_gqa(pd):
    _say(f"reshard GQA pd={pd}")
    n_q, n_kv, d = 16, 4, 8
    ext = (n_q + 2 * n_kv) * d
    G = _logical(ext, 96) if pd == 0 else _logical(96, ext)
    for a, b in [(5, 7), (7, 5), (16, 3)]:
        got, want, _ = _run(G, pd, d, a, b, O.QKV_GQA, n_q, n_kv)
        for s in range(b):
            assert np.array_equal(got[s], want[s])


def test_reshard_round_trip_and_special_values():
    import torch
    _say("reshard round trip with NaN payloads")
    G = _logical(512, 4099)
    G[0, :6] = [0x7FC00001, 0xFFC12345, 0x80000000, 0x00000001, 0x7F800000, 0xFF800000]
    mid, want_mid, src = _run(G, 1, 1, 7, 8)
    for s in range(8):
        assert np.array_equal(mid[s], want_mid[s])
    # go back 8 -> 7 from what the GPU produced
    Gmid = np.concatenate(mid, axis=1)
    assert np.array_equal(Gmid, G)
    back, _, _ = _run(Gmid, 1, 1, 8, 7)
    for r in range(7):
        assert np.array_equal(back[r], src[r])


def test_reshard_one_gpu_share_and_alias_check():
    import torch
    import paper_2504_06095_amd as N
    _say("reshard NULL shards / alias")
    rows, cols, a, b = 64, 700, 7, 8
    G = _logical(rows, cols)
    src_np = [O.cut_shard(G, 1, 1, O.PLAIN, a, r) for r in range(a)]
    want = O.reshard(src_np, 1, 1, O.PLAIN, a, b, cols)
    spec = N.tensor_spec(rows, cols, 1, 1, 4)
    # only source rank 2 is on this GPU: destination elements fed by other ranks stay untouched
    src = [None] * a
    src[2] = torch.from_numpy(src_np[2].view(np.int32)).cuda()
    dst = [torch.full(w.shape, -1, dtype=torch.int32, device="cuda") for w in want]
    N.ntp_reshard_grad(spec, a, b, src, dst)
    torch.cuda.synchronize()
    o2, w2 = O.shard_plan(cols, a, 2)
    for s in range(b):
        do, dw = O.shard_plan(cols, b, s)
        got = dst[s].cpu().numpy().view(np.uint32)
        for j in range(dw):
            fed = o2 <= do + j < o2 + w2
            col = got[:, j]
            assert np.array_equal(col, want[s][:, j]) if fed else (col == 0xFFFFFFFF).all()
    # aliasing source and destination is refused
    full = [torch.from_numpy(s.view(np.int32)).cuda() for s in src_np]
    bad_dst = list(dst)
    bad_dst[0] = full[0][:, : want[0].shape[1]]
    with pytest.raises(N.NtpError) as ei:
        N.ntp_reshard_grad(spec, a, b, full, bad_dst)
    assert ei.value.status == N.binding.NTP_ERR_INVALID_ARG
    # a leading dimension smaller than the shard width is refused
    lib = N.binding.lib()
    import ctypes as C
    sp, sl = (C.c_void_p * a)(*[t.data_ptr() for t in full]), (C.c_int64 * a)(*[1] * a)
    dp, dl = (C.c_void_p * b)(*[t.data_ptr() for t in dst]), (C.c_int64 * b)(*[t.stride(0) for t in dst])
    assert lib.ntp_reshard_grad(N.default_handle().ptr, C.byref(spec), a, b, sp, sl, dp, dl, None) == N.binding.NTP_ERR_INVALID_ARG
