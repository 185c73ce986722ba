"""Host side of the fused gradient -> reshard path (no GPU): the row segments of one source rank against
the oracle's unit lists, for plain and grouped-query layouts."""
import pytest

import paper_2504_06095_amd as N
from oracle import ntp_oracle as O
from paper_2504_06095_amd.binding import NTP_ERR_UNSUPPORTED, NTP_KIND_PLAIN, NTP_KIND_QKV_GQA, NtpError

BASE, STEP = 1 << 40, 1 << 32  # fake, well separated device addresses of the destination shards


def _check(rows, cols, unit, kind, a, b, n_q=0, n_kv=0, absent=()):
    n_units = rows // unit
    okind = O.QKV_GQA if kind == NTP_KIND_QKV_GQA else O.PLAIN
    spec = N.tensor_spec(rows, cols, 0, unit, 4, kind, n_q, n_kv)
    ld = cols + 4
    dst = [None if d in absent else (BASE + d * STEP, ld) for d in range(b)]
    for r in range(a):
        if okind == O.QKV_GQA:
            # a KV head that another source rank holds too: this rank's rows are a partial sum, the fused path refuses
            mine = {u for u in O.unit_list(okind, n_units, a, r, n_q, n_kv) if u >= n_q}
            shared = any(mine & set(O.unit_list(okind, n_units, a, o, n_q, n_kv)) for o in range(a) if o != r)
            if shared:
                with pytest.raises(NtpError) as e:
                    N.ntp_reshard_row_segments(spec, a, r, b, dst)
                assert e.value.status == NTP_ERR_UNSUPPORTED
                continue
        segs = N.ntp_reshard_row_segments(spec, a, r, b, dst)
        got = {}
        for s in segs:
            d, off = divmod(s.dst - BASE, STEP)
            assert 0 <= d < b and s.ld == ld and off % (4 * ld) == 0 and s.rows > 0
            assert s.row_begin % unit == 0 and s.rows % unit == 0
            for q in range(s.rows // unit):
                key = (d, off // (4 * ld) // unit + q)
                assert key not in got
                got[key] = s.row_begin // unit + q
        want = {}
        for d in range(b):
            if d in absent:
                continue
            for j in range(len(O.unit_list(okind, n_units, b, d, n_q, n_kv))):
                sr, sl = O.reshard_source_of(okind, n_units, a, b, d, j, n_q, n_kv)
                if sr == r:
                    want[(d, j)] = sl
        assert got == want, (a, b, r)


@pytest.mark.parametrize("a,b", [(7, 8), (8, 7), (3, 5), (5, 3), (4, 4), (1, 6), (9, 2)])
def test_row_segments_plain(a, b):
    _check(100, 16, 1, NTP_KIND_PLAIN, a, b)
    _check(96, 8, 4, NTP_KIND_PLAIN, a, b)


@pytest.mark.parametrize("a,b", [(5, 7), (7, 5), (16, 3), (3, 16), (4, 4), (2, 7), (4, 16), (1, 3)])
def test_row_segments_gqa(a, b):
    n_q, n_kv, d = 16, 4, 8
    _check((n_q + 2 * n_kv) * d, 24, d, NTP_KIND_QKV_GQA, a, b, n_q, n_kv)
    _check(3 * 12 * d, 24, d, NTP_KIND_QKV_GQA, a, b, 12, 12)  # one KV head per query head: nothing is replicated


def test_row_segments_absent_destinations_and_errors():
    _check(100, 16, 1, NTP_KIND_PLAIN, 7, 8, absent=(1, 5))
    spec = N.tensor_spec(100, 16, 0, 1, 4)
    dst = [(BASE + d * STEP, 16) for d in range(8)]
    with pytest.raises(NtpError):
        N.ntp_reshard_row_segments(spec, 7, 7, 8, dst)  # rank out of range
    with pytest.raises(NtpError):
        N.ntp_reshard_row_segments(N.tensor_spec(16, 100, 1, 1, 4), 7, 0, 8, dst)  # column-partitioned
    with pytest.raises(NtpError):
        N.ntp_reshard_row_segments(N.tensor_spec(100, 16, 0, 1, 2), 7, 0, 8, dst)  # not fp32
    with pytest.raises(NtpError):
        N.ntp_reshard_row_segments(spec, 7, 0, 8, [(BASE + d * STEP, 12) for d in range(8)])  # rows too short
