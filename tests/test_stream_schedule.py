"""Host logic of the sequencer's stream schedule: which call waits for which, worked out from the calls' own reads and writes
(no GPU: the dependency rules are exercised on CPU tensors, nothing is launched)."""
import torch

from paper_1812_10624_amd import api
from paper_1812_10624_amd.netrun import _PARAMS, _WRITES, StreamSchedule


def fresh(n=4):
    sc = StreamSchedule.__new__(StreamSchedule)      # no streams are made: only the bookkeeping of a pass
    sc.n, sc.seq, sc.last_writer, sc.readers = n, 0, {}, {}
    sc.seen = [dict() for _ in range(n)]
    return sc


def conv(sc, s, x, y, ws):
    d = api.conv_desc(1, 4, 4, 4, 4, 1, 1, 1, 0)
    w, b = torch.zeros(4), torch.zeros(4)
    return sc._work_out(s, "stanza_conv_fwd", (d, x, w, b, y, ws), {})


def test_every_entry_point_of_the_table_exists_and_names_real_arguments():
    for name, written in _WRITES.items():
        assert hasattr(api, name)
        assert set(written) <= set(_PARAMS[name]), name


def test_reader_on_another_stream_waits_for_the_writer_and_not_on_the_same_stream():
    sc = fresh()
    x, y, z = torch.zeros(8), torch.zeros(8), torch.zeros(8)
    ws0, ws1 = torch.zeros(4), torch.zeros(4)
    w0, e0 = conv(sc, 0, x, y, ws0)
    assert w0 == []
    w1, e1 = conv(sc, 0, y, z, ws0)                  # same stream: ordered by the stream itself
    assert w1 == []
    w2, e2 = conv(sc, 1, y, torch.zeros(8), ws1)     # another stream reads y: waits for its writer
    assert w2 == [e0]


def test_writer_waits_for_readers_on_other_streams_and_readers_do_not_wait_for_each_other():
    sc = fresh()
    t = torch.zeros(8)
    _, ew = conv(sc, 0, torch.zeros(8), t, torch.zeros(4))
    wa, ea = conv(sc, 1, t, torch.zeros(8), torch.zeros(4))
    wb, eb = conv(sc, 2, t, torch.zeros(8), torch.zeros(4))
    assert wa == [ew] and wb == [ew]                 # two readers: each waits for the writer only
    ww, _ = conv(sc, 0, torch.zeros(8), t, torch.zeros(4))      # writing t again: after both readers
    assert set(map(id, ww)) == {id(ea), id(eb)}


def test_views_of_one_storage_are_one_buffer_and_a_shared_workspace_orders_its_users():
    sc = fresh()
    base = torch.zeros(16)
    _, e0 = conv(sc, 0, torch.zeros(8), base[:8], torch.zeros(4))
    w1, _ = conv(sc, 1, base[8:], torch.zeros(8), torch.zeros(4))
    assert w1 == [e0]
    sc = fresh()
    ws = torch.zeros(4)
    _, e0 = conv(sc, 0, torch.zeros(8), torch.zeros(8), ws)
    w1, _ = conv(sc, 1, torch.zeros(8), torch.zeros(8), ws)
    assert w1 == [e0]


def test_latest_event_of_a_stream_stands_for_its_earlier_ones():
    sc = fresh()
    a, b = torch.zeros(8), torch.zeros(8)
    _, ea = conv(sc, 0, torch.zeros(8), a, torch.zeros(4))
    _, eb = conv(sc, 0, torch.zeros(8), b, torch.zeros(4))
    # stream 1 reads both: one wait, for the later event of stream 0
    d = api.conv_desc(1, 4, 4, 4, 4, 1, 1, 1, 0)
    w, _ = sc._work_out(1, "stanza_add_relu_fwd", (a, b, torch.zeros(8)), {})
    assert w == [eb]
    # and having waited for it, stream 1 does not wait again for anything stream 0 did before
    w2, _ = sc._work_out(1, "stanza_add_relu_fwd", (a, a, torch.zeros(8)), {})
    assert w2 == []


def test_keyword_arguments_count():
    sc = fresh()
    res = torch.zeros(8)
    _, e0 = conv(sc, 0, torch.zeros(8), res, torch.zeros(4))
    w, _ = sc._work_out(1, "stanza_bn_fwd_stats", (torch.zeros(8), torch.zeros(4), torch.zeros(4), torch.zeros(4), torch.zeros(8),
                                                    torch.zeros(4), torch.zeros(4)), {"res": res})
    assert w == [e0]
