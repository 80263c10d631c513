"""Host-only checks of the record / replay hook: modes that never touch a device (pass-through counting, a
replay whose boundary holds no entry), and tape files that must be refused.  No kernel is launched."""
import os
import struct

import pytest

from tests import tape_io


@pytest.fixture(scope="module")
def tm():
    import paper_2412_12636_amd as tm
    if not os.path.exists(tm.LIB_PATH):
        from paper_2412_12636_amd import build
        build.build()
    return tm


def test_pass_through_counts_calls_and_touches_nothing(tm):
    c = tm.tm_comm_open(None, tm.TM_COMM_PASS, tm.TM_SCOPE_TP | tm.TM_SCOPE_PP)
    tm.tm_comm_call(c, tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, 0x1000, 4096)     # never dereferenced
    tm.tm_comm_call(c, tm.TM_COLL_BARRIER, tm.TM_SCOPE_DP, tm.TM_SITE_STEP_END, 0, None, 0)
    st = tm.tm_comm_stats(c)
    assert st["calls"] == 2 and st["native"] == 2 and st["stored"] == 0 and st["skipped"] == 0
    with pytest.raises(tm.TmError) as e:
        tm.tm_comm_rewind(c)
    assert e.value.code == tm.TM_ESTATE
    tm.tm_comm_close(c)


def test_argument_errors(tm):
    for args in ((None, 7, 0), (None, tm.TM_COMM_RECORD, tm.TM_SCOPE_PP), ("/nonexistent-dir/x.tape", tm.TM_COMM_RECORD, 2),
                 (None, tm.TM_COMM_PASS, 8), ("/nonexistent-dir/x.tape", tm.TM_COMM_REPLAY, 2)):
        with pytest.raises(tm.TmError) as e:
            tm.tm_comm_open(*args)
        assert e.value.code == tm.TM_EINVAL and tm.tm_last_error()
    c = tm.tm_comm_open(None, tm.TM_COMM_PASS, 0)
    for args in ((9, tm.TM_SCOPE_PP, 0, 0, None, 0), (tm.TM_COLL_RECV, 3, 0, 0, None, 0), (tm.TM_COLL_RECV, 2, 0, 0, None, 16),
                 (tm.TM_COLL_RECV, 2, 0, 5, None, 0)):
        with pytest.raises(tm.TmError) as e:
            tm.tm_comm_call(c, *args)
        assert e.value.code == tm.TM_EINVAL
    tm.tm_comm_close(c)


def test_replay_loads_only_the_boundary_and_skips_send_and_barrier(tm, tmp_path):
    path = str(tmp_path / "a.tape")
    tape_io.write_tape(path, [(tm.TM_COLL_ALL_REDUCE, tm.TM_SCOPE_TP, tm.TM_SITE_ATTN_OUT, 1, b"\1" * 100),
                              (tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, b"")])
    assert len(tape_io.read_tape(path)) == 2
    c = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, tm.TM_SCOPE_DP)      # nothing on the boundary: nothing loaded
    assert tm.tm_comm_stats(c)["tape_entries"] == 0
    tm.tm_comm_call(c, tm.TM_COLL_ALL_REDUCE, tm.TM_SCOPE_TP, tm.TM_SITE_ATTN_OUT, 1, 0x1000, 100)   # native
    tm.tm_comm_call(c, tm.TM_COLL_BARRIER, tm.TM_SCOPE_DP, tm.TM_SITE_STEP_END, 0, None, 0)
    tm.tm_comm_call(c, tm.TM_COLL_SEND, tm.TM_SCOPE_DP, tm.TM_SITE_Y, 0, 0x1000, 64)
    st = tm.tm_comm_stats(c)
    assert st["native"] == 1 and st["skipped"] == 2
    with pytest.raises(tm.TmError) as e:                               # the boundary's tape is empty
        tm.tm_comm_call(c, tm.TM_COLL_ALL_REDUCE, tm.TM_SCOPE_DP, tm.TM_SITE_GRADS, 0, 0x1000, 64)
    assert e.value.code == tm.TM_ESTATE
    tm.tm_comm_close(c)
    # an entry of zero bytes on the boundary needs no memory either; it must match the call
    c = tm.tm_comm_open(path, tm.TM_COMM_REPLAY, tm.TM_SCOPE_PP)
    assert tm.tm_comm_stats(c)["tape_entries"] == 1
    with pytest.raises(tm.TmError) as e:
        tm.tm_comm_call(c, tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_DY, 1, None, 0)
    assert e.value.code == tm.TM_ESTATE and "site" in e.value.message
    tm.tm_comm_call(c, tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, None, 0)
    tm.tm_comm_rewind(c)
    tm.tm_comm_call(c, tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, None, 0)
    assert tm.tm_comm_stats(c)["stored"] == 2
    tm.tm_comm_close(c)


def test_malformed_tapes_are_refused(tm, tmp_path):
    good = str(tmp_path / "g.tape")
    tape_io.write_tape(good, [(tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, b"\2" * 200)])
    raw = open(good, "rb").read()
    cases = {"magic": b"XXTAPE01" + raw[8:], "short": raw[:40], "payload": raw[:16 + 64 + 100],
             "kind": raw[:16] + struct.pack("<I", 77) + raw[20:]}
    for name, data in cases.items():
        p = str(tmp_path / f"{name}.tape")
        open(p, "wb").write(data)
        with pytest.raises(tm.TmError) as e:
            tm.tm_comm_open(p, tm.TM_COMM_REPLAY, tm.TM_SCOPE_PP)
        assert e.value.code == tm.TM_EINVAL, name
    # the same broken files are fine when their scope is not on the boundary, except for the header
    tm.tm_comm_close(tm.tm_comm_open(str(tmp_path / "payload.tape"), tm.TM_COMM_REPLAY, tm.TM_SCOPE_TP))


def test_record_of_no_stored_call_writes_an_empty_tape(tm, tmp_path):
    path = str(tmp_path / "e.tape")
    c = tm.tm_comm_open(path, tm.TM_COMM_RECORD, tm.TM_SCOPE_PP)
    tm.tm_comm_call(c, tm.TM_COLL_SEND, tm.TM_SCOPE_PP, tm.TM_SITE_Y, 1, 0x1000, 64)      # sends are not stored
    tm.tm_comm_call(c, tm.TM_COLL_ALL_REDUCE, tm.TM_SCOPE_TP, tm.TM_SITE_ATTN_OUT, 1, 0x1000, 64)   # scope not recorded
    tm.tm_comm_call(c, tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, None, 0)          # empty tensor: stored
    assert tm.tm_comm_stats(c)["native"] == 2
    tm.tm_comm_close(c)
    assert tape_io.read_tape(path) == [(tm.TM_COLL_RECV, tm.TM_SCOPE_PP, tm.TM_SITE_X, 1, b"")]
