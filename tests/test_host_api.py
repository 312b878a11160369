"""Host-side logic of the C-ABI library: it loads without a GPU, exports every symbol the header
declares, validates configurations and arguments before any launch, and sizes the workspace."""
import ctypes as C
import os
import re

import pytest

import paper_2502_04077_amd as ap
from paper_2502_04077_amd.binding import ap_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(n_inst=8, g=4, head_dim=128, block=16, hist_len=64, t_cap=32768 + 256, k_blocks=64, n_sink=4,
                n_local=4, c1=8, c2=8, kv_dtype=ap.AP_BF16, flags=0)
    base.update(kw)
    return ap_config(*[base[n] for n, _ in ap_config._fields_])


def _create(**kw):
    lib = ap.load_library()
    h = C.c_void_p()
    rc = lib.ap_create(C.byref(_cfg(**kw)), C.byref(h))
    return rc, h


def test_header_symbols_are_exported():
    lib = ap.load_library()
    header = open(os.path.join(ROOT, "include", "attnpred.h")).read()
    declared = sorted(set(re.findall(r"\b(ap_[a-z_]+)\s*\(", header)))
    assert "ap_step" in declared and "ap_calibrate" in declared
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in attnpred.h but not exported"
    assert sorted(ap.EXPORTS) == declared


def test_create_accepts_the_five_configurations():
    from workloads import CONFIGS
    for w in CONFIGS.values():
        c = ap.Context(n_inst=w.n_inst, g=w.g, head_dim=w.head_dim, block=w.block, hist_len=w.hist_len,
                       t_cap=w.t_cap, k_blocks=w.k_blocks, n_sink=w.n_sink, n_local=w.n_local, c1=w.c1, c2=w.c2,
                       kv_dtype=w.kv_dtype)
        assert c.hist_slots() == w.hist_len + 1
        assert c.nb_cap() == w.nb_cap
        assert c.workspace_bytes() % 16 == 0 and c.workspace_bytes() > 0
        c.close()


@pytest.mark.parametrize("kw,code", [
    (dict(n_inst=0), -1), (dict(t_cap=1000), -1), (dict(n_sink=40, n_local=40), -1), (dict(hist_len=0), -1),
    (dict(block=12), -5), (dict(block=128, t_cap=128 * 300), -5), (dict(g=3), -5), (dict(head_dim=96), -5),
    (dict(c1=8, c2=16), -5), (dict(kv_dtype=7), -5), (dict(k_blocks=20000), -5), (dict(hist_len=300), -5),
    (dict(n_inst=70000), -5),
])
def test_create_rejects_bad_configurations(kw, code):
    rc, h = _create(**kw)
    assert rc == code and not h.value


def test_dense_budget_is_accepted():
    """k = t_cap / b (every block selected) is a valid configuration: attention over the whole context."""
    from workloads import CONFIGS
    w = CONFIGS["cfg2"]
    c = ap.Context(n_inst=128, g=w.g, head_dim=w.head_dim, block=w.block, hist_len=w.hist_len, t_cap=w.t_cap,
                   k_blocks=w.nb_cap, n_sink=0, n_local=0, c1=w.c1, c2=w.c2, kv_dtype=w.kv_dtype)
    assert c.workspace_bytes() > 0
    c.close()


def test_null_and_misaligned_pointers_are_refused_before_any_launch():
    lib = ap.load_library()
    rc, h = _create()
    assert rc == 0
    ok = 4096          # a fake, aligned, non-null address: the call must stop at the weights check
    assert lib.ap_predict(h, None, 0, 100, ok, ok, None) == -1
    assert lib.ap_predict(h, ok + 4, 0, 100, ok, ok, None) == -2
    assert lib.ap_predict(h, ok, 0, 100, ok, ok, None) == -6          # weights not set
    assert lib.ap_select_topk(h, ok, 0, ok, ok, ok, None) == -3       # nb_cur out of range
    assert lib.ap_select_topk(h, ok, 10**6, ok, ok, ok, None) == -3
    assert lib.ap_sparse_decode(h, ok, ok, ok, 0, ok, ok, ok, ok, ok, None) == -3
    assert lib.ap_sparse_decode(h, ok, ok, ok, 10**8, ok, ok, ok, ok, ok, None) == -3
    assert lib.ap_calibrate(h, ok, None, 5, ok, ok, None) == -1
    assert lib.ap_update_history(h, ok, -1, ok, None) == -3
    assert lib.ap_step(h, ok, 0, ok, ok, ok, 5, ok, ok, ok, ok, ok, 0, ok, None) == -6
    assert lib.ap_predict_incremental(h, ok, 0, 100, 100, 9, ok, ok, ok, None) == -6
    assert lib.ap_set_weights(h, ok, 3, None) == -1                   # wrong blob length
    assert lib.ap_stream_read(None, 64, ok, 1, None) == -1
    # the calls of the widened rows stop on the host as well
    assert lib.ap_refresh_selection(h, 10, 5, ok, ok, None) == -3     # nb_prev > nb_cur
    assert lib.ap_refresh_selection(h, 5, 10, None, ok, None) == -1
    assert lib.ap_prefetch_state_bytes(h) == 8 * (3 * 64 + 4) * 4    # n_inst x (3k + 4) int32
    assert lib.ap_prefetch_blocks(h, ok, ok, 10, 0, ok, ok, ok, ok, ok, ok, None) == -3
    assert lib.ap_prefetch_blocks(h, ok, ok, 10, 5, ok, ok, ok, ok, ok, None, None) == -1
    assert lib.ap_prefetch_blocks(h, ok, ok, 10, 5, ok, ok, ok, ok, ok, ok, None) == -1   # not device-readable memory
    assert lib.ap_append_kv(h, ok, ok, -1, ok, ok, ok, ok, None) == -3
    assert lib.ap_append_kv(h, ok, ok + 2, 3, ok, ok, ok, ok, None) == -2
    assert lib.ap_offload_begin(h, ok, 0, ok, ok, 5, ok, ok, ok, ok, ok, ok, ok, ok, ok, None, None) == -6
    assert lib.ap_offload_step(h, ok, 0, ok, ok, ok, ok, ok, 5, 0, ok, ok, ok, ok, ok, 1, ok, ok, ok, ok, ok, ok,
                               None, None) == -6
    assert lib.ap_step(h, ok, 0, ok, ok, ok, 5, ok, ok, ok, ok, ok, 3, ok, None) == -6
    assert lib.ap_destroy(h) == 0
    assert lib.ap_destroy(None) == -1
    for code in range(0, -8, -1):
        assert lib.ap_strerror(code)
