"""Host-only checks of the C-ABI boundary: the library loads, exports what the
header declares, and its host-side size/layout queries behave (no GPU work)."""
import ctypes as C
import os
import re

import pytest

import paper_2512_17452_amd as wg
from paper_2512_17452_amd.binding import _CConfig, _CLayout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(wg.library_path()):
        from paper_2512_17452_amd import build
        build.build(force=True)
    return wg.load_library()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "wgkv.h")).read()
    declared = set(re.findall(r"\b(wgkv_[a-z_]+)\s*\(", hdr))
    assert declared == set(wg.EXPORTED_SYMBOLS)
    for s in declared:
        assert getattr(lib, s) is not None
    assert lib.wgkv_version().startswith(b"wgkv")


def test_query_sizes_and_layout(lib):
    cfg = wg.Config(32, 32, 8, 128, wg.BF16, 16, 256, 8, 8208, 2_300_000)
    cc = cfg.c()
    pb, mb, wb = C.c_size_t(), C.c_size_t(), C.c_size_t()
    assert lib.wgkv_query_sizes(C.byref(cc), 8, 8 * 131072, C.byref(pb), C.byref(mb), C.byref(wb)) == 0
    assert pb.value == 2_300_000 * 2 * 16 * 128 * 2      # [page][K,V][P][d] bf16
    lay = _CLayout()
    assert lib.wgkv_get_meta_layout(C.byref(cc), C.byref(lay)) == 0
    assert lay.n_local_pages == 16 and lay.total_bytes == mb.value
    offs = [lay.seq_len, lay.global_len, lay.local_pt, lay.global_pt, lay.ring_g, lay.free_stack,
            lay.free_top, lay.err_flag, lay.unit_counters, lay.ahead]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert lay.total_bytes - lay.ahead >= 8 * 32 * 8 * 4      # one stamp per (sequence, layer, kv head)
    assert lay.global_len - lay.seq_len >= 8 * 32 * 4
    assert lay.ring_g - lay.global_pt >= 8 * 32 * 8 * 8208 * 4
    assert wb.value > 0


@pytest.mark.parametrize("field,value", [("head_dim", 96), ("page_size", 12), ("n_q_heads", 30), ("dtype", 7),
                                         ("w_local", 0), ("n_pages", 0), ("n_pages", 1 << 31),
                                         ("n_q_heads", 128)])
def test_bad_configs_are_rejected(lib, field, value):
    cfg = wg.Config(2, 32, 8, 128, wg.BF16, 16, 256, 4, 64, 1000)
    setattr(cfg, field, value)
    cc = cfg.c()
    pb = C.c_size_t()
    assert lib.wgkv_query_sizes(C.byref(cc), 1, 16, C.byref(pb), None, None) == -1


def test_null_handles_are_rejected(lib):
    assert lib.wgkv_free_seq(None, 0, None) == -1
    assert lib.wgkv_status(None, None, None, None) == -1
    assert lib.wgkv_set_profile_events(None, None, None) == -1
    assert lib.wgkv_gate_scores(1, 4, 12, 8, None, None, None, None) == -1
    assert lib.wgkv_clear_error(None, None) == -1
    assert lib.wgkv_decode_promote(None, 1, (C.c_int32 * 1)(0), 0.5, None) == -1
    assert lib.wgkv_decode_step(None, 0, 1, (C.c_int32 * 1)(0), None, None, None, 0.5, None, None) == -1
    assert lib.wgkv_prefill_admit_bounded(None, 0, 1, (C.c_int32 * 1)(0), (C.c_int32 * 1)(1), None, None, None, None,
                                          None, 0, 0.5, 4, None, None, 0, None) == -1
    assert lib.wgkv_attend_decode_static(None, 0, 1, (C.c_int32 * 1)(0), None, 1.0, None, None) == -1
    assert lib.wgkv_stream_read_probe(None, 1024, None, None, None, None) == -1
    lib.wgkv_destroy(None)
