"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol include/lckv.h declares,
and finds argument errors before any GPU work.  No compute call is made here."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2405_10637_amd import binding as lk
from paper_2405_10637_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(lk.LIB_PATH), reason="liblckv.so not built")


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lckv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lckv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = declared_functions()
    assert len(names) >= 18
    L = lk.lib()
    for n in names:
        assert hasattr(L, n), "liblckv.so does not export " + n
        assert hasattr(lk, n), "binding has no function " + n
    assert sorted(lk.EXPORTS) == names


def cfg_for(wl, **kw):
    args = dict(L=wl.L, Hq=wl.Hq, Hkv=wl.Hkv, D=wl.D, dtype=lk.LCKV_BF16 if wl.dtype == "bf16" else lk.LCKV_F32,
                B_max=wl.B, T_max=wl.T + 1, warmup_mask=wl.warmup_mask)
    args.update(kw)
    return lk.make_config(**args)


def test_cache_bytes_is_the_footprint_closed_form():
    # slots * B * T * 2 * Hkv * D * elem: the number of cached layers drives memory (Sections 1 and 4.2)
    for wl, slots in [(synth.C1, 2), (synth.C2, 3), (synth.C3, 3), (synth.C5, 11)]:
        T_pad = (wl.T + 1 + 15) // 16 * 16
        want = slots * wl.B * T_pad * 2 * wl.Hkv * wl.D * wl.elem_bytes
        assert lk.lckv_cache_bytes(cfg_for(wl)) == want
    # standard transformer (all layers warmup) needs L slots: the ratio is the paper's memory saving
    full = lk.lckv_cache_bytes(cfg_for(synth.C3, warmup_mask=np.ones(32, np.uint8)))
    assert full == lk.lckv_cache_bytes(cfg_for(synth.C3)) // 3 * 32
    # rule 2 on a sandwich mask has one slot fewer
    assert lk.lckv_cache_bytes(cfg_for(synth.C3, pairing_rule=lk.LCKV_PAIR_LAST_LAYER)) * 3 == \
        lk.lckv_cache_bytes(cfg_for(synth.C3)) * 2
    # paged: blocks * Hkv * 2 pages
    assert lk.lckv_cache_bytes(cfg_for(synth.C4, page_size=16, num_blocks=1000, T_max=0)) == \
        3 * 1000 * 32 * 2 * 16 * 128 * 2


@pytest.mark.parametrize("field,value", [
    ("L", 0), ("Hq", 0), ("Hkv", 3), ("D", 96), ("dtype", 7), ("B_max", 0), ("T_max", 0), ("page_size", 32),
    ("pairing_rule", 5), ("scale", -1.0), ("scale", float("nan")), ("Hkv", 1),
])
def test_bad_config_is_rejected_on_the_host(field, value):
    cfg = cfg_for(synth.C3)
    setattr(cfg, field, value)
    with pytest.raises(lk.LckvError) as e:
        lk.lckv_cache_bytes(cfg)
    assert e.value.code == lk.LCKV_ERR_CONFIG


def test_null_and_misaligned_arguments():
    L = lk.lib()
    out = ctypes.c_size_t(0)
    assert L.lckv_cache_bytes(None, ctypes.byref(out)) == lk.LCKV_ERR_NULL
    cfg = cfg_for(synth.C1)
    assert L.lckv_cache_bytes(ctypes.byref(cfg), None) == lk.LCKV_ERR_NULL
    h = ctypes.c_void_p(None)
    assert L.lckv_cache_alloc(ctypes.byref(cfg), None, 1 << 30, ctypes.byref(h)) == lk.LCKV_ERR_NULL
    assert L.lckv_cache_alloc(ctypes.byref(cfg), 0x1008, 1 << 30, ctypes.byref(h)) == lk.LCKV_ERR_ALIGN
    assert L.lckv_cache_alloc(ctypes.byref(cfg), 0x1000, 100, ctypes.byref(h)) == lk.LCKV_ERR_STORAGE
    assert h.value is None
    cfg2 = cfg_for(synth.C1)
    cfg2.warmup_mask = None
    assert L.lckv_cache_bytes(ctypes.byref(cfg2), ctypes.byref(out)) == lk.LCKV_ERR_NULL
    # a handle that is not a cache
    junk = ctypes.create_string_buffer(4096)
    n = ctypes.c_int32(0)
    assert L.lckv_n_slots(ctypes.addressof(junk), ctypes.byref(n)) == lk.LCKV_ERR_NULL
    assert L.lckv_cache_free(None) == lk.LCKV_ERR_NULL
    assert L.lckv_step(None, None, None, None, None, None, 1, 1, None, 0, None) == lk.LCKV_ERR_NULL


def test_strerror_names_every_code():
    seen = set()
    for code in range(0, -14, -1):
        s = lk.lckv_strerror(code)
        assert s and "unknown" not in s
        seen.add(s)
    assert len(seen) == 14 and "unknown" in lk.lckv_strerror(-99)
