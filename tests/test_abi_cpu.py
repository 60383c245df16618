"""CPU-only checks of the boundary: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

from paper_2308_01320_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "he.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(he_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS), names
    for n in names:
        assert getattr(L, n) is not None


def test_workspace_bytes_is_pure_and_monotone():
    L = binding.lib()
    d = synth.CONFIGS["tiny"]
    c1 = binding.make_config(d)
    c2 = binding.make_config(d, max_batch=8)
    b1, b2 = L.he_workspace_bytes(C.byref(c1)), L.he_workspace_bytes(C.byref(c2))
    assert 0 < b1 < b2
    bad = binding.make_config(d)
    bad.hidden = 250  # not a multiple of n_heads
    assert L.he_workspace_bytes(C.byref(bad)) == 0
    assert L.he_workspace_bytes(None) == 0
    big = binding.make_config(synth.CONFIGS["opt-13b"])
    kv = 2 * 40 * 32 * 512 * 5120 * 2
    assert L.he_workspace_bytes(C.byref(big)) > kv  # at least the KV arena of the headline workload


def test_host_side_argument_errors_need_no_gpu():
    L = binding.lib()
    h = C.c_void_p()
    assert L.he_create(None, None, C.byref(h)) == 1
    assert b"NULL" in L.he_last_error(None)
    cfg = binding.make_config(synth.CONFIGS["tiny"])
    cfg.dtype = 7
    assert L.he_create(C.byref(cfg), None, C.byref(h)) == 1
    cfg = binding.make_config(synth.CONFIGS["tiny"])
    cfg.hidden = 250
    assert L.he_create(C.byref(cfg), None, C.byref(h)) == 2
    cfg = binding.make_config(synth.CONFIGS["tiny"])
    assert L.he_create(C.byref(cfg), None, C.byref(h)) == 1  # weights NULL
    assert L.he_destroy(None) == 0
    assert L.he_reset(None) == 1
    assert L.he_cache_len(None) == -1
    assert L.he_rng_words(0, 0, 0, 0, 4, None, None) == 1
