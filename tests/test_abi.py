"""The C-ABI library loads and exports every entry point include/twist.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "twist.h")).read()
    return sorted(set(re.findall(r"TWIST_API[^;(]*?\b(twist_\w+)\s*\(", text)))


def test_header_declares_the_four_hot_path_calls():
    names = _declared()
    for n in ("twist_sample", "twist_extract", "twist_subnet_fwd_bwd", "twist_aggregate"):
        assert n in names


def test_library_exports_every_declared_symbol():
    path = os.path.join(ROOT, "paper_2511_03983_amd", "libtwist.so")
    assert os.path.exists(path), "build the library first (__graft_entry__.build())"
    lib = ctypes.CDLL(path)
    for n in _declared():
        assert hasattr(lib, n), n
    import paper_2511_03983_amd as tw
    assert sorted(tw.binding.EXPORTS) == _declared()      # the binding covers the same names


def test_host_only_error_paths():
    """Argument checks that run before any device work."""
    import paper_2511_03983_amd as tw
    import synth_inputs as si
    d = tw.desc_from_cfg(si.CFG1)
    h = ctypes.c_void_p()
    assert tw.lib.twist_create(ctypes.byref(d), None, ctypes.byref(h)) == 0
    # size bound of Section 3.1: 4 heads cannot be covered by 2 subnets of 1 head
    sd = tw.SampleDesc(2, 1, 256, None, 0, None, 0, None, 1, 1, 0, 0)
    p = ctypes.c_void_p()
    assert tw.lib.twist_sample(h, ctypes.byref(sd), ctypes.byref(p)) == 2 and not p.value
    assert b"N_full" in tw.lib.twist_last_error(h)
    sd = tw.SampleDesc(2, 5, 256, None, 0, None, 0, None, 1, 1, 0, 0)      # N_sub > N_full
    assert tw.lib.twist_sample(h, ctypes.byref(sd), ctypes.byref(p)) == 2
    sd = tw.SampleDesc(0, 2, 256, None, 0, None, 0, None, 1, 1, 0, 0)      # S = 0
    assert tw.lib.twist_sample(h, ctypes.byref(sd), ctypes.byref(p)) == 1
    tw.lib.twist_destroy(h)
    bad = tw.desc_from_cfg(si.CFG1)
    bad.ffn_granule = 7
    assert tw.lib.twist_create(ctypes.byref(bad), None, ctypes.byref(h)) == 3
