"""CPU-only checks of the C-ABI library: it loads, exports every function the header
declares, validates arguments on the host before any launch, and its saved-bytes
accounting reproduces the paper's memory model."""
import ctypes as C
import os
import re

import pytest

from paper_2305_11624_amd import binding as B
from paper_2305_11624_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "convbn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(convbn_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = _declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(B.EXPORTS)


def test_output_size_and_workspace_queries():
    d = B.make_desc(32, 3, 224, 224, 64, 7, 7, 2, 3)
    assert (B.convbn_hout(d), B.convbn_wout(d)) == (112, 112)
    d = B.make_desc(32, 256, 28, 28, 256, 3, 3, 2, 1)
    assert (B.convbn_hout(d), B.convbn_wout(d)) == (14, 14)
    for mode in (B.MODE_TUNE, B.MODE_EVAL):
        for p in (B.PASS_FWD, B.PASS_BWD):
            assert B.convbn_workspace_bytes(d, mode, p) % 256 == 0
    assert B.convbn_workspace_bytes(d, B.MODE_TUNE, B.PASS_FWD) >= 256 * 2304 * 2
    assert B.convbn_wgrad_parts(d) >= 1 and B.convbn_rsum_parts(d) >= 1


BAD_DESCS = [
    (dict(N=0), B.ERR_SHAPE), (dict(Cin=-1), B.ERR_SHAPE), (dict(stride=0), B.ERR_SHAPE),
    (dict(pad=-1), B.ERR_SHAPE), (dict(kH=9, kW=9, pad=0), B.ERR_SHAPE),
    (dict(dtype=7), B.ERR_UNSUPPORTED), (dict(layout=1), B.ERR_UNSUPPORTED),
    (dict(N=1 << 20, Hin=64, Win=64), B.ERR_UNSUPPORTED),
]


@pytest.mark.parametrize("change,code", BAD_DESCS)
def test_bad_descriptor_is_rejected_before_any_launch(change, code):
    kw = dict(N=2, Cin=8, Hin=8, Win=8, Cout=8, kH=3, kW=3, stride=1, pad=1)
    kw.update(change)
    d = B.make_desc(**kw)
    fake = C.c_void_p(4096)   # never dereferenced: validation fails first
    st = B.lib().convbn_tune_fwd(C.byref(d), fake, fake, None, fake, fake, fake, fake, fake, None,
                                 fake, 1 << 30, None)
    assert st == code, B.convbn_last_error()
    assert B.convbn_workspace_bytes(d, B.MODE_TUNE, B.PASS_FWD) == 0
    assert B.convbn_hout(d) == 0


def test_null_misaligned_and_workspace_errors():
    d = B.make_desc(2, 8, 8, 8, 8, 3, 3, 1, 1)
    L = B.lib()
    ok = C.c_void_p(4096)
    need = B.convbn_workspace_bytes(d, B.MODE_TUNE, B.PASS_FWD)
    assert L.convbn_tune_fwd(None, ok, ok, None, ok, ok, ok, ok, ok, None, ok, need, None) == B.ERR_NULL
    assert L.convbn_tune_fwd(C.byref(d), None, ok, None, ok, ok, ok, ok, ok, None, ok, need, None) == B.ERR_NULL
    assert "x" in B.convbn_last_error()
    assert L.convbn_tune_fwd(C.byref(d), C.c_void_p(4100), ok, None, ok, ok, ok, ok, ok, None, ok, need,
                             None) == B.ERR_UNSUPPORTED
    assert L.convbn_tune_fwd(C.byref(d), ok, ok, None, ok, ok, ok, ok, ok, None, None, 0, None) == B.ERR_WORKSPACE
    assert L.convbn_tune_fwd(C.byref(d), ok, ok, None, ok, ok, ok, ok, ok, None, ok, need - 1, None) == B.ERR_WORKSPACE
    needb = B.convbn_workspace_bytes(d, B.MODE_TUNE, B.PASS_BWD)
    # db given without b
    assert L.convbn_tune_bwd(C.byref(d), ok, ok, None, ok, ok, ok, None, ok, ok, ok, ok, ok, ok, ok, needb,
                             None) == B.ERR_NULL
    assert L.convbn_eval_bwd(C.byref(d), ok, ok, None, ok, ok, ok, None, ok, ok, ok, None, ok, ok, ok,
                             1 << 30, None) == B.ERR_NULL      # y_saved missing
    assert L.convbn_eval_fwd(C.byref(d), ok, ok, None, ok, ok, ok, ok, ok, None, None, 0, None) == B.ERR_NULL


def test_saved_bytes_follow_the_memory_model():
    """App. K.1: Eval keeps Y (N Cout Hout Wout), Tune keeps w' (k^2 Cin Cout); the
    saving per block is their difference."""
    for s in synth.CONFIGS.values():
        d = B.desc_from_shape(s)
        assert B.convbn_saved_bytes(d, B.MODE_EVAL) == s.A_z * s.elem_bytes
        assert B.convbn_saved_bytes(d, B.MODE_TUNE) == s.P * s.elem_bytes
        assert B.convbn_saved_bytes(d, B.MODE_TUNE, refold=True) == 0


def _golden_rows():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_appendix_d_resnet50.txt")):
        if line.strip() and not line.startswith("#"):
            v = line.split()
            rows.append((int(v[0]), int(v[1]), float(v[3]), float(v[5])))
    return rows


@pytest.mark.parametrize("batch,image,eval_gb,tune_gb", _golden_rows())
def test_resnet50_saving_matches_paper_appendix_d(batch, image, eval_gb, tune_gb):
    """The paper's measured Eval-minus-Tune peak memory for ResNet-50 (App. D, fp32) against
    the library's saved-bytes accounting summed over the 53 blocks: agreement within 4 % (3.3 % at batch 16, under 1 % from batch 32 up)
    pins the accounting (Eval keeps every Y, Tune every w')."""
    blocks = synth.resnet50_blocks(N=batch, image=image, dtype="f32")
    assert len(blocks) == 53
    ev = sum(B.convbn_saved_bytes(B.desc_from_shape(s), B.MODE_EVAL) for s in blocks)
    tu = sum(B.convbn_saved_bytes(B.desc_from_shape(s), B.MODE_TUNE) for s in blocks)
    predicted = (ev - tu) / 2 ** 30
    measured = eval_gb - tune_gb
    assert abs(predicted - measured) / measured < 0.04, (predicted, measured)
