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
    (dict(dtype=7), B.ERR_UNSUPPORTED), (dict(layout=1), B.ERR_UNSUPPORTED), (dict(act=16), B.ERR_UNSUPPORTED), (dict(act=4), B.ERR_NULL), (dict(act=8), B.ERR_NULL),
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


def test_transposed_block_queries_and_validation():
    """Output size of the transposed convolution (Hout = (Hin-1) s - 2 p + k), workspace queries and the host-side
    argument checks of its two entry points (nothing is launched: every call fails validation)."""
    d = B.make_desc(32, 256, 28, 28, 128, 2, 2, 2, 0)
    assert (B.convbn_tconv_hout(d), B.convbn_tconv_wout(d)) == (56, 56)
    d4 = B.make_desc(32, 512, 14, 14, 256, 4, 4, 2, 1)
    assert (B.convbn_tconv_hout(d4), B.convbn_tconv_wout(d4)) == (28, 28)
    d3 = B.make_desc(2, 8, 5, 7, 8, 3, 3, 1, 1)
    assert (B.convbn_tconv_hout(d3), B.convbn_tconv_wout(d3)) == (5, 7)
    T, E = B.MODE_TUNE, B.MODE_EVAL
    for m in (T, E):
        for p in (B.PASS_FWD, B.PASS_BWD):
            assert B.convbn_tconv_workspace_bytes(d, m, p) % 256 == 0 and B.convbn_tconv_workspace_bytes(d, m, p) > 0
    # forward keeps the transposed scaled weight in the workspace; backward at least one fp32 copy of dw'
    assert B.convbn_tconv_workspace_bytes(d, T, B.PASS_FWD) >= 256 * 128 * 4 * 2
    assert B.convbn_tconv_workspace_bytes(d, T, B.PASS_BWD) >= 256 * 128 * 4 * 4
    # Eval backward additionally holds dY; what stays alive between the passes: Y (Eval) against w' (Tune)
    assert B.convbn_tconv_workspace_bytes(d, E, B.PASS_BWD) >= 32 * 56 * 56 * 128 * 2
    assert B.convbn_tconv_saved_bytes(d, E) == 32 * 56 * 56 * 128 * 2
    assert B.convbn_tconv_saved_bytes(d, T) == 256 * 128 * 4 * 2 and B.convbn_tconv_saved_bytes(d, T, True) == 0
    L = B.lib()
    ok = C.c_void_p(4096)
    need = B.convbn_tconv_workspace_bytes(d, T, B.PASS_FWD)
    fwd = lambda desc, x=ok, ws=ok, n=need: L.convbn_tconv_tune_fwd(desc, x, ok, None, ok, ok, ok, ok, ok, None, ws, n, None)
    assert fwd(None) == B.ERR_NULL
    assert fwd(C.byref(d), x=None) == B.ERR_NULL
    assert fwd(C.byref(d), x=C.c_void_p(4100)) == B.ERR_UNSUPPORTED
    assert fwd(C.byref(d), ws=None, n=0) == B.ERR_WORKSPACE
    assert fwd(C.byref(d), n=need - 1) == B.ERR_WORKSPACE
    gone = B.make_desc(1, 8, 2, 2, 8, 1, 1, 1, 1)           # padding removes the whole output
    assert fwd(C.byref(gone)) == B.ERR_SHAPE and B.convbn_tconv_hout(gone) == 0
    assert B.convbn_tconv_workspace_bytes(gone, T, B.PASS_FWD) == 0
    needb = B.convbn_tconv_workspace_bytes(d, T, B.PASS_BWD)
    bwd = lambda dx, dW, db, dg, dbt: L.convbn_tconv_tune_bwd(C.byref(d), ok, ok, None, ok, ok, ok, None, ok, dx, dW, db,
                                                             dg, dbt, ok, needb, None)
    assert bwd(ok, ok, ok, ok, ok) == B.ERR_NULL             # db given without b
    assert bwd(ok, ok, None, None, ok) == B.ERR_NULL         # dgamma missing
    assert bwd(None, None, None, None, None) == B.ERR_NULL   # nothing asked for
    assert bwd(ok, None, None, ok, None) == B.ERR_NULL       # dgamma without dW
    assert L.convbn_tconv_eval_fwd(C.byref(d), ok, ok, None, ok, ok, ok, ok, ok, None, ok, need, None) == B.ERR_NULL   # y_saved
    assert L.convbn_tconv_eval_bwd(C.byref(d), ok, ok, None, ok, ok, ok, None, ok, ok, ok, None, ok, ok, ok, 1 << 40,
                                   None) == B.ERR_NULL                                                                   # y_saved


def test_depthwise_block_queries_and_validation():
    """Workspace / saved-bytes queries and host-side argument checks of the depthwise entry points."""
    d = B.make_desc(32, 144, 56, 56, 144, 3, 3, 1, 1)
    T, E = B.MODE_TUNE, B.MODE_EVAL
    for m in (T, E):
        for p in (B.PASS_FWD, B.PASS_BWD):
            assert B.convbn_dw_workspace_bytes(d, m, p) % 256 == 0 and B.convbn_dw_workspace_bytes(d, m, p) > 0
    assert B.convbn_dw_workspace_bytes(d, E, B.PASS_BWD) >= 32 * 56 * 56 * 144 * 2      # dY
    assert B.convbn_dw_saved_bytes(d, E) == 32 * 56 * 56 * 144 * 2                      # Y
    assert B.convbn_dw_saved_bytes(d, T) == 9 * 144 * 2 and B.convbn_dw_saved_bytes(d, T, True) == 0
    bad = B.make_desc(2, 16, 8, 8, 32, 3, 3, 1, 1)                                      # not one filter per channel
    assert B.convbn_dw_workspace_bytes(bad, T, B.PASS_FWD) == 0 and B.convbn_dw_saved_bytes(bad, T) == 0
    L = B.lib()
    ok = C.c_void_p(4096)
    need = B.convbn_dw_workspace_bytes(d, T, B.PASS_FWD)
    fwd = lambda desc, x=ok, ws=ok, n=need: L.convbn_dw_tune_fwd(desc, x, ok, None, ok, ok, ok, ok, ok, None, ws, n, None)
    assert fwd(C.byref(bad)) == B.ERR_SHAPE
    assert fwd(None) == B.ERR_NULL
    assert fwd(C.byref(d), x=None) == B.ERR_NULL
    assert fwd(C.byref(d), x=C.c_void_p(4100)) == B.ERR_UNSUPPORTED
    assert fwd(C.byref(d), ws=None, n=0) == B.ERR_WORKSPACE
    assert fwd(C.byref(d), n=need - 1) == B.ERR_WORKSPACE
    needb = B.convbn_dw_workspace_bytes(d, T, B.PASS_BWD)
    bwd = lambda dx, dW, db, dg, dbt: L.convbn_dw_tune_bwd(C.byref(d), ok, ok, None, ok, ok, ok, None, ok, dx, dW, db, dg,
                                                          dbt, ok, needb, None)
    assert bwd(ok, ok, ok, ok, ok) == B.ERR_NULL             # db given without b
    assert bwd(ok, ok, None, None, ok) == B.ERR_NULL         # dgamma missing
    assert bwd(None, None, None, None, None) == B.ERR_NULL   # nothing asked for
    assert L.convbn_dw_eval_fwd(C.byref(d), ok, ok, None, ok, ok, ok, ok, ok, None, ok, need, None) == B.ERR_NULL   # y_saved


def test_grouped_block_queries_and_validation():
    """Workspace / saved-bytes queries and host-side argument checks of the grouped entry points."""
    d = B.make_desc(32, 128, 56, 56, 128, 3, 3, 1, 1)
    T, E = B.MODE_TUNE, B.MODE_EVAL
    G = 32
    for m in (T, E):
        for p in (B.PASS_FWD, B.PASS_BWD):
            assert B.convbn_grouped_workspace_bytes(d, G, m, p) % 256 == 0 and B.convbn_grouped_workspace_bytes(d, G, m, p) > 0
    assert B.convbn_grouped_workspace_bytes(d, G, E, B.PASS_BWD) >= 32 * 56 * 56 * 128 * 2      # dY
    assert B.convbn_grouped_saved_bytes(d, G, E) == 32 * 56 * 56 * 128 * 2                      # Y
    assert B.convbn_grouped_saved_bytes(d, G, T) == 128 * 9 * 4 * 2 and B.convbn_grouped_saved_bytes(d, G, T, True) == 0
    assert B.convbn_grouped_saved_bytes(d, 1, T) == B.convbn_saved_bytes(d, T)                  # one group: the dense block
    for bad_g in (0, -1, 3, 256):
        assert B.convbn_grouped_workspace_bytes(d, bad_g, T, B.PASS_FWD) == 0 and B.convbn_grouped_saved_bytes(d, bad_g, T) == 0
    L = B.lib()
    ok = C.c_void_p(4096)
    need = B.convbn_grouped_workspace_bytes(d, G, T, B.PASS_FWD)
    fwd = lambda desc, g=G, x=ok, ws=ok, n=need: L.convbn_grouped_tune_fwd(desc, g, x, ok, None, ok, ok, ok, ok, ok, None,
                                                                         ws, n, None)
    assert fwd(C.byref(d), g=3) == B.ERR_SHAPE
    assert fwd(None) == B.ERR_NULL
    assert fwd(C.byref(d), x=None) == B.ERR_NULL
    assert fwd(C.byref(d), x=C.c_void_p(4100)) == B.ERR_UNSUPPORTED
    assert fwd(C.byref(d), ws=None, n=0) == B.ERR_WORKSPACE
    assert fwd(C.byref(d), n=need - 1) == B.ERR_WORKSPACE
    needb = B.convbn_grouped_workspace_bytes(d, G, T, B.PASS_BWD)
    bwd = lambda dx, dW, db, dg, dbt: L.convbn_grouped_tune_bwd(C.byref(d), G, ok, ok, None, ok, ok, ok, None, ok, dx, dW,
                                                               db, dg, dbt, ok, needb, None)
    assert bwd(ok, ok, ok, ok, ok) == B.ERR_NULL             # db given without b
    assert bwd(ok, ok, None, None, ok) == B.ERR_NULL         # dgamma missing
    assert bwd(None, None, None, None, None) == B.ERR_NULL   # nothing asked for
    assert L.convbn_grouped_eval_fwd(C.byref(d), G, ok, ok, None, ok, ok, ok, ok, ok, None, ok, need, None) == B.ERR_NULL   # y_saved


def test_sizes_beyond_32_bit_indexing_are_rejected_on_the_host():
    """The kernels index tensors and buffers of partial sums with 32 bits: larger problems are turned down by the
    host checks (no launch, so this runs without a GPU)."""
    fake = C.c_void_p(4096)
    L = B.lib()
    big = (B.BF16, fake, fake, fake, 1 << 12, 1 << 10, 1 << 10, 8, None)   # 2^35 elements
    assert L.convbn_aux_maxpool_fwd(*big) == B.ERR_UNSUPPORTED, B.convbn_last_error()
    assert L.convbn_aux_maxpool_bwd(*big) == B.ERR_UNSUPPORTED, B.convbn_last_error()
    # every tensor of this block fits, and so do the partial sums its plan would write: accepted, sizes consistent
    d = B.make_desc(N=4, Cin=4096, Hin=14, Win=14, Cout=4096, kH=3, kW=3, stride=1, pad=1, dtype=B.BF16)
    need = B.convbn_workspace_bytes(d, B.MODE_TUNE, B.PASS_BWD)
    assert need > 0 and need % 256 == 0
    assert B.convbn_wgrad_parts(d) * 4096 * 9 * 4096 <= 0x7fffffff
