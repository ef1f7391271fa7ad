"""CPU-only checks of the C ABI: the library loads, exports every function
include/hbp.h declares, and rejects bad descriptors before touching a device."""
import ctypes as C
import os
import re

import pytest

from paper_2501_17086_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hbp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hbp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    lib = B.lib()
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layout_matches_header():
    # field order and sizes as in the header (LP64)
    assert C.sizeof(B.hbp_desc) == 4 * 8 + 8 * 5 + 4 * 2 + 4 * 2 + 8
    assert C.sizeof(B.hbp_buffers) == 8 + 8 * 16 + 8 + 8 + 8 * 7
    assert C.sizeof(B.hbp_optim) == 4 * 8 + 8
    assert C.sizeof(B.hbp_optim_state) == 8 + 8 * 9 + 8 + 8 + 8 * 6


def _desc(**kw):
    base = dict(kind="mlp", dtype="bf16", act="gelu", norm="rms", L=4, N=16, d=64, d_ff=128)
    base.update(kw)
    return B.make_desc(**base)


def test_status_strings():
    for s in range(6):
        assert len(B.status_string(s)) > 0


def test_workspace_size_scales():
    a = B.workspace_size(_desc())
    b = B.workspace_size(_desc(N=32))
    assert a > 0 and b > a
    # v [L,N,d] + da [L,N,d_ff] in bf16 at least
    assert a >= 4 * 16 * (64 + 128) * 2


@pytest.mark.parametrize("field,value,status", [
    ("L", 0, 1), ("N", -1, 1), ("d", 0, 1), ("d", 60, 2), ("d_ff", 100, 2), ("kind", 7, 1), ("dtype", 3, 1),
    ("act", 5, 1), ("norm", 2, 1), ("lambda_kind", 9, 1), ("loss_every_state", 2, 1), ("struct_size", 12, 1),
    ("d_in", 8, 1), ("gamma", -0.1, 1), ("gamma", 1.5, 1), ("gamma", float("nan"), 1), ("post", 3, 1), ("post", -1, 1),
])
def test_bad_descriptor_is_rejected(field, value, status):
    d = _desc()
    setattr(d, field, value)
    n = C.c_size_t(0)
    assert B.lib().hbp_workspace_size(C.byref(d), C.byref(n)) == status


def test_rms_width_limit_and_rnn_needs_input_width():
    n = C.c_size_t(0)
    d = _desc(d=8192)
    assert B.lib().hbp_workspace_size(C.byref(d), C.byref(n)) == 2
    d = _desc(kind="rnn", act="tanh", norm="none", d_in=0)
    assert B.lib().hbp_workspace_size(C.byref(d), C.byref(n)) == 1


def test_relu_after_the_sum_is_for_depth_stacks_with_the_plain_split():
    n = C.c_size_t(0)
    assert B.lib().hbp_workspace_size(C.byref(_desc(post="relu")), C.byref(n)) == 0
    assert B.lib().hbp_workspace_size(C.byref(_desc(post="relu", gamma=0.5)), C.byref(n)) == 2
    d = _desc(kind="rnn", act="tanh", norm="none", d_in=64, post="relu")
    assert B.lib().hbp_workspace_size(C.byref(d), C.byref(n)) == 2
    for alg in (2, 3):
        assert B.lib().hbp_scan_workspace_size(C.byref(_desc(post="relu")), alg, C.byref(n)) == 2
        bufs = B.hbp_buffers(C.sizeof(B.hbp_buffers))
        assert B.lib().hbp_initial_estimate(C.byref(_desc(post="relu")), alg, C.byref(bufs), None) == 2


def test_gated_cell_descriptor_rules():
    n = C.c_size_t(0)
    ok = dict(kind="gated", act="tanh", norm="none", d=64, d_ff=128, d_in=32, lambda_token=True)
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok)), C.byref(n)) == 0 and n.value > 0
    for bad in (dict(d_ff=64), dict(act="gelu"), dict(norm="rms"), dict(lambda_token=False), dict(d_in=0),
                dict(lambda_token=False, lambda_channel=True)):
        assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, **bad})), C.byref(n)) == 1, bad
    assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, "post": "relu"})), C.byref(n)) == 2
    # W2 and dW2 are not part of the cell: NULL passes the pointer checks, a missing lambda does not
    d = _desc(**ok)
    bufs = B.hbp_buffers(C.sizeof(B.hbp_buffers))
    for f in ("W1", "U", "xin", "x", "z", "e", "g", "dW1", "dU", "workspace"):
        setattr(bufs, f, 256)
    bufs.workspace_bytes = n.value
    assert B.lib().hbp_check(C.byref(d), C.byref(bufs)) == 4
    bufs.lambda_ = 256
    assert B.lib().hbp_check(C.byref(d), C.byref(bufs)) == 0


def test_transformer_descriptor_rules():
    n = C.c_size_t(0)
    ok = dict(kind="transformer", L=4, N=64, d=128, d_ff=256, heads=2, seq_len=32)
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok)), C.byref(n)) == 0 and n.value > 0
    for bad in (dict(L=3), dict(heads=0), dict(seq_len=0), dict(seq_len=48), dict(heads=3), dict(d_in=8)):
        assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, **bad})), C.byref(n)) == 1, bad
    # heads must be whole 16-byte vectors; a ReLU or norm after the sum is not built for this kind; the plain
    # kernels (fp32, or heads other than 64 wide) hold a row of scores in LDS
    assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, "post": "rms", "norm": "none"})), C.byref(n)) == 0
    for bad in (dict(d=96, heads=8), dict(post="relu"), dict(post="rms"), dict(dtype="f32", N=16384, seq_len=16384),
                dict(heads=4, N=16384, seq_len=16384)):
        assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, **bad})), C.byref(n)) == 2, bad
    assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, "N": 16384, "seq_len": 16384})), C.byref(n)) == 0
    # the attention's weights and saved state are required pointers
    d = _desc(**ok)
    B.lib().hbp_workspace_size(C.byref(d), C.byref(n))
    bufs = B.hbp_buffers(C.sizeof(B.hbp_buffers))
    for f in ("W1", "W2", "x", "y", "rinv", "z", "dphi", "e", "g", "workspace", "Wqkv", "Wo", "qkv", "attn_o"):
        setattr(bufs, f, 256)
    bufs.workspace_bytes = n.value
    assert B.lib().hbp_check(C.byref(d), C.byref(bufs)) == 4
    bufs.lse = 256
    assert B.lib().hbp_check(C.byref(d), C.byref(bufs)) == 0


def test_lstm_descriptor_rules():
    n = C.c_size_t(0)
    ok = dict(kind="lstm", act="tanh", norm="none", d=64, d_ff=128, d_in=32, lambda_token=True)
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok)), C.byref(n)) == 0 and n.value > 0
    assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, "d_ff": 256})), C.byref(n)) == 1
    assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, "lambda_token": False})), C.byref(n)) == 1
    # both halves of [c | h] must be whole 16-byte vectors
    assert B.lib().hbp_workspace_size(C.byref(_desc(**{**ok, "d": 72, "d_ff": 144})), C.byref(n)) == 2


def test_post_norm_descriptor_rules():
    n = C.c_size_t(0)
    ok = dict(norm="none", post="rms")
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok)), C.byref(n)) == 0
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok, gamma=0.5)), C.byref(n)) == 0
    assert B.lib().hbp_workspace_size(C.byref(_desc(post="rms")), C.byref(n)) == 2          # a norm inside the block too
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok, lambda_token=True)), C.byref(n)) == 2
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok, d=4096 + 8)), C.byref(n)) == 2
    assert B.lib().hbp_workspace_size(C.byref(_desc(**ok, d=4096, gamma=0.5)), C.byref(n)) == 2
    assert B.lib().hbp_scan_workspace_size(C.byref(_desc(**ok)), 3, C.byref(n)) == 2


def test_null_pointers_and_workspace_are_checked_before_launch():
    d = _desc()
    bufs = B.hbp_buffers(C.sizeof(B.hbp_buffers))
    lib = B.lib()
    assert lib.hbp_check(C.byref(d), None) == 0
    assert lib.hbp_check(C.byref(d), C.byref(bufs)) == 4          # W1 NULL
    # fake non-null addresses: validation never dereferences them
    for f in ("W1", "W2", "x", "y", "rinv", "z", "dphi", "e", "g"):
        setattr(bufs, f, 0x1000)
    assert lib.hbp_check(C.byref(d), C.byref(bufs)) == 3          # no workspace
    bufs.workspace = 0x1000
    bufs.workspace_bytes = B.workspace_size(d) - 1
    assert lib.hbp_backward(C.byref(d), 1, C.byref(bufs), None) == 3
    bufs.workspace_bytes = B.workspace_size(d)
    assert lib.hbp_check(C.byref(d), C.byref(bufs)) == 0
    assert lib.hbp_backward(C.byref(d), -2, C.byref(bufs), None) == 1
    assert lib.hbp_param_grads(C.byref(d), C.byref(bufs), None) == 4   # dW1 NULL
    d2 = _desc(lambda_channel=True)
    assert lib.hbp_check(C.byref(d2), C.byref(bufs)) == 4         # lambda NULL
    assert lib.hbp_workspace_size(None, None) == 4


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libhbp.so")
    with pytest.raises(RuntimeError):
        B.lib()


def test_header_compiles_as_c_and_links(tmp_path):
    """include/hbp.h is plain C: a C99 program that fills the two structs positionally, asks for the workspace
    size and has its NULL pointers reported, compiled with gcc against the built library."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_hbp.c"
    src.write_text(r'''
#include "hbp.h"
#include <stdio.h>
int main(void) {
  hbp_desc d = { sizeof d, HBP_MLP, HBP_BF16, HBP_ACT_GELU_ERF, HBP_NORM_RMS, HBP_LAMBDA_CHANNEL, 0, 1e-6f,
                 2, 8, 64, 128, 0, 0.f, HBP_POST_NONE };
  size_t ws = 0;
  if (hbp_workspace_size(&d, &ws) != HBP_OK || ws == 0) return 1;
  hbp_buffers b = { sizeof b };
  b.workspace_bytes = ws;
  if (hbp_check(&d, &b) != HBP_E_NULL) return 2;
  if (hbp_backward(&d, 1, &b, NULL) != HBP_E_NULL) return 3;      /* found before anything is launched */
  printf("%s\n", hbp_status_string(HBP_E_NULL));
  return 0;
}
''')
    exe = tmp_path / "use_hbp"
    libdir = os.path.join(root, "paper_2501_17086_amd")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(root, "include"), str(src),
                        "-L", libdir, "-lhbp", f"-Wl,-rpath,{libdir}", "-o", str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "NULL" in r.stdout
