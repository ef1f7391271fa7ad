"""The entry point that allocates nothing (hbp_initial_estimate_static: the chunked scan with its scratch in a
fixed array inside the library) against the entry point it is a variant of (hbp_initial_estimate with
HBP_SCAN_CHUNKED and a caller's workspace), through the C ABI: two calls in a row on one GPU, the second on a
smaller problem, so that what the first call left in the shared scratch is seen not to matter."""
import ctypes as C

import numpy as np
import pytest

from oracle import hbp_oracle as O
from paper_2501_17086_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

W = synth.WORKLOADS
FIRST = synth.scaled(W["gated_rnn_contractive"], name="static_first", L=300, N=6, d=128, d_ff=128, d_in=64)
SECOND = synth.scaled(W["gated_rnn_contractive"], name="static_second", L=130, N=4, d=64, d_ff=64, d_in=32)
FIRST_TOK = synth.scaled(W["gated_rnn_token_gates"], name="static_first_tok", L=330, N=5, d=128, d_ff=128, d_in=64)
SECOND_TOK = synth.scaled(W["gated_rnn_token_gates"], name="static_second_tok", L=70, N=3, d=72, d_ff=72, d_in=32)


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    from paper_2501_17086_amd import binding
    binding.lib()
    return binding


def _one(B, w):
    inp = synth.make_inputs(w)
    st = H.oracle_stack(w, inp)
    sv = O.forward(st, inp["x0"], inp["xin"])
    p = B.allocate(w, inp)
    ws = torch.zeros(max(B.scan_workspace_size(p.desc, "chunked"), 16), dtype=torch.uint8, device=p.g.device)
    p.g.fill_(float("nan"))
    B.hbp_initial_estimate(p, "chunked", workspace=ws)
    torch.cuda.synchronize()
    ref = p.g.clone()
    p.g.fill_(float("nan"))
    B.hbp_initial_estimate_static(p)
    torch.cuda.synchronize()
    assert torch.equal(p.g, ref), f"{w.name}: the two entry points differ"
    want = O.hbp_backward(st, sv, inp["e"], 0)
    H.assert_close(H.to_np(p.g), want, H.TOL[w.dtype], f"{w.name}: w^0 against the oracle")


@pytest.mark.parametrize("first,second", [(FIRST, SECOND), (FIRST_TOK, SECOND_TOK)])
def test_two_calls_in_a_row_the_second_smaller(B, first, second):
    _one(B, first)
    _one(B, second)


def test_sizes_beyond_the_fixed_scratch_are_refused(B):
    # 16 * ceil(L / 64) * N * d bytes: T = 4096, 32 x 1024 chains is exactly the limit; one more row is not
    ok = B.make_desc("rnn", "bf16", "tanh", "none", L=4096, N=32, d=1024, d_ff=1024, d_in=1024,
                     lambda_channel=True, loss_every_state=True)
    assert B.scan_workspace_size(ok, "chunked") == B.STATIC_SCRATCH_BYTES
    w = SECOND
    inp = synth.make_inputs(w)
    p = B.allocate(w, inp)
    big = B.make_desc("rnn", "bf16", "tanh", "none", L=4096, N=33, d=1024, d_ff=1024, d_in=1024,
                      lambda_channel=True, loss_every_state=True)
    b = p.buffers()
    st = B.lib().hbp_initial_estimate_static(C.byref(big), C.byref(b), None)   # refused before any launch
    assert st == 3
    relu = B.make_desc("mlp", "bf16", "gelu", "rms", L=4, N=8, d=64, d_ff=64, lambda_channel=True, post="relu")
    assert B.lib().hbp_initial_estimate_static(C.byref(relu), C.byref(b), None) == 2
