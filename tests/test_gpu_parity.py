"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs.  Bars: relative L2 of 1e-5 for
fp32 storage, 2e-2 for bf16 storage.

Two set-ups.  "end to end": each side runs its own forward from x_0.  "shared
state": the oracle's forward state, rounded to the storage type, is what both
backward passes read -- the backward calls' own inputs are then identical,
which is the only meaningful comparison for the chaotic RNN (trajectories of
two forwards in different precisions separate after a few hundred steps).
"""
import numpy as np
import pytest

from oracle import hbp_oracle as O
from paper_2501_17086_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m gpu on an MI355X box)")
    from paper_2501_17086_amd import binding
    binding.lib()
    return binding


W = synth.WORKLOADS
CASES = {
    # the small fp32 stack at its full size
    "mlp_small_f32": W["mlp_small_f32"],
    # fp32, ragged in every dimension the kernels tile
    "mlp_f32_ragged": synth.scaled(W["mlp_small_f32"], name="mlp_f32_ragged", L=5, N=203, d=72, d_ff=136,
                                   norm="rms", lam="uniform", lam_lo=0.9, lam_hi=1.0, ks=(0, 1, 3, 5)),
    # reduced copies of the bf16 stacks: several tiles and a ragged tail
    "resnet_like_small": synth.scaled(W["resnet_like"], name="resnet_like_small", L=6, N=333, d=512, d_ff=2048,
                                      w2_scale=1 / np.sqrt(6.0), ks=(0, 1, 2, 4, 6)),
    "resnet_like_odd": synth.scaled(W["resnet_like"], name="resnet_like_odd", L=4, N=130, d=264, d_ff=520,
                                    w2_scale=0.5, ks=(1, 3)),
    "transformer_small": synth.scaled(W["transformer_mlp"], name="transformer_small", L=5, N=257, d=1024,
                                      d_ff=1024, w2_scale=1 / np.sqrt(10.0), ks=(1, 2)),
    "deep_small": synth.scaled(W["deep_large"], name="deep_small", L=4, N=192, d=2048, d_ff=512,
                               w2_scale=1 / np.sqrt(8.0), ks=(1, 3)),
    "rnn_small": synth.scaled(W["gated_rnn_contractive"], name="rnn_small", L=37, N=5, d=256, d_ff=256,
                              d_in=128, ks=(0, 1, 2, 4)),
    "rnn_f32": synth.scaled(W["gated_rnn_contractive"], name="rnn_f32", dtype="f32", L=19, N=3, d=64, d_ff=64,
                            d_in=40, ks=(0, 2, 19)),
    # long chains, few of them: the chunked form of the scan (a ragged last chunk and row group)
    "rnn_long": synth.scaled(W["gated_rnn_contractive"], name="rnn_long", L=300, N=6, d=128, d_ff=128,
                             d_in=64, ks=(0, 1, 3)),
    "mlp_f32_deep": synth.scaled(W["mlp_small_f32"], name="mlp_f32_deep", L=270, N=3, d=64, d_ff=64,
                                 w2_scale=0.1, ks=(0, 2)),
    "rnn_chaotic_small": synth.scaled(W["gated_rnn"], name="rnn_chaotic_small", L=130, N=4, d=512, d_ff=512,
                                      d_in=256, ks=(1, 2, 4)),
    # every contraction on whole 256 x 256 tiles (the aligned GEMM kernel), several tiles per workgroup,
    # contraction lengths of 8 and 16 slices; in the RNN the iterations' row counts are padded to the tile
    "aligned_small": synth.scaled(W["resnet_like"], name="aligned_small", L=12, N=512, d=256, d_ff=512,
                                  w2_scale=1 / np.sqrt(12.0), ks=(0, 1, 2, 5)),
    "rnn_aligned": synth.scaled(W["gated_rnn_contractive"], name="rnn_aligned", L=64, N=8, d=256, d_ff=256,
                                d_in=128, ks=(0, 1, 2, 3)),
    # exact BPTT one step at a time: 40 batch rows (two 32-row blocks, the second ragged) with d != d_ff through the
    # few-row kernel, and a width it does not take (96 is no multiple of 64)
    "rnn_rows_40": synth.scaled(W["gated_rnn_contractive"], name="rnn_rows_40", L=20, N=40, d=192, d_ff=320,
                                d_in=64, ks=(0, 2)),
    "rnn_width_96": synth.scaled(W["gated_rnn_contractive"], name="rnn_width_96", L=12, N=7, d=96, d_ff=160,
                                 d_in=32, ks=(0, 2)),
    # a ReLU after the sum (the original ResNet's residual function): wave-per-row scan with the norm (one and two
    # 512-channel chunks), thread-per-vector scan without, a chain long enough that the chunked form would be
    # picked without the mask, and whole 256-row tiles
    "postact_rms": synth.scaled(W["resnet_postact"], name="postact_rms", L=6, N=333, d=512, d_ff=1024,
                                w2_scale=1 / np.sqrt(6.0), ks=(0, 1, 2, 6)),
    "postact_wide": synth.scaled(W["resnet_postact"], name="postact_wide", L=4, N=130, d=1024, d_ff=512,
                                 w2_scale=0.5, ks=(0, 1, 3)),
    "postact_aligned": synth.scaled(W["resnet_postact"], name="postact_aligned", L=9, N=512, d=256, d_ff=512,
                                    w2_scale=1 / 3.0, ks=(0, 2, 4)),
    "postact_f32_none": synth.scaled(W["resnet_postact"], name="postact_f32_none", dtype="f32", norm="none", L=5,
                                     N=203, d=72, d_ff=136, w2_scale=0.4, loss_every_state=True, ks=(0, 1, 2, 5)),
    "postact_f32_deep": synth.scaled(W["resnet_postact"], name="postact_f32_deep", dtype="f32", norm="none", L=270,
                                     N=3, d=64, d_ff=64, w2_scale=0.1, ks=(0, 2)),
    # the gated recurrent cell (residual coefficient = the cell's own 1 - u): few-row kernels for the steps of exact
    # BPTT and of the forward, fp32, a chain long enough for the chunked scan, a width the few-row kernel does not
    # take, and row counts that are whole 256-row tiles
    "gated_small": synth.scaled(W["gru_cell"], name="gated_small", L=37, N=5, d=128, d_ff=256, d_in=64,
                                ks=(0, 1, 2, 5)),
    "gated_f32": synth.scaled(W["gru_cell"], name="gated_f32", dtype="f32", L=19, N=3, d=64, d_ff=128, d_in=32,
                              ks=(0, 1, 3, 19)),
    "gated_long": synth.scaled(W["gru_cell"], name="gated_long", L=330, N=6, d=128, d_ff=256, d_in=64, ks=(0, 2)),
    "gated_width_72": synth.scaled(W["gru_cell"], name="gated_width_72", L=12, N=7, d=72, d_ff=144, d_in=32,
                                   ks=(0, 2)),
    "gated_aligned": synth.scaled(W["gru_cell"], name="gated_aligned", L=64, N=8, d=256, d_ff=512, d_in=128,
                                  ks=(0, 1, 2, 3)),
    # the standard GRU (reset gate: two dependent products per step and per VJP): few-row kernels, fp32, a long chain
    # (single-pass scan + remainder), a width the few-row kernel does not take, whole 256-row tiles, a loss on the
    # last state only, contractions over tokens in several shares
    "gru_small": synth.scaled(W["gru_std_cell"], name="gru_small", L=37, N=5, d=128, d_ff=384, d_in=64,
                              ks=(0, 1, 2, 5)),
    "gru_f32": synth.scaled(W["gru_std_cell"], name="gru_f32", dtype="f32", L=19, N=3, d=64, d_ff=192, d_in=32,
                            ks=(0, 1, 3, 19)),
    "gru_long": synth.scaled(W["gru_std_cell"], name="gru_long", L=330, N=6, d=128, d_ff=384, d_in=64, ks=(0, 2)),
    "gru_width_72": synth.scaled(W["gru_std_cell"], name="gru_width_72", L=12, N=7, d=72, d_ff=216, d_in=32,
                                 ks=(0, 2)),
    "gru_aligned": synth.scaled(W["gru_std_cell"], name="gru_aligned", L=64, N=8, d=256, d_ff=768, d_in=128,
                                ks=(0, 1, 2, 3)),
    "gru_last_loss": synth.scaled(W["gru_std_cell"], name="gru_last_loss", L=23, N=6, d=64, d_ff=192, d_in=32,
                                  loss_every_state=False, ks=(0, 1, 3)),
    "gru_splitk": synth.scaled(W["gru_std_cell"], name="gru_splitk", L=128, N=64, d=256, d_ff=768, d_in=128,
                               ks=(0, 2)),
    # attention sub-blocks (L = 2 x layers): fp32 with narrow heads (plain kernels), causal and not; bf16 with 64-wide
    # heads (matrix-core kernels) on a sequence length with a ragged last tile of 32, not causal on three tiles, 32-wide
    # heads in bf16 (plain kernels), whole 256-row GEMM tiles with several tiles of queries per sequence, a loss at
    # every state without a norm (e added by the second contraction), contractions over tokens in several shares
    "tfm_f32": synth.scaled(W["gpt2_paper"], name="tfm_f32", dtype="f32", L=4, N=30, seq_len=10, d=32, heads=2,
                            d_ff=64, w1_std=0.0, w2_std=0.0, w2_scale=0.7, lam="uniform", lam_lo=0.8, lam_hi=1.0,
                            ks=(0, 1, 2, 4)),
    "tfm_f32_bidir": synth.scaled(W["gpt2_paper"], name="tfm_f32_bidir", dtype="f32", L=6, N=21, seq_len=7, d=48,
                                  heads=3, d_ff=40, w1_std=0.0, w2_std=0.0, w2_scale=0.7, causal=False, ks=(0, 2, 6)),
    "tfm_small": synth.scaled(W["gpt2_paper"], name="tfm_small", L=6, N=120, seq_len=40, d=128, heads=2, d_ff=256,
                              w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(0, 1, 2, 6)),
    "tfm_bidir": synth.scaled(W["gpt2_paper"], name="tfm_bidir", L=4, N=140, seq_len=70, d=128, heads=2, d_ff=128,
                              w1_std=0.0, w2_std=0.0, w2_scale=0.6, causal=False, ks=(0, 1, 3)),
    "tfm_heads_32": synth.scaled(W["gpt2_paper"], name="tfm_heads_32", L=4, N=66, seq_len=33, d=64, heads=2, d_ff=128,
                                 w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(0, 2)),
    "tfm_aligned": synth.scaled(W["gpt2_paper"], name="tfm_aligned", L=4, N=1024, seq_len=256, d=256, heads=4,
                                d_ff=512, w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(0, 1, 2, 3)),
    "tfm_loss_all": synth.scaled(W["gpt2_paper"], name="tfm_loss_all", L=4, N=96, seq_len=48, d=128, heads=2,
                                 d_ff=256, norm="none", w2_scale=0.5, loss_every_state=True, lam="uniform",
                                 lam_lo=0.8, lam_hi=1.0, ks=(0, 1, 3)),
    # sequences of one token (the softmax is 1: o = v), of exactly one tile, and of five tiles (two workgroups of
    # query tiles, the second with one live wavefront) with and without the causal mask
    "tfm_one_token": synth.scaled(W["gpt2_paper"], name="tfm_one_token", L=4, N=24, seq_len=1, d=128, heads=2, d_ff=128,
                                  w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(0, 2)),
    "tfm_one_tile": synth.scaled(W["gpt2_paper"], name="tfm_one_tile", L=2, N=96, seq_len=32, d=64, heads=1, d_ff=128,
                                 w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(1, 2)),
    "tfm_five_tiles": synth.scaled(W["gpt2_paper"], name="tfm_five_tiles", L=4, N=320, seq_len=160, d=192, heads=3,
                                   d_ff=256, w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(1, 3)),
    "tfm_five_tiles_bidir": synth.scaled(W["gpt2_paper"], name="tfm_five_tiles_bidir", L=2, N=298, seq_len=149, d=128,
                                         heads=2, d_ff=128, w1_std=0.0, w2_std=0.0, w2_scale=0.6, causal=False, ks=(1, 2)),
    # post-norm transformer layers (the norm after each residual sum), run with the gamma split they need
    "tfm_postnorm_f32": synth.scaled(W["gpt2_paper"], name="tfm_postnorm_f32", dtype="f32", L=4, N=36, seq_len=12, d=32,
                                     heads=2, d_ff=64, norm="none", post="rms", w1_std=0.0, w2_std=0.0, w2_scale=0.7,
                                     causal=False, gamma=0.8, ks=(0, 1, 2, 4)),
    "tfm_postnorm": synth.scaled(W["gpt2_paper"], name="tfm_postnorm", L=6, N=150, seq_len=50, d=128, heads=2, d_ff=256,
                                 norm="none", post="rms", w1_std=0.0, w2_std=0.0, w2_scale=0.6, causal=False, gamma=0.8,
                                 ks=(0, 1, 3, 6)),
    "tfm_splitk": synth.scaled(W["gpt2_paper"], name="tfm_splitk", L=2, N=8192, seq_len=128, d=128, heads=2,
                               d_ff=256, w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(0, 2)),
    # the LSTM cell (state [c | h]; the contraction's result lands in the hidden half of v with the full row stride)
    "lstm_small": synth.scaled(W["lstm_cell"], name="lstm_small", L=37, N=5, d=128, d_ff=256, d_in=64,
                               ks=(0, 1, 2, 5)),
    "lstm_f32": synth.scaled(W["lstm_cell"], name="lstm_f32", dtype="f32", L=19, N=3, d=64, d_ff=128, d_in=32,
                             ks=(0, 1, 3, 19)),
    "lstm_long": synth.scaled(W["lstm_cell"], name="lstm_long", L=330, N=6, d=128, d_ff=256, d_in=64, ks=(0, 2)),
    "lstm_width_80": synth.scaled(W["lstm_cell"], name="lstm_width_80", L=12, N=7, d=80, d_ff=160, d_in=32,
                                  ks=(0, 2)),
    "lstm_aligned": synth.scaled(W["lstm_cell"], name="lstm_aligned", L=64, N=8, d=512, d_ff=1024, d_in=128,
                                 ks=(0, 1, 2, 3)),
    # a token count that is no multiple of the 256-row tile: whole tiles on the aligned kernel, the last 88 rows on
    # the general one (resnet_like_small and transformer_small take the same route with one whole tile)
    "ragged_tokens": synth.scaled(W["resnet_like"], name="ragged_tokens", L=3, N=600, d=256, d_ff=512,
                                  w2_scale=1 / np.sqrt(3.0), ks=(0, 1, 3)),
    # post-norm stacks (RMS norm after the sum): one and two 512-channel chunks per row, fp32 without whole tiles and
    # with a loss on every state, whole 256-row tiles
    "postnorm_small": synth.scaled(W["postnorm_mlp"], name="postnorm_small", L=6, N=333, d=512, d_ff=1024,
                                   ks=(0, 1, 2, 6)),
    "postnorm_wide": synth.scaled(W["postnorm_mlp"], name="postnorm_wide", L=4, N=130, d=1024, d_ff=512,
                                  lam="uniform", lam_lo=0.8, lam_hi=1.0, ks=(0, 1, 3)),
    "postnorm_aligned": synth.scaled(W["postnorm_mlp"], name="postnorm_aligned", L=9, N=512, d=256, d_ff=512,
                                     ks=(0, 2, 4)),
    # rows split over four wavefronts (the last one past the width) with one row per workgroup, and over two
    # (the second one partly past the width) with a spare row in the last workgroup
    "postnorm_four_waves": synth.scaled(W["postnorm_mlp"], name="postnorm_four_waves", L=5, N=37, d=1536, d_ff=256,
                                        lam="uniform", lam_lo=0.8, lam_hi=1.0, ks=(0, 1, 3)),
    "postnorm_two_waves_odd": synth.scaled(W["postnorm_mlp"], name="postnorm_two_waves_odd", L=7, N=45, d=640,
                                           d_ff=256, loss_every_state=True, ks=(0, 2, 4)),
    "postnorm_f32": synth.scaled(W["postnorm_mlp"], name="postnorm_f32", dtype="f32", L=5, N=203, d=72, d_ff=136,
                                 w1_std=0.0, w2_std=0.0, lam="uniform", lam_lo=0.8, lam_hi=1.0,
                                 loss_every_state=True, ks=(0, 1, 2, 5)),
    # the cells with a loss on the last state only (g[L] seeded by a copy, no e in the second contraction's epilogue
    # or in the LSTM's elementwise kernel), and a ReLU stack with a norm and a loss on every state (e read by the scan)
    "gated_last_loss": synth.scaled(W["gru_cell"], name="gated_last_loss", L=23, N=6, d=64, d_ff=128, d_in=32,
                                    loss_every_state=False, ks=(0, 1, 3)),
    "lstm_last_loss": synth.scaled(W["lstm_cell"], name="lstm_last_loss", L=23, N=6, d=128, d_ff=256, d_in=32,
                                   loss_every_state=False, ks=(0, 1, 3)),
    "postact_loss_all": synth.scaled(W["resnet_postact"], name="postact_loss_all", L=7, N=96, d=128, d_ff=256,
                                     w2_scale=1 / np.sqrt(7.0), loss_every_state=True, ks=(0, 1, 2, 7)),
    # widths that are no multiple of the 256-wide tile (320 = 256 + 64, 640 = 512 + 128) with 640 tokens: every
    # contraction is split into a part on the aligned kernel and row / column remainders on the general one
    "odd_widths": synth.scaled(W["resnet_like"], name="odd_widths", L=3, N=640, d=320, d_ff=640,
                               w2_scale=1 / np.sqrt(3.0), ks=(0, 1, 3)),
    # a loss on every state of a depth stack (e read by the scan behind the norm's backward), and without a norm
    # (e added by the second contraction's epilogue)
    # coefficients per (block, token, channel): direct scans (depth, RMS and none) and the chunked scan (time)
    "rnn_token_gates": synth.scaled(W["gated_rnn_token_gates"], name="rnn_token_gates", L=40, N=9, d=128, d_ff=128,
                                    d_in=64, ks=(0, 1, 2, 5)),
    "rnn_token_gates_long": synth.scaled(W["gated_rnn_token_gates"], name="rnn_token_gates_long", L=330, N=5, d=128,
                                         d_ff=128, d_in=64, ks=(0, 1, 3)),
    "rnn_token_gates_f32": synth.scaled(W["gated_rnn_token_gates"], name="rnn_token_gates_f32", dtype="f32", L=21,
                                        N=4, d=64, d_ff=64, d_in=24, ks=(0, 2, 21)),
    "mlp_token_gates": synth.scaled(W["resnet_like"], name="mlp_token_gates", lam="sigmoid_full", lam_lo=2.0,
                                    lam_hi=0.7, L=6, N=200, d=256, d_ff=512, w2_scale=1 / np.sqrt(6.0),
                                    ks=(0, 1, 3, 6)),
    "mlp_loss_all": synth.scaled(W["resnet_like"], name="mlp_loss_all", L=7, N=96, d=128, d_ff=256,
                                 loss_every_state=True, w2_scale=1 / np.sqrt(7.0), ks=(0, 1, 3, 7)),
    "mlp_loss_all_nonorm": synth.scaled(W["resnet_like"], name="mlp_loss_all_nonorm", norm="none", L=5, N=256, d=256,
                                        d_ff=256, loss_every_state=True, w2_scale=0.3, ks=(0, 2, 5)),
    # contractions over 8192 and more token rows: the parameter gradients are computed in several shares of the
    # token range (split-K) whose partial sums a second kernel adds up.  Whole 256-wide tiles (the aligned
    # kernel); widths of 320 = 256 + 64 and 640 = 512 + 128 (aligned part plus row / column remainders on the
    # general kernel, each with its own shares); a narrow dU (128 columns: the general kernel alone); the cells.
    "mlp_splitk": synth.scaled(W["resnet_like"], name="mlp_splitk", L=2, N=8192, d=256, d_ff=512,
                               w2_scale=1 / np.sqrt(2.0), ks=(0, 2)),
    "mlp_splitk_odd": synth.scaled(W["resnet_like"], name="mlp_splitk_odd", L=2, N=8192, d=320, d_ff=640,
                                   w2_scale=1 / np.sqrt(2.0), ks=(1,)),
    "rnn_splitk": synth.scaled(W["gated_rnn_contractive"], name="rnn_splitk", L=128, N=64, d=256, d_ff=256,
                               d_in=128, ks=(0, 2)),
    "rnn_splitk_odd": synth.scaled(W["gated_rnn_contractive"], name="rnn_splitk_odd", L=512, N=24, d=320, d_ff=320,
                                   d_in=192, ks=(1,)),
    "gated_splitk": synth.scaled(W["gru_cell"], name="gated_splitk", L=128, N=64, d=256, d_ff=512, d_in=128,
                                 ks=(0, 2)),
    "lstm_splitk": synth.scaled(W["lstm_cell"], name="lstm_splitk", L=128, N=64, d=512, d_ff=1024, d_in=128,
                                ks=(0, 2)),
}
SPLITK_CASES = ["mlp_splitk", "mlp_splitk_odd", "rnn_splitk", "rnn_splitk_odd", "gated_splitk", "lstm_splitk",
                "gru_splitk"]       # (tfm_splitk is listed with the transformer cases)
TFM_CASES = ["tfm_f32", "tfm_f32_bidir", "tfm_small", "tfm_bidir", "tfm_heads_32", "tfm_aligned", "tfm_loss_all",
             "tfm_splitk", "tfm_one_token", "tfm_one_tile", "tfm_five_tiles", "tfm_five_tiles_bidir"]
TFM_POSTNORM = ["tfm_postnorm_f32", "tfm_postnorm"]
GRU_CASES = ["gru_small", "gru_f32", "gru_long", "gru_width_72", "gru_aligned", "gru_last_loss"]


def _setup(B, w):
    inp = synth.make_inputs(w)
    st = H.oracle_stack(w, inp)
    sv = O.forward(st, inp["x0"], inp["xin"])
    p = B.allocate(w, inp)
    return inp, st, sv, p


@pytest.mark.parametrize("name", ["mlp_small_f32", "mlp_f32_ragged", "resnet_like_small", "resnet_like_odd",
                                  "transformer_small", "deep_small", "rnn_small", "rnn_f32", "rnn_token_gates",
                                  "rnn_token_gates_f32", "mlp_token_gates"])
def test_forward_parity(B, name):
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    assert H.rel(H.to_np(p.x), sv["x"]) < tol
    assert H.rel(H.to_np(p.z), sv["z"]) < tol
    if p.dphi is not None:
        assert H.rel(H.to_np(p.dphi), sv["dphi"]) < tol
    if p.y is not None:
        assert H.rel(H.to_np(p.y), sv["y"]) < tol
        assert H.rel(H.to_np(p.rinv), sv["rinv"]) < tol


def _check_backward(B, w, p, st, sv_oracle, inp, tag, exact=True):
    """Every k of the case, then exact BP, each followed by the parameter gradients.  Every state gradient and
    every parameter gradient is compared as a whole, row by row and element by element (helpers.assert_close)."""
    tol = H.TOL[w.dtype]
    xin = inp["xin"]

    def compare(label, want_g):
        kept = H.as_kept(st, sv_oracle, want_g)
        got = H.to_np(p.g)
        err = H.rel(got, kept)
        assert err < tol, f"{tag} {label}: g rel L2 {err:.3e}"
        for l in range(w.L + 1):     # per state: an error confined to one state, row or element must not hide
            H.assert_close(got[l], kept[l], 2 * tol, f"{tag} {label} state {l}", row_factor=2.0, abs_factor=4.0)
        pg = O.param_grads(st, sv_oracle, want_g, xin)
        for nm, t in (("dW1", p.dW1), ("dW2", p.dW2), ("dU", p.dU), ("dWqkv", p.dWqkv), ("dWo", p.dWo)):
            if t is not None:
                H.assert_close(H.to_np(t), pg[nm], tol, f"{tag} {label}: {nm}", row_floor=0.5)

    for k in w.ks:
        B.hbp_backward(p, k)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        compare(f"k={k}", O.hbp_backward(st, sv_oracle, inp["e"], k, gamma=w.gamma))   # the workload's own split
    if not exact:
        return
    B.hbp_exact_backward(p)
    B.hbp_param_grads(p)
    torch.cuda.synchronize()
    compare("exact", O.exact_backward(st, sv_oracle, inp["e"]))


@pytest.mark.parametrize("name", ["mlp_small_f32", "mlp_f32_ragged", "resnet_like_small", "resnet_like_odd",
                                  "transformer_small", "deep_small", "rnn_small", "rnn_f32", "rnn_long",
                                  "mlp_f32_deep", "aligned_small", "rnn_aligned", "mlp_loss_all",
                                  "mlp_loss_all_nonorm", "rnn_token_gates", "rnn_token_gates_long",
                                  "rnn_token_gates_f32", "mlp_token_gates", "rnn_rows_40", "rnn_width_96",
                                  "postact_f32_none", "gated_small", "gated_f32", "gated_long", "gated_width_72",
                                  "gated_aligned", "lstm_small", "lstm_f32", "lstm_long", "lstm_width_80",
                                  "lstm_aligned", "ragged_tokens", "postnorm_f32", "postnorm_small",
                                  "gated_last_loss", "lstm_last_loss", "odd_widths"] + SPLITK_CASES + GRU_CASES
                         + TFM_CASES + ["tfm_postnorm_f32"])
def test_backward_end_to_end(B, name):
    """Own forward on each side, then Highway-BP at every k of the case, exact BP
    and the parameter gradients."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    _check_backward(B, w, p, st, sv, inp, name)


@pytest.mark.parametrize("name", TFM_CASES + TFM_POSTNORM)
def test_forward_of_the_transformer_stack(B, name):
    """States, the MLP sub-blocks' inner state, [q | k | v], the attention's output and its row statistics."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    for l in range(w.L + 1):
        H.assert_close(H.to_np(p.x)[l], sv["x"][l], tol, f"{name} x[{l}]")
    H.assert_close(H.to_np(p.z), sv["z"][1::2], tol, f"{name} z")
    H.assert_close(H.to_np(p.qkv), sv["qkv"][0::2], tol, f"{name} qkv")
    H.assert_close(H.to_np(p.attn_o), sv["o"][0::2], tol, f"{name} attention output")
    want = np.stack([H.attn_row_stats(st, sv["qkv"][l]) for l in range(0, w.L, 2)])
    assert np.abs(H.to_np(p.lse) - want).max() < (1e-4 if w.dtype == "f32" else 0.05)


@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("T", [2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 160, 255, 257])
def test_attention_around_tile_and_workgroup_boundaries(B, T, causal):
    """One layer pair (attention + MLP) on two sequences of every length around the 32-row tiles and the 128-row
    workgroup blocks of the attention kernels: forward state, Highway-BP at k = 1, 2 and all parameter gradients."""
    w = synth.scaled(W["gpt2_paper"], name=f"tfm_T{T}", L=2, N=2 * T, seq_len=T, d=64, heads=1, d_ff=64, w1_std=0.0,
                     w2_std=0.0, w2_scale=0.6, causal=causal, ks=(1, 2))
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    H.assert_close(H.to_np(p.attn_o), sv["o"][0::2], H.TOL[w.dtype], f"{w.name} attention output")
    _check_backward(B, w, p, st, sv, inp, w.name, exact=False)


def test_attention_problem_by_problem_with_a_ragged_problem_count(B):
    """Enough (sequence, head) problems that the attention kernels take their workgroups problem by problem, one XCD
    per problem (grids of 4096 workgroups and more), and a problem count that is no multiple of the eight XCDs:
    forward state and Highway-BP at k = 1 on 2052 sequences of 129 tokens (two blocks of tiles each)."""
    w = synth.scaled(W["gpt2_paper"], name="tfm_many_sequences", L=2, N=2052 * 129, seq_len=129, d=64, heads=1, d_ff=64,
                     w1_std=0.0, w2_std=0.0, w2_scale=0.6, ks=(1,))
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    H.assert_close(H.to_np(p.attn_o), sv["o"][0::2], H.TOL[w.dtype], f"{w.name} attention output")
    _check_backward(B, w, p, st, sv, inp, w.name, exact=False)


@pytest.mark.parametrize("name", ["gated_small", "gated_f32", "gated_width_72", "gated_aligned"])
def test_forward_of_the_gated_cell(B, name):
    """States, both gates ([u | c] side by side) and the residual coefficient 1 - u that the forward writes."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    assert H.rel(H.to_np(p.x), sv["x"]) < tol
    assert H.rel(H.to_np(p.z), np.concatenate([sv["u"], sv["c"]], axis=-1)) < tol
    assert H.rel(H.to_np(p.lam), sv["a"]) < tol


@pytest.mark.parametrize("name", ["gru_small", "gru_f32", "gru_width_72", "gru_aligned"])
def test_forward_of_the_standard_gru(B, name):
    """States, the three gates [z | r | n] and the residual coefficient 1 - z that the forward writes."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    assert H.rel(H.to_np(p.x), sv["x"]) < tol
    assert H.rel(H.to_np(p.z), sv["zrn"]) < tol
    assert H.rel(H.to_np(p.lam), sv["a"]) < tol


@pytest.mark.parametrize("name", ["lstm_small", "lstm_f32", "lstm_width_80", "lstm_aligned"])
def test_forward_of_the_lstm_cell(B, name):
    """States [c | h], the four gates and the residual coefficient [f | 0] that the forward writes."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    assert H.rel(H.to_np(p.x), sv["x"]) < tol
    assert H.rel(H.to_np(p.z), sv["gates"]) < tol
    assert H.rel(H.to_np(p.lam), sv["a"]) < tol
    assert float(p.lam[..., w.d // 2:].abs().max()) == 0.0


@pytest.mark.parametrize("name", ["postnorm_small", "postnorm_wide", "postnorm_f32"])
def test_forward_of_a_post_norm_stack(B, name):
    """Normalised states and the norm's 1/rms of each sum."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    assert H.rel(H.to_np(p.x), sv["x"]) < tol
    assert H.rel(H.to_np(p.rinv), sv["rpost"]) < tol
    assert H.rel(H.to_np(p.z), sv["z"]) < tol


@pytest.mark.parametrize("name", ["postact_rms", "postact_wide", "postact_f32_none", "postact_f32_deep"])
def test_forward_with_relu_after_the_sum(B, name):
    """States and the ReLU's mask.  A sum within rounding of zero may land on the other side in the
    storage type: the masks may differ there and nowhere else."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    torch.cuda.synchronize()
    tol = H.TOL[w.dtype]
    assert H.rel(H.to_np(p.x), sv["x"]) < tol
    assert float(H.to_np(p.x)[1:].min()) >= 0.0
    got = H.mask_bits(p)
    assert np.array_equal(got, (H.to_np(p.x)[1:] > 0).astype(np.float64))
    differ = got != sv["mask"]
    assert differ.mean() < (2e-2 if w.dtype == "bf16" else 1e-4)
    scale = np.sqrt(np.mean(sv["x"][1:] ** 2))
    assert np.all(np.abs(sv["x"][1:][differ]) < 10 * tol * scale)


@pytest.mark.parametrize("name", ["mlp_f32_ragged", "resnet_like_small", "rnn_small", "rnn_chaotic_small",
                                  "postact_rms", "postact_wide", "postact_aligned", "postact_f32_none",
                                  "postact_f32_deep", "gated_small", "gated_long", "lstm_small", "lstm_long",
                                  "postnorm_small", "postnorm_wide", "postnorm_aligned", "postnorm_f32",
                                  "postnorm_four_waves", "postnorm_two_waves_odd",
                                  "postact_loss_all", "gru_small", "gru_long", "tfm_f32", "tfm_small", "tfm_bidir",
                                  "tfm_heads_32"] + TFM_POSTNORM)
def test_backward_shared_state(B, name):
    """Both backward passes read the same (storage-rounded) forward state."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    sv_r = H.oracle_saved_rounded(w, sv)
    sv_r["_stack"] = st
    H.upload_saved(p, w, sv_r)
    # Exact BPTT through the chaotic RNN amplifies storage rounding exponentially
    # with the number of steps (gradient norms grow by orders of magnitude), so
    # the bf16 bar is only meaningful there for the k-iteration estimates; exact
    # BPTT is checked on the contractive variant (rnn_small).
    _check_backward(B, w, p, st, sv_r, inp, name + "/shared", exact=name != "rnn_chaotic_small")


@pytest.mark.parametrize("name,gamma", [("mlp_small_f32", 0.2), ("mlp_f32_ragged", 0.8), ("mlp_f32_ragged", 1.0),
                                        ("resnet_like_small", 0.2), ("resnet_like_small", 1.0),
                                        ("deep_small", 0.5), ("rnn_small", 0.3), ("rnn_f32", 1.0), ("rnn_long", 0.2), ("rnn_long", 1.0),
                                        ("aligned_small", 0.8), ("rnn_token_gates", 0.4),
                                        ("rnn_token_gates_long", 1.0), ("mlp_token_gates", 0.3),
                                        ("gated_small", 0.3), ("gated_long", 1.0), ("gated_f32", 0.6),
                                        ("lstm_small", 0.3), ("lstm_long", 0.7), ("gru_small", 0.3), ("gru_long", 1.0),
                                        ("tfm_f32", 0.2), ("tfm_small", 0.2), ("tfm_small", 1.0), ("tfm_postnorm", 0.5),
                                        ("postnorm_small", 0.5), ("postnorm_wide", 0.8), ("postnorm_f32", 1.0),
                                        ("postnorm_aligned", 0.2), ("postnorm_four_waves", 0.5),
                                        ("postnorm_two_waves_odd", 0.8)])
def test_gamma_iterates(B, name, gamma):
    """The iteration on the re-split pair (J + gamma K, (1 - gamma) K): every k of
    the case against the oracle on a shared forward state; gamma = 1 is the
    fixed-point-iteration baseline.  k >= L gives the exact gradient for any gamma."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    sv_r = H.oracle_saved_rounded(w, sv)
    sv_r["_stack"] = st
    H.upload_saved(p, w, sv_r)
    tol = H.TOL[w.dtype]
    for k in w.ks:
        B.hbp_backward(p, k, gamma=gamma)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        want = O.hbp_backward(st, sv_r, inp["e"], k, gamma=gamma)
        kept = H.as_kept(st, sv_r, want)
        err = H.rel(H.to_np(p.g), kept)
        assert err < tol, f"{name} gamma={gamma} k={k}: g rel L2 {err:.3e}"
        for l in range(w.L + 1):
            n = np.linalg.norm(kept[l])
            if n > 1e-30:   # (at gamma = 1 and a loss on the last state only, states below L - k are exactly 0)
                el = H.rel(H.to_np(p.g[l]), kept[l])
                assert el < 2 * tol, f"{name} gamma={gamma} k={k} state {l}: {el:.3e}"
            else:
                assert float(p.g[l].abs().max()) == 0.0
        pg = O.param_grads(st, sv_r, want, inp["xin"])
        for nm, t in (("dW1", p.dW1), ("dW2", p.dW2), ("dU", p.dU), ("dWqkv", p.dWqkv), ("dWo", p.dWo)):
            if t is not None:
                assert H.rel(H.to_np(t), pg[nm]) < tol, f"{name} gamma={gamma} k={k}: {nm}"
    if w.L <= 40:
        B.hbp_backward(p, w.L, gamma=gamma)
        torch.cuda.synchronize()
        G = O.exact_backward(st, sv_r, inp["e"])
        assert H.rel(H.to_np(p.g), H.as_kept(st, sv_r, G)) < tol


@pytest.mark.parametrize("name", ["mlp_f32_ragged", "resnet_like_small", "rnn_small", "rnn_f32", "rnn_long",
                                  "rnn_token_gates", "rnn_token_gates_long", "mlp_loss_all", "mlp_small_f32"])
@pytest.mark.parametrize("algorithm", ["auto", "sequential", "chunked", "single_pass", "hillis_steele"])
def test_initial_estimate_by_every_form_of_the_scan(B, name, algorithm):
    """w^0 = CumSumProd(e, K): the sequential walk, the chunked three-pass form, the single-pass form with its
    chained look-back and the sweeps of the paper's Algorithm 1 give the oracle's result (and so each other's)
    up to rounding order."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    if algorithm == "single_pass" and w.dtype != "bf16":      # bf16 storage only
        with pytest.raises(B.HbpError) as ei:
            B.scan_workspace_size(p.desc, algorithm)
        assert ei.value.status == 2
        return
    ws = torch.zeros(max(B.scan_workspace_size(p.desc, algorithm), 16), dtype=torch.uint8, device=p.g.device)
    p.g.fill_(float("nan"))
    B.hbp_initial_estimate(p, algorithm, workspace=ws)
    torch.cuda.synchronize()
    want = O.hbp_backward(st, sv, inp["e"], 0)
    assert H.rel(H.to_np(p.g), want) < H.TOL[w.dtype], f"{name} {algorithm}"
    for l in range(w.L + 1):
        if np.linalg.norm(want[l]) > 0:
            assert H.rel(H.to_np(p.g[l]), want[l]) < 2 * H.TOL[w.dtype], f"{name} {algorithm} state {l}"


@pytest.mark.parametrize("name", ["postact_rms", "postact_f32_none", "postact_f32_deep", "postnorm_small",
                                  "postnorm_f32"])
@pytest.mark.parametrize("algorithm", ["auto", "sequential"])
def test_initial_estimate_with_relu_after_the_sum(B, name, algorithm):
    """w^0 along K_l = diag(mask_l lambda_l) on the oracle's forward state (its mask uploaded); the
    chunked form and the sweeps are refused for this residual function."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    sv_r = H.oracle_saved_rounded(w, sv)
    H.upload_saved(p, w, sv_r)
    ws = torch.zeros(max(B.scan_workspace_size(p.desc, algorithm), 16), dtype=torch.uint8, device=p.g.device)
    p.g.fill_(float("nan"))
    B.hbp_initial_estimate(p, algorithm, workspace=ws)
    torch.cuda.synchronize()
    want = H.as_kept(st, sv_r, O.hbp_backward(st, sv_r, inp["e"], 0))
    assert H.rel(H.to_np(p.g), want) < H.TOL[w.dtype], f"{name} {algorithm}"
    for other in ("chunked", "hillis_steele", "single_pass"):
        with pytest.raises(B.HbpError) as ei:
            B.scan_workspace_size(p.desc, other)
        assert ei.value.status == 2


def test_gamma_needs_narrow_rows_with_rms(B):
    d = B.make_desc("mlp", "bf16", "gelu", "rms", L=2, N=8, d=4096, d_ff=64, gamma=0.5)
    assert B.workspace_size(B.make_desc("mlp", "bf16", "gelu", "rms", L=2, N=8, d=4096, d_ff=64)) > 0
    n = __import__("ctypes").c_size_t(0)
    assert B.lib().hbp_workspace_size(__import__("ctypes").byref(d), __import__("ctypes").byref(n)) == 2


def test_k_beyond_L_is_exact_and_deterministic(B):
    w = CASES["resnet_like_odd"]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    B.hbp_backward(p, w.L + 3)
    torch.cuda.synchronize()
    a = p.g.clone()
    B.hbp_backward(p, w.L)
    torch.cuda.synchronize()
    assert torch.equal(a, p.g)
    B.hbp_exact_backward(p)
    torch.cuda.synchronize()
    assert H.rel(H.to_np(a), H.to_np(p.g)) < 1e-2
    # run-to-run determinism (this case's contractions over tokens are short: one share each; the split ones
    # are covered by test_split_parameter_gradients_are_deterministic)
    B.hbp_backward(p, 2)
    B.hbp_param_grads(p)
    torch.cuda.synchronize()
    g1, w1, w2 = p.g.clone(), p.dW1.clone(), p.dW2.clone()
    p.g.zero_(); p.dW1.zero_(); p.dW2.zero_()
    B.hbp_backward(p, 2)
    B.hbp_param_grads(p)
    torch.cuda.synchronize()
    assert torch.equal(g1, p.g) and torch.equal(w1, p.dW1) and torch.equal(w2, p.dW2)


@pytest.mark.parametrize("name", SPLITK_CASES + ["rnn_long", "rnn_token_gates_long", "gated_long", "tfm_splitk", "tfm_small"])
def test_split_parameter_gradients_are_deterministic(B, name):
    """Two runs from scratch give the same bits: the shares of a split contraction are added in a fixed order by
    a second kernel (no atomics), and the chunked scan combines its chunks in a fixed order."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    outs = []
    for _ in range(2):
        for t in (p.g, p.dW1, p.dW2, p.dU, p.dWqkv, p.dWo, p.workspace):
            if t is not None:
                t.fill_(0)
        B.hbp_backward(p, 2)
        B.hbp_param_grads(p)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (p.g, p.dW1, p.dW2, p.dU, p.dWqkv, p.dWo) if t is not None])
    for a, b in zip(*outs):
        assert torch.equal(a, b)


@pytest.mark.parametrize("L,N", [(1, 1), (1, 9), (2, 1), (3, 64)])
def test_degenerate_sizes(B, L, N):
    w = synth.scaled(W["resnet_like"], name="tiny", L=L, N=N, d=64, d_ff=128, w2_scale=1.0, ks=(0, 1, 2))
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)
    _check_backward(B, w, p, st, sv, inp, f"tiny L={L} N={N}")


def test_error_codes_on_device_buffers(B):
    w = CASES["resnet_like_odd"]
    inp, st, sv, p = _setup(B, w)
    with pytest.raises(B.HbpError) as ei:
        B.hbp_backward(p, -1)
    assert ei.value.status == 1
    ws = p.workspace
    p.workspace = ws[: ws.numel() // 2]
    with pytest.raises(B.HbpError) as ei:
        B.hbp_backward(p, 1)
    assert ei.value.status == 3
    p.workspace = ws
    e = p.e
    p.e = None
    with pytest.raises(B.HbpError) as ei:
        B.hbp_exact_backward(p)
    assert ei.value.status == 4
    p.e = e
    B.hbp_forward(p)
    B.hbp_backward(p, 1)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["aligned_small", "rnn_aligned", "gated_small", "postact_rms", "tfm_aligned"])
def test_calls_can_be_captured_in_a_graph_and_replayed(B, name):
    """The backward calls allocate nothing and never synchronise, so a caller may record them into a HIP graph:
    every replay, with eager work and synchronisations between them, gives the eager result bit for bit."""
    w = CASES[name]
    inp, st, sv, p = _setup(B, w)
    B.hbp_forward(p)

    def step():
        B.hbp_backward(p, 2)
        B.hbp_param_grads(p)
    step()
    torch.cuda.synchronize()
    ref_g, ref_w = p.g.clone(), p.dW1.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):       # a first run on the capturing side, as torch's capture protocol asks
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for _ in range(3):
        p.g.fill_(float("nan"))
        p.dW1.fill_(float("nan"))
        B.hbp_exact_backward(p)          # eager work between the replays
        torch.cuda.synchronize()
        p.g.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(p.g, ref_g)
        assert torch.equal(p.dW1, ref_w)
