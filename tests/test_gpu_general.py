"""GPU parity of the general path: Haar transform of any sequence length and with the first token left out of L,
sequency-ordered WHT, DCT, the transformed-bias form, per-block scales.  Every case goes through the C ABI and is
compared with the oracle: codes and scales bit for bit, outputs to the output bar."""
import numpy as np
import pytest

import stamp_testlib as tl
from gen.workloads import Workload, make_inputs
from oracle import stamp_oracle as so

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2510_26771_amd as st
    st.load_library()


def _wl(name, **kw):
    base = dict(batch=1, seq_len=256, d_in=128, d_out=192, xform="haar1d", levels=3, k_hi=16, x_dtype="f32", rho=0.9,
                n_outlier_channels=3, outlier_scale=20.0, w_std=0.05, seed=11)
    base.update(kw)
    return Workload(name, **base)


RAGGED = [
    _wl("rag_100_J3", batch=2, seq_len=100, levels=3, seed=21),
    _wl("rag_333_all", seq_len=333, levels=so.max_ragged_levels(333), k_hi=8, seed=22),
    _wl("rag_2049_J12", seq_len=2049, levels=12, k_hi=64, d_in=256, d_out=130, x_dtype="bf16", seed=23),
    _wl("rag_2047_J5_asym", seq_len=2047, levels=5, k_hi=64, act_quant="asym", mean_shift=1.5, seed=24),
    _wl("rag_7_J3", batch=3, seq_len=7, levels=3, k_hi=1, seed=25),
    _wl("rag_3_J0", seq_len=3, levels=0, k_hi=0, seed=26),
    _wl("skip_256_J8", batch=2, seq_len=256, levels=8, skip_first=True, first_token_scale=100.0, seed=28),
    _wl("skip_1024_J3_k64", seq_len=1024, levels=3, k_hi=64, skip_first=True, first_token_scale=100.0, x_dtype="bf16",
        seed=29),
    _wl("skip_130_J2_asym", seq_len=130, levels=2, k_hi=4, skip_first=True, first_token_scale=50.0, act_quant="asym",
        seed=30),
    _wl("skip_3_J1", seq_len=3, levels=1, k_hi=1, skip_first=True, seed=31),
]


@pytest.mark.parametrize("w", RAGGED, ids=[w.name for w in RAGGED])
def test_haar_any_length_and_first_token_left_out(w):
    tl.full_case(w, with_bias=True, check_unfused=False)


OTHER = [
    _wl("wht_256", batch=2, xform="wht", levels=0, seed=41),
    _wl("wht_2048_asym", xform="wht", levels=0, seq_len=2048, k_hi=64, act_quant="asym", mean_shift=0.5, seed=42),
    _wl("wht_2", xform="wht", levels=0, seq_len=2, k_hi=1, seed=43),
    _wl("dct_256", batch=2, xform="dct", levels=0, seed=44),
    _wl("dct_200", xform="dct", levels=0, seq_len=200, k_hi=8, x_dtype="bf16", seed=45),
    _wl("dct_77_asym", xform="dct", levels=0, seq_len=77, k_hi=5, act_quant="asym", seed=46),
]


@pytest.mark.parametrize("w", OTHER, ids=[w.name for w in OTHER])
def test_wht_and_dct_along_the_tokens(w):
    tl.full_case(w, with_bias=True, check_unfused=False)


def test_bf16_output_on_the_general_path():
    tl.full_case(_wl("rag_500_bf16out", seq_len=500, levels=4, x_dtype="bf16", seed=47), with_bias=True, y_dtype="bf16",
                 check_unfused=False)


TBIAS = [
    _wl("tb_1d_512_J9", batch=2, seq_len=512, levels=9, bias_mode="transformed", seed=51),
    _wl("tb_1d_512_J4", seq_len=512, levels=4, k_hi=32, bias_mode="transformed", seed=52),
    _wl("tb_2d_32_J3", seq_len=1024, xform="haar2d", grid_h=32, grid_w=32, levels=3, bias_mode="transformed", seed=53),
    _wl("tb_2d_32_J5", seq_len=1024, xform="haar2d", grid_h=32, grid_w=32, levels=5, bias_mode="transformed",
        act_quant="asym", seed=54),
    _wl("tb_ident", xform="identity", levels=0, bias_mode="transformed", seed=55),
    _wl("tb_wht", xform="wht", levels=0, bias_mode="transformed", seed=56),
    _wl("tb_dct_100", xform="dct", levels=0, seq_len=100, bias_mode="transformed", seed=57),
    _wl("tb_skip_300_J4", seq_len=300, levels=4, skip_first=True, bias_mode="transformed", seed=58),
]


@pytest.mark.parametrize("w", TBIAS, ids=[w.name for w in TBIAS])
def test_transformed_bias_form(w):
    """Y = L^-1 (Q(LX) W + (L 1) bias^T): same output as adding the bias last, to the output bar."""
    rep = tl.full_case(w, with_bias=True, check_unfused=False)
    assert rep


def test_transformed_bias_without_a_bias_is_the_plain_layer():
    tl.full_case(_wl("tb_nobias", seq_len=512, levels=9, bias_mode="transformed", seed=59), with_bias=False,
                 check_unfused=False)


GROUPED = [
    _wl("g_1d_512_J9", batch=2, seq_len=512, levels=9, group_size=64, d_in=256, seed=61),
    _wl("g_1d_300_J3", seq_len=300, levels=3, group_size=64, d_in=192, d_out=130, x_dtype="bf16", seed=62),
    _wl("g_2d_32_J3", seq_len=1024, xform="haar2d", grid_h=32, grid_w=32, levels=3, k_hi=64, group_size=64, d_in=128,
        d_out=257, seed=63),
    _wl("g_ident", xform="identity", levels=0, group_size=64, d_in=64, seed=64),
    _wl("g_wht", xform="wht", levels=0, group_size=64, seed=65),
    _wl("g_skip", seq_len=257, levels=8, skip_first=True, first_token_scale=100.0, group_size=64, seed=66),
    _wl("g_k0", seq_len=128, levels=7, k_hi=0, group_size=64, seed=67),
    _wl("g_all8", seq_len=64, levels=6, k_hi=64, group_size=64, seed=68),
]


@pytest.mark.parametrize("w", GROUPED, ids=[w.name for w in GROUPED])
def test_per_block_scales(w):
    tl.grouped_case(w, with_bias=True)


def test_per_block_scales_bf16_output():
    tl.grouped_case(_wl("g_bf16", seq_len=512, levels=9, group_size=64, d_in=256, x_dtype="bf16", seed=69),
                    with_bias=True, y_dtype="bf16")


@pytest.mark.parametrize("case", ["ragged", "skip", "wht", "dct", "2d"])
def test_stamp_inverse_on_general_plans(case):
    """stamp_inverse alone on random STaMP-ordered input against the oracle's inverse."""
    import torch
    import paper_2510_26771_amd as st
    kw = dict(batch=2, d_in=64, d_out=96)
    w = {"ragged": _wl("inv_rag", seq_len=301, levels=5, **kw),
         "skip": _wl("inv_skip", seq_len=128, levels=7, skip_first=True, **kw),
         "wht": _wl("inv_wht", seq_len=128, xform="wht", levels=0, **kw),
         "dct": _wl("inv_dct", seq_len=90, xform="dct", levels=0, **kw),
         "2d": _wl("inv_2d", seq_len=256, xform="haar2d", grid_h=16, grid_w=16, levels=2, bias_mode="transformed", **kw)}[case]
    inp = make_inputs(w, with_bias=True)
    plan = st.StampPlan(tl.plan_desc_for(w, "f32"), torch.from_numpy(inp["W"]).cuda(), torch.from_numpy(inp["bias"]).cuda())
    rng = np.random.default_rng(5)
    for ncols in (96, 37):
        Yt = rng.standard_normal((w.batch, w.seq_len, ncols)).astype(np.float32)
        ref = np.stack([so.sequence_inverse(Yt[b], w.xform, w.levels, w.grid_h, w.grid_w, skip_first=w.skip_first)
                        for b in range(w.batch)])
        if ncols == w.d_out:
            ref = ref + inp["bias"][None, None, :]
        Y = torch.empty((w.batch, w.seq_len, ncols), dtype=torch.float32, device="cuda")
        one = -(-(w.batch * w.seq_len * ncols * 4) // 256) * 256
        ws = torch.empty(2 * one, dtype=torch.uint8, device="cuda")
        Ytd = torch.from_numpy(Yt).cuda()
        plan.inverse(Ytd, ncols, Y, ws)
        torch.cuda.synchronize()
        assert np.array_equal(Ytd.cpu().numpy(), Yt), "stamp_inverse wrote its input"
        err = np.max(np.abs(Y.cpu().numpy() - ref)) / np.max(np.abs(ref))
        assert err <= 1e-5, err
    plan.destroy()


@pytest.mark.timeout(600)
def test_full_size_llm_first_token_left_out():
    """The language-model set-up of the appendix "Experimental details": 2048 tokens, three levels, 64 8-bit tokens,
    the first token (the attention sink: scaled by 100 here) left out of the transform; sampled output columns."""
    from dataclasses import replace
    from gen.workloads import WORKLOADS
    w = replace(WORKLOADS["cfg2"], name="cfg2_skip_first_J3", levels=3, skip_first=True)
    rng = np.random.default_rng(77)
    cols = np.unique(np.concatenate([[0, 1, w.d_out - 1],
                                     np.arange(0, w.d_out, 128) + rng.integers(0, 128, size=(w.d_out + 127) // 128)]))
    cols = cols[cols < w.d_out]
    tl.full_case(w, with_bias=True, y_dtype="bf16", cols=cols, check_unfused=False, also_f32_out=True)
