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


RECT = [
    _wl("rect_16x64_J3", batch=2, seq_len=1024, xform="haar2d", grid_h=16, grid_w=64, levels=3, k_hi=16, corr_len=4.0, seed=91),
    _wl("rect_64x16_J4_asym", seq_len=1024, xform="haar2d", grid_h=64, grid_w=16, levels=4, k_hi=4, corr_len=4.0,
        act_quant="asym", mean_shift=0.5, x_dtype="bf16", seed=92),
    _wl("rect_8x32_J1_tb", seq_len=256, xform="haar2d", grid_h=8, grid_w=32, levels=1, k_hi=64, corr_len=3.0,
        bias_mode="transformed", seed=93),
    _wl("rect_2x128_J1", seq_len=256, xform="haar2d", grid_h=2, grid_w=128, levels=1, k_hi=8, corr_len=3.0, seed=94),
]


@pytest.mark.parametrize("w", RECT, ids=[w.name for w in RECT])
def test_2d_haar_on_rectangular_grids(w):
    tl.full_case(w, with_bias=True, check_unfused=False)


def test_rectangular_grid_with_per_block_scales():
    tl.grouped_case(_wl("rect_g64", seq_len=512, xform="haar2d", grid_h=16, grid_w=32, levels=3, k_hi=8, corr_len=4.0,
                        group_size=64, seed=95), with_bias=True, y_dtype="bf16")


# Valid settings on power-of-two sequences and square grids that have no fast-path block structure: served by the
# general path (and identity plans with many 8-bit tokens, which stay on the per-token kernel).
NO_BLOCKS = [
    _wl("k12_of_256", batch=2, seq_len=256, levels=8, k_hi=12, seed=101),                       # k not a power of two
    _wl("blocks_of_2", seq_len=256, levels=8, k_hi=128, seed=102),
    _wl("blocks_of_512", seq_len=1024, levels=10, k_hi=2, x_dtype="bf16", seed=103),
    _wl("top_512", seq_len=4096, levels=3, k_hi=64, d_in=128, d_out=72, seed=104),               # 512 approximations
    _wl("k300_of_512_asym", seq_len=512, levels=3, k_hi=300, act_quant="asym", mean_shift=0.5, seed=105),
    _wl("k0_of_512", seq_len=512, levels=9, k_hi=0, seed=106),
    _wl("all_8bit", seq_len=64, levels=2, k_hi=64, seed=107),
    _wl("grid16_k8", seq_len=256, xform="haar2d", grid_h=16, grid_w=16, levels=4, k_hi=8, corr_len=4.0, seed=108),
    _wl("grid32_J1", batch=2, seq_len=1024, xform="haar2d", grid_h=32, grid_w=32, levels=1, k_hi=16, corr_len=4.0,
        seed=109),                                                                                # 2x2 token blocks
    _wl("grid2_J1", seq_len=4, xform="haar2d", grid_h=2, grid_w=2, levels=1, k_hi=1, corr_len=2.0, seed=110),
    _wl("ident_k300", seq_len=512, xform="identity", levels=0, k_hi=300, seed=111),
    _wl("ident_all_8bit", batch=2, seq_len=100, xform="identity", levels=0, k_hi=100, act_quant="asym", seed=112),
]


@pytest.mark.parametrize("w", NO_BLOCKS, ids=[w.name for w in NO_BLOCKS])
def test_settings_without_the_fast_paths_block_structure(w):
    tl.full_case(w, with_bias=True, check_unfused=w.xform == "identity")


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


def _random_general(seed: int) -> Workload:
    """A valid general-path plan: transform, length, depth, quantizer form and the three switches drawn at random."""
    rng = np.random.default_rng(7000 + seed)
    kind = str(rng.choice(["ragged", "skip", "wht", "dct", "haar_pow2", "haar2d", "identity"]))
    kw = dict(batch=int(rng.integers(1, 4)), d_in=int(rng.integers(1, 9)) * 64, d_out=int(rng.integers(1, 300)),
              seed=8000 + seed, x_dtype=str(rng.choice(["bf16", "f32"])), n_outlier_channels=int(rng.integers(0, 4)),
              outlier_scale=25.0, mean_shift=float(rng.choice([0.0, 0.7])))
    group = 64 if rng.random() < 0.35 else 0
    if not group:
        kw["act_quant"] = str(rng.choice(["sym", "asym"]))
    tbias = "transformed" if rng.random() < 0.4 else "after"
    if kind == "ragged":
        s = int(rng.integers(3, 700))
        if s & (s - 1) == 0:
            s += 1
        w = dict(xform="haar1d", seq_len=s, levels=int(rng.integers(0, so.max_ragged_levels(s) + 1)))
    elif kind == "skip":
        s = int(rng.integers(3, 700))
        w = dict(xform="haar1d", seq_len=s, levels=int(rng.integers(0, so.max_ragged_levels(s - 1) + 1)), skip_first=True,
                 first_token_scale=60.0)
    elif kind == "wht":
        w = dict(xform="wht", seq_len=1 << int(rng.integers(1, 11)), levels=0)
    elif kind == "dct":
        w = dict(xform="dct", seq_len=int(rng.integers(2, 300)), levels=0)
    elif kind == "haar_pow2":   # a plan the fast path would take, sent to the general path by a switch
        J = int(rng.integers(3, 10))
        w = dict(xform="haar1d", seq_len=1 << J, levels=int(rng.integers(1, J + 1)))
        if not group:
            tbias = "transformed"
    elif kind == "haar2d":
        lg = int(rng.integers(2, 6))
        w = dict(xform="haar2d", seq_len=1 << (2 * lg), grid_h=1 << lg, grid_w=1 << lg, levels=int(rng.integers(1, lg + 1)),
                 corr_len=4.0)
        if not group:
            tbias = "transformed"
    else:
        w = dict(xform="identity", seq_len=int(rng.integers(1, 300)), levels=0)
        if not group:
            tbias = "transformed"
    s = w["seq_len"]
    k_hi = int(rng.integers(0, min(s, 64) + 1))
    return _wl(f"rndg{seed}_{kind}", k_hi=k_hi, group_size=group, bias_mode=tbias, **w, **kw)


@pytest.mark.parametrize("seed", range(40))
def test_random_general_plans(seed):
    """Seeded sweep over the general path: every plan it accepts meets the same bars as the fast path's."""
    w = _random_general(seed)
    rng = np.random.default_rng(9000 + seed)
    y_dtype = str(rng.choice(["f32", "bf16"]))
    if w.group_size:
        tl.grouped_case(w, with_bias=True, y_dtype=y_dtype)
    else:
        r = tl.full_case(w, with_bias=True, y_dtype=y_dtype, check_unfused=False)
        assert r["code_mismatches"] == 0


@pytest.mark.parametrize("seed", range(24))
def test_random_haar_plans_of_any_block_structure(seed):
    """Seeded sweep over plain Haar settings (power-of-two sequences, square or rectangular grids) with any depth and
    any number of 8-bit tokens: whichever path serves the plan, the result meets the same bars."""
    rng = np.random.default_rng(7600 + seed)
    kw = dict(batch=int(rng.integers(1, 3)), d_in=int(rng.integers(1, 7)) * 32, d_out=int(rng.integers(1, 260)),
              seed=8600 + seed, x_dtype=str(rng.choice(["bf16", "f32"])), act_quant=str(rng.choice(["sym", "asym"])),
              mean_shift=float(rng.choice([0.0, 0.7])))
    if rng.random() < 0.5:
        J = int(rng.integers(1, 12))
        kw.update(xform="haar1d", seq_len=1 << J, levels=int(rng.integers(1, J + 1)))
    else:
        lh, lw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        kw.update(xform="haar2d", seq_len=1 << (lh + lw), grid_h=1 << lh, grid_w=1 << lw,
                  levels=int(rng.integers(1, min(lh, lw) + 1)), corr_len=4.0)
    s = kw["seq_len"]
    k_hi = int(rng.integers(0, s + 1)) if rng.random() < 0.5 else int(rng.integers(0, min(s, 48) + 1))
    w = _wl(f"rndb{seed}", k_hi=k_hi, **kw)
    y_dtype = str(rng.choice(["f32", "bf16"]))
    general = tl.general_path(tl.plan_desc_for(w, y_dtype))
    tl.log(f"{w.name}: {w.xform} s={s} grid={w.grid_h}x{w.grid_w} J={w.levels} k={k_hi} general={general}")
    r = tl.full_case(w, with_bias=True, y_dtype=y_dtype, check_unfused=not general)
    assert r["code_mismatches"] == 0


def test_general_path_under_hip_graph_capture_and_static_scratch():
    """The general path only enqueues kernels (no allocation, copy or memset): it can be captured into a HIP graph,
    every replay reproduces the eager result bit for bit, and stamp_linear_forward_static runs it from the
    library's static scratch array."""
    import torch
    import paper_2510_26771_amd as st
    for w in (_wl("graph_skip", batch=2, seq_len=300, levels=4, skip_first=True, d_in=160, d_out=300, seed=81),
              _wl("graph_g64_2d", seq_len=256, xform="haar2d", levels=3, grid_h=16, grid_w=16, k_hi=4, d_in=128,
                  d_out=130, group_size=64, seed=82),
              _wl("graph_wht_tb", seq_len=128, xform="wht", levels=0, bias_mode="transformed", act_quant="asym", seed=83)):
        inp = make_inputs(w, with_bias=True)
        plan = st.StampPlan(tl.plan_desc_for(w, "bf16"), torch.from_numpy(inp["W"]).cuda(),
                            torch.from_numpy(inp["bias"]).cuda())
        X = tl.to_device_x(inp, w)
        ws = plan.alloc_workspace()
        Y_eager = torch.zeros((w.batch, w.seq_len, w.d_out), dtype=torch.int16, device="cuda")
        plan.linear_forward(X, Y_eager, ws)
        torch.cuda.synchronize()
        Y = torch.zeros_like(Y_eager)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            plan.linear_forward(X, Y, ws)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                plan.linear_forward(X, Y, ws)
        torch.cuda.current_stream().wait_stream(side)
        for it in range(3):
            Y.fill_(-1)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(Y, Y_eager), f"{w.name}: replay {it} differs from the eager result"
        Y.fill_(-1)
        plan.linear_forward_static(X, Y)
        torch.cuda.synchronize()
        assert torch.equal(Y, Y_eager), f"{w.name}: static scratch and caller workspace disagree"
        plan.destroy()
