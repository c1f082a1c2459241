"""Shared helpers of the GPU parity tests: run the oracle and the HIP library on the same seeded
inputs and compare them step by step.  The oracle is only ever called from here and from tests."""
from __future__ import annotations

import time
from typing import Tuple, Dict, Optional

import numpy as np

from gen import Workload, make_inputs
from oracle import stamp_oracle as so

from paper_2510_26771_amd.marshal import XFORM_CODE, plan_desc_for, to_device_x  # noqa: F401  (used by the tests through this module)


def log(msg: str):
    print(f"[stamp-test {time.strftime('%H:%M:%S')}] {msg}", flush=True)


def unpack_int4(q_lo: np.ndarray) -> np.ndarray:
    """[..., d/2] bytes -> [..., d] int8, low nibble = even channel, two's complement."""
    lo = (q_lo & 0xF).astype(np.int8)
    hi = (q_lo >> 4).astype(np.int8)
    lo = np.where(lo >= 8, lo - 16, lo).astype(np.int8)
    hi = np.where(hi >= 8, hi - 16, hi).astype(np.int8)
    out = np.empty(q_lo.shape[:-1] + (q_lo.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def _has_fast_blocks(d) -> bool:
    """Whether a Haar setting has the block structure the library's fast path serves (include/stamp.h)."""
    pow2 = lambda n: n >= 1 and n & (n - 1) == 0
    # more than 256 top rows: only without top levels (fewer 8-bit tokens than approximations)
    if d.xform == XFORM_CODE["haar1d"]:
        na = d.seq_len >> d.levels
        if d.k_hi >= na and not pow2(d.k_hi):
            return False
        n_top = max(d.k_hi, na)
        return (n_top <= 256 or d.k_hi < na) and d.seq_len // n_top in (8, 16, 32, 64, 128)
    side = d.grid_h >> d.levels
    if d.k_hi >= side * side and not (pow2(d.k_hi) and (d.k_hi.bit_length() - 1) % 2 == 0):
        return False
    n_top = max(d.k_hi, side * side)
    return (n_top <= 256 or d.k_hi < side * side) and d.seq_len // n_top in (16, 64)


def general_path(d) -> bool:
    """Plans the library serves with its general path (transform level by level, rows in STaMP order)."""
    pow2 = d.seq_len & (d.seq_len - 1) == 0
    if (d.xform in (XFORM_CODE["wht"], XFORM_CODE["dct"]) or bool(d.skip_first) or bool(d.bias_mode) or bool(d.group_size)
            or (d.xform == XFORM_CODE["haar1d"] and not pow2) or (d.xform == XFORM_CODE["haar2d"] and d.grid_h != d.grid_w)):
        return True
    return d.xform != XFORM_CODE["identity"] and not _has_fast_blocks(d)


def gpu_codes_in_stamp_order(plan, q_hi, q_lo, scales):
    """Device buffers (physical row order) -> numpy codes [B, s, d], scales [B, s] and (asymmetric plans) offsets
    [B, s] in STaMP order.  Asymmetric plans store code - 2^(b-1); the unsigned code is returned."""
    d = plan.desc
    row = plan.row_of_coeff().astype(np.int64)
    assert sorted(row.tolist()) == list(range(d.seq_len)), "row_of_coeff is not a permutation"
    k = plan.hi_rows()  # rows kept in q_hi: the 8-bit tokens and any further approximation coefficients
    assert k >= d.k_hi
    if d.xform == XFORM_CODE["identity"] or general_path(d):
        assert k == d.k_hi
        assert np.array_equal(row, np.arange(d.seq_len))  # rows are kept in STaMP order (no transform: token order)
    else:
        assert np.array_equal(row[:k], np.arange(k) * (d.seq_len // k))
    qh = q_hi.cpu().numpy()[:, :k]
    # q_lo is tiled [Mp/256][Kp/128][256 rows][64 bytes] (include/stamp.h): back to [batch, seq_len, d/2]
    mp = -(-(d.batch * d.seq_len) // 256) * 256
    kp = -(-d.d_in // 128) * 128
    ql = q_lo.cpu().numpy().reshape(mp // 256, kp // 128, 256, 64).transpose(0, 2, 1, 3).reshape(mp, kp // 2)
    ql = ql[:d.batch * d.seq_len, :d.d_in // 2].reshape(d.batch, d.seq_len, d.d_in // 2)
    sc = scales.cpu().numpy()
    codes = np.empty((d.batch, d.seq_len, d.d_in), dtype=np.int16)
    codes[:, :k] = qh
    codes[:, k:] = unpack_int4(ql[:, row[k:]])
    if k > d.k_hi and d.xform != XFORM_CODE["identity"] and not general_path(d):
        # 4-bit approximations (no top levels): the quantizer also leaves them packed at their physical row of q_lo
        assert np.array_equal(unpack_int4(ql[:, row[d.k_hi:k]]), qh[:, d.k_hi:]), "packed copy of the 4-bit approximations"
    if d.act_quant:
        assert sc.shape == (2, d.batch, d.seq_len)
        codes[:, :d.k_hi] += 128
        codes[:, d.k_hi:] += 8
        assert codes.min() >= 0
        return codes.astype(np.uint8), sc[0][:, row], sc[1][:, row]
    return codes.astype(np.int8), sc[:, row], None


def near_boundary_mask(T: np.ndarray, bits: np.ndarray, asym: bool) -> np.ndarray:
    """Elements whose fp32 value T * inv lies within 1 ulp of a rounding boundary (a half-integer)."""
    if asym:
        qm = np.where(bits == 8, np.float32(255), np.float32(15)).astype(np.float32)
        a = (np.max(T, axis=-1) - np.min(T, axis=-1)).astype(np.float32)
        a = np.where(a == 0, np.abs(np.max(T, axis=-1)), a).astype(np.float32)
    else:
        qm = np.where(bits == 8, np.float32(127), np.float32(7)).astype(np.float32)
        a = np.max(np.abs(T), axis=-1)
    inv = np.zeros_like(a)
    nz = a > 0
    inv[nz] = (np.broadcast_to(qm, a.shape)[nz] / a[nz]).astype(np.float32)
    p = (T * inv[..., None]).astype(np.float32)
    h = np.floor(p) + np.float32(0.5)
    return np.abs(p - h) <= np.spacing(np.abs(p).astype(np.float32))


def compare_codes(gpu_codes, gpu_scales, gpu_zeros, ora: Dict[str, np.ndarray]) -> Dict[str, int]:
    """Scales, offsets and codes must match the oracle bit for bit.  Both sides round the same fp32 products, so even
    the elements that sit within 1 ulp of a rounding boundary agree; if that ever fails, the message says how many
    of the mismatches are such elements (those the bar would tolerate) and how many are not."""
    assert gpu_scales.dtype == np.float32
    bad_scales = int(np.count_nonzero(gpu_scales.view(np.uint32) != ora["scales"].view(np.uint32)))
    assert bad_scales == 0, f"{bad_scales} scales differ from the oracle"
    asym = "zeros" in ora
    if asym:
        assert gpu_zeros is not None and np.array_equal(gpu_zeros, ora["zeros"]), "offsets differ from the oracle"
    assert gpu_codes.dtype == ora["codes"].dtype
    diff = gpu_codes.astype(np.int16) - ora["codes"].astype(np.int16)
    n_mis = int(np.count_nonzero(diff))
    if n_mis:
        near = near_boundary_mask(ora["T"], ora["bits"][None, :].repeat(gpu_codes.shape[0], 0), asym)
        outside = int(((diff != 0) & ~near).sum())
        raise AssertionError(f"{n_mis} codes differ from the oracle: {n_mis - outside} within 1 ulp of a rounding "
                             f"boundary, {outside} away from one; largest step {int(np.abs(diff).max())}")
    return {"code_mismatches": 0, "near_boundary_mismatches": 0}


def run_oracle(w: Workload, inp: dict, cols: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Oracle results; with `cols` the GEMM / inverse run on those output columns only."""
    qa = so.quantize_activation(inp["X_f32"], w.xform, w.levels, w.k_hi, w.bits_hi, w.bits_lo, w.grid_h, w.grid_w,
                                act_quant=w.act_quant, skip_first=w.skip_first)
    qw, sw = so.quantize_weight(inp["W"], w.bits_w)
    bias = inp["bias"]
    if cols is not None:
        qw_c, sw_c = qw[:, cols], sw[cols]
        bias_c = None if bias is None else bias[cols]
    else:
        qw_c, sw_c, bias_c = qw, sw, bias
    out = so.linear_from_codes(qa["codes"], qa["scales"], qw_c, sw_c, w.xform, w.levels, w.grid_h, w.grid_w, bias_c,
                               zeros=qa.get("zeros"), skip_first=w.skip_first, bias_mode=w.bias_mode)
    out.update(qa)
    out.update({"qw": qw, "sw": sw})
    return out


# fp32 evaluation-order slack of the dequantization + inverse transform, relative to max|Y_ref|: the two
# sides may order the at most r + J + 3 <= 20 roundings of an output differently (each <= 2^-24 of the column's
# largest coefficient); 64 * 2^-24 leaves a factor of three.  Observed: 1e-7 .. 3e-7.
FP32_ORDER_SLACK = 64.0 * 2.0 ** -24


def check_output(y_gpu: np.ndarray, y_ref: np.ndarray, y_is_bf16: bool, what: str, stats: Optional[dict] = None) -> float:
    """Output bar.  fp32 stores: max |y - ref| <= 1e-3 * max|ref| (the stated tolerance), plainly.
    bf16 stores: the library rounds its fp32 result g to bf16; |g - ref| <= delta = FP32_ORDER_SLACK * max|ref|
    and rounding is monotonic, so every stored value must lie between the oracle's rounding of ref - delta and
    of ref + delta (for all but the elements within delta of a rounding boundary that is the oracle's own bf16
    value; the others are its bf16 neighbour).  The number of stored values that differ from round_to_bf16(ref)
    is reported in stats["bf16_nonidentical"]."""
    assert np.isfinite(y_gpu).all(), f"{what}: non-finite output"
    ref64 = y_ref.astype(np.float64)
    scale = float(np.max(np.abs(ref64)))
    err = np.abs(y_gpu.astype(np.float64) - ref64)
    if not y_is_bf16:
        assert float(err.max()) <= 1e-3 * scale, f"{what}: max err {float(err.max()):.3e} vs scale {scale:.3e}"
    else:
        delta = FP32_ORDER_SLACK * scale
        lo = so.round_to_bf16((ref64 - delta).astype(np.float32))
        hi = so.round_to_bf16((ref64 + delta).astype(np.float32))
        y = y_gpu.astype(np.float32)
        bad = int(np.count_nonzero((y < lo) | (y > hi)))
        assert bad == 0, (f"{what}: {bad} bf16 outputs outside [bf16(ref - delta), bf16(ref + delta)], "
                          f"max err {float(err.max()):.3e} vs scale {scale:.3e}")
        nonid = int(np.count_nonzero(y != so.round_to_bf16(y_ref.astype(np.float32))))
        if stats is not None:
            stats["bf16_nonidentical"] = stats.get("bf16_nonidentical", 0) + nonid
            stats["bf16_compared"] = stats.get("bf16_compared", 0) + int(y.size)
    return float(err.max() / scale) if scale > 0 else 0.0


def y_to_numpy(Y, y_is_bf16: bool) -> np.ndarray:
    import torch
    if y_is_bf16:
        return Y.contiguous().view(torch.bfloat16).float().cpu().numpy()
    return Y.cpu().numpy()


def full_case(w: Workload, with_bias: bool = False, y_dtype: str = "f32", cols: Optional[np.ndarray] = None,
              check_acc: bool = True, check_unfused: bool = True,
              engines: Tuple[str, ...] = ("fp6", "int8"), also_f32_out: bool = False) -> Dict[str, float]:
    """Everything the ABI exposes, on one workload, against the oracle, under each GEMM engine.
    also_f32_out: a second plan with fp32 output runs the fused path on the same inputs and is held to the
    plain 1e-3 bar (for cases whose main plan stores bf16)."""
    import torch
    import paper_2510_26771_amd as st

    log(f"case {w.name}: B={w.batch} s={w.seq_len} d={w.d_in} N={w.d_out} {w.xform} k={w.k_hi} x={w.x_dtype} "
        f"y={y_dtype} bias={with_bias} seed={w.seed} act_quant={w.act_quant}")
    inp = make_inputs(w, with_bias=with_bias)
    ora = run_oracle(w, inp, cols)
    log("oracle done")
    Xd = to_device_x(inp, w)
    Wd = torch.from_numpy(inp["W"]).cuda()
    bd = None if inp["bias"] is None else torch.from_numpy(inp["bias"]).cuda()
    plan = st.StampPlan(plan_desc_for(w, y_dtype), Wd, bd)
    report: Dict[str, float] = {}

    # weights
    qw, sw = plan.debug_weight_codes()
    assert np.array_equal(qw, ora["qw"]), "weight codes differ"
    assert np.array_equal(sw.view(np.uint32), ora["sw"].view(np.uint32)), "weight scales differ"

    # activation codes and scales
    ws = plan.alloc_workspace()
    q_hi, q_lo, scales = plan.alloc_act_buffers()
    plan.quantize_act(Xd, q_hi, q_lo, scales, ws)
    torch.cuda.synchronize()
    codes, sc, zs = gpu_codes_in_stamp_order(plan, q_hi, q_lo, scales)
    report.update(compare_codes(codes, sc, zs, ora))
    log(f"codes ok: {report}")

    # integer accumulators
    sel = slice(None) if cols is None else cols
    cols_t = None if cols is None else torch.from_numpy(np.asarray(cols, dtype=np.int64)).cuda()

    def pick(t3):  # [B, s, N] device tensor -> the compared columns, on the host
        return (t3 if cols_t is None else t3.index_select(2, cols_t)).cpu()

    if check_acc:
        if w.act_quant == "asym":
            # the library multiplies the STORED codes, code - 2^(b-1)
            shift = np.where(np.arange(w.seq_len) < w.k_hi, 128, 8).astype(np.int16)
            stored = ora["codes"].astype(np.int16) - shift[None, :, None]
            ref_acc = np.stack([so.int_gemm(stored[b], ora["qw"][:, sel]) for b in range(w.batch)])
        else:
            ref_acc = ora["acc"]
        for engine in engines:
            plan.set_gemm_engine(engine)
            acc = torch.full((w.batch * w.seq_len, w.d_out), -(2 ** 31), dtype=torch.int32, device="cuda")
            plan.debug_gemm_acc(q_hi, q_lo, acc)
            torch.cuda.synchronize()
            acc_np = pick(acc.view(w.batch, w.seq_len, w.d_out)).numpy()
            assert np.array_equal(acc_np, ref_acc), f"integer sums differ (engine {engine})"
            del acc
        log("accumulators ok")

    # the whole layer, fused (default) and unfused
    y_bf16 = y_dtype == "bf16"
    ydt = torch.int16 if y_bf16 else torch.float32
    y_ref = ora["Y"]
    y_first = None
    for engine in engines:
        plan.set_gemm_engine(engine)
        for unfused in ([False, True] if check_unfused else [False]):
            plan.set_unfused(unfused)
            ws = plan.alloc_workspace()
            Y = torch.zeros((w.batch, w.seq_len, w.d_out), dtype=ydt, device="cuda")
            plan.linear_forward(Xd, Y, ws)
            torch.cuda.synchronize()
            y_np = y_to_numpy(pick(Y), y_bf16)
            tag = ("unfused" if unfused else "fused") + "_" + engine
            report[f"y_relerr_{tag}"] = check_output(y_np, y_ref, y_bf16, f"{w.name} {tag}", report)
            # and from the separately quantized activation
            Y2 = torch.zeros_like(Y)
            plan.linear_forward_q(q_hi, q_lo, scales, Y2, ws)
            torch.cuda.synchronize()
            if plan.hi_rows() > w.k_hi > 0 and engine == "fp6" and not unfused:
                # 4-bit approximations: stamp_linear_forward takes them through the 4-bit rows' GEMM, the entry point
                # for caller-packed codes through the 8-bit rows' one, whose split depth may round differently
                check_output(y_to_numpy(pick(Y2), y_bf16), y_ref, y_bf16, f"{w.name} {tag} forward_q", {})
                yf, yf2 = torch.from_numpy(y_to_numpy(Y, y_bf16)), torch.from_numpy(y_to_numpy(Y2, y_bf16))
                assert float((yf - yf2).abs().max()) <= (2.0 ** -7 if y_bf16 else 1e-5) * float(yf.abs().max())
            else:
                assert torch.equal(Y, Y2), "linear_forward and quantize_act + linear_forward_q disagree"
            if not unfused:
                # both engines compute the same integer sums, so the outputs agree bit for bit
                # (plans with 4-bit approximations: the FP6 engine takes them through its own GEMM, see above)
                if y_first is None:
                    y_first = Y
                elif plan.hi_rows() > w.k_hi > 0:
                    yf, yf1 = torch.from_numpy(y_to_numpy(Y, y_bf16)), torch.from_numpy(y_to_numpy(y_first, y_bf16))
                    assert float((yf - yf1).abs().max()) <= (2.0 ** -7 if y_bf16 else 1e-5) * float(yf.abs().max())
                else:
                    assert torch.equal(Y, y_first), f"engine {engine} and engine {engines[0]} disagree"
            del Y2, ws
    del y_first
    plan.destroy()
    if also_f32_out and y_bf16:
        plan32 = st.StampPlan(plan_desc_for(w, "f32"), Wd, bd)
        ws = plan32.alloc_workspace()
        for engine in engines:
            plan32.set_gemm_engine(engine)
            Y = torch.zeros((w.batch, w.seq_len, w.d_out), dtype=torch.float32, device="cuda")
            plan32.linear_forward(Xd, Y, ws)
            torch.cuda.synchronize()
            report[f"y_relerr_f32out_{engine}"] = check_output(pick(Y).numpy(), y_ref, False, f"{w.name} f32 out {engine}")
            del Y
        plan32.destroy()
    log(f"outputs ok: {report}")
    return report


def grouped_case(w: Workload, with_bias: bool = False, y_dtype: str = "f32") -> Dict[str, float]:
    """Per-block (group_size = 64) scales: weight codes and scales, activation codes and scales bit for bit, the
    layer's output to the output bar, and quantize_act + linear_forward_q against linear_forward."""
    import torch
    import paper_2510_26771_amd as st

    assert w.group_size == 64
    log(f"grouped case {w.name}: B={w.batch} s={w.seq_len} d={w.d_in} N={w.d_out} {w.xform} J={w.levels} k={w.k_hi} "
        f"x={w.x_dtype} y={y_dtype} bias={with_bias} seed={w.seed} skip_first={w.skip_first}")
    inp = make_inputs(w, with_bias=with_bias)
    ora = so.stamp_linear_forward_grouped(inp["X_f32"], inp["W"], w.xform, w.levels, w.k_hi, 64, w.bits_hi, w.bits_lo,
                                          w.bits_w, w.grid_h, w.grid_w, inp["bias"], skip_first=w.skip_first)
    log("oracle done")
    Xd = to_device_x(inp, w)
    Wd = torch.from_numpy(inp["W"]).cuda()
    bd = None if inp["bias"] is None else torch.from_numpy(inp["bias"]).cuda()
    plan = st.StampPlan(plan_desc_for(w, y_dtype), Wd, bd)
    qw, swg = plan.debug_weight_codes()
    assert np.array_equal(qw, ora["qw"]), "weight codes differ"
    assert np.array_equal(swg.view(np.uint32), ora["swg"].view(np.uint32)), "weight scales differ"
    assert plan.hi_rows() == w.seq_len
    assert np.array_equal(plan.row_of_coeff(), np.arange(w.seq_len))

    ws = plan.alloc_workspace()
    q_hi, q_lo, scales = plan.alloc_act_buffers()
    plan.quantize_act(Xd, q_hi, q_lo, scales, ws)
    torch.cuda.synchronize()
    sc = scales.cpu().numpy()
    assert np.array_equal(sc.view(np.uint32), ora["scales"].view(np.uint32)), "activation scales differ"
    codes = q_hi.cpu().numpy()
    n_mis = int(np.count_nonzero(codes != ora["codes"]))
    assert n_mis == 0, f"{n_mis} activation codes differ"

    y_bf16 = y_dtype == "bf16"
    Y = torch.zeros((w.batch, w.seq_len, w.d_out), dtype=torch.int16 if y_bf16 else torch.float32, device="cuda")
    plan.linear_forward(Xd, Y, ws)
    torch.cuda.synchronize()
    report: Dict[str, float] = {}
    report["y_relerr"] = check_output(y_to_numpy(Y, y_bf16), ora["Y"], y_bf16, w.name, report)
    Y2 = torch.zeros_like(Y)
    plan.linear_forward_q(q_hi, q_lo, scales, Y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2), "linear_forward and quantize_act + linear_forward_q disagree"
    plan.destroy()
    log(f"outputs ok: {report}")
    return report
