"""Benchmark: one "step" = one pass over every operator class of the hot path at full workload size.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints ONE JSON line.  `value` is the whole-step throughput: algorithmic HBM bytes of all operators in the
step divided by the wall-clock time of the step (inputs already resident in HBM).  `per_op` gives each
operator's own time (HIP events inside the timed region), GB/s, fraction of the 8 TB/s peak and elements/s.
`roofline` describes the operator that takes the largest share of the step.  `cpu_baseline` is the CPU oracle
timed on a bounded sample of the same step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_GBPS = 8000.0
MiB = 1 << 20
# HBM bytes per launch from the hardware counters (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE; the text summary under
# profiles/ has the commands and the copy calibration: bytes = 2.0 x FETCH_SIZE KiB + 1.0 x WRITE_SIZE KiB).  An entry
# is valid only for the kernel version it was measured on: remove it when that kernel changes.
PMC_TRAFFIC_BYTES = {"index_select_f32": (2 * 2122803 + 4194442) * 1024,
                     "gather_f32": (2 * 277623 + 16384) * 1024}


def build_ops(torch, B):
    """Returns a list of dicts: name, kernel, row (scope-table step), bytes, elems, fn."""
    dev = "cuda"
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    F32, BF16, I64, I32 = torch.float32, torch.bfloat16, torch.int64, torch.int32

    def randn(shape, dtype=F32, std=1.0):
        x = torch.randn(shape, device=dev, dtype=F32, generator=g)
        if std != 1.0:
            x.mul_(std)
        return x.to(dtype)

    def randint(shape, lo, hi, dtype=I64):
        return torch.randint(lo, hi + 1, shape, device=dev, dtype=I64, generator=g).to(dtype)

    ops = []

    def add(name, row, kernel, nbytes, elems, fn, extra=False):
        ops.append(dict(name=name, row=row, kernel=kernel, bytes=int(nbytes), elems=int(elems), fn=fn, extra=extra))

    def extra(name, row, kernel, nbytes, elems, fn):
        """An alternative kernel for a workload the step already covers: timed after the step, not part of `value`."""
        add(name, row, kernel, nbytes, elems, fn, extra=True)

    # ---- workload 1: broadcast add, rotating outputs so the 64 MiB result is not an Infinity-Cache hit
    a1, b1 = randn((4096, 1)), randn((1, 4096))
    outs1 = [torch.empty((4096, 4096), device=dev) for _ in range(9)]
    state = {"i": 0}

    REP1 = 9     # an 11 us kernel between two events mostly measures the events: launch it 9 times back to back

    # descriptors built once, as a C caller would hold them: per call the binding then only crosses into the library
    d_a1, d_b1, d_outs1 = B.desc(a1), B.desc(b1), [B.desc(o) for o in outs1]

    def f_bcast():
        for _ in range(REP1):
            state["i"] = (state["i"] + 1) % len(outs1)
            B.tx_add(d_outs1[state["i"]], d_a1, d_b1, 1)
    # The same 9 launches replayed from a HIP graph are timed outside the step (a 9-node graph replays no faster than
    # 9 calls through the binding: 12.7 against 11.6 us per launch; a 36-node graph reaches 11.3 us).
    f_bcast()
    torch.cuda.synchronize()
    graph1 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph1):
        f_bcast()
    nb1 = REP1 * (4096 * 4096 * 4 + 2 * 4096 * 4)
    add("add_bcast_f32[4096,1]+[1,4096] x9", "a3", "ew_bcast_kernel", nb1, REP1 * 4096 * 4096, f_bcast)
    extra("add_bcast_f32[4096,1]+[1,4096] x9 (graph replay)", "a3", "ew_bcast_kernel", nb1, REP1 * 4096 * 4096, graph1.replay)

    # ---- workload 2: elementwise sweep at [8192,8192]
    N = 8192
    n2 = N * N
    xf, yf, of = randn((N, N), std=3.0), randn((N, N), std=3.0), torch.empty((N, N), device=dev)
    xb, ob = xf.to(BF16), torch.empty((N, N), device=dev, dtype=BF16)
    xi, yi, oi = randint((N, N), -1000, 1000), randint((N, N), -1000, 1000), torch.empty((N, N), device=dev, dtype=I64)
    obool = torch.empty((N, N), device=dev, dtype=torch.bool)
    cond = torch.rand((N, N), device=dev, generator=g) < 0.5
    add("exp_f32", "a3", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("exp", of, xf))
    add("add_f32", "a3", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_add(of, xf, yf, 1))
    add("gelu_bf16", "a3", "ew_vec_kernel", n2 * 4, n2, lambda: B.tx_unary("gelu", ob, xb))
    add("gelu_f32", "a3", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("gelu", of, xf))
    add("sigmoid_f32", "a3", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("sigmoid", of, xf))
    add("tanh_f32", "a3", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("tanh", of, xf))
    add("add_i64", "a3", "ew_vec_kernel", n2 * 24, n2, lambda: B.tx_add(oi, xi, yi, 1))
    add("eq_f32", "a3", "ew_vec_kernel", n2 * 9, n2, lambda: B.tx_binary("eq", obool, xf, yf))
    add("where_f32", "a3", "ew_vec_kernel", n2 * 13, n2, lambda: B.tx_where(of, cond, xf, yf))
    add("add_bf16+f32_mixed", "a4", "ew_vec_kernel", n2 * 10, n2, lambda: B.tx_add(of, xb, yf, 1))
    wide = randn((N, 2 * N), std=3.0)
    tall = randn((2 * N, N), std=3.0)
    add("add_f32_step2_inner", "a4", "ew_generic_kernel", n2 * 12, n2, lambda: B.tx_add(of, wide[:, ::2], yf, 1))
    add("add_f32_step2_outer", "a4", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_add(of, tall[::2], yf, 1))
    col = randn((N, 1), std=3.0)
    add("add_f32_expand_row", "a4", "ew_vec_kernel", n2 * 8 + N * 4, n2, lambda: B.tx_add(of, col.expand(N, N), yf, 1))
    add("add_f32_transposed", "a5", "ew_tile_kernel", n2 * 12, n2, lambda: B.tx_add(of, xf.t(), yf, 1))
    add("mul_bf16_transposed", "a5", "ew_tile_kernel", n2 * 6, n2, lambda: B.tx_binary("mul", ob, xb.t(), xb))

    def forced(path, fn):                 # the same call with a dispatch path forced (alternatives, for A/B measurements)
        def run():
            B.tx_force_path(path)
            try:
                fn()
            finally:
                B.tx_force_path(None)
        return run

    # alternatives of kernels in the step, timed outside it: what each design choice is measured against
    extra("add_f32_transposed_via_generic_path", "a5", "ew_generic_kernel", n2 * 12, n2,
          forced("generic", lambda: B.tx_add(of, xf.t(), yf, 1)))
    extra("add_f32_plain_cached_loads", "a3", "ew_vec_kernel", n2 * 12, n2, forced("vec-cached", lambda: B.tx_add(of, xf, yf, 1)))
    extra("add_bcast_f32_vec_kernel_one_vector_per_lane x9", "a3", "ew_vec_kernel", nb1, REP1 * 4096 * 4096, forced("vec-narrow", f_bcast))
    extra("add_bcast_f32_vec_kernel_four_vectors_per_lane x9", "a3", "ew_vec_kernel", nb1, REP1 * 4096 * 4096, forced("vec-wide", f_bcast))
    # data-moving shape operators, timed outside the step
    extra("copy_f32_contiguous", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_copy(of, xf))
    extra("copy_f32_to_bf16", "f1", "ew_vec_kernel", n2 * 6, n2, lambda: B.tx_copy(ob, xf))
    extra("copy_f32_transposed", "f1", "ew_tile_kernel", n2 * 8, n2, lambda: B.tx_copy(of, xf.t()))
    extra("flip_f32_dim0", "f1", "remap_copy_kernel", n2 * 8, n2, lambda: B.tx_flip(of, xf, [0]))
    extra("flip_f32_dim1", "f1", "remap_copy_kernel", n2 * 8, n2, lambda: B.tx_flip(of, xf, [1]))
    extra("roll_f32_dim0", "f1", "remap_copy_kernel", n2 * 8, n2, lambda: B.tx_roll(of, xf, [1234], [0]))
    extra("tril_f32", "f1", "remap_copy_kernel", n2 * 8, n2, lambda: B.tx_tri(of, xf, 0, False))
    # second batch of elementwise operators (same iterator paths), timed outside the step
    extra("sub_f32", "f1", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_sub(of, xf, yf, 1))
    extra("minimum_f32", "f1", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_binary("minimum", of, xf, yf))
    extra("lt_f32", "f1", "ew_vec_kernel", n2 * 9, n2, lambda: B.tx_binary("lt", obool, xf, yf))
    extra("log1p_f32", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("log1p", of, xf))
    extra("expm1_f32", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("expm1", of, xf))
    extra("logsigmoid_f32", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_unary("logsigmoid", of, xf))
    extra("logsigmoid_bf16", "f1", "ew_vec_kernel", n2 * 4, n2, lambda: B.tx_unary("logsigmoid", ob, xb))
    for third in ("sin", "exp2", "rsqrt", "silu", "round"):
        extra(third + "_f32", "f1", "ew_vec_kernel", n2 * 8, n2, (lambda o: (lambda: B.tx_unary(o, of, xf)))(third))
    extra("isfinite_f32", "f1", "ew_vec_kernel", n2 * 5, n2, lambda: B.tx_unary("isfinite", obool, xf))
    extra("atan2_f32", "f1", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_binary("atan2", of, xf, yf))
    extra("pow_f32", "f1", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_binary("pow", of, xf, yf))
    for fourth in ("relu", "hardswish", "erf", "tan", "mish"):
        extra(fourth + "_f32", "f1", "ew_vec_kernel", n2 * 8, n2, (lambda o: (lambda: B.tx_unary(o, of, xf)))(fourth))
    extra("relu_bf16", "f1", "ew_vec_kernel", n2 * 4, n2, lambda: B.tx_unary("relu", ob, xb))
    for name, params in (("leaky_relu", (0.01,)), ("elu", (1.0,)), ("softplus", (1.0, 20.0)), ("hardshrink", (0.5,))):
        extra(name + "_f32", "f1", "ew_vec_kernel", n2 * 8, n2, (lambda o, p: (lambda: B.tx_unary_param(o, of, xf, *p)))(name, params))
    extra("elu_bf16", "f1", "ew_vec_kernel", n2 * 4, n2, lambda: B.tx_unary_param("elu", ob, xb, 1.0))
    extra("addcmul_f32", "f1", "ew_vec_kernel", n2 * 16, n2, lambda: B.tx_ternary("addcmul", of, xf, yf, tall[:N], 0.5))
    extra("lerp_f32_scalar_weight", "f1", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_ternary("lerp", of, xf, yf, None, 0.3))
    for fourth in ("fmax", "remainder", "floor_divide", "hypot", "logaddexp"):
        extra(fourth + "_f32", "f1", "ew_vec_kernel", n2 * 12, n2, (lambda o: (lambda: B.tx_binary(o, of, xf, yf)))(fourth))
    extra("clamp_f32", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_clamp(of, xf, -0.5, 0.75))
    extra("clamp_bf16", "f1", "ew_vec_kernel", n2 * 4, n2, lambda: B.tx_clamp(ob, xb, -0.5, 0.75))
    extra("logical_and_f32", "f1", "ew_vec_kernel", n2 * 9, n2, lambda: B.tx_binary("logical_and", obool, xf, yf))
    extra("logical_not_f32", "f1", "ew_vec_kernel", n2 * 5, n2, lambda: B.tx_unary("logical_not", obool, xf))
    extra("add_bf16_out_f32_cast", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_add(of, xb, xb, 1))
    extra("add_bf16_f32_in_place", "f1", "ew_vec_kernel", n2 * 8, n2, lambda: B.tx_add(ob, ob, xf, 1))

    # ---- workload 3: reductions over x[64,4096,1024]
    R = (64, 4096, 1024)
    nr = 64 * 4096 * 1024
    rf = randn(R)
    rb = rf.to(BF16)
    ri = randint(R, -(2 ** 20), 2 ** 20)

    def reducer(op, x, dims, out_shape, out_dtype, param=1.0):
        out = torch.empty(out_shape, device=dev, dtype=out_dtype)
        nb = B.tx_reduce_workspace_bytes(op, out, x, dims)
        ws = B.workspace(nb) if nb else None
        return lambda: B.tx_reduce(op, out, x, dims, False, param, ws)

    add("sum_f32_dim-1", "a6", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("sum", rf, -1, (64, 4096), F32))
    add("argmax_f32_dim-1", "a6", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 8, nr, reducer("argmax", rf, -1, (64, 4096), I64))
    add("var_f32_dim-1", "a6", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("var", rf, -1, (64, 4096), F32))
    add("sum_bf16_dim-1", "a6", "reduce_rows_kernel", nr * 2 + 64 * 4096 * 2, nr, reducer("sum", rb, -1, (64, 4096), BF16))
    add("sum_f32_dim0", "a7", "reduce_cols_kernel", nr * 4 + 4096 * 1024 * 4, nr, reducer("sum", rf, 0, (4096, 1024), F32))
    add("amax_bf16_dim0", "a7", "reduce_cols_kernel", nr * 2 + 4096 * 1024 * 2, nr, reducer("amax", rb, 0, (4096, 1024), BF16))
    add("sum_f32_dims(0,2)", "a8", "reduce_rows_kernel", nr * 4 + 4096 * 4, nr, reducer("sum", rf, (0, 2), (4096,), F32))
    add("sum_f32_all", "a9", "reduce_rows_kernel", nr * 4 + 4, nr, reducer("sum", rf, None, (), F32))
    add("sum_i64_all", "a9", "reduce_rows_kernel", nr * 8 + 8, nr, reducer("sum", ri, None, (), I64))
    add("prod_f32_all", "a9", "reduce_rows_kernel", nr * 4 + 4, nr, reducer("prod", rf, None, (), F32))
    # second batch of reductions, timed outside the step
    extra("amin_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("amin", rf, -1, (64, 4096), F32))
    extra("argmin_f32_dim0", "f1", "reduce_cols_kernel", nr * 4 + 4096 * 1024 * 8, nr, reducer("argmin", rf, 0, (4096, 1024), I64))
    extra("std_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("std", rf, -1, (64, 4096), F32))
    extra("logsumexp_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr,
          reducer("logsumexp", rf, -1, (64, 4096), F32))
    extra("logsumexp_bf16_dim0", "f1", "reduce_cols_kernel", nr * 2 + 4096 * 1024 * 2, nr,
          reducer("logsumexp", rb, 0, (4096, 1024), BF16))
    extra("all_i64_all_dims", "f1", "reduce_rows_kernel", nr * 8 + 1, nr, reducer("all", ri, None, (), torch.bool))
    extra("any_f32_dims(0,2)", "f1", "reduce_rows_kernel", nr * 4 + 4096, nr, reducer("any", rf, (0, 2), (4096,), torch.bool))
    extra("nanmean_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("nanmean", rf, -1, (64, 4096), F32))
    extra("nansum_bf16_dim0", "f1", "reduce_cols_kernel", nr * 2 + 4096 * 1024 * 2, nr, reducer("nansum", rb, 0, (4096, 1024), BF16))
    extra("count_nonzero_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 8, nr,
          reducer("count_nonzero", rf, -1, (64, 4096), I64))
    extra("norm2_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("norm", rf, -1, (64, 4096), F32, 2.0))
    extra("norm2_f32_dim0", "f1", "reduce_cols_kernel", nr * 4 + 4096 * 1024 * 4, nr, reducer("norm", rf, 0, (4096, 1024), F32, 2.0))
    extra("norm_inf_bf16_all", "f1", "reduce_rows_kernel", nr * 2 + 2, nr, reducer("norm", rb, None, (), BF16, float("inf")))
    extra("norm3_f32_dim-1", "f1", "reduce_rows_kernel", nr * 4 + 64 * 4096 * 4, nr, reducer("norm", rf, -1, (64, 4096), F32, 3.0))

    # ---- workload 4: softmax [32768,4096], cumsum [4096,65536]
    S = (32768, 4096)
    ns = S[0] * S[1]
    sf = randn(S, std=4.0)
    sf[torch.rand(S, device=dev, generator=g) < 0.001] = float("-inf")
    sb = sf.to(BF16)
    osf, osb = torch.empty(S, device=dev), torch.empty(S, device=dev, dtype=BF16)
    add("softmax_f32", "a10", "softmax_wave_kernel", ns * 8, ns, lambda: B.tx_softmax(osf, sf, -1, False))
    add("log_softmax_bf16", "a10", "softmax_wave_kernel", ns * 4, ns, lambda: B.tx_softmax(osb, sb, -1, True))
    extra("softmax_f32_wave_per_row", "a10", "softmax_wave_kernel", ns * 8, ns,
          forced("softmax-wave", lambda: B.tx_softmax(osf, sf, -1, False)))
    extra("log_softmax_bf16_wave_per_row", "a10", "softmax_wave_kernel", ns * 4, ns,
          forced("softmax-wave", lambda: B.tx_softmax(osb, sb, -1, True)))
    # fused row-normalisation and loss operators (Appendix B.3, B.1), timed outside the step; the softmax
    # tensors double as inputs (layer_norm) and the sweep tensors as probabilities (binary_cross_entropy)
    lw, lb = randn((S[1],)), randn((S[1],))
    lwb, lbb = lw.to(BF16), lb.to(BF16)
    lx = randn(S, std=2.0)
    lxb = lx.to(BF16)
    extra("layer_norm_f32[32768,4096]", "f2", "layer_norm_row_kernel", ns * 8, ns, lambda: B.tx_layer_norm(osf, lx, 1, lw, lb))
    extra("layer_norm_bf16[32768,4096]", "f2", "layer_norm_row_kernel", ns * 4, ns,
          lambda: B.tx_layer_norm(osb, lxb, 1, lwb, lbb))
    extra("layer_norm_f32[32768,4096]_workgroup_per_row", "f2", "layer_norm_rows_kernel", ns * 8, ns,
          forced("layer-norm-block", lambda: B.tx_layer_norm(osf, lx, 1, lw, lb)))
    extra("layer_norm_bf16[32768,4096]_workgroup_per_row", "f2", "layer_norm_rows_kernel", ns * 4, ns,
          forced("layer-norm-block", lambda: B.tx_layer_norm(osb, lxb, 1, lwb, lbb)))
    extra("layer_norm_f32[32768,4096]_wave_per_row", "f2", "layer_norm_rows_kernel", ns * 8, ns,
          forced("layer-norm-wave", lambda: B.tx_layer_norm(osf, lx, 1, lw, lb)))
    extra("layer_norm_bf16[32768,4096]_wave_per_row", "f2", "layer_norm_rows_kernel", ns * 4, ns,
          forced("layer-norm-wave", lambda: B.tx_layer_norm(osb, lxb, 1, lwb, lbb)))
    l2 = lx.view(131072, 1024)
    o2 = osf.view(131072, 1024)
    extra("layer_norm_f32[131072,1024]", "f2", "layer_norm_rows_kernel", ns * 8, ns,
          lambda: B.tx_layer_norm(o2, l2, 1, lw[:1024], lb[:1024]))
    l3 = lx.view(8192, 16384)
    o3 = osf.view(8192, 16384)
    extra("layer_norm_f32[8192,16384]_long_rows", "f2", "layer_norm_generic_kernel", ns * 8, ns,
          lambda: B.tx_layer_norm(o3, l3, 1))
    px, pt = torch.sigmoid(xf), torch.rand((N, N), device=dev, generator=g)
    pxb, ptb = px.to(BF16), pt.to(BF16)
    pw = torch.rand((N,), device=dev, generator=g)
    oscalar, oscalar_b = torch.empty((), device=dev), torch.empty((), device=dev, dtype=BF16)
    wsb = B.workspace(B.tx_binary_cross_entropy_workspace_bytes(oscalar, px, pt, pw, "mean"))
    extra("bce_mean_f32", "f2", "bce_partial_kernel", n2 * 8, n2,
          lambda: B.tx_binary_cross_entropy(oscalar, px, pt, None, "mean", wsb))
    extra("bce_mean_f32_class_weight", "f2", "bce_partial_kernel", n2 * 8, n2,
          lambda: B.tx_binary_cross_entropy(oscalar, px, pt, pw, "mean", wsb))
    extra("bce_sum_bf16", "f2", "bce_partial_kernel", n2 * 4, n2,
          lambda: B.tx_binary_cross_entropy(oscalar_b, pxb, ptb, None, "sum", wsb))
    extra("bce_none_f32", "f2", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_binary_cross_entropy(of, px, pt, None, "none"))
    wsl = B.workspace(B.tx_loss_workspace_bytes("mse", oscalar, xf, yf, "mean", 1.0))
    extra("mse_loss_mean_f32", "f2", "bce_partial_kernel", n2 * 8, n2, lambda: B.tx_loss("mse", oscalar, xf, yf, "mean", 1.0, wsl))
    extra("huber_loss_mean_f32", "f2", "bce_partial_kernel", n2 * 8, n2, lambda: B.tx_loss("huber", oscalar, xf, yf, "mean", 1.0, wsl))
    extra("smooth_l1_loss_sum_bf16", "f2", "bce_partial_kernel", n2 * 4, n2,
          lambda: B.tx_loss("smooth_l1", oscalar_b, pxb, ptb, "sum", 0.5, wsl))
    extra("l1_loss_none_f32", "f2", "ew_vec_kernel", n2 * 12, n2, lambda: B.tx_loss("l1", of, xf, yf, "none"))

    # softmax / cumsum along a dim that is not the innermost one (column kernels), timed outside the step
    sT, oT = sf.view(4096, 32768), osf.view(4096, 32768)
    extra("softmax_f32_dim0[4096,32768]", "f3", "softmax_cols_kernel", ns * 8, ns, lambda: B.tx_softmax(oT, sT, 0, False))
    s3, o3d = sf.view(64, 4096, 512), osf.view(64, 4096, 512)
    extra("log_softmax_f32_dim1[64,4096,512]", "f3", "softmax_cols_kernel", ns * 8, ns, lambda: B.tx_softmax(o3d, s3, 1, True))
    sC, oC = sf.view(512, 128, 2048), osf.view(512, 128, 2048)       # softmax over 128 channels
    extra("softmax_f32_dim1[512,128,2048]", "f3", "softmax_cols_reg_kernel", ns * 8, ns, lambda: B.tx_softmax(oC, sC, 1, False))
    extra("softmax_f32_dim1[512,128,2048]_two_reads", "f3", "softmax_cols_kernel", ns * 8, ns,
          forced("softmax-cols", lambda: B.tx_softmax(oC, sC, 1, False)))
    wsc = B.workspace(max(B.tx_cumsum_workspace_bytes(oT, lx.view(4096, 32768), 0),
                          B.tx_cumsum_workspace_bytes(osf.view(65536, 2048), lx.view(65536, 2048), 0)))
    extra("cumsum_f32_dim0[4096,32768]", "f3", "colscan_lookback_kernel", ns * 8, ns,
          lambda: B.tx_cumsum(oT, lx.view(4096, 32768), 0, wsc))
    extra("cumsum_f32_dim0[65536,2048]", "f3", "colscan_lookback_kernel", ns * 8, ns,
          lambda: B.tx_cumsum(osf.view(65536, 2048), lx.view(65536, 2048), 0, wsc))
    extra("cumsum_f32_dim0[4096,32768]_three_passes", "f3", "colscan_apply_kernel", ns * 8, ns,
          forced("scan-cols-3pass", lambda: B.tx_cumsum(oT, lx.view(4096, 32768), 0, wsc)))
    extra("cumsum_f32_dim0[65536,2048]_three_passes", "f3", "colscan_apply_kernel", ns * 8, ns,
          forced("scan-cols-3pass", lambda: B.tx_cumsum(osf.view(65536, 2048), lx.view(65536, 2048), 0, wsc)))

    C = (4096, 65536)
    nc = C[0] * C[1]
    cf, ci = randn(C), randint(C, -100, 100)
    ocf, oci = torch.empty(C, device=dev), torch.empty(C, device=dev, dtype=I64)
    wsf = B.workspace(B.tx_cumsum_workspace_bytes(ocf, cf, -1))
    wsi = B.workspace(B.tx_cumsum_workspace_bytes(oci, ci, -1))
    add("cumsum_f32", "a11", "cumsum_lookback_kernel", nc * 8, nc, lambda: B.tx_cumsum(ocf, cf, -1, wsf))
    add("cumsum_i64", "a11", "cumsum_lookback_kernel", nc * 16, nc, lambda: B.tx_cumsum(oci, ci, -1, wsi))

    def carry_f32():         # the same scan forced through the one-workgroup-per-row kernel (register carry)
        B.tx_force_path("scan-carry")
        try:
            B.tx_cumsum(ocf, cf, -1, wsf)
        finally:
            B.tx_force_path(None)
    extra("cumsum_f32_row_carry", "a11", "cumsum_carry_kernel", nc * 8, nc, carry_f32)
    extra("cumsum_f32_look_back_16KiB_tiles", "a11", "cumsum_lookback_kernel", nc * 8, nc,
          forced("scan-lookback-narrow", lambda: B.tx_cumsum(ocf, cf, -1, wsf)))
    wsp = B.workspace(B.tx_scan_workspace_bytes("cumprod", ocf, cf, -1))
    extra("cumprod_f32", "f3", "cumsum_lookback_kernel", nc * 8, nc, lambda: B.tx_scan("cumprod", ocf, cf, -1, wsp))
    extra("logcumsumexp_f32", "f3", "cumsum_lookback_kernel", nc * 8, nc, lambda: B.tx_scan("logcumsumexp", ocf, cf, -1, wsp))
    # few long rows: every row has to be spread over the whole chip
    cl = randn((8, 1 << 24))
    ocl = torch.empty_like(cl)
    wsl = B.workspace(B.tx_cumsum_workspace_bytes(ocl, cl, -1))
    add("cumsum_f32_8_long_rows", "a11", "cumsum_lookback_kernel", cl.numel() * 8, cl.numel(),
        lambda: B.tx_cumsum(ocl, cl, -1, wsl))

    # ---- workload 5: indexing on src[1048576,256]
    NS, W, ND = 1048576, 256, 65536
    src = rf.view(-1)[: NS * W].view(NS, W)           # 1 GiB of N(0,1): reuse the reduction input
    nidx = 4194304
    idx = torch.randint(0, NS, (nidx,), device=dev, dtype=I64, generator=g)
    osel = torch.empty((nidx, W), device=dev)
    add("index_select_f32", "a12", "index_select_rows_kernel", nidx * (8 + 2 * W * 4), nidx * W,
        lambda: B.tx_index_select(osel, src, 0, idx))
    gidx = torch.randint(0, NS, (16384, W), device=dev, dtype=I64, generator=g)
    ogat = torch.empty((16384, W), device=dev)
    add("gather_f32", "a13", "gather_kernel", 16384 * W * 16, 16384 * W, lambda: B.tx_gather(ogat, src, 0, gidx))
    from paper_2512_10977_amd import inputs as I
    rows = I.zipf_rows(NS, ND, 1.1, seed=4).to(dev)
    eidx = rows.unsqueeze(1).expand(NS, W)
    src_i = ri.view(-1)[: NS * W].view(NS, W).to(I32)
    dst_i = torch.zeros((ND, W), device=dev, dtype=I32)
    wsi32 = B.workspace(B.tx_scatter_add_workspace_bytes(dst_i, 0, eidx, src_i, True))
    add("scatter_add_i32_rows", "a14", "seg_rows_kernel", NS * (W * 4 + 8) + 2 * ND * W * 4, NS * W,
        lambda: B.tx_scatter_add_(dst_i, 0, eidx, src_i, True, wsi32))
    # integer atomics, timed outside the step (the dispatcher does not choose them for the row-index workload):
    # the same workload with one atomic per element, and the secondary configuration with a materialised index
    NE = 131072
    midx = I.zipf_rows(NE * W, ND, 1.1, seed=9).reshape(NE, W).to(dev)
    src_e = src_i[:NE]

    def forced_atomic():
        B.tx_force_path("scatter-atomic")
        try:
            B.tx_scatter_add_(dst_i, 0, eidx, src_i, True, wsi32)
        finally:
            B.tx_force_path(None)
    extra("scatter_add_i32_atomic_per_element", "a14", "scatter_add_atomic_kernel", NS * (W * 4 + 8) + 2 * ND * W * 4,
          NS * W, forced_atomic)
    extra("scatter_add_i32_atomic_elem_index[131072,256]", "a14", "scatter_add_atomic_kernel", NE * W * (4 + 8 + 8), NE * W,
          lambda: B.tx_scatter_add_(dst_i, 0, midx, src_e, True, None))
    dst_f = torch.zeros((ND, W), device=dev)
    wss = B.workspace(B.tx_scatter_add_workspace_bytes(dst_f, 0, eidx, src, True))
    add("scatter_add_f32_sorted", "a15", "seg_rows_kernel", NS * (W * 4 + 8) + 2 * ND * W * 4, NS * W,
        lambda: B.tx_scatter_add_(dst_f, 0, eidx, src, True, wss))
    mask = torch.rand((NS, W), device=dev, generator=g) < 0.3
    omf = osel[:NS]
    add("masked_fill_f32", "a16", "ew_vec_kernel", NS * W * 9, NS * W, lambda: B.tx_masked_fill(omf, src, mask, -1.0))
    # further indexing operators, timed outside the step
    wsia = B.workspace(B.tx_index_add_workspace_bytes(dst_f, 0, rows, src, True))
    extra("index_add_f32_rows_alpha", "f3", "seg_rows_kernel", NS * (W * 4 + 8) + 2 * ND * W * 4, NS * W,
          lambda: B.tx_index_add_(dst_f, 0, rows, src, 0.5, True, wsia))
    wsfe = B.workspace(B.tx_scatter_add_workspace_bytes(dst_f, 0, midx, src[:NE], True))
    extra("scatter_add_f32_sorted_elem_index[131072,256]", "a15", "seg_reduce_kernel", NE * W * (4 + 8 + 8), NE * W,
          lambda: B.tx_scatter_add_(dst_f, 0, midx, src[:NE], True, wsfe))
    wsrr = B.workspace(B.tx_scatter_reduce_workspace_bytes(dst_f, 0, eidx, src, "amax", True))
    extra("scatter_reduce_amax_f32_rows", "f3", "seg_rows_kernel", NS * (W * 4 + 8) + 2 * ND * W * 4, NS * W,
          lambda: B.tx_scatter_reduce_(dst_f, 0, eidx, src, "amax", True, wsrr))
    NR = 131072                                      # element-wise paths: one sort entry per element, so a smaller source
    eidx_r = eidx[:NR].contiguous()                  # a materialised index: element keys
    wssr = B.workspace(B.tx_scatter_reduce_workspace_bytes(dst_f, 0, eidx_r, src[:NR], "amax", True))
    extra("scatter_reduce_amax_f32_elem_index[131072,256]", "f3", "seg_reduce_kernel", NR * W * (4 + 8 + 8), NR * W,
          lambda: B.tx_scatter_reduce_(dst_f, 0, eidx_r, src[:NR], "amax", True, wssr))
    wsip = B.workspace(B.tx_index_put_workspace_bytes(dst_f, [rows[:NR]], src[:NR], True))
    extra("index_put_accumulate_f32_rows[131072,256]", "f3", "seg_rows_kernel", NR * (W * 4 + 8) + 2 * ND * W * 4, NR * W,
          lambda: B.tx_index_put_(dst_f, [rows[:NR]], src[:NR], True, wsip))
    prm = torch.randperm(ND, device=dev, generator=g)
    extra("index_put_assign_f32_rows[65536,256]", "f3", "index_put_kernel", ND * (W * 8 + 8), ND * W,
          lambda: B.tx_index_put_(dst_f, [prm], src[:ND], False, None))
    flat = src.view(-1)
    tidx = torch.randint(-flat.numel(), flat.numel(), (16384 * W,), device=dev, dtype=I64, generator=g)
    otake = ogat.view(-1)
    extra("take_f32", "f3", "take_kernel", tidx.numel() * 16, tidx.numel(), lambda: B.tx_take(otake, src, tidx))
    bounds = torch.randn((65536,), device=dev, generator=g).sort().values
    bvals = torch.randn((4096, 4096), device=dev, generator=g)
    obkt = torch.empty((4096, 4096), device=dev, dtype=I64)
    extra("bucketize_f32[4096,4096]_in_65536", "f3", "searchsorted_kernel", bvals.numel() * 12 + 65536 * 4, bvals.numel(),
          lambda: B.tx_searchsorted(obkt, bounds, bvals, False))
    cnt = torch.zeros((1,), device=dev, dtype=I64)
    osel1 = osel.view(-1)[: NS * W]
    nsel = int(mask.sum().item())
    wsm = B.workspace(B.tx_masked_select_workspace_bytes(osel1, cnt, src, mask))
    extra("masked_select_f32_p0.3", "f3", "select_write_kernel", NS * W * 5 + nsel * 4, NS * W,
          lambda: B.tx_masked_select(osel1, cnt, src, mask, wsm))
    def fused():
        B.tx_force_path("select-fused")
        try:
            B.tx_masked_select(osel1, cnt, src, mask, wsm)
        finally:
            B.tx_force_path(None)
    extra("masked_select_f32_p0.3_single_pass_look_back", "f3", "select_fused_quad_kernel", NS * W * 5 + nsel * 4, NS * W, fused)
    sparse = torch.where(mask, src, torch.zeros((), device=dev))
    onz = torch.empty((NS * W // 2, 2), device=dev, dtype=I64)
    wsn = B.workspace(B.tx_nonzero_workspace_bytes(onz, cnt, sparse))
    extra("nonzero_f32_p0.3", "f3", "nonzero_fused_kernel", NS * W * 4 + nsel * 16, NS * W,
          lambda: B.tx_nonzero(onz, cnt, sparse, wsn))
    extra("nonzero_f32_p0.3_three_passes", "f3", "select_write_kernel", NS * W * 4 + nsel * 16, NS * W,
          forced("select-3pass", lambda: B.tx_nonzero(onz, cnt, sparse, wsn)))
    # 1 GiB probes: the simplest kernels of the library on known traffic (what a copy, a pure read and a pure write sustain)
    pn = 1 << 28
    px1 = rf.view(-1)[:pn]
    py1 = osel.view(-1)[:pn]
    extra("probe_copy_f32_1GiB", "-", "ew_vec_kernel", 2 * pn * 4, pn, lambda: B.tx_copy(py1, px1))
    pout0 = torch.empty((), device=dev)
    pws = B.workspace(B.tx_reduce_workspace_bytes("sum", pout0, px1, None))
    extra("probe_read_sum_f32_1GiB", "-", "reduce_rows_kernel", pn * 4, pn, lambda: B.tx_reduce("sum", pout0, px1, None, False, 1.0, pws))
    par, pbr = randn((16384, 1)), randn((1, 16384))
    py2 = py1.view(16384, 16384)
    extra("probe_write_bcast_add_f32_1GiB", "-", "ew_vec_kernel", pn * 4, pn, lambda: B.tx_add(py2, par, pbr, 1))
    return ops


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(torch, budget_s=2.0):
    """The oracle on a bounded slice of each of the five workloads, timed twice: with every host thread OpenMP
    hands out, and with one thread.  Returns (summary for the headline line, per-workload table for the side file).
    A workload's rate is its algorithmic bytes over its time; slices are cut along the outermost independent dim."""
    from oracle import oracle as O
    from paper_2512_10977_amd import inputs as I
    F32 = torch.float32
    a, b = I.broadcast_add_inputs(4096, 4096, 0)
    x = I.typed((1024, 8192), F32, seed=1)
    y = I.typed((1024, 8192), F32, seed=2)
    y2 = y.reshape(8192, 1024)
    n = x.numel()
    r = I.reduction_input((8, 4096, 1024), F32, seed=2)
    s = I.softmax_logits((2048, 4096), F32, seed=3)
    c = I.cumsum_input((256, 65536), F32, seed=3)
    src = r.view(-1, 256)[:65536]
    idx = I.uniform_indices(262144, 65536, seed=4)
    rows = I.zipf_rows(65536, 4096, 1.1, seed=4)
    dst = torch.zeros((4096, 256))
    m = I.bernoulli_mask((65536, 256), 0.3, seed=4)
    workloads = [
        ("1 broadcast add", "full size [4096,1]+[1,4096]", [(4096 * 4096 * 4 + 2 * 4096 * 4, lambda: O.binary("add", a, b))]),
        ("2 elementwise sweep", "1/8: exp, add, add with a transposed input on [1024,8192] f32",
         [(n * 8, lambda: O.unary("exp", x)), (n * 12, lambda: O.binary("add", x, y)),
          (n * 12, lambda: O.binary("add", x.t(), y2))]),
        ("3 reductions", "1/8: sum over dim -1 and over dim 0 of [8,4096,1024] f32",
         [(r.numel() * 4, lambda: O.reduce("sum", r, -1)), (r.numel() * 4, lambda: O.reduce("sum", r, 0))]),
        ("4 softmax + cumsum", "1/16: softmax [2048,4096], cumsum [256,65536] f32",
         [(s.numel() * 8, lambda: O.softmax(s)), (c.numel() * 8, lambda: O.cumsum(c))]),
        ("5 indexing", "1/16: index_select 262144 rows, scatter_add 65536 Zipf rows into 4096, masked_fill [65536,256]",
         [(262144 * (8 + 2048), lambda: O.index_select(src, 0, idx)),
          (65536 * (1024 + 8) + 2 * 4096 * 1024, lambda: O.scatter_add_(dst, 0, rows.unsqueeze(1).expand(65536, 256), src)),
          (65536 * 256 * 9, lambda: O.masked_fill(src, m, -1.0))]),
    ]
    all_threads = O.num_threads()
    table = []
    tot = {all_threads: [0, 0.0], 1: [0, 0.0]}
    try:
        for name, what, items in workloads:
            row = {"workload": name, "sample": what}
            for threads in (all_threads, 1):
                O.set_num_threads(threads)
                nbytes, passes = 0, 0
                t0 = time.perf_counter()
                while passes == 0 or (time.perf_counter() - t0 < budget_s and passes < 200):
                    for item_bytes, fn in items:
                        fn()
                        nbytes += item_bytes
                    passes += 1
                dt = time.perf_counter() - t0
                row["GB/s_%s" % ("1_thread" if threads == 1 else "all_threads")] = round(nbytes / dt / 1e9, 3)
                row["s_per_pass_%s" % ("1_thread" if threads == 1 else "all_threads")] = round(dt / passes, 4)
                tot[threads][0] += nbytes
                tot[threads][1] += dt
            table.append(row)
    finally:
        O.set_num_threads(all_threads)
    summary = {"value": round(tot[all_threads][0] / tot[all_threads][1] / 1e9, 3), "unit": "GB/s", "cores": all_threads,
               "kind": "oracle", "value_1_thread": round(tot[1][0] / tot[1][1] / 1e9, 3),
               "seconds": round(tot[all_threads][1] + tot[1][1], 1), "nproc": os.cpu_count(), "cpu": cpu_model(),
               "sample": "oracle over 1/8-1/16 slices of workloads 2-5 and all of workload 1, about %g s each at %d "
                         "threads and at 1 thread; per-workload table in the side file" % (budget_s, all_threads)}
    return summary, table


# Kernel behind each dispatch path the step takes (paths are what the library reports for its last launch).
PATH_KERNEL = {"vec": "ew_vec_kernel", "vec-bcast": "ew_bcast_kernel", "tile": "ew_tile_vec_kernel", "tile-scalar": "ew_tile_kernel", "generic": "ew_generic_kernel",
               "rows-wave": "reduce_rows_kernel", "rows-half": "reduce_rows_kernel", "rows-block": "reduce_rows_kernel", "rows-split": "reduce_rows_kernel",
               "cols": "reduce_cols_kernel", "cols-split": "reduce_cols_kernel", "softmax-wave": "softmax_wave_kernel",
               "scan-lookback-wide": "cumsum_lookback_kernel", "scan-lookback": "cumsum_lookback_kernel",
               "scan-carry": "cumsum_carry_kernel", "scan-cols-lookback": "colscan_lookback_kernel", "index-put-rows": "index_put_rows_kernel", "nonzero-fused": "nonzero_fused_kernel",
               "softmax-cols-reg": "softmax_cols_reg_kernel", "softmax-cols": "softmax_cols_kernel", "scan-cols-3pass": "colscan_apply_kernel", "softmax-row": "softmax_row_kernel", "index-select-rows": "index_select_rows_kernel",
               "gather": "gather_kernel", "scatter-sort-rows": "seg_rows_kernel", "scatter-atomic": "scatter_add_atomic_kernel"}


def op_row(op, ms):
    gbps = op["bytes"] / (ms * 1e-3) / 1e9
    return {"op": op["name"], "row": op["row"], "path": op.get("path", ""), "kernel": op["kernel"], "us": round(ms * 1e3, 2),
            "GB/s": round(gbps, 1), "frac_of_peak": round(gbps / PEAK_GBPS, 4),
            "Gelem/s": round(op["elems"] / (ms * 1e-3) / 1e9, 2), "bytes": op["bytes"]}


def headline(result):
    """The one JSON line the harness reads: short enough to survive a truncated log tail (the per-operator tables
    go to the side file).  Raises if it grows past 1500 characters."""
    keep = ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
            "vs_baseline", "dtype", "data", "config", "frac_of_peak", "elements_per_s", "roofline", "cpu_baseline", "side_file")
    line = json.dumps({k: result[k] for k in keep if k in result}, separators=(",", ":"))
    if len(line) > 1500 or "\n" in line:
        raise ValueError("headline JSON line is %d characters; the limit is 1500" % len(line))
    return line


def time_launches(torch, fn, count, warm):
    """Average time in ms of `count` back-to-back launches (events on the launch stream), after `warm` warm-ups."""
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(count):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / count


def time_median(torch, fn, count):
    """Median time in ms of `count` launches in a row, one event after each (a host stall between two launches then
    lengthens one sample, not the figure)."""
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(count + 1)]
    ev[0].record()
    for i in range(count):
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(count))
    return t[count // 2]


def measurement_detail(torch, B):
    """Numbers beside the step: workload 1 with rotating and with one output buffer and as a single launch;
    1 GiB probes (copy, pure read, pure write) that show what this GPU sustains on the simplest kernels."""
    dev = "cuda"
    F32 = torch.float32
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    a1 = torch.randn((4096, 1), device=dev, generator=g)
    b1 = torch.randn((1, 4096), device=dev, generator=g)
    outs = [torch.empty((4096, 4096), device=dev) for _ in range(9)]
    state = {"i": 0}
    nb1 = 4096 * 4096 * 4 + 2 * 4096 * 4

    def rotating():
        state["i"] = (state["i"] + 1) % len(outs)
        B.tx_add(outs[state["i"]], a1, b1, 1)

    def rate(nbytes, ms):
        return {"us": round(ms * 1e3, 2), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                "frac_of_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_GBPS, 4)}

    detail = {"timing": "HIP events around 27 back-to-back launches after 9 warm-ups, divided by 27; "
                        "single launch = events around one launch after a device synchronisation, median of 9"}
    w1 = {"rotating_9_outputs": rate(nb1, time_launches(torch, rotating, 27, 9)),
          "one_output_buffer": rate(nb1, time_launches(torch, lambda: B.tx_add(outs[0], a1, b1, 1), 27, 9))}
    singles = []
    for _ in range(9):
        torch.cuda.synchronize()
        singles.append(time_launches(torch, rotating, 1, 0))
    w1["single_launch"] = rate(nb1, sorted(singles)[4])
    detail["workload_1_add[4096,1]+[1,4096]"] = w1
    n = 1 << 28
    x = torch.empty(n, device=dev, dtype=F32).normal_(generator=g)
    y = torch.empty_like(x)
    probes = {"tx_copy_f32_1GiB (1 read + 1 write)": rate(2 * n * 4, time_launches(torch, lambda: B.tx_copy(y, x), 10, 3)),
              "device_memcpy_1GiB (1 read + 1 write)": rate(2 * n * 4, time_launches(torch, lambda: y.copy_(x), 10, 3))}
    out0 = torch.empty((), device=dev)
    ws = B.workspace(B.tx_reduce_workspace_bytes("sum", out0, x, None))
    probes["tx_reduce_sum_all_f32_1GiB (pure read)"] = rate(n * 4, time_launches(
        torch, lambda: B.tx_reduce("sum", out0, x, None, False, 1.0, ws), 10, 3))
    ar = torch.randn((16384, 1), device=dev, generator=g)
    br = torch.randn((1, 16384), device=dev, generator=g)
    y2 = y.view(16384, 16384)
    probes["tx_add_[16384,1]+[1,16384]_1GiB (pure write)"] = rate(n * 4, time_launches(
        torch, lambda: B.tx_add(y2, ar, br, 1), 10, 3))
    detail["probes_1GiB"] = probes
    return detail


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the operators timed outside the step")
    ap.add_argument("--no-detail", action="store_true", help="skip the extra measurements of workload 1 and the 1 GiB probes")
    ap.add_argument("--only", default="", help="comma-separated substrings: run only the operators whose name matches "
                                               "(for profiling single kernels; the JSON line then covers that subset)")
    ap.add_argument("--calibrate", action="store_true",
                    help="add a plain 1 GiB device-to-device copy to the step (known traffic, to scale profiler counters)")
    ap.add_argument("--side-file", default=os.path.join("gpurun_out", "bench_per_op.json"),
                    help="where the per-operator tables go (relative to the repository root)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one MI355X: every operator here runs on a single GPU; --gpus %d is not supported "
              "(see DESIGN.md for how the path would shard)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2512_10977_amd import binding as B
    B.lib()
    torch.cuda.set_device(0)
    ops = build_ops(torch, B)
    if args.only:
        pats = [p for p in args.only.split(",") if p]
        ops = [o for o in ops if any(p in o["name"] for p in pats)]
    extras = [] if args.no_extras else [o for o in ops if o["extra"]]
    ops = [o for o in ops if not o["extra"]]
    if args.calibrate:
        ca = torch.empty(1 << 28, device="cuda", dtype=torch.float32).normal_()
        cb = torch.empty_like(ca)
        ops.append(dict(name="calibration_copy_1GiB", row="-", kernel="device copy", bytes=2 << 30, elems=1 << 28,
                        fn=lambda: cb.copy_(ca), extra=False))
    torch.cuda.synchronize()

    def label(op):                                  # the path the dispatcher took, and the kernel behind it
        if op["kernel"] != "device copy" and "graph replay" not in op["name"]:
            op["path"] = B.tx_last_path()
            op["kernel"] = PATH_KERNEL.get(op["path"], op["kernel"])

    for w in range(max(1, args.warmup)):
        for op in ops:
            op["fn"]()
            if w == 0:
                label(op)
    torch.cuda.synchronize()
    # Instrumented pass (not the timed one): one event after every operator (and one at the head of each step); an
    # operator's time is the distance between the event before it and the event after it, so consecutive operators
    # share a marker instead of each being bracketed by a pair of its own (a marker is a barrier on the stream, about
    # 2 us during which nothing runs: 45 of them are 2 % of a step, which is why they stay out of the timed pass).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(ops) + 1)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        events[k][0].record()
        for j, op in enumerate(ops):
            op["fn"]()
            events[k][j + 1].record()
    torch.cuda.synchronize()
    wall_marked = time.perf_counter() - t0
    med_ms = [sorted(events[k][j].elapsed_time(events[k][j + 1]) for k in range(args.steps))[args.steps // 2] for j in range(len(ops))]
    jdom = max(range(len(ops)), key=lambda j: med_ms[j]) if ops else -1
    # Timed pass: exactly `steps` steps between two synchronisations, with one pair of events per step, around the
    # operator that takes the largest share of the step (the roofline object of the headline is measured here).
    dom_events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        for j, op in enumerate(ops):
            if j == jdom:
                dom_events[k][0].record()
            op["fn"]()
            if j == jdom:
                dom_events[k][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    outside = []
    for op in extras:                        # alternatives the dispatcher did not choose: one warm-up, the median of five launches
        op["fn"]()
        label(op)
        outside.append(op_row(op, time_median(torch, op["fn"], 5)))
    step_bytes = sum(op["bytes"] for op in ops)
    step_elems = sum(op["elems"] for op in ops)
    per_op = []
    for j, op in enumerate(ops):
        # the table's figure is the median over the steps: the distance between two events also holds any time the
        # stream sat idle because the host fell behind (one such stall, about 1 ms, in one step of ten, doubled an
        # operator's mean in one run); the mean and the minimum are kept beside it
        times = sorted(events[k][j].elapsed_time(events[k][j + 1]) for k in range(args.steps))
        row = op_row(op, times[len(times) // 2])
        row["us_min"], row["us_mean"] = round(times[0] * 1e3, 2), round(sum(times) / args.steps * 1e3, 2)
        per_op.append(row)
    for r in per_op:                         # stored counter readings: traffic and the rate in bytes actually moved
        if r["op"] in PMC_TRAFFIC_BYTES:
            t = PMC_TRAFFIC_BYTES[r["op"]]
            r["hbm_traffic_bytes_counters"] = t
            r["frac_of_peak_in_traffic_bytes"] = round(t / (r["us"] * 1e-6) / 1e9 / PEAK_GBPS, 4)
    # (--only may leave the step empty: the line then describes the selected operators timed outside it)
    if jdom >= 0:                            # the dominant operator as the timed pass saw it
        dom = op_row(ops[jdom], sum(a.elapsed_time(b) for a, b in dom_events) / args.steps)
    else:
        dom = max(outside or [op_row({"name": "none", "row": "", "kernel": "", "bytes": 0, "elems": 0}, 1e-3)], key=lambda r: r["us"])
    ms_step = wall / args.steps * 1e3
    value = step_bytes / (wall / args.steps) / 1e9
    side = os.path.join(ROOT, args.side_file)
    result = {
        "metric": "achieved HBM GB/s (algorithmic bytes / time) over one pass of all operator classes on one GPU",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "all five workloads at full size: add [4096,1]+[1,4096]; elementwise [8192,8192]; "
                               "reductions [64,4096,1024]; softmax [32768,4096]; cumsum [4096,65536]; "
                               "indexing on src[1048576,256]", "ops_per_step": len(ops)},
        "frac_of_peak": round(value / PEAK_GBPS, 4),
        "elements_per_s": round(step_elems / (wall / args.steps), 1),
        "roofline": {"bound": "hbm", "kernel": dom["kernel"], "op": dom["op"], "achieved": dom["GB/s"],
                     "peak": PEAK_GBPS, "unit": "GB/s", "frac": dom["frac_of_peak"],
                     "traffic": PMC_TRAFFIC_BYTES.get(dom["op"]), "algorithmic_bytes": dom["bytes"],
                     "avg_us": dom["us"]},
        "side_file": args.side_file,
        "ms_per_step_with_operator_events": round(wall_marked / args.steps * 1e3, 3),
        "per_op": per_op,
        "per_op_outside_step": outside,
    }
    if not args.only and not args.no_detail:
        result["measurement_detail"] = measurement_detail(torch, B)
    if not args.no_cpu_baseline:
        result["cpu_baseline"], result["cpu_baseline_per_workload"] = cpu_baseline(torch)
    try:                                       # the tables: a file, never the line the harness parses
        os.makedirs(os.path.dirname(side), exist_ok=True)
        with open(side, "w") as f:
            json.dump(result, f, indent=1)
    except OSError as e:
        print("could not write %s: %s" % (side, e), file=sys.stderr)
    sys.stdout.flush()
    print(headline(result), flush=True)


if __name__ == "__main__":
    main()
