#!/usr/bin/env python3
"""Benchmark of the HALO low-precision linear layer on one MI355X.

One "step" = one pass of the whole hot path on config c2 (Llama-3-8B attention projection, tokens 2048,
4096 x 4096, HALO-1): rotate+quantise X and W, INT8 forward GEMM with dequant epilogue, then both backward
products (quantise E twice, two INT8 GEMMs on the saved codes, dequantise + un-rotate).  All inputs are
resident in HBM before the timed region; outputs, saved codes and the workspace are preallocated.

Prints ONE JSON line.  `value` = 6*b*n*m INT8 operations / step time of c2 (effective TOPS of the whole layer,
quantisation and Hadamard overheads included).  `roofline` describes the kernel that takes the most time in
that step; `kernels` lists every kernel family with its own roofline fraction; `cpu_baseline` is the numpy
oracle timed on the host cores.  `configs` carries the same kind of record for c3 (MLP down projection, HALO-2)
and c4 (the seven linears of a decoder layer at 8192 tokens: seven forwards, then seven backwards, back to back
on one stream, q/k/v and gate/up sharing one quantised activation), and for c5, the MXFP6 forward product.  `mfma_ceiling` is the INT8 MFMA rate the
machine sustains on constant, on random and on the step's own operand bytes with nothing else running
(halo_mfma_i8_probe); `copy_GBs` a plain device copy, the practical HBM ceiling.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
INT8_PEAK_TOPS = 5000.0      # MI355X dense INT8 MFMA, published (5.0 POP/s)
METRIC = "HALO linear fwd+bwd INT8 TOPS at Llama-3-8B shapes; Hadamard+quant GB/s"


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=100)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--config", default="c2", help="headline workload: c2 (default) or c3")
    p.add_argument("--extra-configs", default="c3,c4,c5,c6,c7,c8", help="comma list of further configs reported under `configs`")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--kernel-iters", type=int, default=50, help="launches per kernel for the per-kernel timings")
    p.add_argument("--pmc-target", default="",
                   help="run ONE kernel family --steps times and exit (for rocprofv3 --pmc runs): gemm_fwd, gemm_ex, "
                        "gemm_g, gemm_pair, rowquant_x, rowquant_w, rowquant_xw, quant_dual, unrotate_ex, unrotate_g, copy")
    p.add_argument("--step-only", action="store_true",
                   help="time the step loop of --config only (no per-kernel loops, no oracle, no extra configs): what a "
                        "kernel-trace profile of the step needs")
    return p.parse_args()


def time_launches(fn, iters, warm=5):
    """Average duration (ms) of fn() launches, measured with HIP events on the stream the kernels run on."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def time_steps(step, steps, warmup):
    import torch
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        return 1


# ------------------------------------------------------------------------------------------------ single linear
class Linear:
    """Device state of one linear of a config: inputs, saved codes, outputs, workspace."""

    def __init__(self, cfg, which, dev, share_x_from=None, out_bufs=None):
        import numpy as np
        import torch
        from paper_2501_02625_amd import binding, inputs
        self.cfg, self.lin = cfg, cfg.linears[which]
        self.b, self.m, self.n, self.level = cfg.tokens, self.lin.m, self.lin.n, cfg.level
        b, m, n = self.b, self.m, self.n
        self.hm = cfg.had_block_m(m) if self.level >= 1 else 0
        self.hb = (b & -b) if self.level >= 2 else 0
        sub = cfg.seed * 1000 + which
        to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        self.host = {}
        if share_x_from is None:
            self.host["X"] = inputs.make_activations(b, m, cfg.outlier_frac, sub)
            self.X = to_dev(self.host["X"])
            Xq = torch.empty((b, m), dtype=torch.int8, device=dev)
            s_x = torch.empty((b,), dtype=torch.float32, device=dev)
        else:
            self.X = None
            Xq, s_x = share_x_from.state.Xq, share_x_from.state.s_x
        self.host["W"] = inputs.make_weights(n, m, sub)
        self.host["E"] = inputs.make_errors(b, n, sub)
        self.W, self.E = to_dev(self.host["W"]), to_dev(self.host["E"])
        self.desc = binding.make_desc(b, m, n, self.level, torch.bfloat16, had_block_m=self.hm,
                                      scale_mode=binding.HALO_SCALE_PER_TENSOR if cfg.per_tensor else binding.HALO_SCALE_PER_ROW)
        self.state = binding.LinearState(Xq, s_x, torch.empty((n, m), dtype=torch.int8, device=dev),
                                         torch.empty((n,), dtype=torch.float32, device=dev))
        alloc = lambda key, shape: (out_bufs.setdefault(key, torch.empty(shape, dtype=torch.bfloat16, device=dev))
                                    if out_bufs is not None else torch.empty(shape, dtype=torch.bfloat16, device=dev))
        self.Y = alloc(("Y", b, n), (b, n))
        self.EX = alloc(("EX", b, m), (b, m))
        self.G = alloc(("G", n, m), (n, m))
        self.ws_bytes = binding.halo_linear_workspace_bytes(self.desc)
        self.ops = 6.0 * b * n * m

    def fwd(self, binding, ws=None):
        binding.halo_linear_fwd(self.desc, self.X, self.W, state=self.state, Y=self.Y, workspace=ws)

    def bwd(self, binding, ws):
        binding.halo_linear_bwd(self.desc, self.E, self.state, workspace=ws, EX=self.EX, G=self.G)


def kernel_timings(L, it, dev, copy_gbs):
    """Per-kernel timings of one linear's step: list of records with roofline fractions."""
    import torch
    from paper_2501_02625_amd import binding
    lib = binding.load_library()
    b, m, n, level, hm, hb = L.b, L.m, L.n, L.level, L.hm, L.hb
    state, X, W, E, Y, EX, G = L.state, L.X, L.W, L.E, L.Y, L.EX, L.G
    kernels = []

    # the quantised E of the step itself (so that the GEMMs are timed on the operand data the workload has)
    if level <= 1:
        Eq, s_e, EqT, s_g = binding.halo_quant_dual(E, fold_cols=state.s_w, fold_rows=state.s_x)
    else:
        Eq, s_e = binding.halo_hadamard_quant(E, had_block_left=hb, fold=state.s_w)
        EqT, s_g = binding.halo_hadamard_quant(E, axis=binding.HALO_QUANT_COLS_T, fold=state.s_x)
    acc_bm = torch.empty((b, m), dtype=torch.int32, device=dev)
    acc_nm = torch.empty((n, m), dtype=torch.int32, device=dev)

    def add_gemm(name, fn, ops, shape):
        ms = time_launches(fn, it)
        tops = ops / (ms * 1e-3) / 1e12
        kernels.append(dict(name=name, bound="mfma", ms=ms, achieved=tops, peak=INT8_PEAK_TOPS, unit="TOP/s",
                            frac=tops / INT8_PEAK_TOPS, shape=shape))

    add_gemm("gemm_fwd_nt(Xq,Wq)->Y", lambda: binding.halo_gemm_i8(state.Xq, state.Wq, trans_b=True, row_scale=state.s_x,
                                                                   col_scale=state.s_w, out=Y), 2.0 * b * n * m, [b, n, m])
    if level == 0:
        add_gemm("gemm_ex_nn(Eq,Wq)->EX", lambda: binding.halo_gemm_i8(Eq, state.Wq, trans_b=False, row_scale=s_e, out=EX),
                 2.0 * b * m * n, [b, m, n])
        add_gemm("gemm_g_nn(EqT,Xq)->G", lambda: binding.halo_gemm_i8(EqT, state.Xq, trans_b=False, row_scale=s_g, out=G),
                 2.0 * n * m * b, [n, m, b])
    else:
        add_gemm("gemm_ex_nn(Eq,Wq)->acc", lambda: binding.halo_gemm_i8(Eq, state.Wq, trans_b=False, out_dtype=None,
                                                                        acc_out=acc_bm), 2.0 * b * m * n, [b, m, n])
        add_gemm("gemm_g_nn(EqT,Xq)->acc", lambda: binding.halo_gemm_i8(EqT, state.Xq, trans_b=False, out_dtype=None,
                                                                        acc_out=acc_nm), 2.0 * n * m * b, [n, m, b])
        # what halo_linear_bwd actually launches: both products in one kernel
        g1 = binding.gemm_desc(Eq, state.Wq, trans_b=False, acc_out=acc_bm)
        g2 = binding.gemm_desc(EqT, state.Xq, trans_b=False, acc_out=acc_nm)
        add_gemm("gemm_bwd_pair(E_X,G)->acc", lambda: binding.halo_gemm_i8_pair(g1, g2), 4.0 * b * m * n,
                 [[b, m, n], [n, m, b]])

    def add_hbm(name, fn_for, bytes_per_launch, nbuf, passes=None):
        # rotate over nbuf distinct buffer sets so the 256 MB last-level cache cannot hold the working set
        fns = [fn_for(i) for i in range(nbuf)]
        counter = [0]

        def run():
            fns[counter[0] % nbuf]()
            counter[0] += 1
        ms = time_launches(run, max(it, nbuf * 2))
        gbs = bytes_per_launch / (ms * 1e-3) / 1e9
        rec = dict(name=name, bound="hbm", ms=ms, achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS,
                   frac_of_copy=gbs / copy_gbs if copy_gbs else None, bytes=bytes_per_launch, rotating_buffers=nbuf)
        if passes:
            rec["passes"] = passes
        kernels.append(rec)

    def nrot(nbytes):
        return max(2, int((768 << 20) // max(nbytes, 1)) + 1)

    # row rotate+quantise of X (F1) and W (F2): 2 B read + 1 B written per element + 4 B per row
    for nm, T, rows in (("hadamard_quant_rows(X)", X, b), ("hadamard_quant_rows(W)", W, n)):
        if T is None:
            continue
        nbytes = rows * m * 3 + rows * 4
        k = nrot(nbytes)
        srcs = [T] + [T.clone() for _ in range(k - 1)]
        qs = [torch.empty((rows, m), dtype=torch.int8, device=dev) for _ in range(k)]
        ss = [torch.empty((rows,), dtype=torch.float32, device=dev) for _ in range(k)]
        add_hbm(nm, lambda i, srcs=srcs, qs=qs, ss=ss: (lambda: binding.halo_hadamard_quant(
            srcs[i], had_block=hm, out_q=qs[i], out_scale=ss[i])), nbytes, k)
        del srcs, qs, ss
    # the same kernel on a tensor large enough to amortise launch and ramp (scale reference, not part of the step)
    if hm and m <= 4096:
        big_rows = 32768
        nbytes = big_rows * m * 3 + big_rows * 4
        k = 3
        srcs = [torch.randn((big_rows, m), device=dev).to(torch.bfloat16) for _ in range(k)]
        qs = [torch.empty((big_rows, m), dtype=torch.int8, device=dev) for _ in range(k)]
        ss = [torch.empty((big_rows,), dtype=torch.float32, device=dev) for _ in range(k)]
        add_hbm("hadamard_quant_rows(%dx%d, scale reference)" % (big_rows, m), lambda i, srcs=srcs, qs=qs, ss=ss: (
            lambda: binding.halo_hadamard_quant(srcs[i], had_block=hm, out_q=qs[i], out_scale=ss[i])), nbytes, k)
        del srcs, qs, ss
    # E for E_X (B1/B2) and E^T for G (B5)
    nbytes = b * n * 3 + b * 4
    k = nrot(nbytes)
    srcs = [E] + [E.clone() for _ in range(k - 1)]
    qs = [torch.empty((b, n), dtype=torch.int8, device=dev) for _ in range(k)]
    ss = [torch.empty((b,), dtype=torch.float32, device=dev) for _ in range(k)]
    wsq = torch.empty((max(1, lib.halo_hadamard_quant_workspace_bytes(b, n, 0, hb)),), dtype=torch.uint8, device=dev)
    add_hbm("hadamard_quant_rows(E,fold=s_w%s)" % (",left" if hb else ""), lambda i: (lambda: binding.halo_hadamard_quant(
        srcs[i], had_block_left=hb, fold=state.s_w, out_q=qs[i], out_scale=ss[i], workspace=wsq)), nbytes, k,
        passes="left-hand rotation: two strided passes with an fp32 intermediate, then the row quantiser" if hb else None)
    qts = [torch.empty((n, b), dtype=torch.int8, device=dev) for _ in range(k)]
    sts = [torch.empty((n,), dtype=torch.float32, device=dev) for _ in range(k)]
    wsc = torch.empty((max(256, lib.halo_hadamard_quant_workspace_bytes(b, n, 1, 0)),), dtype=torch.uint8, device=dev)
    add_hbm("hadamard_quant_cols_t(E,fold=s_x)", lambda i: (lambda: binding.halo_hadamard_quant(
        srcs[i], axis=binding.HALO_QUANT_COLS_T, fold=state.s_x, out_q=qts[i], out_scale=sts[i], workspace=wsc)),
        b * n * 3 + n * 4, k)
    if level <= 1:
        wsd = torch.empty((lib.halo_quant_dual_workspace_bytes(b, n),), dtype=torch.uint8, device=dev)
        add_hbm("quant_dual(E,fold=s_w|s_x)", lambda i: (lambda: binding.halo_quant_dual(
            srcs[i], fold_cols=state.s_w, fold_rows=state.s_x, out_q=qs[i], row_scale=ss[i], out_qt=qts[i],
            col_scale=sts[i], workspace=wsd)), b * n * 4 + (b + n) * 4, k)
    del srcs, qs, ss, qts, sts
    if level >= 1:
        for nm, rows, acc, left, out in (("dequant_unrotate(acc->EX%s)" % (",left" if hb else ""), b, acc_bm, hb, EX),
                                         ("dequant_unrotate(acc->G)", n, acc_nm, 0, G)):
            nbytes = rows * m * (4 + 2)
            k = nrot(nbytes)
            accs = [acc] + [acc.clone() for _ in range(k - 1)]
            outs = [torch.empty((rows, m), dtype=torch.bfloat16, device=dev) for _ in range(k)]
            scale = torch.rand((rows,), dtype=torch.float32, device=dev)
            wsu = torch.empty((max(1, lib.halo_dequant_unrotate_workspace_bytes(rows, m, left)),), dtype=torch.uint8,
                              device=dev)
            add_hbm(nm, lambda i, accs=accs, outs=outs, scale=scale, wsu=wsu, left=left: (lambda: binding.halo_dequant_unrotate(
                accs[i], scale, had_block=hm, had_block_left=left, out=outs[i], workspace=wsu)), nbytes, k,
                passes=("stand-alone entry point: strided passes from the int32 accumulators, then the row pass; inside the "
                        "layer the product's epilogue runs the eight low strides and one strided pass is left") if left else None)
            del accs, outs
    return kernels


def oracle_slice(cfg, which_list, tokens):
    """The numpy oracle on the first `tokens` tokens of the given linears (all in/out features); seconds, ops."""
    from oracle import halo_oracle as orc
    from paper_2501_02625_amd import inputs
    secs, ops = 0.0, 0.0
    for which in which_list:
        lin = cfg.linears[which]
        t = inputs.make_linear_inputs(cfg, which, tokens=tokens, need_error=True)
        hm = cfg.had_block_m(lin.m) if cfg.level >= 1 else 0
        hb = (tokens & -tokens) if cfg.level >= 2 else 0
        Xr, Wr, Er = (orc.bf16_bits_to_real(t[k]) for k in ("X", "W", "E"))
        c0 = time.perf_counter()
        f = orc.forward(Xr, Wr, cfg.level, hm, per_tensor=cfg.per_tensor)
        orc.backward_input(Er, f["Wq"], f["s_w"], cfg.level, hm, hb, per_tensor=cfg.per_tensor)
        orc.backward_weight(Er, f["Xq"], f["s_x"], cfg.level, hm, per_tensor=cfg.per_tensor)
        secs += time.perf_counter() - c0
        ops += 6.0 * tokens * lin.n * lin.m
    return secs, ops


def run_single(key, args, dev, copy_gbs, with_kernels, with_oracle):
    import torch
    from paper_2501_02625_amd import binding, inputs
    cfg = inputs.CONFIGS[key]
    L = Linear(cfg, 0, dev)
    ws = torch.empty((max(L.ws_bytes, 1),), dtype=torch.uint8, device=dev)

    def step():
        L.fwd(binding, ws if cfg.per_tensor else None)
        L.bwd(binding, ws)
    ms = time_steps(step, args.steps, args.warmup)
    with_kernels = with_kernels and not cfg.per_tensor       # the per-kernel loops time the per-row entry points
    rec = dict(workload="%s: tokens %d, linear %dx%d (n x m), HALO-%d, INT8%s, bf16 in/out, fwd + both bwd products"
                        % (key, L.b, L.n, L.m, L.level, ", one scale per tensor" if cfg.per_tensor else ""),
               b=L.b, m=L.m, n=L.n, level=L.level, had_block_m=L.hm, had_block_b=L.hb, ops_per_step=L.ops,
               ms_per_step=ms, value=L.ops / (ms * 1e-3) / 1e12, unit="TOPS")
    kernels = None
    if with_kernels:
        kernels = kernel_timings(L, args.kernel_iters, dev, copy_gbs)
        rec["kernels"] = kernels
    if with_oracle:
        if key == "c2":
            secs, ops = oracle_slice(cfg, [0], L.b)
            sample = "the full c2 step once"
        else:
            tokens = 512
            secs, ops = oracle_slice(cfg, [0], tokens)
            sample = "the first %d of %d tokens of %s (all features; left block = %d), extrapolated by operation count" % (
                tokens, L.b, key, tokens)
        nt = blas_threads()
        rec["cpu_baseline"] = dict(value=ops / secs / 1e12, unit="TOPS", cores=nt, kind="oracle", seconds=secs,
                                   sample=sample + " (numpy oracle; elementwise parts single-threaded, integer GEMMs "
                                                   "carried by a %d-thread fp64 BLAS matmul)" % nt)
    return rec, L, kernels


def run_layer(key, args, dev, with_oracle):
    """Config c4: every linear of the decoder layer, forwards then backwards back to back on one stream."""
    import torch
    from paper_2501_02625_amd import binding, inputs
    cfg = inputs.CONFIGS[key]
    out_bufs = {}
    Ls, by_name = [], {}
    for i, lin in enumerate(cfg.linears):
        L = Linear(cfg, i, dev, share_x_from=by_name.get(lin.shares_input_with), out_bufs=out_bufs)
        L.host = None                                    # the host copies are not needed any more
        Ls.append(L)
        by_name[lin.name] = L
    ws = torch.empty((max(L.ws_bytes for L in Ls),), dtype=torch.uint8, device=dev)

    def step():
        for L in Ls:
            L.fwd(binding)
        for L in reversed(Ls):
            L.bwd(binding, ws)
    steps = max(3, min(args.steps, 20))
    ms = time_steps(step, steps, max(2, min(args.warmup, 5)))
    ops = sum(L.ops for L in Ls)
    rec = dict(workload="%s: tokens %d, the seven linears of a Llama-3-8B decoder layer (%s), HALO-%d, INT8, bf16 in/out, "
                        "7 forwards then 7 backwards on one stream, one quantised activation shared by q/k/v and by gate/up"
                        % (key, cfg.tokens, ", ".join("%s %dx%d" % (l.name, l.n, l.m) for l in cfg.linears), cfg.level),
               b=cfg.tokens, level=cfg.level, ops_per_step=ops, steps=steps, ms_per_step=ms,
               value=ops / (ms * 1e-3) / 1e12, unit="TOPS")
    if with_oracle:
        tokens = 256
        which = [i for i, l in enumerate(cfg.linears) if l.name in ("q", "k", "down")]
        secs, sops = oracle_slice(cfg, which, tokens)
        nt = blas_threads()
        rec["cpu_baseline"] = dict(value=sops / secs / 1e12, unit="TOPS", cores=nt, kind="oracle", seconds=secs,
                                   sample="the first %d of %d tokens of the linears q, k and down (left block = %d), "
                                          "extrapolated by operation count (numpy oracle, %d-thread fp64 BLAS)"
                                          % (tokens, cfg.tokens, tokens, nt))
    del Ls, out_bufs, ws
    torch.cuda.empty_cache()
    return rec


def run_mx6(key, args, dev, copy_gbs, with_oracle):
    """Config c5: the MXFP6 forward product (rotate + microscaling FP6 quantise of X and W, scaled-MFMA GEMM)."""
    import numpy as np
    import torch
    from paper_2501_02625_amd import binding, inputs
    cfg = inputs.CONFIGS[key]
    lin = cfg.linears[0]
    b, m, n = cfg.tokens, lin.m, lin.n
    hm = min(m & -m, 4096)
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    X = to_dev(inputs.make_activations(b, m, cfg.outlier_frac, cfg.seed))
    W = to_dev(inputs.make_weights(n, m, cfg.seed))
    xc = torch.empty((b, m // 32 * 24), dtype=torch.uint8, device=dev); xs = torch.empty((b, m // 32), dtype=torch.uint8, device=dev)
    wc = torch.empty((n, m // 32 * 24), dtype=torch.uint8, device=dev); ws = torch.empty((n, m // 32), dtype=torch.uint8, device=dev)
    Y = torch.empty((b, n), dtype=torch.bfloat16, device=dev)

    def step():
        binding.halo_mx6_quant(X, had_block=hm, out_codes=xc, out_scales=xs)
        binding.halo_mx6_quant(W, had_block=hm, out_codes=wc, out_scales=ws)
        binding.halo_gemm_mx6(xc, xs, wc, ws, out=Y)
    ms = time_steps(step, args.steps, args.warmup)
    ops = 2.0 * b * m * n
    it = args.kernel_iters
    kernels = []
    for nm, T, rows, oc, osc in (("mx6_quant(X)", X, b, xc, xs), ("mx6_quant(W)", W, n, wc, ws)):
        kms = time_launches(lambda: binding.halo_mx6_quant(T, had_block=hm, out_codes=oc, out_scales=osc), it)
        nbytes = rows * m * (2 + 0.75) + rows * (m // 32)
        gbs = nbytes / (kms * 1e-3) / 1e9
        kernels.append(dict(name=nm, bound="hbm", ms=kms, achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s", frac=gbs / HBM_PEAK_GBS,
                            frac_of_copy=gbs / copy_gbs if copy_gbs else None, bytes=nbytes))
    kms = time_launches(lambda: binding.halo_gemm_mx6(xc, xs, wc, ws, out=Y), it)
    tf = ops / (kms * 1e-3) / 1e12
    kernels.append(dict(name="gemm_mx6(Xc,Wc)->Y", bound="mfma", ms=kms, achieved=tf, peak=10100.0, unit="TFLOP/s",
                        frac=tf / 10100.0, shape=[b, n, m]))
    rec = dict(workload="%s: MXFP6 forward product, X %dx%d, W %dx%d, FWHT over K, FP6 E3M2 elements with an E8M0 scale "
                        "per 32 along K, fp32 accumulation, bf16 in/out" % (key, b, m, n, m),
               b=b, m=m, n=n, ops_per_step=ops, ms_per_step=ms, value=ops / (ms * 1e-3) / 1e12, unit="TFLOP/s",
               kernels=kernels)
    if with_oracle:
        from oracle import mxfp6_oracle as mxo
        from oracle import halo_oracle as orc
        tokens = 256
        Xr = orc.bf16_bits_to_real(inputs.make_activations(tokens, m, cfg.outlier_frac, cfg.seed))
        Wr = orc.bf16_bits_to_real(inputs.make_weights(n, m, cfg.seed))
        c0 = time.perf_counter()
        mxo.forward_mxfp6(Xr, Wr, hm)
        secs = time.perf_counter() - c0
        rec["cpu_baseline"] = dict(value=2.0 * tokens * m * n / secs / 1e12, unit="TFLOP/s", cores=blas_threads(), kind="oracle",
                                   seconds=secs, sample="the first %d of %d tokens against the full weight matrix, "
                                   "extrapolated by operation count (numpy oracle)" % (tokens, b))
    return rec


def run_peft(key, args, dev, with_oracle, with_parts=True):
    """Config c8: the HALO-PEFT module, frozen quantised weight + LoRA adapters; a step is its forward pass and its
    backward pass (E_X and both adapter gradients)."""
    import numpy as np
    import torch
    from paper_2501_02625_amd import binding, inputs
    cfg = inputs.CONFIGS[key]
    lin = cfg.linears[0]
    b, m, n, rank = cfg.tokens, lin.m, lin.n, cfg.peft_rank
    hm = cfg.had_block_m(m) if cfg.level >= 1 else 0
    hb = cfg.had_block_b() if cfg.level >= 2 else 0
    t = inputs.make_linear_inputs(cfg)
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    X, W, E, U, V = (to_dev(t[k]) for k in ("X", "W", "E", "U", "V"))
    Wq, s_w = binding.halo_hadamard_quant(W, had_block=hm)            # once, before fine-tuning: not part of a step
    del W
    desc = binding.make_desc(b, m, n, cfg.level, torch.bfloat16, had_block_m=hm, had_block_b=hb)
    ws = torch.empty((binding.halo_peft_workspace_bytes(desc, rank),), dtype=torch.uint8, device=dev)
    Y = torch.empty((b, n), dtype=torch.bfloat16, device=dev)
    T = torch.empty((b, rank), dtype=torch.float32, device=dev)
    EX = torch.empty((b, m), dtype=torch.bfloat16, device=dev)
    GU = torch.empty((rank, m), dtype=torch.float32, device=dev)
    GV = torch.empty((n, rank), dtype=torch.float32, device=dev)

    fwd = lambda: binding.halo_peft_fwd(desc, X, Wq, s_w, U, V, workspace=ws, Y=Y, T=T)
    bwd = lambda: binding.halo_peft_bwd(desc, E, X, T, Wq, s_w, U, V, workspace=ws, EX=EX, GU=GU, GV=GV)

    def step():
        fwd()
        bwd()
    ms = time_steps(step, args.steps, args.warmup)
    ops = float(cfg.gemm_ops())
    it = args.kernel_iters
    # the same two large products without the adapters (plain layer on the frozen weight, E_X only), for the cost of the
    # low-rank branch
    state = binding.LinearState(torch.empty((b, m), dtype=torch.int8, device=dev), torch.empty((b,), dtype=torch.float32, device=dev),
                                Wq, s_w)
    lws = torch.empty((max(binding.halo_linear_workspace_bytes(desc), 1),), dtype=torch.uint8, device=dev)
    parts = None if not with_parts else dict(
        fwd=time_launches(fwd, it),
        bwd=time_launches(bwd, it),
        bwd_ex_only=time_launches(lambda: binding.halo_peft_bwd(desc, E, X, T, Wq, s_w, U, V, workspace=ws, EX=EX,
                                                                 want_gu=False, want_gv=False), it),
        bwd_adapter_gradients_only=time_launches(lambda: binding.halo_peft_bwd(desc, E, X, T, Wq, s_w, U, V, workspace=ws,
                                                                                GU=GU, GV=GV, want_ex=False), it),
        plain_fwd_frozen_weight=time_launches(lambda: binding.halo_linear_fwd(desc, X, None, state=state, Y=Y), it),
        plain_bwd_ex_only=time_launches(lambda: binding.halo_linear_bwd(desc, E, state, workspace=lws, EX=EX, want_g=False), it),
    )
    rec = dict(workload="%s: HALO-PEFT, tokens %d, frozen INT8 weight %dx%d (n x m), LoRA rank %d, HALO-%d forms of F and E, "
                        "bf16 in/out, fwd + bwd (E_X, G_U, G_V)" % (key, b, n, m, rank, cfg.level),
               b=b, m=m, n=n, rank=rank, level=cfg.level, had_block_m=hm, had_block_b=hb, ops_per_step=ops, ms_per_step=ms,
               value=ops / (ms * 1e-3) / 1e12, unit="TOPS", ms_parts=parts)
    if with_oracle:
        from oracle import halo_oracle as orc
        tokens = 512
        ts = inputs.make_linear_inputs(cfg, tokens=tokens)
        Xr, Wr, Er, Ur, Vr = (orc.bf16_bits_to_real(ts[k]) for k in ("X", "W", "E", "U", "V"))
        base = orc.forward(np.zeros((16, m), np.float32), Wr, cfg.level, hm)
        c0 = time.perf_counter()
        orc.peft_forward(Xr, base["Wq"], base["s_w"], Ur, Vr, cfg.level, hm)
        orc.peft_backward(Er, Xr, base["Wq"], base["s_w"], Ur, Vr, cfg.level, hm, tokens)
        secs = time.perf_counter() - c0
        rec["cpu_baseline"] = dict(value=ops * tokens / b / secs / 1e12, unit="TOPS", cores=blas_threads(), kind="oracle",
                                   seconds=secs, sample="the first %d of %d tokens (all features; left block = %d), "
                                   "extrapolated by operation count (numpy oracle)" % (tokens, b, tokens))
    return rec


def measure_copy(dev):
    import torch
    src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev)
    dsts = [torch.empty_like(src) for _ in range(3)]
    c = [0]

    def run():
        dsts[c[0] % 3].copy_(src)
        c[0] += 1
    ms = time_launches(run, 20)
    return 2.0 * src.numel() / (ms * 1e-3) / 1e9


def measure_mfma_ceiling(dev, real_codes):
    """INT8 MFMA rate with nothing else running, by operand data (halo_mfma_i8_probe)."""
    import torch
    from paper_2501_02625_amd import binding
    sink = torch.zeros((4,), dtype=torch.int32, device=dev)
    out = {}
    g = torch.Generator(device="cpu").manual_seed(0)
    operands = {"constant": torch.ones((4096,), dtype=torch.int8),
                "uniform_random": torch.randint(-127, 128, (4096,), dtype=torch.int8, generator=g),
                "workload_codes": real_codes}
    iters = 4096
    for name, t in operands.items():
        t = t.to(dev).contiguous()
        ops = [0.0]

        def run():
            ops[0] = binding.halo_mfma_i8_probe(t, iters, sink)
        ms = time_launches(run, 4, warm=2)
        out[name] = ops[0] / (ms * 1e-3) / 1e12
    out["unit"] = "TOP/s"
    out["what"] = "256 workgroups x 8 wavefronts x %d x 16 v_mfma_i32_32x32x32_i8 on 4 KB of operand bytes, no memory traffic" % iters
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2501_02625_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    binding.load_library()          # raises if libhalo.so is missing: there is no fallback
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    assert len(inputs.CONFIGS[args.config].linears) == 1, "--config names a single-linear workload (c2, c3)"

    if inputs.CONFIGS[args.config].peft_rank and not args.step_only:
        print("bench.py: %s is reported under `configs` of the default run; alone it runs with --step-only" % args.config,
              file=sys.stderr)
        sys.exit(2)

    if args.pmc_target:
        pmc_run(args, dev)
        return

    if args.step_only:
        if inputs.CONFIGS[args.config].peft_rank:
            rec = run_peft(args.config, args, dev, False, with_parts=False)
        else:
            rec, _, _ = run_single(args.config, args, dev, None, False, False)
        print(json.dumps({"metric": METRIC, "value": rec["value"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
                          "warmup": args.warmup, "ms_per_step": rec["ms_per_step"], "higher_is_better": True,
                          "step_only": True, "config": {"workload": rec["workload"]}}))
        return

    copy_gbs = measure_copy(dev)
    rec, L, kernels = run_single(args.config, args, dev, copy_gbs, True, not args.no_cpu_baseline)
    ceiling = measure_mfma_ceiling(dev, L.state.Wq.flatten()[:4096].cpu())

    # the kernel that takes the most time in the step: single-product timings of the two backward GEMMs are listed
    # for reference only, the step runs them as one paired launch
    in_step = [k for k in kernels if "scale reference" not in k["name"] and
               not (L.level >= 1 and k["name"] in ("gemm_ex_nn(Eq,Wq)->acc", "gemm_g_nn(EqT,Xq)->acc"))]
    dominant = max(in_step, key=lambda k: k["ms"])
    # HBM traffic of the dominant kernel from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.config)
    if os.path.exists(tpath):
        with open(tpath) as f:
            tj = json.load(f)
        tk = tj["kernels"].get(dominant["name"])
        if tk:
            traffic = tk["fetch_bytes"] + tk["write_bytes"]
            traffic_source = "profiles/traffic_%s.json (%s)" % (args.config, tj.get("measured_at", "rocprofv3 --pmc"))
    roofline = dict(kernel=dominant["name"], bound=dominant["bound"], achieved=dominant["achieved"], peak=dominant["peak"],
                    unit=dominant["unit"], frac=dominant["frac"], traffic=traffic, traffic_source=traffic_source,
                    avg_ms=dominant["ms"])
    if dominant["bound"] == "mfma":
        roofline["sustained_ceiling"] = ceiling["uniform_random"]
        roofline["frac_of_sustained_ceiling"] = dominant["achieved"] / ceiling["uniform_random"]
    hq = [k for k in kernels if k["name"].startswith("hadamard_quant_rows(W)")][0]
    hq_big = [k for k in kernels if "scale reference" in k["name"]]

    extras = {}
    for key in [k for k in args.extra_configs.split(",") if k and k != args.config]:
        cfg = inputs.CONFIGS[key]
        del L
        L = None
        torch.cuda.empty_cache()
        if key == "c5":
            r = run_mx6(key, args, dev, copy_gbs, not args.no_cpu_baseline)
        elif cfg.peft_rank:
            r = run_peft(key, args, dev, not args.no_cpu_baseline)
        elif len(cfg.linears) == 1:
            r, Lx, _ = run_single(key, args, dev, copy_gbs, True, not args.no_cpu_baseline)
            del Lx
        else:
            r = run_layer(key, args, dev, not args.no_cpu_baseline)
        extras[key] = r
        torch.cuda.empty_cache()

    out = {
        "metric": METRIC,
        "value": rec["value"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": rec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {k: rec[k] for k in ("workload", "b", "m", "n", "level", "had_block_m", "had_block_b", "ops_per_step")},
        "hadamard_quant_GBs": hq["achieved"],
        "hadamard_quant_GBs_note": "fused FWHT+absmax+INT8 kernel on W (%d x %d, the larger tensor of the step); "
                                   "at 32768 rows the same kernel reaches %s GB/s; a plain device copy reaches %.0f GB/s" % (
                                       rec["n"], rec["m"], ("%.0f" % hq_big[0]["achieved"]) if hq_big else "n/a", copy_gbs),
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": rec.get("cpu_baseline"),
        "copy_GBs": copy_gbs,
        "mfma_ceiling": ceiling,
        "configs": extras,
        "device": torch.cuda.get_device_name(0),
    }
    print(json.dumps(out))


def pmc_run(args, dev):
    """One kernel family, a few launches, nothing else: the dispatches a counter run should see."""
    import torch
    from paper_2501_02625_amd import binding, inputs
    cfg = inputs.CONFIGS[args.config]
    L = Linear(cfg, 0, dev)
    b, m, n, hm, hb, state = L.b, L.m, L.n, L.hm, L.hb, L.state
    lib = binding.load_library()
    L.fwd(binding)
    Eq_, s_e_, EqT_, s_g_ = binding.halo_quant_dual(L.E, fold_cols=state.s_w, fold_rows=state.s_x)
    acc1 = torch.empty((b, m), dtype=torch.int32, device=dev)
    acc2 = torch.empty((n, m), dtype=torch.int32, device=dev)
    sc1 = torch.rand((b,), dtype=torch.float32, device=dev)
    sc2 = torch.rand((n,), dtype=torch.float32, device=dev)
    src = torch.empty((64 << 20,), dtype=torch.uint8, device=dev)
    dst = torch.empty_like(src)
    wsd = torch.empty((lib.halo_quant_dual_workspace_bytes(b, n),), dtype=torch.uint8, device=dev)
    qd = [torch.empty((b, n), dtype=torch.int8, device=dev), torch.empty((b,), dtype=torch.float32, device=dev),
          torch.empty((n, b), dtype=torch.int8, device=dev), torch.empty((n,), dtype=torch.float32, device=dev)]
    targets = {
        "gemm_fwd": lambda: binding.halo_gemm_i8(state.Xq, state.Wq, trans_b=True, row_scale=state.s_x, col_scale=state.s_w, out=L.Y),
        "gemm_ex": lambda: binding.halo_gemm_i8(Eq_, state.Wq, trans_b=False, out_dtype=None, acc_out=acc1),
        "gemm_g": lambda: binding.halo_gemm_i8(EqT_, state.Xq, trans_b=False, out_dtype=None, acc_out=acc2),
        "gemm_pair": lambda: binding.halo_gemm_i8_pair(binding.gemm_desc(Eq_, state.Wq, trans_b=False, acc_out=acc1),
                                                       binding.gemm_desc(EqT_, state.Xq, trans_b=False, acc_out=acc2)),
        "rowquant_x": lambda: binding.halo_hadamard_quant(L.X, had_block=hm, out_q=state.Xq, out_scale=state.s_x),
        "rowquant_w": lambda: binding.halo_hadamard_quant(L.W, had_block=hm, out_q=state.Wq, out_scale=state.s_w),
        "rowquant_xw": lambda: L.fwd(binding),
        "quant_dual": lambda: binding.halo_quant_dual(L.E, fold_cols=state.s_w, fold_rows=state.s_x, out_q=qd[0], row_scale=qd[1],
                                                      out_qt=qd[2], col_scale=qd[3], workspace=wsd),
        "unrotate_ex": lambda: binding.halo_dequant_unrotate(acc1, sc1, had_block=hm, out=L.EX),
        "unrotate_g": lambda: binding.halo_dequant_unrotate(acc2, sc2, had_block=hm, out=L.G),
        "copy": lambda: dst.copy_(src),      # plain device copy of 64 MiB: calibrates FETCH_SIZE / WRITE_SIZE
    }
    fn = targets[args.pmc_target]
    for _ in range(args.steps):
        fn()
    torch.cuda.synchronize()
    print(json.dumps({"pmc_target": args.pmc_target, "launches": args.steps}))


if __name__ == "__main__":
    main()
