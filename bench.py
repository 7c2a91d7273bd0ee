#!/usr/bin/env python3
"""Benchmark of the HALO low-precision linear layer on one MI355X.

One "step" = one pass of the whole hot path on config c2 (Llama-3-8B attention projection, tokens 2048,
4096 x 4096, HALO-1): rotate+quantise X and W, INT8 forward GEMM with dequant epilogue, then both backward
products (quantise E twice, two INT8 GEMMs on the saved codes, dequantise + un-rotate).  All inputs are
resident in HBM before the timed region; outputs, saved codes and the workspace are preallocated.

Prints ONE JSON line.  `value` = 6*b*n*m INT8 operations / step time (effective TOPS of the whole layer,
quantisation and Hadamard overheads included).  `roofline` describes the kernel that takes the most time in
the step; `kernels` lists every kernel family with its own roofline fraction; `cpu_baseline` is the numpy
oracle timed on the host cores on the same workload.
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


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=100)
    p.add_argument("--warmup", type=int, default=20)
    p.add_argument("--config", default="c2", help="workload key from paper_2501_02625_amd.inputs.CONFIGS (single-linear ones)")
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--kernel-iters", type=int, default=50, help="launches per kernel for the per-kernel timings")
    p.add_argument("--pmc-target", default="",
                   help="run ONE kernel family --steps times and exit (for rocprofv3 --pmc runs): gemm_fwd, gemm_ex, "
                        "gemm_g, gemm_pair, rowquant_x, rowquant_w, quant_dual, unrotate_ex, unrotate_g, copy")
    p.add_argument("--step-only", action="store_true",
                   help="time the step loop only (no per-kernel loops, no oracle): what a kernel-trace profile of the step needs")
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


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives are part of it); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2501_02625_amd import binding, inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    binding.load_library()          # raises if libhalo.so is missing: there is no fallback
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = inputs.CONFIGS[args.config]
    assert len(cfg.linears) == 1, "bench.py times single-linear configs"
    lin = cfg.linears[0]
    b, m, n, level = cfg.tokens, lin.m, lin.n, cfg.level
    host = inputs.make_linear_inputs(cfg, need_error=True)
    to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    X, W, E = to_dev(host["X"]), to_dev(host["W"]), to_dev(host["E"])

    desc = binding.make_desc(b, m, n, level, torch.bfloat16)
    hm = min(m & -m, 4096) if level >= 1 else 0
    hb = (b & -b) if level >= 2 else 0
    state = binding.LinearState(torch.empty((b, m), dtype=torch.int8, device=dev),
                                torch.empty((b,), dtype=torch.float32, device=dev),
                                torch.empty((n, m), dtype=torch.int8, device=dev),
                                torch.empty((n,), dtype=torch.float32, device=dev))
    Y = torch.empty((b, n), dtype=torch.bfloat16, device=dev)
    EX = torch.empty((b, m), dtype=torch.bfloat16, device=dev)
    G = torch.empty((n, m), dtype=torch.bfloat16, device=dev)
    ws = torch.empty((binding.halo_linear_workspace_bytes(desc),), dtype=torch.uint8, device=dev)

    def step():
        binding.halo_linear_fwd(desc, X, W, state=state, Y=Y)
        binding.halo_linear_bwd(desc, E, state, workspace=ws, EX=EX, G=G)

    if args.pmc_target:
        # One kernel family, a few launches, nothing else: the dispatches a counter run should see.
        Eq_ = torch.randint(-127, 128, (b, n), dtype=torch.int8, device=dev)
        EqT_ = torch.randint(-127, 128, (n, b), dtype=torch.int8, device=dev)
        acc1 = torch.empty((b, m), dtype=torch.int32, device=dev)
        acc2 = torch.empty((n, m), dtype=torch.int32, device=dev)
        sc1 = torch.rand((b,), dtype=torch.float32, device=dev)
        sc2 = torch.rand((n,), dtype=torch.float32, device=dev)
        binding.halo_linear_fwd(desc, X, W, state=state, Y=Y)
        src = torch.empty((64 << 20,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        wsd = torch.empty((binding.load_library().halo_quant_dual_workspace_bytes(b, n),), dtype=torch.uint8, device=dev)
        qd = [torch.empty((b, n), dtype=torch.int8, device=dev), torch.empty((b,), dtype=torch.float32, device=dev),
              torch.empty((n, b), dtype=torch.int8, device=dev), torch.empty((n,), dtype=torch.float32, device=dev)]
        targets = {
            "gemm_fwd": lambda: binding.halo_gemm_i8(state.Xq, state.Wq, trans_b=True, row_scale=state.s_x, col_scale=state.s_w, out=Y),
            "gemm_ex": lambda: binding.halo_gemm_i8(Eq_, state.Wq, trans_b=False, out_dtype=None, acc_out=acc1),
            "gemm_g": lambda: binding.halo_gemm_i8(EqT_, state.Xq, trans_b=False, out_dtype=None, acc_out=acc2),
            "gemm_pair": lambda: binding.halo_gemm_i8_pair(binding.gemm_desc(Eq_, state.Wq, trans_b=False, acc_out=acc1),
                                                           binding.gemm_desc(EqT_, state.Xq, trans_b=False, acc_out=acc2)),
            "rowquant_x": lambda: binding.halo_hadamard_quant(X, had_block=hm, out_q=state.Xq, out_scale=state.s_x),
            "rowquant_w": lambda: binding.halo_hadamard_quant(W, had_block=hm, out_q=state.Wq, out_scale=state.s_w),
            "quant_dual": lambda: binding.halo_quant_dual(E, fold_cols=state.s_w, fold_rows=state.s_x, out_q=qd[0], row_scale=qd[1],
                                                          out_qt=qd[2], col_scale=qd[3], workspace=wsd),
            "unrotate_ex": lambda: binding.halo_dequant_unrotate(acc1, sc1, had_block=hm, out=EX),
            "unrotate_g": lambda: binding.halo_dequant_unrotate(acc2, sc2, had_block=hm, out=G),
            "copy": lambda: dst.copy_(src),      # plain device copy of 64 MiB: calibrates FETCH_SIZE / WRITE_SIZE
        }
        fn = targets[args.pmc_target]
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"pmc_target": args.pmc_target, "launches": args.steps}))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ops = 6.0 * b * n * m
    value = ops / (ms_per_step * 1e-3) / 1e12

    if args.step_only:
        print(json.dumps({"metric": "HALO linear fwd+bwd INT8 TOPS at Llama-3-8B shapes; Hadamard+quant GB/s",
                          "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": ms_per_step, "higher_is_better": True, "step_only": True}))
        return

    # ---------------------------------------------------------------- per-kernel timings (HIP events)
    it = args.kernel_iters
    kernels = []

    def add_gemm(name, A, B, trans_b, M, N, K, **kw):
        ms = time_launches(lambda: binding.halo_gemm_i8(A, B, trans_b=trans_b, **kw), it)
        tops = 2.0 * M * N * K / (ms * 1e-3) / 1e12
        kernels.append(dict(name=name, bound="mfma", ms=ms, achieved=tops, peak=INT8_PEAK_TOPS, unit="TOP/s",
                            frac=tops / INT8_PEAK_TOPS, shape=[M, N, K]))

    Eq = torch.randint(-127, 128, (b, n), dtype=torch.int8, device=dev)
    EqT = torch.randint(-127, 128, (n, b), dtype=torch.int8, device=dev)
    acc_bm = torch.empty((b, m), dtype=torch.int32, device=dev)
    acc_nm = torch.empty((n, m), dtype=torch.int32, device=dev)
    add_gemm("gemm_fwd_nt(Xq,Wq)->Y", state.Xq, state.Wq, True, b, n, m, row_scale=state.s_x, col_scale=state.s_w, out=Y)
    if level == 0:
        add_gemm("gemm_ex_nn(Eq,Wq)->EX", Eq, state.Wq, False, b, m, n, out=EX)
        add_gemm("gemm_g_nn(EqT,Xq)->G", EqT, state.Xq, False, n, m, b, out=G)
    else:
        add_gemm("gemm_ex_nn(Eq,Wq)->acc", Eq, state.Wq, False, b, m, n, out_dtype=None, acc_out=acc_bm)
        add_gemm("gemm_g_nn(EqT,Xq)->acc", EqT, state.Xq, False, n, m, b, out_dtype=None, acc_out=acc_nm)
        # what halo_linear_bwd actually launches: both products in one kernel
        g1 = binding.gemm_desc(Eq, state.Wq, trans_b=False, acc_out=acc_bm)
        g2 = binding.gemm_desc(EqT, state.Xq, trans_b=False, acc_out=acc_nm)
        ms = time_launches(lambda: binding.halo_gemm_i8_pair(g1, g2), it)
        tops = 4.0 * b * m * n / (ms * 1e-3) / 1e12
        kernels.append(dict(name="gemm_bwd_pair(E_X,G)->acc", bound="mfma", ms=ms, achieved=tops, peak=INT8_PEAK_TOPS,
                            unit="TOP/s", frac=tops / INT8_PEAK_TOPS, shape=[[b, m, n], [n, m, b]]))

    def add_hbm(name, fn_for, bytes_per_launch, nbuf):
        # rotate over nbuf distinct buffer sets so the 256 MB last-level cache cannot hold the working set
        fns = [fn_for(i) for i in range(nbuf)]
        counter = [0]

        def run():
            fns[counter[0] % nbuf]()
            counter[0] += 1
        ms = time_launches(run, max(it, nbuf * 2))
        gbs = bytes_per_launch / (ms * 1e-3) / 1e9
        kernels.append(dict(name=name, bound="hbm", ms=ms, achieved=gbs, peak=HBM_PEAK_GBS, unit="GB/s",
                            frac=gbs / HBM_PEAK_GBS, bytes=bytes_per_launch, rotating_buffers=nbuf))

    def nrot(nbytes):
        return max(2, int((768 << 20) // max(nbytes, 1)) + 1)

    # row rotate+quantise of X (F1) and W (F2): 2 B read + 1 B written per element + 4 B per row
    for nm, T, rows in (("hadamard_quant_rows(X)", X, b), ("hadamard_quant_rows(W)", W, n)):
        nbytes = rows * m * 3 + rows * 4
        k = nrot(nbytes)
        srcs = [T] + [T.clone() for _ in range(k - 1)]
        qs = [torch.empty((rows, m), dtype=torch.int8, device=dev) for _ in range(k)]
        ss = [torch.empty((rows,), dtype=torch.float32, device=dev) for _ in range(k)]
        add_hbm(nm, lambda i, srcs=srcs, qs=qs, ss=ss: (lambda: binding.halo_hadamard_quant(
            srcs[i], had_block=hm, out_q=qs[i], out_scale=ss[i])), nbytes, k)
        del srcs, qs, ss
    # the same kernel on a tensor large enough to amortise launch and ramp (scale reference, not part of the step)
    if hm:
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
    wsq = torch.empty((max(1, binding.load_library().halo_hadamard_quant_workspace_bytes(b, n, 0, hb)),), dtype=torch.uint8, device=dev)
    add_hbm("hadamard_quant_rows(E,fold=s_w%s)" % (",left" if hb else ""), lambda i: (lambda: binding.halo_hadamard_quant(
        srcs[i], had_block_left=hb, fold=state.s_w, out_q=qs[i], out_scale=ss[i], workspace=wsq)), nbytes, k)
    qts = [torch.empty((n, b), dtype=torch.int8, device=dev) for _ in range(k)]
    sts = [torch.empty((n,), dtype=torch.float32, device=dev) for _ in range(k)]
    wsc = torch.empty((n * 4 + 256,), dtype=torch.uint8, device=dev)
    add_hbm("hadamard_quant_cols_t(E,fold=s_x)", lambda i: (lambda: binding.halo_hadamard_quant(
        srcs[i], axis=binding.HALO_QUANT_COLS_T, fold=state.s_x, out_q=qts[i], out_scale=sts[i], workspace=wsc)),
        b * n * 3 + n * 4, k)
    if level <= 1:
        wsd = torch.empty((binding.load_library().halo_quant_dual_workspace_bytes(b, n),), dtype=torch.uint8, device=dev)
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
            wsu = torch.empty((max(1, binding.load_library().halo_dequant_unrotate_workspace_bytes(rows, m, left)),),
                              dtype=torch.uint8, device=dev)
            add_hbm(nm, lambda i, accs=accs, outs=outs, scale=scale, wsu=wsu, left=left: (lambda: binding.halo_dequant_unrotate(
                accs[i], scale, had_block=hm, had_block_left=left, out=outs[i], workspace=wsu)), nbytes, k)
            del accs, outs

    # the kernel that takes the most time in the step: single-product timings of the two backward GEMMs are listed
    # for reference only, the step runs them as one paired launch
    in_step = [k for k in kernels if "scale reference" not in k["name"] and
               not (level >= 1 and k["name"] in ("gemm_ex_nn(Eq,Wq)->acc", "gemm_g_nn(EqT,Xq)->acc"))]
    dominant = max(in_step, key=lambda k: k["ms"])
    # HBM traffic of the dominant kernel from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary (config c2 only)
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic_%s.json" % args.config)
    if os.path.exists(tpath):
        with open(tpath) as f:
            tk = json.load(f)["kernels"].get(dominant["name"])
        if tk:
            traffic = tk["fetch_bytes"] + tk["write_bytes"]
    roofline = dict(kernel=dominant["name"], bound=dominant["bound"], achieved=dominant["achieved"], peak=dominant["peak"],
                    unit=dominant["unit"], frac=dominant["frac"], traffic=traffic, avg_ms=dominant["ms"])
    hq = [k for k in kernels if k["name"].startswith("hadamard_quant_rows(W)")][0]
    hq_big = [k for k in kernels if "scale reference" in k["name"]]

    # ---------------------------------------------------------------- oracle on the host cores
    cpu_baseline = None
    if not args.no_cpu_baseline:
        from oracle import halo_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            blas_threads = 1
        Xr, Wr, Er = (orc.bf16_bits_to_real(host[k]) for k in ("X", "W", "E"))
        c0 = time.perf_counter()
        f = orc.forward(Xr, Wr, level, hm)
        orc.backward_input(Er, f["Wq"], f["s_w"], level, hm, hb)
        orc.backward_weight(Er, f["Xq"], f["s_x"], level, hm)
        c1 = time.perf_counter()
        cpu_baseline = dict(value=ops / (c1 - c0) / 1e12, unit="TOPS", cores=blas_threads, kind="oracle",
                            seconds=c1 - c0,
                            sample="the full %s step once (numpy oracle; elementwise parts single-threaded, "
                                   "integer GEMMs carried by a %d-thread fp64 BLAS matmul)" % (args.config, blas_threads))

    out = {
        "metric": "HALO linear fwd+bwd INT8 TOPS at Llama-3-8B shapes; Hadamard+quant GB/s",
        "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: tokens %d, linear %dx%d (n x m), HALO-%d, INT8, bf16 in/out, fwd + both bwd products"
                               % (args.config, b, n, m, level),
                   "b": b, "m": m, "n": n, "level": level, "had_block_m": hm, "had_block_b": hb,
                   "ops_per_step": ops},
        "hadamard_quant_GBs": hq["achieved"],
        "hadamard_quant_GBs_note": "fused FWHT+absmax+INT8 kernel on W (%d x %d, the larger tensor of the step); "
                                   "at 32768 rows the same kernel reaches %s GB/s" % (
                                       n, m, ("%.0f" % hq_big[0]["achieved"]) if hq_big else "n/a"),
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu_baseline,
        "device": torch.cuda.get_device_name(0),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
