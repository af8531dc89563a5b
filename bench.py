#!/usr/bin/env python3
"""Decode benchmark of the multi-tenant BitDelta linear stack on one MI355X.

Workload: the linears of Llama-2-7B (32 decoder layers x q,k,v,o,gate,up,down), one fp16 base model shared by
B = 16 tenants, each tenant with its own 1-bit delta of every matrix, one decode token per tenant.  A step is
one pass over the whole stack, i.e. B tokens decoded; every layer has its own weights (25.9 GB in total), so
nothing is served from cache.  Deltas are produced by bd_compress from synthetic fine-tuned weights and, like
the base, re-laid into the serving layout (bd_tile_signs / bd_tile_base) before the timed region: compression
and re-layout are offline (their rate is reported under "extras").  --path chooses the serving path:
  tiled-fused  (default) 4 launches per layer: q,k,v in one grouped call, o, gate+up in one grouped call, down
  tiled        7 launches per layer, bd_linear_multitenant_tiled
  rowmajor     7 launches per layer, bd_linear_multitenant on the row-major tensors

Prints ONE JSON line: decode tokens/s, the HBM roofline of the decode kernel, and the CPU oracle timed on the
host cores on one layer of the same workload.

Other workloads and options (each prints one JSON line of its own):
  --workload prefill   8 tenants x 512 tokens through the matrix-core GEMM (--variant 4/5/6/7 picks the kernel; the
                       merged one-product form, variant 8, is timed beside it)
  --workload hotswap   one tenant's delta set from pinned host memory into the serving layout while B tenants decode
  --mix 6,4,3,1,1,1    a mixed decode batch (tokens per active tenant; the other resident tenants idle)
  --planes K           K sign planes per tenant (iterated compression)
  --base int8          8-bit round-to-nearest base weights
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
def measured_traffic(model, tenants, path, library_version):
    """HBM bytes per launch of the decode kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by what
    the same counters read for a plain copy of known size).  The figure lives in the rocprofv3 summary under profiles/
    (a line "traffic-record: model=.. tenants=.. path=.. library_version=.. bytes_per_launch=.."), next to the commands
    that produced it; it is reported only for the library version it was measured on, otherwise None."""
    import glob
    import re
    for f in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic.md"))):
        for line in open(f):
            if not line.startswith("traffic-record:"):
                continue
            kv = dict(re.findall(r"(\w+)=(\S+)", line))
            if (kv.get("model") == model and kv.get("path") == path and int(kv.get("tenants", -1)) == tenants
                    and int(kv.get("library_version", -1)) == library_version):
                return float(kv["bytes_per_launch"])
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--tenants", type=int, default=16, help="B: tenants = decode tokens per step")
    ap.add_argument("--layers", type=int, default=32, help="decoder layers in the stack (32 = Llama-2-7B)")
    ap.add_argument("--model", choices=["7b", "70b"], default="7b")
    ap.add_argument("--variant", type=int, default=0, help="row-major path: kernel variant (0 = library's choice)")
    ap.add_argument("--path", choices=["tiled-fused", "tiled", "rowmajor"], default="tiled-fused")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-extras", action="store_true", help="skip naive baseline, read probe, compress rate")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--per-linear", action="store_true", help="also time each linear shape on its own")
    ap.add_argument("--workload", choices=["decode", "prefill", "hotswap"], default="decode",
                    help="prefill: 8 tenants x 512 tokens on the 4096x11008 and 11008x4096 linears (matrix-core GEMM)")
    ap.add_argument("--mix", type=str, default="",
                    help="mixed decode batch: tokens per active tenant, e.g. 6,4,3,1,1,1 (tenants 0.. of the B resident "
                         "ones; the others stay idle); default: one token per tenant")
    ap.add_argument("--base", choices=["fp16", "int8"], default="fp16",
                    help="int8: 8-bit round-to-nearest base weights (one scale per output row), deltas taken against them")
    ap.add_argument("--planes", type=int, default=1,
                    help="sign planes per tenant (iterated compression); a token then takes that many of a launch's columns")
    ap.add_argument("--shared-signs", action="store_true",
                    help="diagnostic: every tenant's table entry points at tenant 0's sign tensors (same launches, same arithmetic, "
                         "same requests to L2, a third of the HBM bytes at B = 16); the reported GB/s stay the nominal ones")
    ap.add_argument("--calibrate", action="store_true",
                    help="only run a 1 GiB copy and a 1 GiB read three times: known sizes against which the "
                         "profiler's HBM byte counters are scaled")
    return ap.parse_args()


MFMA_F16_PEAK_TFLOPS = 2500.0
MERGED_VARIANT = 8


def run_prefill(args, torch, bd, synth, dev, with_variants=False):
    """8 tenants x 512 tokens through bd_linear_multitenant on an up- and a down-projection of Llama-2-7B: one
    step = both linears; reports TFLOP/s of the two products (base and delta) against the dense fp16 MFMA peak."""
    B, per = 8, 512
    T = B * per
    tok = [t for t in range(B) for _ in range(per)]
    tok_arr = bd._tok_array(tok)
    mats = []
    ws_c = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, 1, 32, 1), dev)
    for name, out, inn in [("up", 11008, 4096), ("down", 4096, 11008)]:
        base = synth.base_weight(out, inn, device=dev, tag=("pf", name))
        packed, alphas = [], []
        for t in range(B):
            ft = synth.finetuned_weight(base, tag=("pf", name, t))
            p, a = bd.compress(base, ft, workspace=ws_c)
            packed.append(p)
            alphas.append(a)
        x = synth.activations(T, inn, device=dev, tag=("pf", name))
        y = torch.empty((T, out), dtype=torch.float16, device=dev)
        ws = bd.new_workspace(bd.workspace_bytes(bd.OP_LINEAR_MULTITENANT, T, out, inn, B), dev)
        mats.append((x, base, bd.TenantTable(packed, alphas), y, ws, out, inn))

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def time_steps(variant):
        def step():
            for x, base, table, y, ws, _, _ in mats:
                bd.linear_multitenant(x, base, table, tok, y=y, tok_array=tok_arr, workspace=ws, variant=variant)
        for _ in range(max(args.warmup, 1)):
            step()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps
    ms = time_steps(args.variant)
    flops = sum(2.0 * 2.0 * T * inn * out for *_, out, inn in mats)      # base + delta products
    one_product = args.variant == MERGED_VARIANT                          # asked for by name: its own flops only
    tflops = (flops / 2 if one_product else flops) / (ms * 1e-3) / 1e12
    # The same two linears as ONE product each on W + alpha S, the sum formed in fp16 on the way to the matrix cores
    # (variant 8): half the flops, and a result that differs from the two-product form by one fp16 rounding per weight.
    ms_m = time_steps(MERGED_VARIANT)
    merged = {"ms_per_step": round(ms_m, 4), "tokens_per_s": round(T / (ms_m * 1e-3), 1),
              "TFLOP/s": round(flops / 2 / (ms_m * 1e-3) / 1e12, 1),
              "frac": round(flops / 2 / (ms_m * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
              "note": "one GEMM on W + alpha S (fp16 sum): the flops of a dense fine-tuned model only"}
    # The same step on the serving layout of the decode path (bd_linear_multitenant_tiled_gemm): one copy of the base and
    # of every delta for decode and prefill.
    tiled_mats = []
    for x, base, table, y, ws, out, inn in mats:
        ttable = bd.TiledTenantTable([bd.tile_signs(p, out, inn) for p in table.packed], table.alpha)
        ws_t = bd.new_workspace(bd.workspace_bytes(bd.OP_LINEAR_TILED_GEMM, T, out, inn, B), dev)
        tiled_mats.append((x, bd.tile_base(base), ttable, y, ws_t, out))

    def time_tiled(one_product):
        def step():
            for x, wt, ttable, y, ws_t, out in tiled_mats:
                bd.linear_multitenant_tiled_gemm(x, wt, out, ttable, tok, one_product=one_product, y=y, workspace=ws_t, tok_array=tok_arr)
        for _ in range(max(args.warmup, 1)):
            step()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            step()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps
    ms_t2, ms_t1 = time_tiled(False), time_tiled(True)
    serving_layout = {"two_products_ms_per_step": round(ms_t2, 4), "two_products_TFLOP/s": round(flops / (ms_t2 * 1e-3) / 1e12, 1),
                      "one_product_ms_per_step": round(ms_t1, 4), "one_product_tokens_per_s": round(T / (ms_t1 * 1e-3), 1),
                      "note": "bd_linear_multitenant_tiled_gemm: W and signs read from the tiled tensors the decode kernel uses"}
    del tiled_mats
    variants = None
    if with_variants:
        # the 128 x 128 tile GEMM on the up projection: one plane (variant 4), two planes per tenant, the 8-bit base
        x, base, table, y, ws, out, inn = mats[0]
        ws_g = bd.new_workspace(bd.workspace_bytes(bd.OP_LINEAR_GEMM, T, out, inn, B), dev)
        planes, alphas = [], []
        for t in range(B):
            ft = synth.finetuned_weight(base, tag=("pf", "up", t))
            p, a = bd.compress_iterated(base, ft, 2, workspace=ws_c)
            planes.append(p)
            alphas.append(a)
        ptable = bd.PlaneTable(planes, torch.stack(alphas))
        q, qs = bd.quantize_base_q8(base)
        qp, qa = [], []
        for t in range(B):
            ft = synth.finetuned_weight(base, tag=("pf", "up", t))
            p, a = bd.compress_q8(q, qs, ft, workspace=ws_c)
            qp.append(p)
            qa.append(a)
        qtable = bd.TenantTable(qp, qa)
        calls = {
            "one_plane_128x128": lambda: bd.linear_multitenant(x, base, table, tok, y=y, tok_array=tok_arr, workspace=ws, variant=4),
            "two_planes_128x128": lambda: bd.linear_multitenant_gemm_kbit(x, base, ptable, tok, y=y, workspace=ws_g, tok_array=tok_arr),
            "int8_base_128x128": lambda: bd.linear_multitenant_gemm_q8(x, q, qs, qtable, tok, y=y, workspace=ws_g, tok_array=tok_arr),
        }
        variants = {}
        for name, fn in calls.items():
            fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) / args.steps * 1e3
            variants[name] = {"us_per_launch": round(us, 1), "TFLOP/s": round(2.0 * 2.0 * T * inn * out / (us * 1e-6) / 1e12, 1)}
    return {
        **({"variants_up_projection": variants} if variants else {}),
        "merged_form": merged,
        "serving_layout": serving_layout,
        "metric": "prefill tokens/s, fused fp16 base + 1-bit delta linear, 8 tenants x 512 tokens",
        "value": round(T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 in, f32 accumulate", "data": "synthetic",
        "config": {"workload": "prefill: 8 tenants x 512 tokens, linears 4096->11008 and 11008->4096 (one step = both)",
                   "tenants": B, "tokens": T},
        "roofline": {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(tflops / MFMA_F16_PEAK_TFLOPS, 4), "traffic": None, "kernel": {4: "linear_prefill_kernel", MERGED_VARIANT: "linear_prefill_merged_kernel"}.get(args.variant, "linear_prefill_big_kernel"),
                     "flops_per_launch": flops / (4 if one_product else 2), "avg_launch_us": round(ms * 1e3 / 2, 2),
                     # counting only the flops of a dense fine-tuned model (2 T in out per linear): half of the above
                     # (all of it for the one-product kernel)
                     "achieved_useful": round(tflops if one_product else tflops / 2, 1),
                     "frac_useful": round((tflops if one_product else tflops / 2) / MFMA_F16_PEAK_TFLOPS, 4),
                     "useful_fraction_note": "one product on W + alpha S" if one_product else
                                             "half of the flops are the base product, half the +-1 delta product"},
    }


def run_hotswap(args, torch, bd, dev, incoming, k, B, step, ms_decode_alone):
    """One tenant's delta set (every matrix of the stack) from pinned host memory into the serving layout, alone and
    while the decode stack keeps running on the main stream."""
    outs, ins = [m[0] for m in incoming], [m[1] for m in incoming]
    image = bd.delta_image_build([m[2] for m in incoming], [m[3] for m in incoming], outs, ins, k, pinned=True)
    nbytes = image.numel()
    arena = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    tiled = [[torch.empty(bd.tiled_signs_bytes(o, i) // 4, dtype=torch.int32, device=dev) for _ in range(k)]
             for o, i in zip(outs, ins)]
    alphas = [torch.zeros(B * k, dtype=torch.float32, device=dev) for _ in outs]
    side = torch.cuda.Stream()

    def swap():
        bd.delta_upload(image, arena, stream=side)
        bd.delta_install(image, arena, 0, B, tiled, alphas, stream=side)

    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            fn()
            side.synchronize()
            e0.record(side)
            for _ in range(reps):
                fn()
            e1.record(side)
        side.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_upload = timed(lambda: bd.delta_upload(image, arena, stream=side), 3)
    ms_install = timed(lambda: bd.delta_install(image, arena, 0, B, tiled, alphas, stream=side), 3)
    ms_swap_alone = timed(swap, 3)
    # the same swap with decode steps running back to back on the main stream
    torch.cuda.synchronize()
    d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_swaps, n_steps = 3, 0
    d0.record()
    with torch.cuda.stream(side):
        s0.record(side)
        for _ in range(n_swaps):
            swap()
        s1.record(side)
    main_stream = torch.cuda.current_stream()
    while not s1.query():
        step()
        main_stream.synchronize()      # no backlog: every counted step overlaps the swaps
        n_steps += 1
    d1.record()
    torch.cuda.synchronize()
    ms_swap_busy = s0.elapsed_time(s1) / n_swaps
    ms_decode_busy = d0.elapsed_time(d1) / max(n_steps, 1)
    print(json.dumps({
        "metric": "delta hot swap: one tenant's delta set from pinned host memory into the serving layout, decode running",
        "value": round(ms_swap_busy, 3), "unit": "ms per swap", "n_gpus": 1, "steps": n_swaps, "warmup": 1,
        "ms_per_step": round(ms_swap_busy, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32 sign words", "data": "synthetic",
        "config": {"workload": f"llama-2-{args.model} stack, {len(outs)} matrices, {k} plane(s), image of {nbytes / 1e6:.1f} MB; "
                               f"B={B} tenants decoding meanwhile"},
        "swap": {"image_MB": round(nbytes / 1e6, 1), "upload_ms_alone": round(ms_upload, 3),
                 "upload_GBps_alone": round(nbytes / ms_upload / 1e6, 2), "install_ms_alone": round(ms_install, 3),
                 "swap_ms_alone": round(ms_swap_alone, 3), "swap_ms_while_decoding": round(ms_swap_busy, 3),
                 "host_to_device_GBps_while_decoding": round(nbytes / ms_swap_busy / 1e6, 2)},
        "decode": {"ms_per_step_alone": round(ms_decode_alone, 4), "ms_per_step_during_swaps": round(ms_decode_busy, 4),
                   "steps_during_swaps": n_steps,
                   "slowdown": round(ms_decode_busy / ms_decode_alone, 4)},
    }))


def build_stack(args, torch, bd, synth, dev, shapes, sigma, n_layers, n_res, k, q8, keep_rowmajor, tag0="L", timing=None):
    """Base weights + n_res compressed deltas per matrix for n_layers layers, resident in HBM in the serving layout
    (and row-major as well for the first keep_rowmajor layers).  Returns (layers, incoming) with
    layers[li] = [(name, out, in, base, table, w_tiled, tiled_table), ...]."""
    layers, incoming = [], []
    ws = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, 1, 32, 1), dev)
    for li in range(n_layers):
        mats = []
        for name, out, inn in shapes:
            base = synth.base_weight(out, inn, device=dev, tag=(tag0, li, name))
            if q8:
                qb, qscale = bd.quantize_base_q8(base)
            packed, alphas = [], []
            for t in range(n_res):
                ft = synth.finetuned_weight(base, sigma=sigma, tag=(tag0, li, name, t))
                if q8:
                    p, a = bd.compress_q8(qb, qscale, ft, workspace=ws)
                else:
                    p, a = bd.compress(base, ft, workspace=ws) if k == 1 else bd.compress_iterated(base, ft, k, workspace=ws)
                packed.append(p)
                alphas.append(a)
                del ft
            if args.workload == "hotswap":       # one more fine-tune per matrix: the tenant that will be swapped in
                ft = synth.finetuned_weight(base, sigma=sigma, tag=(tag0, li, name, "incoming"))
                p, a = bd.compress_iterated(base, ft, k, workspace=ws)
                incoming.append((out, inn, p.cpu(), a.cpu()))
                del ft, p
            table = bd.TenantTable(packed, alphas) if k == 1 else None
            wt = ttable = None
            if k != 1:
                wt = bd.tile_base(base)
                ttable = bd.TiledPlaneTable([[bd.tile_signs(p[j], out, inn) for j in range(k)] for p in packed],
                                            torch.stack(alphas))
                base = None
            else:
                wt = bd.tile_base_q8(qb, qscale) if q8 else bd.tile_base(base)
                tiles = [bd.tile_signs(p, out, inn) for p in packed]
                if getattr(args, "shared_signs", False):
                    tiles = [tiles[0]] * len(tiles)
                ttable = bd.TiledTenantTable(tiles, table.alpha)
                if li >= keep_rowmajor:
                    base = table = None
                elif q8:
                    base = (qb, qscale)   # the row-major 8-bit base: what bd_linear_multitenant_q8 takes
            mats.append((name, out, inn, base, table, wt, ttable))
        layers.append(mats)
    return layers, incoming


def make_plans(args, bd, layers, xs, ys, tok, tok_arr, path, k, q8):
    """One list of launch closures per layer for the given serving path."""
    plans = []
    for mats in layers:
        by = {m[0]: m for m in mats}
        plan = []
        if path == "rowmajor" and q8:
            for name, out, inn, base, table, _, _ in mats:
                plan.append(lambda inn=inn, base=base, table=table, y=ys[(name, out)]: bd.linear_multitenant_q8(
                    xs[inn], base[0], base[1], table, tok, y=y, tok_array=tok_arr))
        elif path == "rowmajor":
            for name, out, inn, base, table, _, _ in mats:
                plan.append(lambda inn=inn, base=base, table=table, y=ys[(name, out)]: bd.linear_multitenant(
                    xs[inn], base, table, tok, y=y, variant=args.variant, tok_array=tok_arr))
        elif path == "tiled":
            for name, out, inn, _, _, wt, ttable in mats:
                plan.append(lambda inn=inn, out=out, wt=wt, ttable=ttable, y=ys[(name, out)]: bd.linear_multitenant_tiled(
                    xs[inn], wt, out, ttable, tok, y=y, tok_array=tok_arr))
        else:
            def grouped(names):
                ms = [by[n] for n in names]
                yl = [ys[(m[0], m[1])] for m in ms]
                if k != 1:
                    g = bd.TiledPlaneGroup([m[5] for m in ms], [m[1] for m in ms], [m[6] for m in ms])
                    return lambda g=g, yl=yl, inn=ms[0][2]: bd.linear_multitenant_tiled_group_kbit(
                        xs[inn], g, tok, ys=yl, tok_array=tok_arr)
                g = bd.TiledGroup([m[5] for m in ms], [m[1] for m in ms], [m[6] for m in ms])
                if q8:
                    return lambda g=g, yl=yl, inn=ms[0][2]: bd.linear_multitenant_tiled_group_q8(xs[inn], g, tok, ys=yl,
                                                                                                  tok_array=tok_arr)
                return lambda g=g, yl=yl, inn=ms[0][2]: bd.linear_multitenant_tiled_group(xs[inn], g, tok, ys=yl,
                                                                                           tok_array=tok_arr)

            def single(n):
                m = by[n]
                if k != 1:
                    return lambda m=m: bd.linear_multitenant_tiled_kbit(xs[m[2]], m[5], m[1], m[6], tok,
                                                                        y=ys[(m[0], m[1])], tok_array=tok_arr)
                if q8:
                    return lambda m=m: bd.linear_multitenant_tiled_q8(xs[m[2]], m[5], m[1], m[6], tok, y=ys[(m[0], m[1])],
                                                                      tok_array=tok_arr)
                return lambda m=m: bd.linear_multitenant_tiled(xs[m[2]], m[5], m[1], m[6], tok, y=ys[(m[0], m[1])],
                                                               tok_array=tok_arr)
            plan = [grouped(["q", "k", "v"]), single("o"), grouped(["gate", "up"]), single("down")]
        plans.append(plan)
    return plans


def stack_bytes(shapes, n_layers, T, n_active, k, q8):
    """Algorithmic bytes of one pass: W once, each active delta (k planes) once, x and y of every linear."""
    P = sum(o * i for _, o, i in shapes)
    xy_bytes = sum(T * (i + o) * 2 for _, o, i in shapes)
    base_bytes = (1.0 * P + 4.0 * sum(o for _, o, _ in shapes)) if q8 else 2.0 * P   # int8: one byte per weight + a scale per row
    return n_layers * (base_bytes + n_active * k * P / 8.0 + xy_bytes)


def capture_and_time(torch, plans, steps, warmup, use_graph=True):
    """Runs the launches of `plans` once eagerly (kernel attributes are set on first use, outside any capture),
    captures them into a HIP graph, and times `steps` replays with events on the current stream.
    Returns (ms per step, step function, graph or None)."""
    def run_stack():
        for plan in plans:
            for launch in plan:
                launch()
    run_stack()
    torch.cuda.synchronize()
    graph = None
    if use_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                run_stack()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                run_stack()
        except Exception as e:   # noqa: BLE001
            print(f"bench.py: graph capture failed ({e}); launching eagerly", file=sys.stderr)
            graph = None
    step = graph.replay if graph is not None else run_stack
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    wall0 = time.time()
    e0.record()
    for _ in range(steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall = time.time() - wall0
    return e0.elapsed_time(e1) / steps, step, graph, wall


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no collective); use --gpus 1. "
              "Over several GPUs the path would shard by output rows, with one all-gather of y per linear.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2402_10193_amd import binding as bd
    from paper_2402_10193_amd import synth

    if not os.path.exists(bd.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    bd.lib()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate:
        src = torch.empty(1 << 28, dtype=torch.int32, device=dev).random_(0, 1 << 30)
        dst = torch.empty_like(src)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for _ in range(3):
            bd.probe_copy(dst, src)
            bd.probe_read(src, sink)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate": "3 x bd_probe_copy and bd_probe_read of 1 GiB"}))
        return
    if args.workload == "prefill":
        print(json.dumps(run_prefill(args, torch, bd, synth, dev, with_variants=not args.no_extras)))
        return
    B, n_layers = args.tenants, args.layers
    shapes = synth.LLAMA2_7B_LAYER if args.model == "7b" else synth.LLAMA2_70B_LAYER
    sigma = 0.002 if args.model == "7b" else 0.001
    tok = synth.one_token_per_tenant(B)
    if args.mix:
        counts = [int(c) for c in args.mix.split(",")]
        assert len(counts) <= B and all(c > 0 for c in counts), "--mix: at most B positive counts"
        tok = [t for t, c in enumerate(counts) for _ in range(c)]
        args.no_extras = args.no_cpu = True      # the baselines below are defined for one token per tenant
    T, n_active = len(tok), len(set(tok))
    k = args.planes
    q8 = args.base == "int8"
    if q8:
        assert args.path in ("tiled-fused", "rowmajor") and k == 1 and args.workload == "decode", "--base int8: tiled-fused or rowmajor decode, one plane"
        args.no_extras = args.no_cpu = True
    if k != 1:
        assert args.path == "tiled-fused", "--planes needs the tiled-fused path"
        args.no_extras = args.no_cpu = True
    if args.workload == "hotswap":
        args.no_extras = args.no_cpu = True
    tok_arr = bd._tok_array(tok)
    # The sweep over the number of tenants (in the extras) needs up to 32 of them resident; the headline run then
    # simply uses the first B.  A tenant without a token costs a launch nothing.
    sweep = (not args.no_extras) and args.model == "7b" and n_layers == 32
    n_res = max(B, 32) if sweep else B
    keep_rowmajor = n_layers if args.path == "rowmajor" else (min(4, n_layers) if not args.no_extras else 0)

    # ---- build the stack: base weights + compressed deltas per matrix, all resident in HBM
    t_setup = time.time()
    layers, incoming = build_stack(args, torch, bd, synth, dev, shapes, sigma, n_layers, n_res, k, q8, keep_rowmajor)
    xs = {inn: synth.activations(T, inn, device=dev, tag=("bench", inn)) for _, _, inn in shapes}
    ys = {(name, out): torch.empty((T, out), dtype=torch.float16, device=dev) for name, out, _ in shapes}
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    plans = make_plans(args, bd, layers, xs, ys, tok, tok_arr, args.path, k, q8)
    launches_per_step = sum(len(p) for p in plans)
    P = sum(o * i for _, o, i in shapes)
    bytes_per_step = stack_bytes(shapes, n_layers, T, n_active, k, q8)

    ms_per_step, step, graph, wall = capture_and_time(torch, plans, args.steps, args.warmup, not args.no_graph)
    tokens_per_s = T / (ms_per_step * 1e-3)
    achieved_gbs = bytes_per_step / (ms_per_step * 1e-3) / 1e9

    # distribution over single steps (a pass of its own, after the timed region: one event pair per step)
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in pairs:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in pairs)

    if args.workload == "hotswap":
        run_hotswap(args, torch, bd, dev, incoming, k, B, step, ms_per_step)
        return

    kernel_name = {"rowmajor": "linear_decode_rowmajor_kernel"}.get(args.path, "linear_decode_tiled_kernel")
    result = {
        "metric": "decode tokens/s, fused fp16 base + 1-bit delta linear stack, B tenants",
        "value": round(tokens_per_s, 2),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 in, f32 accumulate",
        "data": "synthetic",
        "config": {
            "workload": f"llama-2-{args.model} linear stack: {n_layers} layers x (q,k,v,o,gate,up,down), "
                        f"B={B} tenants, " + (f"mixed decode batch of {T} tokens ({args.mix} per active tenant), "
                                               if args.mix else "one decode token per tenant, ")
                        + (f"distinct {k}-plane delta per (tenant, matrix)" if k != 1 else "distinct 1-bit delta per (tenant, matrix)"),
            "tenants": B, "resident_tenants": n_res, "tokens": T, "active_tenants": n_active, "planes": k, "base": args.base,
            "layers": n_layers, "launches_per_step": launches_per_step,
            "launch": "hip graph replay" if graph is not None else "eager",
            "path": args.path, "kernel_variant": args.variant,
            **({"shared_signs": True} if args.shared_signs else {}),
        },
        "roofline": {
            "bound": "hbm",
            "achieved": round(achieved_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved_gbs / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(args.model, B, args.path, bd.version()) if n_layers == 32 and not args.mix and k == 1 and not q8 and not args.shared_signs else None,
            "kernel": kernel_name,
            "bytes_per_launch": round(bytes_per_step / launches_per_step, 1),
            "avg_launch_us": round(ms_per_step * 1e3 / launches_per_step, 3),
        },
        "step_ms_single": {"median": round(per_step[len(per_step) // 2], 4), "min": round(per_step[0], 4),
                           "max": round(per_step[-1], 4)},
        "wall_s_timed_region": round(wall, 4),
        "setup_s": round(t_setup, 1),
    }
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    extras = {}
    if args.per_linear:
        per = {}
        for name, out, inn in [s for s in shapes if s[0] in ("q", "k", "gate", "down")]:
            mats = [(m[3], m[4]) for L in layers for m in L if m[0] == name and m[3] is not None]
            if not mats:    # the row-major tensors are kept only with --path rowmajor
                continue
            for base, table in mats[:2]:
                bd.linear_multitenant(xs[inn], base, table, tok, y=ys[(name, out)], variant=args.variant, tok_array=tok_arr)
            torch.cuda.synchronize()
            e0.record()
            reps = 0
            for _ in range(4):
                for base, table in mats:
                    bd.linear_multitenant(xs[inn], base, table, tok, y=ys[(name, out)], variant=args.variant,
                                          tok_array=tok_arr)
                    reps += 1
            e1.record()
            e1.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            nbytes = 2.0 * out * inn + B * out * inn / 8.0 + B * (inn + out) * 2
            per[name] = {"us": round(us, 2), "GB/s": round(nbytes / us / 1e3, 1)}
        extras["per_linear_eager"] = per

    if not args.no_extras:
        # (a) read ceiling: a pure 128-bit streaming read over 4 GiB
        buf = torch.empty(1 << 30, dtype=torch.int32, device=dev)
        buf.random_(0, 1 << 30)
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        bd.probe_read(buf, sink)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            bd.probe_read(buf, sink)
        e1.record()
        e1.synchronize()
        extras["read_probe_GBs"] = round(5 * buf.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        del buf

        # (b) the naive system of the paper (Sec. 4.3): every tenant keeps a full fp16 copy of the model.  Layers 0 and 1
        # are materialised for every resident tenant and timed in turn, so that no pass finds its weights in the
        # memory-side cache; n tenants = the first n copies.
        n_naive_layers = min(2, keep_rowmajor)
        naive = []
        for li in range(n_naive_layers):
            nl = []
            for name, out, inn, base, table, _, _ in layers[li]:
                wts = [bd.materialize(base, table.packed[t], table.alpha[t:t + 1]) for t in range(n_res)]
                nl.append((name, out, inn, wts))
            naive.append(nl)

        def naive_ms_per_layer(n):
            toks = list(range(n))
            ta = bd._tok_array(toks)
            xn = {inn: xs[inn][:n] if n <= T else synth.activations(n, inn, device=dev, tag=("bench", inn, n)) for _, _, inn in shapes}
            yn = {(name, out): torch.empty((n, out), dtype=torch.float16, device=dev) for name, out, _ in shapes}
            tabs = [[(name, out, inn, bd.WeightTable(wts[:n])) for name, out, inn, wts in nl] for nl in naive]

            def run(which):
                for name, out, inn, wt in which:
                    bd.linear_naive(xn[inn], wt, toks, y=yn[(name, out)], tok_array=ta)
            for t_ in tabs:
                run(t_)
            torch.cuda.synchronize()
            reps = 3
            e0.record()
            for _ in range(reps):
                for t_ in tabs:
                    run(t_)
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) / (reps * len(tabs))

        def naive_entry(n, ms_bitdelta_step):
            ms_layer = naive_ms_per_layer(n)
            return {"ms_per_layer": round(ms_layer, 4),
                    "tokens_per_s_stack": round(n / (ms_layer * 1e-3 * n_layers), 2),
                    "GB/s": round(n * 2.0 * P / (ms_layer * 1e-3) / 1e9, 1),
                    "bitdelta_speedup": round(ms_layer / (ms_bitdelta_step / n_layers), 3),
                    "byte_ratio": round(n * 2.0 * P * n_layers / stack_bytes(shapes, n_layers, n, n, 1, False), 3)}
        if naive:
            ent = naive_entry(B, ms_per_step)
            ent["note"] = "two layers measured (B full fp16 copies each), stack figure = x layers"
            extras["naive_per_tenant_fp16"] = ent

        # (c) config 3: the sweep over the number of tenants, same stack, one token per tenant, graph replay
        def timed_stack(lyrs, shp, toks, path, steps=10, warmup=2):
            ta = bd._tok_array(toks)
            n = len(toks)
            xs_ = {inn: synth.activations(n, inn, device=dev, tag=("bench", inn, n)) for _, _, inn in shp}
            ys_ = {(name, out): torch.empty((n, out), dtype=torch.float16, device=dev) for name, out, _ in shp}
            pl = make_plans(args, bd, lyrs, xs_, ys_, toks, ta, path, 1, False)
            ms, _, g, _ = capture_and_time(torch, pl, steps, warmup, not args.no_graph)
            nb = stack_bytes(shp, len(lyrs), n, len(set(toks)), 1, False)
            gbs = nb / (ms * 1e-3) / 1e9
            del g
            return {"ms_per_step": round(ms, 4), "tokens_per_s": round(n / (ms * 1e-3), 1), "GB/s": round(gbs, 1),
                    "frac": round(gbs / HBM_PEAK_GBS, 4), "launches_per_step": sum(len(p) for p in pl)}
        if sweep and k == 1 and not q8:
            sw = {}
            for n in (1, 2, 4, 8, 32):
                ent = timed_stack(layers, shapes, list(range(n)), "tiled-fused")
                if naive:
                    nv = naive_entry(n, ent["ms_per_step"])
                    ent["naive_tokens_per_s"] = nv["tokens_per_s_stack"]
                    ent["speedup_vs_naive"] = nv["bitdelta_speedup"]
                    ent["byte_ratio"] = nv["byte_ratio"]
                sw[str(n)] = ent
            extras["tenant_sweep_7b"] = sw
            # the same stack through the other two entry points: 7 launches per layer on the tiled layout, and the
            # row-major bd_linear_multitenant (its tensors are kept for the first layers only)
            extras["path_tiled_7_launches"] = timed_stack(layers, shapes, tok, "tiled")
            if keep_rowmajor > 0:
                ent = timed_stack(layers[:keep_rowmajor], shapes, tok, "rowmajor")
                ent["layers"] = keep_rowmajor
                extras["path_rowmajor_bd_linear_multitenant"] = ent
        del naive

        # (d) the compressor: whole calls back to back (outputs and workspace allocated beforehand)
        cshape = [(n_, o, i) for n_, o, i in shapes if n_ in ("q", "gate")]
        for name, out, inn in cshape:
            cb = [synth.base_weight(out, inn, device=dev, tag=("C", j, name)) for j in range(4)]
            cf = [synth.finetuned_weight(b, sigma=sigma, tag=("C", j, name, 0)) for j, b in enumerate(cb)]
            pk = torch.empty((out, inn // 32), dtype=torch.int32, device=dev)
            al = torch.empty((1,), dtype=torch.float32, device=dev)
            wsc = bd.new_workspace(bd.workspace_bytes(bd.OP_COMPRESS, 0, out, inn, 1), dev)
            for b_, f_ in zip(cb, cf):
                bd.compress(b_, f_, packed=pk, alpha=al, workspace=wsc)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(5):
                for b_, f_ in zip(cb, cf):
                    bd.compress(b_, f_, packed=pk, alpha=al, workspace=wsc)
            e1.record()
            e1.synchronize()
            extras[f"compress_GBs_{out}x{inn}"] = round(20 * out * inn * 4.125 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
            del cb, cf
        extras["compress_GBs"] = extras.get("compress_GBs_11008x4096")
        if not q8 and k == 1:
            # the same compressor with the matrices of a layer in one call (bd_compress_batch): whole-call rate
            cb_bases = [synth.base_weight(out, inn, device=dev, tag=("L", 0, name)) for name, out, inn in shapes]
            cb_fts = [synth.finetuned_weight(b, sigma=sigma, tag=("L", 0, name, 0)) for b, (name, _, _) in zip(cb_bases, shapes)]
            ws_b = bd.new_workspace(bd.COMPRESS_BATCH_MAX * bd.workspace_bytes(bd.OP_COMPRESS, 0, 1, 32, 1), dev)
            best = None
            for _ in range(4):
                e0.record()
                bd.compress_batch(cb_bases, cb_fts, workspace=ws_b)
                e1.record()
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None or ms < best else best
            extras["compress_batch_GBs"] = round(sum(o * i for _, o, i in shapes) * 4.125 / (best * 1e-3) / 1e9, 1)
            del cb_bases, cb_fts

        if sweep and k == 1 and not q8:
            # (e) config 4: Llama-2-70B layer shapes, 32 tenants, sigma 0.001; two layers so that nothing is served from cache
            del layers, plans, step, graph
            torch.cuda.empty_cache()
            shapes70 = synth.LLAMA2_70B_LAYER
            l70, _ = build_stack(args, torch, bd, synth, dev, shapes70, 0.001, 2, 32, 1, False, 0, tag0="L70")
            extras["llama2_70b_layers"] = {str(n): timed_stack(l70, shapes70, list(range(n)), "tiled-fused", steps=20, warmup=3)
                                           for n in (16, 32)}
            extras["llama2_70b_layers"]["layers"] = 2
            del l70
            torch.cuda.empty_cache()
            # (f) config 5: prefill, 8 tenants x 512 tokens through the matrix-core GEMM
            pf = run_prefill(args, torch, bd, synth, dev)
            extras["prefill_8x512"] = {"tokens_per_s": pf["value"], "ms_per_step": pf["ms_per_step"],
                                       "TFLOP/s": pf["roofline"]["achieved"], "frac": pf["roofline"]["frac"],
                                       "TFLOP/s_fine_tuned_model_only": pf["roofline"]["achieved_useful"],
                                       "frac_fine_tuned_model_only": pf["roofline"]["frac_useful"],
                                       "merged_form": pf["merged_form"], "serving_layout": pf["serving_layout"]}
    result["extras"] = extras

    # ---- the oracle on the host cores, one layer of the same workload
    if not args.no_cpu:
        from oracle import ref
        rng = np.random.default_rng(synth.DEFAULT_SEED)
        t_cpu, layer_passes = 0.0, 0
        cpu_inputs = []
        for name, out, inn in shapes:
            wb = (rng.standard_normal((out, inn), dtype=np.float32) * 0.02).astype(np.float16)
            xb = rng.standard_normal((B, inn), dtype=np.float32).astype(np.float16)
            packed = [rng.integers(0, 2**32, size=(out, inn // 32), dtype=np.uint64).astype(np.uint32) for _ in range(B)]
            cpu_inputs.append((xb, wb, packed, np.full(B, 0.0016, dtype=np.float32)))
        while t_cpu < 10.0 and layer_passes < 64:      # about 10 s of oracle work
            for xb, wb, packed, alphas in cpu_inputs:
                t0 = time.time()
                ref.linear_multitenant(xb, wb, packed, alphas, tok)
                t_cpu += time.time() - t0
            layer_passes += 1
        result["cpu_baseline"] = {
            "value": round(B * layer_passes / (t_cpu * n_layers), 4),
            "unit": "tokens/s",
            "cores": ref.num_threads(),
            "kind": "oracle",
            "sample": f"one decoder layer at full shape (7 linears, B={B}; iid weights and sign words), {layer_passes} passes, "
                      f"{t_cpu:.2f} s of oracle time; stack rate = layer rate / {n_layers}",
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
