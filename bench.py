#!/usr/bin/env python3
"""Benchmark of the client-side ZGR step on one MI355X.

One step = the whole hot path on one synthetic batch already resident in HBM:
perturb +eps Z, forward, perturb -2 eps Z, forward, restore +eps Z, form g,
update theta <- theta - lr g Z (four streaming passes over all parameters and
two forward passes).  Prints one JSON line with the throughput, the roofline
of the dominant kernel (HIP-event timed inside the timed region) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

COPY_BYTES = 1 << 30
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "cfg5_hbm_traffic.json")
HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


ALU_PEAK_DATASHEET = 256 * 4 * 32 * 2.4e9 / 1e12   # T lane-instr/s: 32 lanes per SIMD at 2.4 GHz (157.3 TFLOP/s fp32 at 2 flops per FMA)


def load_traffic():
    """Per-launch counter figures of the committed counter runs (HBM bytes fetched / written, vector instructions),
    or {} when the kernel sources changed since they were taken."""
    try:
        from paper_2601_12917_amd.build import source_digest
        rec = json.load(open(TRAFFIC_FILE))
        return rec["kernels"] if rec.get("source_digest") == source_digest() else {}
    except Exception:
        return {}


def kernel_valu(traffic, prefix):
    """SQ_INSTS_VALU (wave instructions) per launch of the kernels whose name starts with prefix, or None."""
    sel = [v for k, v in traffic.items() if k.startswith(prefix) and "valu_insts" in v]
    n = sum(v["launches"] for v in sel)
    return sum(v["valu_insts"] * v["launches"] for v in sel) / n if n else None


def measured_ceilings(torch, B, dtype_code):
    """Live on this machine: wave64 issue rate of a simple vector instruction (v_fma_f32, 8 waves per SIMD), the
    bare in-place read-modify-write stream over 1 GiB of the storage type, and the matrix core alone (bf16 32x32x16
    on register operands, 4 accumulators, one wave per SIMD) with the clock the chip holds under it."""
    from paper_2601_12917_amd import ceilings as Cl
    lib = B.lib()
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    cpi, ghz, rate = Cl.issue_rate(lib, B, torch, 0, 1, 8, n_cu=n_cu)
    gbs, _ = Cl.stream_rate(lib, B, torch, 1 << 30, dtype_code, 0, n_cu * 8)
    _, mghz, mrate = Cl.issue_rate(lib, B, torch, Cl.N_VECTOR_OPS, 4, 1, iters=4096, n_cu=n_cu)
    return {"simple_issue_T_lane_instr_per_s": rate * 64 / 1e12, "simple_issue_cycles_per_instruction": cpi, "shader_ghz": ghz, "rmw_stream_GBs": gbs,
            "mfma_bf16_alone_TFLOPs": mrate * Cl.MFMA_FLOPS / 1e12, "mfma_bf16_alone_ghz": mghz}


def forward_gemm_flops(cfg):
    """Algorithmic FLOPs of the GEMM launches of one forward pass (linear layers + vocabulary projection)."""
    M, d, ff = cfg.batch * cfg.seq, cfg.d_model, cfg.d_ff
    per_layer = 2.0 * M * (4 * d * d + 2 * d * ff)
    head = 2.0 * M * d * cfg.vocab if cfg.arch == 1 else 0.0      # the classifier's head is a reduction kernel, not a GEMM launch
    return cfg.n_layer * per_layer + head


def kernel_traffic(traffic, prefix):
    """Measured HBM bytes (fetch + write) per launch, averaged over the kernels whose name starts with prefix."""
    sel = [v for k, v in traffic.items() if k.startswith(prefix)]
    n = sum(v["launches"] for v in sel)
    if not n:
        return None
    return sum((v["fetch_bytes"] + v["write_bytes"]) * v["launches"] for v in sel) / n


def cpu_baseline(cfg, specs, budget_note=True):
    """Times the oracle (as it stands) on a bounded sample of the workload and scales to steps/s."""
    import zgr_inputs as I
    from oracle import forward as F
    from oracle import perturbation as P
    threads = os.cpu_count() or 1
    try:
        import threadpoolctl
        infos = threadpoolctl.threadpool_info()
        if infos:
            threads = max(i.get("num_threads", 1) for i in infos)
    except Exception:
        pass
    d, ff, V, T = cfg.d_model, cfg.d_ff, cfg.vocab, cfg.seq
    rng = np.random.default_rng(0)
    # (i) one perturbation pass over the guided matrices of one block
    layer0 = [sp for sp in specs if sp.guided and sp.layer == 0]
    t_pass, sampled = 0.0, 0
    for sp in layer0:
        q, _ = np.linalg.qr(rng.standard_normal((sp.rows, cfg.k)))
        U = q.astype(np.float32)
        W = (rng.standard_normal((sp.rows, sp.cols)) * 0.02).astype(np.float32)
        t0 = time.perf_counter()
        Z = P.hybrid_z(cfg.seed, 0, sp.tensor_id, sp.rows, sp.cols, U, cfg.k, cfg.alpha)
        P.axpy_inplace_value(W, np.float32(cfg.eps), Z, cfg.dtype)
        t_pass += time.perf_counter() - t0
        sampled += sp.numel
        del Z, W
    total_params = sum(s.numel for s in specs)
    # (ii) two transformer blocks + the vocabulary projection and loss on a quarter of the batch
    nb, nl = max(1, cfg.batch // 4), min(2, cfg.n_layer)
    one = I.shrink(cfg, name="cpu_sample", n_layer=nl, batch=nb)
    sspecs = I.tensor_specs(one)
    Pd = {s.name: (rng.standard_normal((s.rows, s.cols)) * 0.02) for s in sspecs}
    for n in [f"l{i}.ln1_g" for i in range(nl)] + [f"l{i}.ln2_g" for i in range(nl)] + ["lnf_g"]:
        Pd[n] = Pd[n] + 1.0
    tok = rng.integers(0, V, size=(nb, T))
    lm = cfg.arch == I.ARCH_DECODER_LM
    lengths = None if lm else rng.integers(32, T + 1, size=(nb,))
    t0 = time.perf_counter()
    x = Pd["tok_emb"][tok] + Pd["pos_emb"][:T][None]
    for i in range(nl):
        x = F.block(x, Pd, i, cfg.n_head, lm, lengths, cfg.ln_eps, cfg.act, cfg.post_ln)
    t_layers = time.perf_counter() - t0
    t0 = time.perf_counter()
    h = F.layer_norm(x, Pd["lnf_g"], Pd["lnf_b"], cfg.ln_eps)
    if lm:
        logp = F.log_softmax(h[:, :-1] @ Pd["tok_emb"].T)
        float(-np.take_along_axis(logp, tok[:, 1:, None], axis=-1).mean())
    else:
        logp = F.log_softmax(h[:, 0] @ Pd["cls_w"].T + Pd["cls_b"].reshape(-1))
        float(-logp[:, 0].mean())
    t_head = time.perf_counter() - t0
    fwd = (cfg.batch / nb) * (cfg.n_layer / nl * t_layers + t_head)
    step_s = 4.0 * t_pass * total_params / sampled + 2.0 * fwd
    return {"value": 1.0 / step_s, "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": (f"one perturbation pass over the {len(layer0)} guided matrices of one block ({sampled} parameters, {t_pass:.2f} s) scaled to "
                       f"{total_params} parameters x 4 passes; {nl} blocks ({t_layers:.2f} s) and the final projection + loss ({t_head:.2f} s) on "
                       f"{nb} sequences of {T} tokens, scaled to {cfg.n_layer} blocks x {cfg.batch} sequences x 2 forwards")}


def gemm_shapes(args, torch, I, B):
    """Every projection shape of the config's forward pass through zgr_debug_gemm, one at a time: [M, K] x [N, K]^T with the
    epilogue the forward uses (0 bias + store, 1 bias + GELU, 2 bias + residual add into fp32).  The fused cross-entropy
    product has no debug entry; it is timed inside the step only."""
    import ctypes as C
    cfg = I.CONFIGS[args.config]
    if cfg.arch == I.ARCH_LINEAR_LSQ:
        print("bench.py --gemm-shapes: needs a transformer config", file=sys.stderr)
        sys.exit(2)
    dt = args.gemm_dtype or cfg.dtype            # the config's shapes in either storage type
    tdt, code = (torch.bfloat16, 1) if dt == "bf16" else (torch.float32, 0)
    if not os.path.exists(B.LIB_PATH):
        from paper_2601_12917_amd.build import build
        build()
    lib = B.lib()
    dev = torch.device("cuda:0")
    M, d, ff = cfg.batch * cfg.seq, cfg.d_model, cfg.d_ff
    shapes = [("qkv", M, 3 * d, d, 0), ("attention output", M, d, d, 2), ("fc1 + gelu", M, ff, d, 1), ("fc2", M, d, ff, 2)]
    g = torch.Generator(device="cpu").manual_seed(0)
    st = torch.cuda.current_stream().cuda_stream
    rows = []
    # two rounds over the shapes, the second one kept: the first launches of a fresh process run while the clock ramps
    for rnd, (name, m, n, k, epi) in [(r, sh) for r in range(2) for sh in shapes]:
        A = (torch.randn(m, k, generator=g) * 0.5).to(tdt).to(dev)
        W = (torch.randn(n, k, generator=g) * 0.05).to(tdt).to(dev)
        bias = (torch.randn(n, generator=g) * 0.1).to(tdt).to(dev)
        out = torch.zeros(m, n, device=dev, dtype=torch.float32 if epi == 2 else tdt)
        def run():
            B.check(lib.zgr_debug_gemm(code, A.data_ptr(), W.data_ptr(), bias.data_ptr(), out.data_ptr(), epi, m, n, k, st))
        def timed(fn, reps=max(args.steps, 20)):
            for _ in range(max(args.warmup, 3)):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps * 1e3
        us = timed(run)
        row = {"shape": name, "M": m, "N": n, "K": k, "epilogue": epi, "us": us, "tflops": 2.0 * m * n * k / us / 1e6, "launches_per_forward": cfg.n_layer}
        if args.with_library:
            lus = timed(lambda: torch.matmul(A, W.t()))
            row["library_us"] = lus
            row["library_tflops"] = 2.0 * m * n * k / lus / 1e6
        if rnd:
            rows.append(row)
    tot_us = sum(r["us"] * r["launches_per_forward"] for r in rows)
    tot_fl = sum(2.0 * r["M"] * r["N"] * r["K"] * r["launches_per_forward"] for r in rows)
    print(json.dumps({"metric": "forward GEMM shapes", "config": {"workload": cfg.name}, "dtype": dt, "data": "synthetic (random operands)",
                      "shapes": rows, "weighted_tflops": tot_fl / tot_us / 1e6, "peak_tflops": MFMA_PEAK_TFLOPS[dt]}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--gauss-bits", type=int, default=32)
    ap.add_argument("--non-guided", action="store_true", help="non-guided round of Algorithm 1: no bases, Z = G for every tensor")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true", help="also run the plain 1 GiB copy kernel that HBM traffic counters are scaled by")
    ap.add_argument("--no-profile", action="store_true", help="leave the HIP-event timing of kernel classes off")
    ap.add_argument("--q4-basis", action="store_true",
                    help="send the bases compressed: quantise every basis to 4-bit codes on the device and let the kernels restore them while loading")
    ap.add_argument("--stream-bases", action="store_true",
                    help="keep the bases in pinned host memory and stream them layer by layer during every pass (with --q4-basis: as 4-bit codes)")
    ap.add_argument("--batched-update", type=int, default=4,
                    help="also time zgr_apply_updates over this many (step, g) pairs against as many zgr_apply_update calls (0: skip)")
    ap.add_argument("--no-fused-line", action="store_true",
                    help="skip the second, shorter measurement with config.fuse_restore_update = 1 (three passes over the parameters per step)")
    ap.add_argument("--profile-every", type=int, default=5,
                    help="HIP events bracket every kernel launch on one timed step in this many (two event records per "
                         "launch cost about 8 %% of a step, so they are sampled inside the timed region rather than kept on)")
    ap.add_argument("--act", choices=["gelu", "relu"], default=None, help="feed-forward activation (default: the config's, erf-GELU)")
    ap.add_argument("--post-ln", action="store_true", help="post-LayerNorm blocks (LayerNorm after each residual sum and on the embeddings)")
    ap.add_argument("--batch", type=int, default=None, help="sequences per batch (default: the config's)")
    ap.add_argument("--seq", type=int, default=None, help="tokens per sequence (default: the config's; at most the model's max_pos)")
    ap.add_argument("--cloud", action="store_true",
                    help="also time the cloud block of Algorithm 1 on the same model and batch: one backward pass, and the basis of one matrix from three gradient snapshots")
    ap.add_argument("--gemm-shapes", action="store_true",
                    help="instead of the step: time each forward GEMM shape of the config on its own (random bf16 operands, HIP events) and print one JSON line")
    ap.add_argument("--gemm-dtype", choices=["bf16", "f32"], default=None, help="with --gemm-shapes: storage type of the operands (default: the config's)")
    ap.add_argument("--with-library", action="store_true", help="with --gemm-shapes: also time torch.matmul (the vendor library) on the same operands, as context")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import zgr_inputs as I
    from paper_2601_12917_amd import binding as B
    from paper_2601_12917_amd.workloads import inputs_of, make_batch_arrays, make_session, session_batch
    if args.gemm_shapes:
        return gemm_shapes(args, torch, I, B)
    if not os.path.exists(B.LIB_PATH):
        from paper_2601_12917_amd.build import build
        build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    cfg = I.CONFIGS[args.config]
    if args.act is not None or args.post_ln:
        cfg = I.shrink(cfg, act=args.act or cfg.act, post_ln=bool(args.post_ln) or cfg.post_ln)
    if args.batch is not None or args.seq is not None:
        cfg = I.shrink(cfg, batch=args.batch or cfg.batch, seq=args.seq or cfg.seq)
        if cfg.batch < 1 or cfg.seq < 2 or cfg.seq > cfg.max_pos:
            print("bench.py: --batch / --seq outside the model's limits (seq <= max_pos = %d)" % cfg.max_pos, file=sys.stderr)
            sys.exit(2)
    t0 = time.perf_counter()
    specs, values, bases = inputs_of(cfg)
    if args.non_guided:
        bases = [None] * len(bases)
        for sp in specs:
            sp.guided = False
    arrays = make_batch_arrays(cfg)
    sess = make_session(cfg, specs, values, bases, bits=args.gauss_bits)
    batch = session_batch(sess, cfg, arrays)
    if args.stream_bases:
        layers = {}
        for i, sp in enumerate(specs):
            if sp.guided and bases[i] is not None:
                layers.setdefault(sp.layer, []).append(i)
        for layer, idx in layers.items():
            if args.q4_basis:
                q = [sess.quantize_basis(bases[i], cfg.k) for i in idx]
                sess.set_layer_bases_host(idx, [x[0] for x in q], cfg.k, codes=True, lams=[x[1] for x in q], deltas=[x[2] for x in q])
            else:
                sess.set_layer_bases_host(idx, [bases[i] for i in idx], cfg.k)
    elif args.q4_basis:
        for i, sp in enumerate(specs):
            if sp.guided:
                sess.compress_basis(i)
    setup_s = time.perf_counter() - t0

    def one_step(i):
        lp, lm, g = sess.step(i, batch)
        sess.apply_update(i, g, cfg.lr)
        return lp, lm, g

    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()
    lib = B.lib()
    every = max(1, args.profile_every)
    profiled_steps = 0
    if not args.no_profile:
        sess.profile_enable(True)          # clears the totals
        lib.zgr_profile_pause(sess.ctx, 1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    last = None
    for i in range(args.steps):
        sample = (not args.no_profile) and (i % every == every - 1 or args.steps < every and i == args.steps - 1)
        if sample:
            lib.zgr_profile_pause(sess.ctx, 0)
            profiled_steps += 1
        last = one_step(args.warmup + i)
        if sample:
            lib.zgr_profile_pause(sess.ctx, 1)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = sess.profile_read() if not args.no_profile else {}
    if args.calibrate_copy:
        src = torch.zeros(COPY_BYTES, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            B.check(B.lib().zgr_debug_copy(dst.data_ptr(), src.data_ptr(), COPY_BYTES, torch.cuda.current_stream().cuda_stream))
        torch.cuda.synchronize()
        del src, dst
    traffic = load_traffic()
    ms_per_step = 1e3 * elapsed / args.steps
    steps_per_s = args.steps / elapsed

    es = 4 if cfg.dtype == "f32" else 2
    guided_elems = sum(s.numel for s in specs if s.guided)
    flat_elems = sum(s.numel for s in specs if not s.guided)
    u_bytes = sum(s.rows * cfg.k * (0.5 if args.q4_basis else 4) for s in specs if s.guided)
    out = {
        "metric": "ZGR steps/sec", "value": steps_per_s, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {I.CONFIGS[args.config].n_layer}-layer d={cfg.d_model} {'decoder' if cfg.arch == I.ARCH_DECODER_LM else 'encoder classifier'}, batch {cfg.batch} x seq {cfg.seq}, "
                               f"{'ReLU feed-forward, ' if cfg.act == 'relu' else ''}{'post-LayerNorm blocks, ' if cfg.post_ln else ''}guided rank k={cfg.k} (basis sent with {cfg.k_full} columns{', 4-bit codes' if args.q4_basis else ''}{', streamed from host memory per layer' if args.stream_bases else ''}), gauss_bits={args.gauss_bits}"
                   if cfg.arch != I.ARCH_LINEAR_LSQ else f"{cfg.name}: linear least squares {cfg.lsq_out}x{cfg.lsq_in}",
                   "params": int(guided_elems + flat_elems), "tokens_per_step": int(cfg.batch * max(cfg.seq, 1))},
        "tokens_per_s": steps_per_s * cfg.batch * max(cfg.seq, 1),
        "last_losses": None if last is None else [last[0], last[1], last[2]],
        "setup_s": setup_s, "profiled_steps": profiled_steps,
    }
    if prof:
        kern = {}
        for name, (ms, n) in prof.items():
            if n:
                kern[name] = {"ms_total": ms, "launches": int(n), "ms_avg": ms / n}
        out["kernel_ms"] = kern
        # perturbation pass over the guided matrices: read + write every element once, plus one read of U
        if "perturb_tile" in kern:
            k1 = kern["perturb_tile"]
            bytes_per_launch = 2.0 * guided_elems * es + u_bytes
            gbs = bytes_per_launch / (k1["ms_avg"] * 1e-3) / 1e9
            out["roofline_perturb"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                                       "traffic": kernel_traffic(traffic, "perturb_tile"), "kernel": "perturb_tile_mfma_kernel" if cfg.k >= 16 else "perturb_tile_kernel",
                                       "bytes_per_launch": bytes_per_launch}
        if "perturb_flat" in kern:
            k1 = kern["perturb_flat"]
            gbs = 2.0 * flat_elems * es / (k1["ms_avg"] * 1e-3) / 1e9
            out["roofline_perturb_flat"] = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                                            "traffic": kernel_traffic(traffic, "perturb_flat"), "kernel": "perturb_flat_kernel"}
        # What really bounds the perturbation passes: vector-ALU issue.  Achieved = vector instructions executed (the
        # SQ_INSTS_VALU counter of the committed counter run, valid while the kernel sources are unchanged) over the
        # measured launch time; peak = the issue rate of a simple wave64 instruction measured on this machine just now
        # (the data-sheet figure, 32 lanes per SIMD at 2.4 GHz, beside it).  The mix also holds half-rate multiplies and
        # conversions and quarter-rate transcendentals, so 1.0 is not reachable; profiles/mi355x_ceilings.md has the rates.
        ceil = measured_ceilings(torch, B, 0 if cfg.dtype == "f32" else 1)
        out["ceilings"] = ceil
        for name, elems, key in (("perturb_tile", guided_elems, "roofline_perturb"), ("perturb_flat", flat_elems, "roofline_perturb_flat")):
            if name in kern and key in out and elems:
                out[key]["frac_of_rmw_stream"] = out[key]["achieved"] / ceil["rmw_stream_GBs"]
                valu = kernel_valu(traffic, name)
                if valu:
                    ach = valu * 64 / (kern[name]["ms_avg"] * 1e-3) / 1e12
                    out[key]["alu"] = {"bound": "alu", "achieved": ach, "peak": ceil["simple_issue_T_lane_instr_per_s"], "unit": "T lane-instr/s",
                                       "frac": ach / ceil["simple_issue_T_lane_instr_per_s"], "peak_datasheet": ALU_PEAK_DATASHEET,
                                       "valu_instructions_per_philox_call": valu * 64 / (elems / (4.0 if args.gauss_bits == 32 else 8.0))}
        if "gemm" in kern and cfg.arch != I.ARCH_LINEAR_LSQ:
            gm = kern["gemm"]
            flops_per_launch = 2.0 * profiled_steps * forward_gemm_flops(cfg) / gm["launches"]
            tf = flops_per_launch / (gm["ms_avg"] * 1e-3) / 1e12
            peak = MFMA_PEAK_TFLOPS[cfg.dtype]
            gemm_roof = {"bound": "mfma", "achieved": tf, "peak": peak, "unit": "TFLOP/s", "frac": tf / peak, "traffic": kernel_traffic(traffic, "gemm_"),
                         "kernel": "gemm_bf16_kernel" if cfg.dtype == "bf16" else "gemm_f32_kernel", "flops_per_launch": flops_per_launch}
            if cfg.dtype == "bf16":
                gemm_roof["frac_of_mfma_alone"] = tf / ceil["mfma_bf16_alone_TFLOPs"]
            out["roofline_gemm"] = gemm_roof
        # the dominant kernel of the step carries the headline roofline
        dom = max(kern, key=lambda n: kern[n]["ms_total"])
        out["roofline"] = {"gemm": out.get("roofline_gemm"), "perturb_tile": out.get("roofline_perturb"),
                           "perturb_flat": out.get("roofline_perturb_flat")}.get(dom) or out.get("roofline_gemm") or out.get("roofline_perturb")
        out["dominant_kernel_class"] = dom
    if prof and "perturb_tile" in out.get("kernel_ms", {}) and cfg.arch != I.ARCH_LINEAR_LSQ and u_bytes:
        # Sec. 3.4: the share of a layer's basis that would have to travel as 4-bit codes for the transfer to hide
        # under that layer's part of a perturbation pass, for a few link speeds (the restore is fused into the
        # pass and costs nothing measurable: a pass over 4-bit bases takes the same time).
        layer_bytes = sum(s.rows * cfg.k * 4 for s in specs if s.guided) / I.CONFIGS[args.config].n_layer   # uncompressed fp32 basis
        t_cc = out["kernel_ms"]["perturb_tile"]["ms_avg"] * 1e-3 / I.CONFIGS[args.config].n_layer
        links = {"10 Mbit/s": 1.25e6, "1 Gbit/s": 1.25e8, "100 Gbit/s": 1.25e10, "PCIe 5 x16 (64 GB/s)": 6.4e10}
        out["dtc_policy"] = {"layer_basis_bytes": layer_bytes, "t_cc_s": t_cc, "theta": 0.125,
                             "omega": {name: dict(zip(("omega", "hidden"), B.dtc_omega(layer_bytes, bw, t_cc, 0.0, 0.125))) for name, bw in links.items()}}
    if args.batched_update > 0:
        # edge-server aggregation over n (step, g) pairs: one pass per 8 perturbations against n single passes
        nb = args.batched_update
        bsteps = list(range(1000, 1000 + nb))
        bg = [1e-3 * (1 + i) for i in range(nb)]
        def timed(fn, reps=3):
            fn(); torch.cuda.synchronize()
            t = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return 1e3 * (time.perf_counter() - t) / reps
        def sequential():
            for st, g in zip(bsteps, bg):
                sess.apply_update(st, g, cfg.lr)
        ms_seq = timed(sequential)
        ms_bat = timed(lambda: sess.apply_updates(bsteps, bg, cfg.lr))
        out["batched_update"] = {"n": nb, "ms_batched": ms_bat, "ms_sequential": ms_seq, "speedup": ms_seq / ms_bat,
                                 "perturbations_per_s": nb / (ms_bat * 1e-3),
                                 "hbm_bytes_algorithmic": 2.0 * (guided_elems + flat_elems) * es * ((nb + 7) // 8) + u_bytes * ((nb + 7) // 8)}
    if args.cloud:
        # cloud block of Algorithm 1 (not part of `value`): back-propagation over the same batch, then the rank-k basis of the
        # first guided matrix from the gradients of three batches (three subspace sweeps)
        from paper_2601_12917_amd.session import cloud_basis_device
        sess.cloud_backward(batch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, grads = sess.cloud_backward(batch)
        torch.cuda.synchronize()
        bw_s = time.perf_counter() - t0
        gi = next(i for i, sp in enumerate(specs) if sp.guided)
        snaps = [grads[gi]]
        for seed in (1, 2):
            snaps.append(sess.cloud_backward(session_batch(sess, cfg, make_batch_arrays(cfg, seed)))[1][gi])
        del grads
        omega = torch.randn(snaps[0].shape[1], cfg.k, device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(0))
        cloud_basis_device(snaps, cfg.k, omega, 3)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        _, dep = cloud_basis_device(snaps, cfg.k, omega, 3)
        torch.cuda.synchronize()
        out["cloud"] = {"backward_s": bw_s, "backward_workspace_GB": B.lib().zgr_cloud_backward_workspace(sess.ctx, cfg.batch, cfg.seq) / 1e9,
                        "basis_ms": 1e3 * (time.perf_counter() - t0), "basis_of": specs[gi].name, "basis_shape": list(snaps[0].shape), "k": cfg.k,
                        "snapshots": 3, "subspace_sweeps": 3, "dependent_columns": dep}
        del snaps
    sess.close()
    del sess, batch
    if not args.no_fused_line:
        # the same step with the restoring pass and the update fused into one pass (3 instead of 4 passes over theta);
        # reported beside the headline value, which keeps the client block and the edge-server update separate
        fs = make_session(cfg, specs, values, bases, bits=args.gauss_bits, fuse_lr=cfg.lr)
        fb = session_batch(fs, cfg, arrays)
        for i in range(max(1, args.warmup)):
            fs.step(i, fb)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fs.step(args.warmup + i, fb)
        torch.cuda.synchronize()
        fe = time.perf_counter() - t0
        out["fused_restore_update"] = {"value": args.steps / fe, "unit": "steps/s", "ms_per_step": 1e3 * fe / args.steps,
                                       "passes_over_parameters": 3}
        fs.close()
        del fs, fb
    del values
    if not args.no_cpu_baseline and cfg.arch != I.ARCH_LINEAR_LSQ:
        out["cpu_baseline"] = cpu_baseline(cfg, specs)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
