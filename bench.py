#!/usr/bin/env python3
"""Benchmark of the SAGE-KV hot path on one MI355X.

One "step" = the whole path over one synthetic batch: the eviction pass (score, softmax, GQA
combine, top-k, gather) over every layer and KV head of the cache, followed by the config's
decode steps (append + attention over the reduced cache, all layers per step).  Inputs are
seeded, generated on the device and resident in HBM before the timed region.

Prints ONE JSON line.  `value` is the algorithmic bytes of a step (K once + survivors of K and V
read and written + indices, plus the reduced K and V once per decode step) divided by the step
time; the two halves of the metric (select GB/s, decode tokens/s) and their fractions of the
8 TB/s HBM peak are reported beside it.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def algorithmic_bytes(cfg, budget=None):
    """(select bytes per pass, decode bytes per decode step, score-kernel bytes per launch)."""
    e, d = cfg.elem_bytes, cfg.head_dim
    budget = cfg.budget if budget is None else budget
    per_row = cfg.L * d * e + 4 * budget * d * e + 4 * budget
    select = cfg.rows * per_row
    decode = 2 * cfg.rows * budget * d * e
    score = cfg.rows * cfg.L * d * e
    return select, decode, score


def read_traffic(cfg_name, key="traffic_bytes_per_launch"):
    """HBM bytes per launch of the score kernel (or, with another key, of the decode kernel) from the
    committed rocprofv3 --pmc summary, if present."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{cfg_name}_pmc.txt")
    if not os.path.exists(path):
        return None
    m = re.search(rf"^{key}:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def cpu_model():
    """Model string of the host CPU; virtual machines often shorten the name, so family / model /
    stepping and the CPU counts go with it."""
    info = {}
    try:
        for line in open("/proc/cpuinfo"):
            if ":" in line:
                k, v = (x.strip() for x in line.split(":", 1))
                if k in ("model name", "vendor_id", "cpu family", "model", "stepping") and k not in info:
                    info[k] = v
    except OSError:
        pass
    name = info.get("model name", "unknown")
    extra = ", ".join(f"{k} {info[k]}" for k in ("vendor_id", "cpu family", "model", "stepping") if k in info)
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return f"{name} ({extra}; {os.cpu_count()} logical CPUs, {usable} usable by this process)"


def cpu_baseline(cfg, K_dev, V_dev, select_repeats, decode_seconds):
    """Times the CPU oracle, as it stands, on the WHOLE workload: the eviction pass over every layer
    (K and V of one layer at a time are copied from the device, which holds the bench's own inputs;
    the copies are not timed), `select_repeats` times, then decode steps over all layers for about
    decode_seconds.  Returns the baseline record and the oracle's kept indices of every row."""
    import numpy as np

    import synth
    from oracle import ref

    q = synth.q_last_host(cfg)
    P = cfg.n_problems
    t_sel = 0.0
    Kc_all, Vc_all, kept_all = [], [], []
    t_one = None
    for p in range(P):
        Kp, Vp = synth.torch_to_host(K_dev[p:p + 1], cfg.dtype), synth.torch_to_host(V_dev[p:p + 1], cfg.dtype)
        qp = np.ascontiguousarray(q[p:p + 1])
        for _ in range(select_repeats):
            t0 = time.perf_counter()
            Kc, Vc, kept = ref.select(cfg.dtype, ref.GROUP_SUM, qp, Kp, Vp, cfg.n_sink, cfg.n_recent, cfg.k)
            t_sel += time.perf_counter() - t0
        if p == 0:  # one row = one oracle thread (its only parallel loop is over rows)
            K1, V1 = np.ascontiguousarray(Kp[:, :1]), np.ascontiguousarray(Vp[:, :1])
            q1 = np.ascontiguousarray(qp[:, : cfg.G])
            t0 = time.perf_counter()
            ref.select(cfg.dtype, ref.GROUP_SUM, q1, K1, V1, cfg.n_sink, cfg.n_recent, cfg.k)
            t_one = time.perf_counter() - t0
        Kc_all.append(Kc), Vc_all.append(Vc), kept_all.append(kept)
        del Kp, Vp
    t_pass = t_sel / select_repeats
    Kc, Vc, kept = np.concatenate(Kc_all), np.concatenate(Vc_all), np.concatenate(kept_all)
    t_dec, n_dec = 0.0, 0
    while t_dec < decode_seconds:
        qs, kn, vn = synth.decode_inputs_host(cfg, n_dec % max(cfg.decode_steps, 1))
        t0 = time.perf_counter()
        ref.append(cfg.dtype, Kc, Vc, kn, vn, cfg.n_sink + cfg.k, cfg.n_recent)
        ref.decode_attn(cfg.dtype, ref.GROUP_SUM, qs, Kc, Vc, cfg.budget)
        t_dec += time.perf_counter() - t0
        n_dec += 1
    one_row_bytes = algorithmic_bytes(cfg)[0] // cfg.rows
    sel_b, dec_b, _ = algorithmic_bytes(cfg)
    # same mix as a bench step: one eviction pass + cfg.decode_steps decode steps
    t_step = t_pass + cfg.decode_steps * t_dec / n_dec
    return {
        "value": (sel_b + cfg.decode_steps * dec_b) / t_step / 1e9,
        "unit": "GB/s",
        "cores": ref.threads(),
        "kind": "oracle",
        "cpu_model": cpu_model(),
        "select_GBps_one_thread": one_row_bytes / t_one / 1e9,
        "sample": f"the whole workload: the eviction pass over all {cfg.n_layers} layers ({cfg.rows} rows of L={cfg.L}) "
                  f"x{select_repeats} ({t_sel:.1f} s), then {n_dec} decode steps over all layers ({t_dec:.1f} s); value = "
                  f"bytes of (1 pass + {cfg.decode_steps} steps) / (pass time + {cfg.decode_steps} x step time)",
        "select_GBps": sel_b / t_pass / 1e9,
        "select_ms_all_layers": t_pass * 1e3,
        "decode_tokens_per_s": cfg.batch / (t_dec / n_dec),
    }, kept


def select_layer_sequential(sk, torch, cfg, head_mode, Bt, q_last, K, V, Kc, Vc, kept):
    """The eviction pass in the order a prefill produces the cache: one call per layer (batch x KV
    heads rows), one after the other on one stream.  In a model each call would overlap the next
    layer's prefill; here they run back to back.  Reported beside the headline, never as it."""
    lb = cfg.batch
    sl0 = slice(0, lb)
    ldesc = sk.select_desc(q_last[sl0], K[sl0], V[sl0], cfg.n_sink, cfg.n_recent, cfg.k, Bt, head_mode=head_mode)
    lws = torch.empty(sk.sagekv_select_workspace_bytes(ldesc), dtype=torch.uint8, device="cuda")

    def run():
        for l in range(cfg.n_layers):
            sl = slice(l * lb, (l + 1) * lb)
            sk.sagekv_select(ldesc, q_last[sl], K[sl], V[sl], Kc[sl], Vc[sl], kept[sl], None, lws)

    run()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    run()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    return {"calls": cfg.n_layers, "ms_all_layers": round(ms, 4), "ms_per_layer": round(ms / cfg.n_layers, 4)}


def layer_sequential(sk, torch, cfg, head_mode, Bt, q_steps, kn_steps, vn_steps, Kc, Vc, out, n_steps):
    """Decode in the dependency order of a real model: one call per layer (its batch x KV heads
    rows only), layers one after the other.  Timed eagerly (one library call per layer from
    Python) and as one HIP graph of the same calls.  Reported beside the headline, never as it."""
    lb = cfg.batch
    ldesc = sk.decode_desc(lb, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.dtype, cfg.n_sink, cfg.k,
                           cfg.n_recent, Bt, head_mode=head_mode)
    lws = torch.empty(max(sk.sagekv_decode_workspace_bytes(ldesc), 16), dtype=torch.uint8, device="cuda")

    def run():
        for t in range(n_steps):
            for l in range(cfg.n_layers):
                sl = slice(l * lb, (l + 1) * lb)
                sk.sagekv_decode_step(ldesc, q_steps[t][sl], kn_steps[t][sl], vn_steps[t][sl], Kc[sl], Vc[sl], t,
                                      out[sl], lws)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_steps

    res = {"steps": n_steps, "launches_per_token": cfg.n_layers}
    ms = timed(run)
    res["eager_ms_per_token"] = round(ms, 4)
    res["eager_tokens_per_s"] = round(cfg.batch / (ms * 1e-3), 1)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    ms = timed(graph.replay)
    res["graph_ms_per_token"] = round(ms, 4)
    res["graph_tokens_per_s"] = round(cfg.batch / (ms * 1e-3), 1)

    # the serving-loop form: the append count on the device (one ring state per layer), so the recorded
    # steps can be replayed for any token
    rings = torch.zeros((cfg.n_layers, 2), dtype=torch.int32, device="cuda")

    def run_ring():
        for t in range(n_steps):
            for l in range(cfg.n_layers):
                sl = slice(l * lb, (l + 1) * lb)
                sk.sagekv_decode_step_ring(ldesc, q_steps[t][sl], kn_steps[t][sl], vn_steps[t][sl], Kc[sl], Vc[sl],
                                           rings[l], out[sl], lws)

    ring_graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(ring_graph):
        run_ring()
    rings.zero_()
    ms = timed(ring_graph.replay)
    res["ring_graph_ms_per_token"] = round(ms, 4)
    res["ring_graph_tokens_per_s"] = round(cfg.batch / (ms * 1e-3), 1)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C3", help="C2, C3 (default: the 128K Llama-3.1-8B-shaped target), C4, C5")
    ap.add_argument("--decode-steps", type=int, default=None, help="decode steps per step (default: the config's)")
    ap.add_argument("--per-query-budget", type=int, default=0, metavar="B",
                    help="paper-literal head mode: one top-k per query head with the appendix's split of a token "
                         "budget B (sink B/4, k = pow2floor(B/2G) per head, recent = rest) instead of the config's")
    ap.add_argument("--page-size", type=int, default=0, metavar="T",
                    help="hold K and V in shuffled pages of T tokens (block-table layout) and run the paged entry point")
    ap.add_argument("--q-heads", type=int, default=0, metavar="HQ",
                    help="override the config's number of query heads (a multiple of its KV heads): other group sizes")
    ap.add_argument("--dense", action="store_true", help="force the dense eviction path (every token's score is written)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the timed region, run one plain 1 GiB device-to-device copy (a reference of "
                         "known size for rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--layer-sequential-steps", type=int, default=8,
                    help="decode steps of the untimed-in-value extra figure that launches one layer at a time")
    ap.add_argument("--cpu-select-repeats", type=int, default=3,
                    help="how often the oracle's eviction pass over the whole workload is timed (about 1-2 s each at C3)")
    ap.add_argument("--cpu-decode-seconds", type=float, default=5.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (rows are independent; no collectives are built). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2503_08879_amd as sk
    import synth

    cfg = synth.CONFIGS[args.config]
    if args.q_heads:
        assert args.q_heads % cfg.n_kv_heads == 0
        cfg = cfg.with_(n_q_heads=args.q_heads)
    head_mode, lists = sk.GROUP_SUM, 1
    if args.per_query_budget:
        n_sink, kk, n_recent = sk.sagekv_paper_budget(args.per_query_budget, cfg.G)
        cfg = cfg.with_(n_sink=n_sink, k=kk, n_recent=n_recent)
        head_mode, lists = sk.PER_QUERY, cfg.G
        args.no_cpu_baseline = True
    n_dec = cfg.decode_steps if args.decode_steps is None else args.decode_steps
    torch.cuda.set_device(0)
    dev = "cuda"
    S, W, k = cfg.n_sink, cfg.n_recent, cfg.k
    Bt = S + lists * k + W

    # ---- inputs, resident in HBM
    q_last, K, V, _ = synth.kv_device(cfg, dev)
    td = synth.torch_dtype(cfg.dtype)
    P, Hq, Hkv, d = cfg.n_problems, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    q_steps = torch.empty((max(n_dec, 1), P, Hq, d), dtype=td, device=dev)
    kn_steps = torch.empty((max(n_dec, 1), P, Hkv, d), dtype=td, device=dev)
    vn_steps = torch.empty((max(n_dec, 1), P, Hkv, d), dtype=td, device=dev)
    synth.fill_device(q_steps, synth.stream_key(cfg.seed, synth.T_QSTEP))
    synth.fill_device(kn_steps, synth.stream_key(cfg.seed, synth.T_KNEW))
    synth.fill_device(vn_steps, synth.stream_key(cfg.seed, synth.T_VNEW))

    pages = None
    if args.page_size:
        ps = args.page_size
        assert cfg.L % ps == 0, "bench pages must divide L"
        per = cfg.L // ps
        gen = torch.Generator(device="cpu").manual_seed(cfg.seed)
        perm = torch.randperm(P * per, generator=gen).to(dev)
        table = perm.to(torch.int32).view(P, per).contiguous()

        def paged(X):
            src = X.view(P, Hkv, per, ps, d).permute(0, 2, 1, 3, 4).reshape(P * per, Hkv, ps, d)
            pool = torch.empty_like(src)
            pool[perm] = src
            return pool

        K, V = paged(K), paged(V)
        torch.cuda.synchronize()

    # ---- outputs and workspaces (allocated once, outside the timed region)
    if args.page_size:
        sdesc, pages = sk.paged_select_desc(q_last, K, V, table, cfg.L, S, W, k, Bt, head_mode=head_mode,
                                            flags=sk.SELECT_DENSE if args.dense else 0)
    else:
        sdesc = sk.select_desc(q_last, K, V, S, W, k, Bt, head_mode=head_mode,
                               flags=sk.SELECT_DENSE if args.dense else 0)
    sws = torch.empty(sk.sagekv_select_workspace_bytes(sdesc), dtype=torch.uint8, device=dev)
    Kc = torch.zeros((P, Hkv, Bt, d), dtype=td, device=dev)
    Vc = torch.zeros((P, Hkv, Bt, d), dtype=td, device=dev)
    kept = torch.zeros((P, Hkv, Bt), dtype=torch.int32, device=dev)
    ddesc = sk.decode_desc(P, Hq, Hkv, d, cfg.dtype, S, k, W, Bt, head_mode=head_mode)
    dws = torch.empty(sk.sagekv_decode_workspace_bytes(ddesc), dtype=torch.uint8, device=dev)
    out = torch.empty((P, Hq, d), dtype=torch.float32, device=dev)

    def one_step_select():
        if pages is not None:
            sk.sagekv_select_paged(sdesc, pages, q_last, K, V, Kc, Vc, kept, None, sws)
        else:
            sk.sagekv_select(sdesc, q_last, K, V, Kc, Vc, kept, None, sws)

    def one_step(ev=None):
        if ev:
            ev[0].record()
        one_step_select()
        if ev:
            ev[1].record()
        for t in range(n_dec):
            sk.sagekv_decode_step(ddesc, q_steps[t], kn_steps[t], vn_steps[t], Kc, Vc, t, out, dws)
        if ev:
            ev[2].record()

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    # ---- timed region: exactly --steps steps
    # Only the score kernel is bracketed by the library's events inside the timed region: every event
    # record idles the GPU for ~10 us, a fully instrumented pass is ~3 % slower (that one runs afterwards).
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    sk.sagekv_stage_timing_stages(["score"], decode=False)
    sk.sagekv_stage_timing_enable(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    sel_all = [e[0].elapsed_time(e[1]) for e in events]
    dec_all = [e[1].elapsed_time(e[2]) for e in events]
    sel_ms, dec_ms = float(np.mean(sel_all)), float(np.mean(dec_all))
    score_ms = float(np.mean([sk.sagekv_stage_timing_read(0, i)[sk.binding.STAGES.index("score")]
                              for i in range(args.steps)]))
    # stage breakdown: separate, fully instrumented passes outside the timed region
    n_brk = min(args.steps, 10)
    sk.sagekv_stage_timing_stages(None, decode=False)
    sk.sagekv_stage_timing_enable(n_brk)
    for i in range(n_brk):
        one_step_select()
    torch.cuda.synchronize()
    stage_ms = np.array([sk.sagekv_stage_timing_read(0, i) for i in range(n_brk)]).mean(axis=0)
    sk.sagekv_stage_timing_enable(0)
    sk.sagekv_stage_timing_stages(None, decode=True)

    sel_b, dec_b, score_b = algorithmic_bytes(cfg, Bt)
    ms_per_step = elapsed / args.steps * 1e3
    total_b = sel_b + n_dec * dec_b
    value = total_b / (ms_per_step * 1e-3) / 1e9
    sel_gbps = sel_b / (sel_ms * 1e-3) / 1e9
    dec_tok_s = (n_dec * cfg.batch) / (dec_ms * 1e-3) if n_dec else None
    dec_gbps = (n_dec * dec_b) / (dec_ms * 1e-3) / 1e9 if n_dec else None
    redone = sk.sagekv_select_redone_rows(sdesc, sws)
    score_gbps = score_b / (score_ms * 1e-3) / 1e9

    result = {
        "metric": "select pass GB/s + compressed decode-attn tokens/s, % of HBM roofline",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == synth.BF16 else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: {cfg.n_layers} layers x batch {cfg.batch}, {Hq}q/{Hkv}kv heads, head_dim {d}, "
                        f"L={cfg.L}, budget {Bt} = {S} sink + {lists}x{k} top-k + {W} recent, {n_dec} decode steps per step"
                        + (", one top-k per query head" if lists > 1 else "")
                        + (f", K and V in shuffled pages of {args.page_size} tokens" if args.page_size else "")
                        + (", dense eviction path forced" if args.dense else ""),
            "rows": cfg.rows,
            "step": "1 eviction pass over the whole cache + the decode steps",
        },
        "frac_hbm": round(value / HBM_PEAK_GBPS, 4),
        "select": {"ms": round(sel_ms, 4), "ms_median": round(float(np.median(sel_all)), 4), "GBps": round(sel_gbps, 1), "frac_hbm": round(sel_gbps / HBM_PEAK_GBPS, 4),
                   "algorithmic_bytes": sel_b, "rows_redone_by_dense_path": redone,
                   "stage_ms": {n: round(float(v), 4) for n, v in zip(sk.binding.STAGES, stage_ms)},
                   "stage_ms_from": "separate fully instrumented passes (an event pair per stage; each event "
                                    "record idles the GPU ~10 us, so their sum exceeds select.ms)"},
        "decode": {"tokens_per_s": None if dec_tok_s is None else round(dec_tok_s, 1),
                   "ms_per_token": None if not n_dec else round(dec_ms / n_dec, 5),
                   "ms_per_token_median": None if not n_dec else round(float(np.median(dec_all)) / n_dec, 5),
                   "GBps": None if dec_gbps is None else round(dec_gbps, 1),
                   "frac_hbm": None if dec_gbps is None else round(dec_gbps / HBM_PEAK_GBPS, 4),
                   "algorithmic_bytes_per_token": dec_b},
    }
    # per kernel: algorithmic bytes of one launch / its average duration (HIP events on the launch stream)
    score_roof = {"kernel": "score_mfma_kernel (the one pass over K of the eviction pass)", "bound": "hbm",
                  "achieved": round(score_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                  "frac": round(score_gbps / HBM_PEAK_GBPS, 4), "avg_ms": round(score_ms, 4),
                  "algorithmic_bytes": score_b, "traffic": None if pages is not None else read_traffic(cfg.name),
                  "traffic_from": f"profiles/hbm_traffic_{cfg.name}_pmc.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                  "command, scaled by a 1 GiB copy; read from the committed summary, not measured in this run)"}
    roofs = [score_roof]
    if n_dec:
        dec_roof = {"kernel": "decode kernel (one launch = append + attention over all rows)", "bound": "hbm",
                    "achieved": round(dec_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(dec_gbps / HBM_PEAK_GBPS, 4), "avg_ms": round(dec_ms / n_dec, 5),
                    "algorithmic_bytes": dec_b,
                    "traffic": read_traffic(cfg.name, "decode_traffic_bytes_per_launch") if lists == 1 else None,
                    "traffic_from": score_roof["traffic_from"]}
        roofs.append(dec_roof)
    # the kernel the step spends most of its time in
    result["roofline"] = max(roofs, key=lambda r: r["avg_ms"] * (n_dec if r is not score_roof else 1))
    result["roofline_kernels"] = roofs
    if args.layer_sequential_steps > 0 and pages is None:
        result["select"]["layer_sequential"] = select_layer_sequential(sk, torch, cfg, head_mode, Bt, q_last, K, V,
                                                                       Kc, Vc, kept)
    if n_dec and args.layer_sequential_steps > 0:
        result["decode"]["layer_sequential"] = layer_sequential(
            sk, torch, cfg, head_mode, Bt, q_steps, kn_steps, vn_steps, Kc, Vc, out,
            min(n_dec, args.layer_sequential_steps))
    if not args.no_cpu_baseline and pages is None:
        base, kept_ref = cpu_baseline(cfg, K, V, args.cpu_select_repeats, args.cpu_decode_seconds)
        # free check: the sampled layers' kept sets must be the oracle's
        one_step()
        torch.cuda.synchronize()
        got = kept[: kept_ref.shape[0]].cpu().numpy()
        base["kept_sets_equal_oracle_rows"] = int((got == kept_ref).all(axis=-1).sum())
        base["rows_checked"] = int(kept_ref.shape[0] * kept_ref.shape[1])
        result["cpu_baseline"] = base
    print(json.dumps(result))


if __name__ == "__main__":
    main()
