#!/usr/bin/env python3
"""Benchmark of the fused decoder-block forward on one MI355X.

One "step" is one whole forward of a workload: [embedding ->] L fused decoder layers (norm, QKV
GEMM, [RoPE,] fused causal attention, out GEMM + residual, norm, MLP GEMMs with fused activation /
residual) -> final norm [-> tied LM head], on synthetic seeded inputs that are resident in HBM
before the timed region.

Headline (`value`, `config`, `roofline`, `cpu_baseline`): the largest single-GPU configuration, the
32-layer Llama-8B-shaped prefill of 1 x 4096 tokens in bf16 (`--workload` picks another).
`per_config` then carries all five evaluation configurations, each with its step time, latency
distribution, tokens/s, fraction of the matrix or HBM peak, and the per-operator breakdown of one
step measured with HIP events INSIDE the step (the library records an event on the launch stream
after every operator of its launch list), and `generation` the prompt + decode-loop workload.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
PEAK_F32_TFLOPS = 157.3        # MI355X fp32 matrix / vector peak
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E peak
METRIC = "decoder-block tokens/s; fused attention+GEMM TFLOP/s as % of MI355X peak"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=["c1", "c2", "c3", "c4", "c5"],
                    help="the headline workload (value, roofline, cpu_baseline)")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip per_config and generation (profiling runs of one workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="stop adding oracle samples once this much CPU time is spent (headline; a third "
                         "of it for each other configuration)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="launch a plain copy of known size, then three steps of the headline workload, and "
                         "exit: the program to run under `rocprofv3 --pmc FETCH_SIZE` / `WRITE_SIZE`")
    ap.add_argument("--traffic-summarize", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="turn the two counter_collection.csv files of the probe runs of --workload into its "
                         "entry of profiles/hbm_traffic.json (no GPU needed)")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------
# HBM traffic per kernel from hardware counters (collected offline, see --traffic-probe)
# ---------------------------------------------------------------------------------------------

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")
COPY_BYTES = 256 << 20          # the probe's copy kernel reads and writes this many bytes


def kernel_source_digest():
    """SHA-256 over every kernel source of the library: a counter record made before any of them
    changed is not reported any more."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2604_16498_amd", "csrc", "*.h*"))):
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def recorded_traffic(workload, inst):
    """(bytes per launch, label) measured for kernel instantiation `inst` inside a step of
    `workload`, or (None, why) when there is no record or the kernel sources have changed since."""
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, "no counter record"
    digest = kernel_source_digest()
    if rec.get("source_sha256") != digest:
        return None, "kernel sources changed since the counters were taken"
    ent = rec.get("workloads", {}).get(workload, {}).get("kernels", {}).get(inst)
    if ent is None:
        return None, "no counter record for this kernel"
    return (round(ent["fetch_bytes_per_launch"] + ent["write_bytes_per_launch"]),
            "recorded: profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of "
            "`bench.py --traffic-probe`), sources sha256 %s" % digest[:16])


def short_kernel_name(name):
    """'void forge::(anonymous namespace)::gemm_bf16_pers_kernel<256, 256, 2, 4, 4, 0>(...)' ->
    'gemm_bf16_pers<256,256,2,4,4,0>'."""
    import re
    m = re.match(r"_ZN5forge12_GLOBAL__N_1\d+([a-z_0-9]+?)_kernelI(.*?)E+v", name)   # not demangled by the profiler
    if m:
        a = m.group(2).replace("DF16b", "bf16,").replace("Li", "").replace("Lb", "").replace("E", ",").strip(",")
        return "%s<%s>" % (m.group(1), a)
    m = re.search(r"(\w+?)_kernel<([^>]*)>", name)
    if m:
        return "%s<%s>" % (m.group(1), m.group(2).replace(" ", ""))
    m = re.search(r"(\w+?)_kernel\b", name)
    return m.group(1) if m else name[:60]


def summarize_traffic(fetch_csv, write_csv):
    """FETCH_SIZE / WRITE_SIZE are reported in KiB per dispatch; both are scaled by what the same
    counter reads for the copy kernel of COPY_BYTES (read once, written once)."""
    import csv

    def per_kernel(path, counter):
        acc = {}
        with open(path) as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] != counter:
                    continue
                acc.setdefault((r["Kernel_Name"], r["Dispatch_Id"]), 0.0)
                acc[(r["Kernel_Name"], r["Dispatch_Id"])] += float(r["Counter_Value"])
        out = {}
        for (name, _), v in acc.items():
            out.setdefault(name, []).append(v)
        return out

    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    ck = "__amd_rocclr_copyBuffer"     # what a device-to-device tensor copy of raw bytes runs
    if ck not in fetch or ck not in write:
        raise SystemExit("no copy kernel found in %s" % fetch_csv)
    # skip the first launch of every kernel (cold caches, first-touch)
    mean = lambda v: sum(v[1:]) / max(1, len(v) - 1) if len(v) > 1 else v[0]
    # the runtime's copy kernel also serves small transfers: keep the probe's large copies only
    big = lambda v: [x for x in v if x > 0.5 * max(v)]
    f_scale = COPY_BYTES / (mean(big(fetch[ck])) * 1024.0)
    w_scale = COPY_BYTES / (mean(big(write[ck])) * 1024.0)
    kernels = {}
    for k in fetch:
        if "forge" not in k:
            continue
        kernels[short_kernel_name(k)] = {
            "launches": len(fetch[k]),
            "fetch_bytes_per_launch": mean(fetch[k]) * 1024.0 * f_scale,
            "write_bytes_per_launch": mean(write.get(k, [0.0])) * 1024.0 * w_scale,
        }
    return {"copy_kernel": ck[:80], "copy_bytes": COPY_BYTES, "fetch_scale": f_scale, "write_scale": w_scale,
            "kernels": kernels}


# ---------------------------------------------------------------------------------------------
# model construction (device memory plumbing only)
# ---------------------------------------------------------------------------------------------

def build_model(wl, F, torch, I, share=None):
    """Weights, descriptors, caches, workspace and the input of one workload on the GPU.
    share: a model built for a workload of the same layer shape and depth, whose weights are reused
    (the decode configuration runs on the prefill configuration's model)."""
    sh = wl.block
    dt = torch.bfloat16 if wl.bf16 else torch.float32
    big = sh.d_model >= 4096          # 8B-shaped: draw on the device (host generation takes minutes)
    g = torch.Generator(device="cuda").manual_seed(I.BASE_SEED * 1000 + wl.cid)

    def dev(a):
        if a is None:
            return None
        t = torch.from_numpy(a)
        return (t.to(torch.bfloat16) if wl.bf16 else t).cuda()

    def dev_normal(shape, std):
        return (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * std).to(dt)

    if share is not None:
        layers, mw = share["layers"], share["mw"]
    else:
        layers = []
        for l in range(wl.layers):
            if not big:
                w = {k: dev(v) for k, v in I.block_weights(sh, wl.cid, l, wl.bf16, wl.bias_std).items()}
            else:
                d = sh.d_model
                w = {
                    "norm1_g": torch.ones(d, device="cuda", dtype=dt), "norm1_b": None,
                    "w_qkv": dev_normal((sh.qkv_out, d), 0.02), "b_qkv": None,
                    "w_o": dev_normal((d, sh.q_heads * sh.head_dim), 0.02), "b_o": None,
                    "norm2_g": torch.ones(d, device="cuda", dtype=dt), "norm2_b": None,
                    "w_up": dev_normal((sh.up_out, d), 0.02), "b_up": None,
                    "w_down": dev_normal((d, sh.d_ff), 0.02), "b_down": None,
                }
            layers.append(w)
        mw = {k: dev(v) for k, v in I.model_weights(wl).items()}
    descs = [F.make_block_desc(sh, w) for w in layers]
    # logits rows padded to a multiple of 8 elements (16-byte aligned rows, the usual vocabulary
    # padding); the padding columns are never written or read
    logits_ld = (wl.vocab + 7) // 8 * 8
    model = F.make_model_desc(descs, mw, logits_ld=logits_ld)

    B, S = wl.batch, wl.seq
    cap = wl.pos0 + S
    cap = (cap + 63) // 64 * 64
    kshape = (wl.layers, B, sh.kv_heads, cap, sh.head_dim)
    if wl.pos0:
        kc = torch.randn(kshape, generator=g, device="cuda", dtype=torch.float32).to(dt)
        vc = torch.randn(kshape, generator=g, device="cuda", dtype=torch.float32).to(dt)
    else:
        kc = torch.zeros(kshape, device="cuda", dtype=dt)
        vc = torch.zeros_like(kc)
    if wl.vocab:
        ids_host = I.token_ids(wl.cid, B, S, wl.vocab)
        inp = torch.from_numpy(ids_host).cuda()
        out = torch.empty(B, S, logits_ld, device="cuda", dtype=dt)
    else:
        ids_host = None
        inp = dev(I.hidden_states(wl))
        out = torch.empty(B, S, sh.d_model, device="cuda", dtype=dt)
    ws = F.workspace(F.forge_model_workspace_bytes(model, B, S, cap))
    return dict(model=model, inp=inp, out=out, kc=kc, vc=vc, ws=ws, descs=descs, ids_host=ids_host,
                layers=layers, mw=mw, cap=cap, logits_ld=logits_ld)


# ---------------------------------------------------------------------------------------------
# algorithmic work
# ---------------------------------------------------------------------------------------------

def step_flops(wl):
    sh = wl.block
    T = wl.batch * wl.seq
    hd = sh.q_heads * sh.head_dim
    gemm = 2.0 * T * (sh.qkv_out * sh.d_model + sh.d_model * hd + sh.up_out * sh.d_model
                      + sh.d_model * sh.d_ff) * wl.layers
    if wl.vocab:
        gemm += 2.0 * T * wl.vocab * sh.d_model
    # causal attention: only the keys a query may see (lower triangle incl. diagonal)
    pairs = wl.batch * sum(wl.pos0 + s + 1 for s in range(wl.seq))
    attn = 4.0 * sh.q_heads * sh.head_dim * pairs * wl.layers
    return gemm, attn


def step_bytes(wl):
    """Algorithmic HBM bytes of one step of the bandwidth-bound (decode) workload: every weight
    and every cached K/V row is read once."""
    sh = wl.block
    es = 2 if wl.bf16 else 4
    hd = sh.q_heads * sh.head_dim
    wbytes = (sh.qkv_out * sh.d_model + sh.d_model * hd + sh.up_out * sh.d_model + sh.d_model * sh.d_ff) * es
    kvbytes = 2 * wl.batch * sh.kv_heads * (wl.pos0 + wl.seq) * sh.head_dim * es
    return (wbytes + kvbytes) * wl.layers


def operator_work(wl, F, torch, logits_ld):
    """name -> (bound, algorithmic flops or bytes of ONE launch, kernel instantiation) for every
    operator of the launch list.  Prompt-sized projections and attention are matrix-core bound
    (2 M N K flops; attention: the lower triangle only); everything of a decode step, the norms,
    RoPE and the embedding are HBM bound (bytes that must move once)."""
    sh = wl.block
    es = 2 if wl.bf16 else 4
    dt = torch.bfloat16 if wl.bf16 else torch.float32
    T = wl.batch * wl.seq
    d, hd, F_ = sh.d_model, sh.q_heads * sh.head_dim, sh.d_ff
    decode = wl.seq == 1 and wl.pos0 > 0
    _, attn_fl = step_flops(wl)
    G = sh.q_heads // sh.kv_heads

    def gemm(N, K, act, mode, ldy=0):
        nw = 2 * N if act == "swiglu" else N
        var = F.forge_gemm_variant(T, N, K, act, dt, ldy=ldy)
        inst = "%s,%d,%d>" % (var[:-1], F.ACT[act], mode) if var.endswith(">") and wl.bf16 and "+" not in var else var
        if decode:
            return ("hbm", float(nw) * K * es, inst)
        return ("mfma", 2.0 * T * nw * K, inst)

    qkv = gemm(sh.qkv_out, d, "none", 1)
    if sh.use_rope and wl.bf16 and wl.seq > 1 and T > 64:
        # a bf16 prompt rotates q and k in the epilogue of its QKV projection (cos / sin table kernel
        # + the head-split kernels in their rotating form, by columns: whole rounds of 256-tiles, the
        # rest on 128-tiles)
        qkv = (qkv[0], qkv[1], "rope_table + gemm_bf16_pers<256,256,2,4,0,3> + gemm_bf16_pers<128,128,2,2,0,3>")
    ops = {
        "norm": ("hbm", 2.0 * T * d * es, "residual_norm"),
        "gemm_qkv": qkv,
        "rope_q": ("hbm", 2.0 * T * hd * es, "rope"),
        "rope_k": ("hbm", 2.0 * T * sh.kv_heads * sh.head_dim * es, "rope"),
        "out_proj": gemm(d, hd, "none", 0),
        "mlp_up": gemm(F_, d, sh.mlp_act, 0),
        "mlp_down": gemm(d, F_, "none", 0),
        "embed": ("hbm", 3.0 * T * d * es, "embed"),
    }
    if decode:
        ops["attention"] = ("hbm", 2.0 * wl.batch * sh.kv_heads * (wl.pos0 + 1) * sh.head_dim * es,
                            "attn_decode<%d,%d>" % (sh.head_dim, G))
    else:
        ops["attention"] = ("mfma", attn_fl / wl.layers,
                            "attn_prefill<%d,false>" % sh.head_dim if wl.bf16 else "attn_f32<%d>" % sh.head_dim)
    if wl.vocab:
        ops["lm_head"] = gemm(wl.vocab, d, "none", 0, ldy=logits_ld)
    return ops


def name_operators(trace):
    """[(forge_op name, ms)] of one step -> [(operator name, ms)]: the two residual projections of a
    layer are told apart by their order (output projection first, MLP down second)."""
    out, res_seen = [], 0
    for op, ms in trace:
        if op == "gemm_qkv":
            res_seen = 0
        if op == "gemm_res":
            name = "out_proj" if res_seen == 0 else "mlp_down"
            res_seen += 1
        else:
            name = {"gemm_act": "mlp_up", "gemm": "lm_head", "attn": "attention"}.get(op, op)
        out.append((name, ms))
    return out


# ---------------------------------------------------------------------------------------------
# measurement of one workload
# ---------------------------------------------------------------------------------------------

def percentiles(ds):
    ds = sorted(ds)
    n = len(ds)
    return {"steps": n, "mean": round(sum(ds) / n, 4), "p50": round(ds[n // 2], 4),
            "p90": round(ds[int(n * 0.9)], 4), "p99": round(ds[min(n - 1, int(n * 0.99))], 4)}


def measure(wl, m, F, torch, steps, warmup, latency_steps=50, traced_steps=3, with_compiled=True):
    """Times `steps` steps after `warmup` (wall clock around a synchronised region), then, outside
    that region: the latency distribution of single steps, the per-operator breakdown of traced
    steps, and the same step through the compiled executor."""
    sh = wl.block
    pos0 = wl.pos0

    def step():
        F.forge_model_forward(m["model"], m["inp"], m["out"], m["kc"], m["vc"], pos0, m["ws"])

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    tokens = wl.batch * wl.seq
    gemm_fl, attn_fl = step_flops(wl)
    decode = wl.seq == 1 and wl.pos0 > 0
    peak_tf = PEAK_BF16_TFLOPS if wl.bf16 else PEAK_F32_TFLOPS

    res = {"workload": wl.name, "dtype": "bf16" if wl.bf16 else "f32", "layers": wl.layers, "batch": wl.batch,
           "seq_len": wl.seq, "kv_pos0": wl.pos0, "steps": steps, "warmup": warmup,
           "ms_per_step": round(ms_per_step, 4), "tokens_per_s": round(tokens / (ms_per_step * 1e-3), 1)}
    if decode:
        gbs = step_bytes(wl) / (ms_per_step * 1e-3) / 1e9
        res["step_hbm_gbs"] = round(gbs, 1)
        res["step_frac_of_hbm_peak"] = round(gbs / PEAK_HBM_GBS, 4)
    else:
        tf = (gemm_fl + attn_fl) / (ms_per_step * 1e-3) / 1e12
        res["step_tflops"] = round(tf, 1)
        res["step_frac_of_peak"] = round(tf / peak_tf, 4)

    # ---- latency of single steps: HIP events around each -----------------------------------------
    evs = []
    for _ in range(latency_steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        step()
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    res["latency_ms"] = percentiles([a.elapsed_time(b) for a, b in evs])

    # ---- per-operator breakdown: the library's own event after every operator of the list ----------
    work = operator_work(wl, F, torch, m["logits_ld"])
    cap_ops = 16 * wl.layers + 8
    table = {}
    traced_total = 0.0
    for _ in range(traced_steps):
        F.forge_trace_start(cap_ops)
        step()
        tr = name_operators(F.forge_trace_stop(cap_ops))
        for name, ms in tr:
            t = table.setdefault(name, {"launches": 0, "ms": 0.0})
            t["launches"] += 1
            t["ms"] += ms
            traced_total += ms
    ops = {}
    for name, t in table.items():
        bound, per_launch, inst = work[name]
        avg_s = t["ms"] * 1e-3 / t["launches"]
        e = {"kernel": inst, "launches_per_step": t["launches"] // traced_steps,
             "avg_us": round(avg_s * 1e6, 2), "share_of_step": round(t["ms"] / traced_total, 4), "bound": bound}
        if bound == "mfma":
            e["tflops"] = round(per_launch / avg_s / 1e12, 1)
            e["frac"] = round(per_launch / avg_s / 1e12 / peak_tf, 4)
        else:
            e["gbs"] = round(per_launch / avg_s / 1e9, 1)
            e["frac"] = round(per_launch / avg_s / 1e9 / PEAK_HBM_GBS, 4)
        e["_per_launch"] = per_launch
        e["_avg_s"] = avg_s
        ops[name] = e
    n_ops = sum(t["launches"] for t in table.values()) // traced_steps
    res["traced_step_ms"] = round(traced_total / traced_steps, 4)
    # what recording an event after every operator adds to a step, per operator (the operators'
    # durations above include it: they are upper bounds of the kernels' own times)
    res["trace_overhead_us_per_operator"] = round(
        (traced_total / traced_steps - res["latency_ms"]["mean"]) * 1e3 / max(1, n_ops), 2)
    res["traced_steps"] = traced_steps
    dom = max(ops, key=lambda k: ops[k]["share_of_step"])
    res["dominant_operator"] = dom
    res["operators"] = ops

    # ---- the same step through the compiled executor (static buffer plan + HIP graph replay) -------
    if with_compiled:
        cm = F.CompiledModel(m["model"], wl.batch, wl.seq, pos0, m["cap"])
        cws = F.workspace(cm.workspace_bytes())
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        cm.bind(m["inp"], m["out"], m["kc"], m["vc"], cws, side)
        for _ in range(warmup):
            cm.run(side)
        side.synchronize()
        c0 = time.perf_counter()
        for _ in range(steps):
            cm.run(side)
        side.synchronize()
        c_ms = (time.perf_counter() - c0) * 1e3 / steps
        # host time to enqueue one step (the calls return before the GPU is done)
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        for _ in range(5):
            step()
        h_plain = (time.perf_counter() - h0) / 5
        torch.cuda.synchronize()
        h0 = time.perf_counter()
        for _ in range(5):
            cm.run(side)
        h_comp = (time.perf_counter() - h0) / 5
        side.synchronize()
        ni, nr, _, nb = cm.counts()
        res["compiled"] = {"ms_per_step": round(c_ms, 4), "host_enqueue_us": round(h_comp * 1e6, 1),
                           "plain_host_enqueue_us": round(h_plain * 1e6, 1), "instructions": ni, "registers": nr,
                           "buffers": nb, "rho_buf": round(1 - nb / nr, 3),
                           "workspace_bytes": cm.workspace_bytes(), "plain_workspace_bytes": m["ws"].numel()}
        cm.close()
        del cws
        torch.cuda.synchronize()
    return res


def int8_weights(wl, m, F, torch, steps, warmup):
    """The same step on int8 weights (quantised by the library's own kernel): the decode step streams
    them as they are, the prompt-sized step writes each weight out as bf16 into the workspace first."""
    layers8 = []
    for w in m["layers"]:
        d = dict(w)
        for wn, sn in (("w_qkv", "s_qkv"), ("w_o", "s_o"), ("w_up", "s_up"), ("w_down", "s_down")):
            d[wn], d[sn] = F.forge_quantize_int8(w[wn])
        layers8.append(d)
    descs8 = [F.make_block_desc(wl.block, d) for d in layers8]
    model8 = F.make_model_desc(descs8, m["mw"], logits_ld=m["logits_ld"])
    ws8 = F.workspace(F.forge_model_workspace_bytes(model8, wl.batch, wl.seq, m["cap"]))

    def step8():
        F.forge_model_forward(model8, m["inp"], m["out"], m["kc"], m["vc"], wl.pos0, ws8)

    for _ in range(warmup):
        step8()
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    for _ in range(steps):
        step8()
    torch.cuda.synchronize()
    ms8 = (time.perf_counter() - c0) * 1e3 / steps
    shb = wl.block
    wbytes8 = (shb.qkv_out * shb.d_model + shb.d_model * shb.q_heads * shb.head_dim + shb.up_out * shb.d_model
               + shb.d_model * shb.d_ff) * wl.layers
    kvbytes = 2 * wl.batch * shb.kv_heads * (wl.pos0 + wl.seq) * shb.head_dim * 2 * wl.layers
    out = {"ms_per_step": round(ms8, 4), "tokens_per_s": round(wl.batch * wl.seq / (ms8 * 1e-3), 1),
           "weights": "int8 per-row symmetric, bf16 activations",
           "algorithmic_gb_per_step": round((wbytes8 + kvbytes) / 1e9, 2),
           "hbm_gbs": round((wbytes8 + kvbytes) / (ms8 * 1e-3) / 1e9, 1)}
    del layers8, descs8, model8, ws8
    torch.cuda.synchronize()
    return out


def generation(wl, m, F, torch, I, prompt=128, new_tokens=64):
    """The paper's language-modelling workload shape (Sec. "Datasets": a 128-token prompt, then 64
    generated tokens) on the token model of `wl`, whole batch: one prefill, then the decode step
    recorded once (positions in device memory) and replayed 64 times.  The ids fed back are
    synthetic (sampling is not part of the path)."""
    sh = wl.block
    B = wl.batch
    cap = (prompt + new_tokens + 63) // 64 * 64
    dt = torch.bfloat16
    ids = torch.from_numpy(I.token_ids(wl.cid, B, prompt + new_tokens, wl.vocab)).cuda()
    kc = torch.zeros(wl.layers, B, sh.kv_heads, cap, sh.head_dim, device="cuda", dtype=dt)
    vc = torch.zeros_like(kc)
    ld = m["logits_ld"]
    lg_p = torch.empty(B, prompt, ld, device="cuda", dtype=dt)
    ws_p = F.workspace(F.forge_model_workspace_bytes(m["model"], B, prompt, cap))
    p_ids = ids[:, :prompt].contiguous()

    def prefill():
        F.forge_model_forward(m["model"], p_ids, lg_p, kc, vc, 0, ws_p)

    for _ in range(3):
        prefill()
    evs = []
    for _ in range(10):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        prefill()
        e1.record()
        evs.append((e0, e1))
    torch.cuda.synchronize()
    pre = sorted(a.elapsed_time(b) for a, b in evs)

    # one padded window alone (batch 1): the shape of the paper's classification workload (windows
    # padded to 128 tokens, one at a time); right padding under the causal mask needs no mask tensor
    lg_1 = torch.empty(1, prompt, ld, device="cuda", dtype=dt)
    ids_1 = p_ids[:1].contiguous()
    k1, v1 = kc[:, :1].contiguous(), vc[:, :1].contiguous()
    ws_1 = F.workspace(F.forge_model_workspace_bytes(m["model"], 1, prompt, cap))

    def timed(fn, n=20):
        """p50 of n single calls, HIP events on torch's current stream."""
        for _ in range(3):
            fn()
        ev = []
        for _ in range(n):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            ev.append((e0, e1))
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in ev)[n // 2]

    w_plain = timed(lambda: F.forge_model_forward(m["model"], ids_1, lg_1, k1, v1, 0, ws_1))
    cw = F.CompiledModel(m["model"], 1, prompt, 0, cap)
    ws_c = F.workspace(cw.workspace_bytes())
    wside = torch.cuda.Stream()
    wside.wait_stream(torch.cuda.current_stream())
    cw.bind(ids_1, lg_1, k1, v1, ws_c, wside)
    wside.synchronize()
    with torch.cuda.stream(wside):
        w_graph = timed(lambda: cw.run(wside))
    cw.close()
    window = {"batch": 1, "tokens": prompt, "plain_ms_p50": round(w_plain, 4), "graph_replay_ms_p50": round(w_graph, 4),
              "tokens_per_s": round(prompt / (min(w_plain, w_graph) * 1e-3), 1)}

    max_pos = prompt + new_tokens - 1
    cm = F.CompiledModel(m["model"], B, 1, max_pos, cap)
    ws = F.workspace(cm.workspace_bytes())
    tok = torch.empty(B, 1, dtype=torch.int32, device="cuda")
    logits = torch.empty(B, 1, ld, device="cuda", dtype=dt)
    seq_pos = torch.full((B,), prompt, dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    tok.copy_(ids[:, prompt:prompt + 1])
    torch.cuda.synchronize()
    cm.bind_decode(tok, logits, kc, vc, seq_pos, ws, side)
    side.synchronize()
    per_step, totals = [], []
    for rep in range(3):                          # the first loop warms up
        seq_pos.fill_(prompt)
        torch.cuda.synchronize()
        evs = []
        with torch.cuda.stream(side):
            t0 = time.perf_counter()
            for i in range(new_tokens):
                tok.copy_(ids[:, prompt + i:prompt + i + 1])     # the "sampled" token of the previous step
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                cm.run(side)
                e1.record()
                seq_pos.add_(1)                                  # the positions advance on the device
                evs.append((e0, e1))
            side.synchronize()
            t1 = time.perf_counter()
        if rep:
            per_step += [a.elapsed_time(b) for a, b in evs]
            totals.append((t1 - t0) * 1e3)
    cm.close()
    ds = sorted(per_step)
    loop_ms = sum(totals) / len(totals)
    total_ms = pre[len(pre) // 2] + loop_ms
    return {"workload": "%s: batch %d, %d-token prompt + %d decode steps" % (wl.name.split("_b")[0], B, prompt, new_tokens),
            "prefill_ms_p50": round(pre[len(pre) // 2], 4),
            "decode_step_ms": {"p50": round(ds[len(ds) // 2], 4), "p99": round(ds[min(len(ds) - 1, int(len(ds) * 0.99))], 4),
                               "mean": round(sum(ds) / len(ds), 4)},
            "decode_loop_ms": round(loop_ms, 3),
            "generated_tokens_per_s": round(B * new_tokens / (loop_ms * 1e-3), 1),
            "end_to_end_tokens_per_s": round(B * (prompt + new_tokens) / (total_ms * 1e-3), 1),
            "launcher": "forge_model_forward (prompt), forge_compiled_bind_decode graph replay (steps)",
            "single_window": window}


# ---------------------------------------------------------------------------------------------

def main():
    args = parse()
    if args.traffic_summarize:
        from paper_2604_16498_amd import inputs as I
        rec = summarize_traffic(*args.traffic_summarize)
        try:
            with open(TRAFFIC_FILE) as f:
                full = json.load(f)
        except (OSError, ValueError):
            full = {}
        digest = kernel_source_digest()
        if full.get("source_sha256") != digest:
            full = {"source_sha256": digest, "workloads": {}}
        full["workloads"][I.WORKLOADS[int(args.workload[1])].name] = rec
        with open(TRAFFIC_FILE, "w") as f:
            json.dump(full, f, indent=1)
        print(json.dumps(rec, indent=1))
        return
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_16498_amd import binding as F
    from paper_2604_16498_amd import inputs as I
    F.lib()                                    # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    log = lambda msg: print("[bench] %s" % msg, file=sys.stderr, flush=True)

    head_id = int(args.workload[1])
    wl = I.WORKLOADS[head_id]
    models = {}

    def model_of(cid):
        """8B-shaped prefill and decode share one set of weights."""
        if cid not in models:
            share = models.get(4 if cid == 5 else 5 if cid == 4 else None)
            models[cid] = build_model(I.WORKLOADS[cid], F, torch, I, share=share)
        return models[cid]

    m = model_of(head_id)
    log("built %s" % wl.name)
    if args.traffic_probe:
        src = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        for _ in range(3):
            F.forge_model_forward(m["model"], m["inp"], m["out"], m["kc"], m["vc"], wl.pos0, m["ws"])
        torch.cuda.synchronize()
        return

    head = measure(wl, m, F, torch, args.steps, args.warmup)
    log("measured %s: %.4f ms/step" % (wl.name, head["ms_per_step"]))
    if head_id in (4, 5):
        head["int8_weights"] = int8_weights(wl, m, F, torch, args.steps, args.warmup)

    # ---- roofline of the dominant kernel of the headline workload, timed inside the step ----------
    dom = head["dominant_operator"]
    dop = head["operators"][dom]
    traffic, traffic_label = recorded_traffic(wl.name, dop["kernel"])
    if dop["bound"] == "mfma":
        peak, unit, achieved = (PEAK_BF16_TFLOPS if wl.bf16 else PEAK_F32_TFLOPS), "TFLOP/s", dop["tflops"]
    else:
        peak, unit, achieved = PEAK_HBM_GBS, "GB/s", dop["gbs"]
    roofline = {"bound": dop["bound"], "achieved": achieved, "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": traffic, "traffic_source": traffic_label,
                "kernel": dop["kernel"], "operator": dom,
                "algorithmic_%s_per_launch" % ("flops" if dop["bound"] == "mfma" else "bytes"): dop["_per_launch"],
                "avg_launch_us": dop["avg_us"], "launches_timed": dop["launches_per_step"] * head["traced_steps"],
                "timed": "HIP events recorded by the library on the launch stream after every operator, inside "
                         "%d whole steps (forge_trace_start / forge_trace_stop)" % head["traced_steps"]}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(wl, m, args.cpu_seconds)
        log("oracle timed on %s" % wl.name)

    # ---- every evaluation configuration, and the generation loop ------------------------------------
    per_config, gen = [], None
    if not args.headline_only:
        for cid in (1, 2, 3, 4, 5):
            if cid == head_id:
                r = head
            else:
                w2 = I.WORKLOADS[cid]
                m2 = model_of(cid)
                log("built %s" % w2.name)
                st, wu = (200, 20) if cid == 1 else (20, 5)
                r = measure(w2, m2, F, torch, st, wu, traced_steps=10 if cid == 1 else 3)
                if cid in (4, 5):
                    r["int8_weights"] = int8_weights(w2, m2, F, torch, st, wu)
                if not args.no_cpu_baseline:
                    r["cpu_baseline"] = cpu_baseline(w2, m2, args.cpu_seconds / 3)
                log("measured %s: %.4f ms/step" % (w2.name, r["ms_per_step"]))
            per_config.append(r)
            if cid == 2:
                gen = generation(I.WORKLOADS[2], model_of(2), F, torch, I)
                if not args.no_cpu_baseline:
                    gen["cpu_baseline"] = cpu_generation(I.WORKLOADS[2], args.cpu_seconds / 3)
                log("generation loop measured")
        models.clear()

    def public(r):
        r = dict(r)
        r["operators"] = {k: {a: b for a, b in v.items() if not a.startswith("_")} for k, v in r["operators"].items()}
        return r

    sh = wl.block
    line = {
        "metric": METRIC,
        "value": head["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if wl.bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "layers": wl.layers, "batch": wl.batch, "seq_len": wl.seq,
                   "kv_pos0": wl.pos0, "d_model": sh.d_model, "parallelism": "single-gpu"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "headline": public(head),
        "per_config": [public(r) for r in per_config],
        "generation": gen,
    }
    print(json.dumps(line))


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(wl, m, budget_s):
    """Time the oracle as it stands on whole sequences of the workload until ~budget_s is spent."""
    import numpy as np
    from oracle import forge_oracle as O
    from paper_2604_16498_amd import inputs as I
    cores = oracle_threads()
    sh = wl.block
    if sh.d_model >= 2048:
        # 1.3B- and 8B-shaped: one layer of one sequence, scaled by the layer count (the embedding
        # and the LM head of the 1.3B shape, 7 % of its flops, are left out of the sample)
        w = {k: (None if v is None else v.float().cpu().numpy()) for k, v in m["layers"][0].items()}
        x = I.normal(wl.cid, 0, "x", (1, wl.seq, sh.d_model), 1.0, bf16=wl.bf16)
        if wl.pos0:
            kc = m["kc"][0, :1].float().cpu().numpy().astype(np.float64)
            vc = m["vc"][0, :1].float().cpu().numpy().astype(np.float64)
            t0 = time.perf_counter()
            O.decoder_block(sh, w, x, kc, vc, pos0=wl.pos0)
        else:
            t0 = time.perf_counter()
            O.decoder_block(sh, w, x)
        dt_ = (time.perf_counter() - t0) * wl.layers
        return {"value": round(wl.seq / dt_, 3), "unit": "tokens/s", "cores": cores, "kind": "oracle",
                "sample": "1 layer x 1 sequence timed (%.1f s), multiplied by %d layers (extrapolated)"
                          % (dt_ / wl.layers, wl.layers)}
    layers = [I.block_weights(sh, wl.cid, l, wl.bf16, wl.bias_std) for l in range(wl.layers)]
    mw = I.model_weights(wl)
    done, t_used = 0, 0.0
    while done < wl.batch and t_used < budget_s:
        t0 = time.perf_counter()
        if wl.vocab:
            O.gpt_forward(sh, layers, mw, ids=m["ids_host"][done:done + 1])
        else:
            O.gpt_forward(sh, layers, mw, x=I.hidden_states(wl)[done:done + 1])
        t_used += time.perf_counter() - t0
        done += 1
    return {"value": round(done * wl.seq / t_used, 2), "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d sequences of %d tokens, all %d layers%s, %.1f s" % (
                done, wl.batch, wl.seq, wl.layers, " + LM head" if wl.vocab else "", t_used)}


def cpu_generation(wl, budget_s, prompt=128, new_tokens=64):
    """The oracle has no KV cache (neither has the paper): generating 64 tokens after a 128-token
    prompt is 64 causal forwards of growing length; a bounded number of them is timed and the rest
    extrapolated by the token count."""
    from oracle import forge_oracle as O
    from paper_2604_16498_amd import inputs as I
    sh = wl.block
    layers = [I.block_weights(sh, wl.cid, l, wl.bf16, wl.bias_std) for l in range(wl.layers)]
    mw = I.model_weights(wl)
    ids = I.token_ids(wl.cid, 1, prompt + new_tokens, wl.vocab)
    t_used, done_tokens, n = 0.0, 0, 0
    total_tokens = sum(prompt + i for i in range(new_tokens))
    for i in range(new_tokens):
        if t_used >= budget_s:
            break
        t0 = time.perf_counter()
        O.gpt_forward(sh, layers, mw, ids=ids[:, :prompt + i])
        t_used += time.perf_counter() - t0
        done_tokens += prompt + i
        n += 1
    est = t_used * total_tokens / done_tokens
    return {"value": round(new_tokens / est, 3), "unit": "generated tokens/s (one sequence)", "cores": oracle_threads(),
            "kind": "oracle", "sample": "%d of %d growing-length forwards timed (%.1f s), the rest extrapolated by "
                                        "token count" % (n, new_tokens, t_used)}


if __name__ == "__main__":
    main()
