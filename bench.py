#!/usr/bin/env python3
"""Benchmark of the FCCO loss step (fwd + bwd) on one MI355X.

A "step" is one fastclip_step call: similarity strips, exp sums, state update of u by dataset index,
gradient contractions, temperature gradient, over one batch of synthetic embeddings that already sit
in HBM.  Prints ONE JSON line: anchors/s for the whole step, the roofline of the dominant kernel
(per-kernel durations from HIP events recorded by the library on its launch stream), the per-phase
times, the step replayed from a HIP graph, the state-update kernel on 2^24 indices against the HBM
roofline, the same step written with stock PyTorch-ROCm ops on the same GPU (context), and the CPU oracle
timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_FLOPS = 2.5e15     # MI355X dense bf16 MFMA
PEAK_HBM_BYTES = 8.0e12      # MI355X HBM3E

def source_digest():
    """First 16 hex digits of the SHA-256 over the library's sources (csrc/*, include/*): names the build a profile
    was taken on."""
    import hashlib
    h = hashlib.sha256()
    for sub in (os.path.join("paper_2407_01445_amd", "csrc"), "include"):
        for f in sorted(os.listdir(os.path.join(ROOT, sub))):
            if f.endswith((".hip", ".hpp", ".h")):
                h.update(f.encode())
                h.update(open(os.path.join(ROOT, sub, f), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic():
    """HBM bytes per launch that rocprofv3 --pmc runs of this script measured (FETCH_SIZE, WRITE_SIZE in KiB per
    dispatch, each scaled by what the same counter reads for a device copy of known size).  The summaries under
    profiles/ carry one line per kernel of the form
        bench-traffic: workload=cfg4 kernel=k_strips_bf16 fetch_KiB=.. fetch_scale=.. write_KiB=.. write_scale=.. source=<digest> date=..
    Returns {(workload, kernel): dict(bytes, source, date, file)}."""
    import re
    out = {}
    pdir = os.path.join(ROOT, "profiles")
    for f in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not f.endswith((".md", ".txt")):
            continue
        for line in open(os.path.join(pdir, f)):
            if "bench-traffic:" not in line:
                continue
            kv = dict(re.findall(r"(\w+)=(\S+)", line.split("bench-traffic:", 1)[1]))
            try:
                nbytes = (float(kv["fetch_KiB"]) * float(kv["fetch_scale"]) +
                          float(kv["write_KiB"]) * float(kv["write_scale"])) * 1024.0
            except (KeyError, ValueError):
                continue
            out[(kv.get("workload"), kv.get("kernel"))] = dict(bytes=nbytes, source=kv.get("source"), date=kv.get("date"),
                                                              file="profiles/" + f)
    return out


def traffic_fields(table, workload, kernel, digest):
    """`traffic` of a roofline object: the profiled HBM bytes per launch if the profile was taken on this very build of
    the sources, else null with the reason."""
    hit = table.get((workload, kernel))
    if hit is None:
        return {"traffic": None, "traffic_source": "no rocprofv3 counter run of this kernel and workload under profiles/"}
    if hit["source"] != digest:
        return {"traffic": None, "traffic_source": "%s (%s) was taken on sources %s, this build is %s: not carried over"
                                                   % (hit["file"], hit["date"], hit["source"], digest)}
    return {"traffic": round(hit["bytes"], 1), "traffic_source": "%s, %s, same sources (%s)" % (hit["file"], hit["date"], digest)}


def algorithmic_flops(B, b, d, gathered=False):
    """Flop the method needs per step and phase (recomputation and padding not counted): one
    'unit' = 2 b B d.  Full batch (b == B): similarity once, then W T and W^T I.  Local share:
    two strips, two anchor-side contractions, and the local contrast-side block (4 b^2 d); with
    gathered state the contrast side runs over all B anchors, whose weights share the rows of the
    anchor-side sum (one weight matrix per side: still two contractions)."""
    unit = 2.0 * b * B * d
    if b == B:
        return {"strips": unit, "contract": 2 * unit}
    if gathered:
        return {"strips": 2 * unit, "contract": 2 * unit}
    return {"strips": 2 * unit, "contract": 2 * unit + 4.0 * b * b * d}


def stock_ops_step(torch, img, txt, idx, u_img, u_txt, tau1, tau2, *, off, b, gamma, eps, rho, version, scale):
    """The same step (local-anchor mode) written with stock PyTorch-ROCm tensor ops on the GPU: bf16 matmuls for the
    two similarity strips and the two gradient contractions, fp32 element-wise ops, index_select / index_copy_ for the
    state (Eq. 1, Eqs. 2-10).  Context for the timing only: the product never calls it, nothing is checked to the
    parity bar against it.  tau1, tau2: [b] temperatures of the anchors (a global temperature repeated)."""
    B = img.shape[0]
    M = float(B - 1)
    Il, Tl = img[off:off + b], txt[off:off + b]
    ar = torch.arange(b, device=img.device)
    diag = (Il.float() * Tl.float()).sum(1)

    def side(A, X, tau_a, u):
        Z = (A @ X.T).float() - diag[:, None]
        E = torch.exp(Z / tau_a[:, None])
        E[ar, off + ar] = 0.0
        g, h = E.sum(1) / M, (Z * E).sum(1) / M
        u_old = u.index_select(0, idx)
        u_new = torch.where(u_old == 0, g, (1.0 - gamma) * u_old + gamma * g)
        u.index_copy_(0, idx, u_new)
        c = 1.0 / (b * M * (eps + u_new))
        if version == 0:
            c = c / tau_a
        return E, g, h, u_new, c

    E1, g1, h1, u1, c1 = side(Il, txt, tau1, u_img)
    E2, g2, h2, u2, c2 = side(Tl, img, tau2, u_txt)
    W1, W2 = c1[:, None] * E1, c2[:, None] * E2
    loc1 = W1[:, off:off + b].clone()
    W1[:, off:off + b] += W2[:, off:off + b].T          # contrast side of the local text anchors (Eqs. 3 / 5 / 7)
    W2[:, off:off + b] += loc1.T
    dd = (M * (c1 * g1 + c2 * g2))[:, None]
    d_img = (W1.to(img.dtype) @ txt).float() - dd * Tl.float()
    d_txt = (W2.to(img.dtype) @ img).float() - dd * Il.float()
    l1, l2 = torch.log(eps + u1), torch.log(eps + u2)
    if version == 2:
        loss = (tau1 * (l1 + rho) + tau2 * (l2 + rho)).sum() / b
        d_tau = (scale * (l1 + rho - h1 / (tau1 * (eps + u1))), scale * (l2 + rho - h2 / (tau2 * (eps + u2))))
    else:
        t = tau1[0]
        hs = (h1 / (eps + u1) + h2 / (eps + u2)).sum()
        if version == 0:
            loss, d_tau = (l1 + l2).sum() / b, -hs / (b * t * t)
        else:
            loss = t * (l1 + l2).sum() / b + (2.0 * rho * t if version == 3 else 0.0)
            d_tau = (l1 + l2).sum() / b + 2.0 * rho - hs / (b * t)
    return loss, d_img, d_txt, d_tau


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000, help="timed steps (0.3 s of GPU work at cfg4)")
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps before them; the shader clock needs some 50 steps after idle to settle")
    ap.add_argument("--prewarm", type=int, default=300,
                    help="steps run before the warm-up steps, untimed and reported as prewarm_steps: they bring the shader "
                         "clock from its idle state to the one it holds under this load, so that a short timed window "
                         "measures the steady state")
    ap.add_argument("--workload", default="cfg4", help="cfg1..cfg4 (bf16 workloads of BASELINE.json)")
    ap.add_argument("--dense-state", action="store_true",
                    help="keep the per-sample state of FastCLIP-v2 workloads as separate dense arrays instead of one "
                         "32-byte record per sample")
    ap.add_argument("--gathered", action="store_true",
                    help="time the step with FASTCLIP_GATHERED_STATE (contrast side over every global anchor); "
                         "not the headline workload")
    ap.add_argument("--update-tau", action="store_true",
                    help="time fastclip_step_update_tau (the step with the temperature update fused in, AdamW) instead of "
                         "fastclip_step; not the headline workload")
    ap.add_argument("--tiles", type=int, choices=(128, 256), default=None,
                    help="ask for this tile size (FASTCLIP_TILES_128 / FASTCLIP_TILES_256) instead of the library's choice; "
                         "not the headline configuration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-state-bench", action="store_true")
    ap.add_argument("--no-stock-ops", action="store_true", help="skip timing the step written with stock PyTorch ops")
    ap.add_argument("--strip-ablations", action="store_true",
                    help="only run the measurement variants of the strip kernel (parts compiled out, in-kernel cycle "
                         "counters) on the workload and print their table as JSON")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a device-to-device copy of 1 GiB a few times (reference for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch

    from paper_2407_01445_amd import binding as fc
    from paper_2407_01445_amd.workloads import WORKLOADS, draw_indices, make_embeddings, step_seed

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if args.calibrate_copy:
        n = 1 << 28                                    # 2^28 fp32 = 1 GiB read + 1 GiB written per copy
        src = torch.rand(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "copy", "bytes_read": 4 * n, "bytes_written": 4 * n, "copies": 5}))
        return
    fc.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    name = args.workload
    w = WORKLOADS[name]
    B, b, off, d, N, version = w["B"], w["b"], w["off"], w["d"], w["N"], w["version"]
    K, W = args.steps, args.warmup

    # ---- inputs, resident in HBM before anything is timed
    img32, txt32 = make_embeddings(step_seed(name, 0), B, d, w["noise"], w["dtype"])
    tdt = torch.bfloat16 if w["dtype"] == "bf16" else torch.float32
    img, txt = torch.from_numpy(img32).to(tdt).to(dev), torch.from_numpy(txt32).to(tdt).to(dev)
    f32 = dict(dtype=torch.float32, device=dev)
    tau = torch.full((1,), w["tau"], **f32)
    # per-sample state.  FastCLIP-v2 keeps u_1, u_2, tau_1, tau_2 and the temperatures' optimizer moments per sample: by
    # default they are the fields {u_1, tau_1, m_1, v_1, u_2, tau_2, m_2, v_2} of one 32-byte record per sample (one
    # memory sector per sample and direction instead of one line per array); the other versions keep u_1, u_2 only.
    records = None
    if version == fc.V2 and not args.dense_state:
        records = torch.zeros(N, 8, **f32)
        u_img, tau_img, m_img, v_img, u_txt, tau_txt, m_txt, v_txt = (records[:, i] for i in range(8))
        tau_img.fill_(w["tau"])
        tau_txt.fill_(w["tau"])
        stride = 8
    else:
        u_img, u_txt = torch.zeros(N, **f32), torch.zeros(N, **f32)
        tau_img = torch.full((N,), w["tau"], **f32) if version == fc.V2 else None
        tau_txt = torch.full((N,), w["tau"], **f32) if version == fc.V2 else None
        m_img = v_img = m_txt = v_txt = None
        stride = 1
    d_img, d_txt = torch.empty(b, d, **f32), torch.empty(b, d, **f32)
    loss, d_tau = torch.empty(1, **f32), torch.empty(1, **f32)
    d_tau_img, d_tau_txt = torch.empty(b, **f32), torch.empty(b, **f32)
    gath = {}
    if args.gathered:
        rs = np.random.default_rng(step_seed(name, 77))
        mk = lambda lo, hi: torch.from_numpy(rs.uniform(lo, hi, B).astype(np.float32)).to(dev)
        gath = dict(u_glob_img=mk(0.05, 2.0), u_glob_txt=mk(0.05, 2.0))
        if version == fc.V2:
            gath.update(tau_glob_img=mk(0.05, 0.1), tau_glob_txt=mk(0.05, 0.1))
    n_sets = min(W + 2 * K, 128)      # distinct index sets, used in turn
    idx_sets = [torch.from_numpy(draw_indices(step_seed(name, t) + 500, b, N)).to(dev) for t in range(n_sets)]
    KE = min(K, 50)                   # steps of the per-step and per-kernel HIP-event legs

    def gamma_at(t):
        g = w["gamma"]
        return fc.fastclip_gamma_cosine(t, 1, g[1], g[2]) if isinstance(g, tuple) else g

    def cfg_at(t):
        return fc.make_config(version=version, emb_dtype=fc.BF16 if w["dtype"] == "bf16" else fc.F32, B=B, b=b,
                              off=off, d=d, N=N, gamma=gamma_at(t), eps=w["eps"], rho=w["rho"], tau_grad_scale=1.0 / N,
                              flags=(fc.GATHERED_STATE if args.gathered else 0) |
                                    {None: 0, 128: fc.TILES_128, 256: fc.TILES_256}[args.tiles], state_stride=stride)

    def bufs_at(t):
        return fc.make_buffers(img_glob=img, txt_glob=txt, idx=idx_sets[t % n_sets], u_img=u_img, u_txt=u_txt, tau=tau,
                               tau_img=tau_img, tau_txt=tau_txt, d_img=d_img, d_txt=d_txt, loss=loss, d_tau=d_tau,
                               d_tau_img=d_tau_img, d_tau_txt=d_tau_txt, **gath)

    ws = torch.empty(fc.fastclip_workspace_bytes(cfg_at(0)), dtype=torch.uint8, device=dev)
    cfgs = [cfg_at(t) for t in range(W + K + KE)]
    bufs = [bufs_at(t) for t in range(W + K + KE)]
    digest = source_digest()
    traffic = profiled_traffic()
    if args.strip_ablations:
        mws = torch.empty(fc.fastclip_workspace_bytes(cfgs[0]) + fc.MEASURE_STRIPS_EXTRA_BYTES, dtype=torch.uint8, device=dev)
        for t in range(args.prewarm):
            fc.fastclip_step(cfgs[0], bufs[0], ws)
        names = {0: "complete kernel", 1: "no global->LDS requests", 2: "no LDS operand reads", 3: "no requests, no operand reads",
                 4: "no epilogue", 7: "MFMAs and barriers only"}
        rows = []
        for abl, label in names.items():
            for _ in range(20):                 # keep the clock where the step holds it
                fc.fastclip_step(cfgs[0], bufs[0], ws)
            r = fc.fastclip_measure_strips(cfgs[0], bufs[0], mws, abl, reps=20)
            stages = r["stages_per_workgroup"]
            rows.append({"ablation": abl, "what": label, "us_per_launch": round(r["ms"] * 1e3, 2), "ghz": round(r["ghz"], 3),
                         "cycles_older_wave": round(r["cycles_older_wave"]), "cycles_younger_wave": round(r["cycles_younger_wave"]),
                         "cycles_between_tiles": round(r["cycles_between_tiles"]),
                         "cycles_per_stage_in_the_loops": round((r["cycles_older_wave"] - r["cycles_between_tiles"]) / stages, 1),
                         "stages_per_workgroup": stages, "workgroups": r["workgroups"]})
        print(json.dumps({"strip_ablations": rows, "workload": name, "sources": digest,
                          "note": "2048 cycles of matrix-core time per 64-deep stage and SIMD (64 MFMAs of 32 cycles)"}))
        return

    step = lambda t: fc.fastclip_step(cfgs[t], bufs[t], ws)
    if args.update_tau:      # Alg. 1 line 12 fused into the step: temperatures and their AdamW moments stepped in place
        # the moment arrays stay referenced here for the whole run: the library is handed their addresses only
        if version == fc.V2:
            moments = [m_img, v_img, m_txt, v_txt] if records is not None else [torch.zeros(N, **f32) for _ in range(4)]
            tst = fc.make_tau_state(tau_img=tau_img, tau_txt=tau_txt, m_img=moments[0], v_img=moments[1],
                                    m_txt=moments[2], v_txt=moments[3])
        else:
            moments = [torch.zeros(1, **f32) for _ in range(2)]
            tst = fc.make_tau_state(tau=tau, m=moments[0], v=moments[1])
        upd = lambda t: fc.make_tau_update(optimizer=fc.TAU_ADAMW, step=t + 1, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8,
                                           tau_min=0.01, state_stride=stride)
        step = lambda t: fc.fastclip_step_update_tau(cfgs[t], bufs[t], upd(t), tst, ws)

    # ---- untimed: bring the clock to its state under load (reported, not counted as warm-up); then the W warm-up
    # steps, then exactly K timed steps bracketed by synchronisation
    for t in range(args.prewarm):
        step(t % (W + K))
    for t in range(W):
        step(t)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(W, W + K):
        step(t)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / K
    anchors_per_s = b * K / (t1 - t0)
    assert torch.isfinite(loss).all() and torch.isfinite(d_img).all()

    # ---- spread of single steps: HIP events around each of K more steps (torch's current stream is the launch stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(KE)]
    for i in range(KE):
        t = W + i
        evs[i][0].record()
        fc.fastclip_step(cfgs[t], bufs[t], ws)
        evs[i][1].record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    step_ms = {"mean": round(sum(per_step) / KE, 5), "min": round(per_step[0], 5), "p50": round(per_step[KE // 2], 5),
               "steps": KE}

    # ---- the step replayed from a HIP graph (it allocates nothing and records no memset): what a training loop that
    # captures its iteration sees; same index set every replay, the state keeps evolving
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step(W)
    for _ in range(max(min(W, 20), 20)):      # the first replays of a graph are slower than the later ones
        graph.replay()
    torch.cuda.synchronize()
    KG = max(K, 200)                          # enough replays that the host's part of a replay is not what is timed
    g0 = time.perf_counter()
    for _ in range(KG):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - g0) * 1e3 / KG
    del graph

    # ---- per-kernel durations: the library records HIP events around every kernel on its launch stream
    phase_ms = {}
    for t in range(W + K, W + K + KE):
        for _ in range(3):          # the timed step starts on a busy GPU, as the steps of the timed loop do
            fc.fastclip_step(cfgs[t], bufs[t], ws)
        for k, v in fc.fastclip_step_timed(cfgs[t], bufs[t], ws).items():
            phase_ms[k] = phase_ms.get(k, 0.0) + v / KE
    # An event pair around a kernel is not free: the bracketed kernels of a step add up to more than the step takes without
    # events.  That surplus, shared equally among the bracketed kernels, is what one pair costs; it is subtracted, and the
    # raw figures are printed beside the corrected ones.
    raw_phase_ms = dict(phase_ms)
    n_bracketed = sum(1 for v in raw_phase_ms.values() if v > 0)
    event_cost_ms = max(0.0, (sum(raw_phase_ms.values()) - ms_per_step) / max(n_bracketed, 1))
    phase_ms = {k: (max(v - event_cost_ms, 0.0) if v > 0 else 0.0) for k, v in raw_phase_ms.items()}
    alg = algorithmic_flops(B, b, d, args.gathered)
    dom = max(("strips", "contract"), key=lambda k: phase_ms.get(k, 0.0))
    achieved = alg[dom] / (phase_ms[dom] * 1e-3) / 1e12
    plan = fc.fastclip_describe(cfgs[0])           # which tiles the library runs this workload on
    kernel_of = {"strips": "k_strips_t128_bf16", "contract": "k_contract_t128_bf16"} if plan["tile"] == 128 else \
                {"strips": "k_strips_bf16", "contract": "k_contract_bf16"}
    roofline = {"kernel": kernel_of[dom], "bound": "mfma",
                "achieved": round(achieved, 2), "peak": PEAK_BF16_FLOPS / 1e12, "unit": "TFLOP/s",
                "frac": round(achieved * 1e12 / PEAK_BF16_FLOPS, 4),
                **(traffic_fields(traffic, name, kernel_of[dom], digest) if not (args.gathered or args.update_tau)
                   else {"traffic": None, "traffic_source": "not profiled in this mode"}),
                "algorithmic_flop_per_launch": alg[dom], "avg_launch_ms": round(phase_ms[dom], 5),
                "avg_launch_ms_with_event_cost": round(raw_phase_ms[dom], 5), "event_cost_ms_per_kernel": round(event_cost_ms, 5),
                "timing": "HIP events around each kernel on the launch stream, %d extra steps, each behind 3 untimed ones; "
                          "the cost of an event pair (sum of the bracketed kernels minus the step timed without events, per "
                          "kernel) subtracted" % KE}
    # what the matrix cores deliver on this machine in the same launch shape with nothing else in the way (a committed
    # measurement kernel: 256 workgroups x 8 waves, two per SIMD, register operands, no memory traffic)
    mws = torch.empty(256 * 128 + 2048, dtype=torch.uint8, device=dev)
    for _ in range(3):
        mc = fc.fastclip_measure_mfma_ceiling(256, 4096, mws)
    roofline["mfma_ceiling"] = {"measured_tflops": round(mc["tflops"], 1), "clock_ghz_under_load": round(mc["ghz"], 3),
                                "cycles_per_mfma_seen_by_a_wave": round(mc["cycles_per_mfma"], 2),
                                "frac_of_peak": round(mc["tflops"] * 1e12 / PEAK_BF16_FLOPS, 4),
                                "kernel_frac_of_measured_ceiling": round(achieved / mc["tflops"], 4),
                                "kind": "k_mfma_ceiling: independent 32x32x16 bf16 MFMAs on pseudo-random register operands"}
    # what the two MFMA kernels execute: whole 256-row tiles, two strips unless the whole batch is local in whole
    # tiles on more tiles than compute units (one similarity pass), two contractions over the padded column range
    up = lambda x, m: (x + m - 1) // m * m
    tile = plan["tile"]
    executed = {"strips": (1 if plan["single_pass"] else 2) * 2.0 * up(b, tile) * up(B, tile) * d,
                "contract": 2 * 2.0 * up(b, tile) * up(B, 64) * up(d, tile)}
    gemm_ms = phase_ms["strips"] + phase_ms["contract"]
    gemm_phases = {"algorithmic_tflops": round((alg["strips"] + alg["contract"]) / (gemm_ms * 1e-3) / 1e12, 2),
                   "frac_of_bf16_peak": round((alg["strips"] + alg["contract"]) / (gemm_ms * 1e-3) / PEAK_BF16_FLOPS, 4),
                   "strips_tflops": round(alg["strips"] / (phase_ms["strips"] * 1e-3) / 1e12, 2),
                   "contract_tflops": round(alg["contract"] / (phase_ms["contract"] * 1e-3) / 1e12, 2),
                   "executed_tflops": round((executed["strips"] + executed["contract"]) / (gemm_ms * 1e-3) / 1e12, 2)}

    out = {"metric": "FCCO loss fwd+bwd anchors/sec", "value": round(anchors_per_s, 1), "unit": "anchors/s",
           "n_gpus": 1, "steps": K, "warmup": W, "prewarm_steps": args.prewarm, "ms_per_step": round(ms_per_step, 5),
           "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": w["dtype"], "data": "synthetic",
           "config": {"workload": "%s: b=%d local anchors x B=%d global pairs, d=%d %s, N=%d state entries, "
                                  "FastCLIP-v%d%s" % (name, b, B, d, w["dtype"], N, version,
                                                      (", gathered state of all workers" if args.gathered else "") +
                                                      (", temperature update fused in" if args.update_tau else "")),
                      "B": B, "b": b, "off": off, "d": d, "N": N, "version": version,
                      "state_layout": "one 32-byte record {u_1, tau_1, m_1, v_1, u_2, tau_2, m_2, v_2} per sample"
                                      if records is not None else "dense arrays",
                      "plan": plan},
           "sources": digest,
           "step_ms_hip_events": step_ms, "step_ms_hip_graph_replay": round(graph_ms, 5), "roofline": roofline, "gemm_phases": gemm_phases,
           "phase_ms": {k: round(v, 5) for k, v in phase_ms.items()},
           "phase_ms_with_event_cost": {k: round(v, 5) for k, v in raw_phase_ms.items()}}

    # ---- context: the same step with stock PyTorch-ROCm ops on this GPU (what framework tensor ops give)
    if not (args.no_stock_ops or args.gathered or args.update_tau):
        us1, us2 = torch.zeros(N, **f32), torch.zeros(N, **f32)
        tau_of = lambda t, arr: arr.index_select(0, idx_sets[t % n_sets]) if version == fc.V2 else tau.expand(b)
        run = lambda t: stock_ops_step(torch, img, txt, idx_sets[t % n_sets], us1, us2, tau_of(t, tau_img), tau_of(t, tau_txt), off=off,
                                       b=b, gamma=gamma_at(t), eps=w["eps"], rho=w["rho"], version=version, scale=1.0 / N)
        # one step of each from the same fresh state: the two must tell the same story (a sanity check, not parity)
        if records is not None:
            rec_c = torch.zeros(N, 8, **f32)
            uc1, tc1, uc2, tc2 = rec_c[:, 0], rec_c[:, 1], rec_c[:, 4], rec_c[:, 5]
            tc1.fill_(w["tau"])
            tc2.fill_(w["tau"])
        else:
            rec_c, uc1, uc2, tc1, tc2 = None, torch.zeros(N, **f32), torch.zeros(N, **f32), tau_img, tau_txt
        fc.fastclip_step(cfgs[0], fc.make_buffers(img_glob=img, txt_glob=txt, idx=idx_sets[0], u_img=uc1, u_txt=uc2, tau=tau,
                                                  tau_img=tc1, tau_txt=tc2, d_img=d_img, d_txt=d_txt, loss=loss,
                                                  d_tau=d_tau, d_tau_img=d_tau_img, d_tau_txt=d_tau_txt), ws)
        s_loss, s_dimg, _, _ = run(0)
        torch.cuda.synchronize()
        loss_diff = abs(float(s_loss) - float(loss)) / abs(float(loss))
        grad_diff = float((s_dimg - d_img).abs().max() / d_img.abs().max())
        del uc1, uc2, tc1, tc2, rec_c
        Ks = min(K, 20)
        for t in range(1, 3):
            run(t)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for t in range(3, 3 + Ks):
            run(t)
        e1.record()
        torch.cuda.synchronize()
        stock_ms = e0.elapsed_time(e1) / Ks
        out["stock_ops_baseline"] = {"value": round(b / (stock_ms * 1e-3), 1), "unit": "anchors/s",
                                     "ms_per_step": round(stock_ms, 4), "steps": Ks,
                                     "kind": "the same step with stock PyTorch-ROCm ops on the same GPU: bf16 matmul, "
                                             "fp32 element-wise, index_select / index_copy_; context, not the product",
                                     "speedup_of_this_library": round(stock_ms / ms_per_step, 2),
                                     "loss_rel_diff": float("%.3g" % loss_diff), "d_img_rel_inf_diff": float("%.3g" % grad_diff)}
        del us1, us2

    # ---- the state phase on its own on many indices: the HBM-bound part of the method.  fastclip_state_phase runs the
    # kernel and the per-anchor code of the step's state phase (FastCLIP-v2: gather of u and tau by dataset index, Eq. 1,
    # coefficients, Eq. 9, loss partials, and the AdamW step of the same samples' temperatures) given the sums over the
    # contrasts, on the workload's N samples.
    if not args.no_state_bench:
        ev = lambda: torch.cuda.Event(enable_timing=True)
        # the step's buffers are no longer needed: the state of N samples is allocated three times over below
        del cfgs, bufs, step
        if records is not None:
            del u_img, tau_img, m_img, v_img, u_txt, tau_txt, m_txt, v_txt, records
        else:
            del u_img, u_txt, tau_img, tau_txt
        torch.cuda.empty_cache()

        def timed(fn, reps=10):
            for _ in range(2):
                fn()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        # what a plain streaming copy reaches on this machine (1 GiB read + 1 GiB written): the practical HBM ceiling
        src = torch.empty(1 << 28, **f32)
        dst = torch.empty_like(src)
        copy_ms = timed(lambda: dst.copy_(src), reps=5)
        copy_gbps = 2.0 * src.numel() * 4 / (copy_ms * 1e-3) / 1e9
        del src, dst
        n_max = min(1 << 24, N)          # distinct indices: at most N of them
        perm = torch.randperm(N, device=dev)[:n_max].contiguous()
        sums = torch.rand(4, n_max, **f32) * 100 + 1
        coef = torch.empty(3, n_max, **f32)
        o_t1, o_t2 = torch.empty(n_max, **f32), torch.empty(n_max, **f32)
        s_loss = torch.empty(1, **f32)
        sws = torch.empty(fc.fastclip_state_phase_workspace_bytes(n_max), dtype=torch.uint8, device=dev)
        # algorithmic bytes per index of this work: idx 8, four sums 16, the sample's eight state words read 32 and
        # written 32, the three coefficients 12, the two temperature gradients 8
        ALG = 108.0
        FIELDS = ("u_img", "tau_img", "m_img", "v_img", "u_txt", "tau_txt", "m_txt", "v_txt")

        def run_layout(layout, n_list):
            if layout == "dense":
                fld = {k: torch.zeros(N, **f32) for k in FIELDS}
                sstride = 1
            else:
                sstride = 16 if layout == "records16" else 8
                rec = torch.zeros(N, sstride, **f32)
                fld = {k: rec[:, i] for i, k in enumerate(FIELDS)}
            fld["tau_img"].fill_(w["tau"])
            fld["tau_txt"].fill_(w["tau"])
            tst = fc.make_tau_state(**{k: fld[k] for k in FIELDS if not k.startswith("u_")})
            upd = fc.make_tau_update(optimizer=fc.TAU_ADAMW, step=10, lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8,
                                     tau_min=0.01, state_stride=sstride)
            res = []
            for n_idx in n_list:
                scfg = fc.make_config(version=fc.V2, emb_dtype=fc.BF16, B=B, b=n_idx, off=0, d=8, N=N, gamma=0.5,
                                      eps=w["eps"], rho=w["rho"], tau_grad_scale=1.0 / N, state_stride=sstride)
                sbuf = fc.make_buffers(idx=perm, u_img=fld["u_img"], u_txt=fld["u_txt"], tau_img=fld["tau_img"],
                                       tau_txt=fld["tau_txt"], loss=s_loss, d_tau_img=o_t1, d_tau_txt=o_t2)
                ms = timed(lambda: fc.fastclip_state_phase(scfg, sbuf, upd, tst, sums, coef, sws))
                res.append({"n_idx": n_idx, "ms": round(ms, 5), "algorithmic_GBps": round(ALG * n_idx / (ms * 1e-3) / 1e9, 1)})
            assert torch.isfinite(s_loss).all()
            if layout == "records8":     # the same records, read and written back with nothing else in the way
                ms = timed(lambda: fc.fastclip_measure_record_rmw(perm, n_list[-1], N, rec, sstride))
                res.append({"n_idx": n_list[-1], "ms": round(ms, 5), "Grecords_per_s": round(n_list[-1] / (ms * 1e-3) / 1e9, 2)})
            return res

        sweep = run_layout("records8", sorted({min(b, n_max), min(1 << 15, n_max), min(1 << 20, n_max), n_max}))
        bare = sweep.pop()
        n_idx, ms = sweep[-1]["n_idx"], sweep[-1]["ms"]
        su = {"kernel": "k_state", "workload": "state phase of FastCLIP-v2 with the AdamW step of the temperatures on %d "
                                               "distinct random samples of N = %d, one 32-byte record per sample" % (n_idx, N),
              "n_idx": n_idx, "N": N, "ms": round(ms, 4), "bound": "hbm",
              "achieved": round(ALG * n_idx / (ms * 1e-3) / 1e9, 1), "peak": PEAK_HBM_BYTES / 1e9, "unit": "GB/s",
              "frac": round(ALG * n_idx / (ms * 1e-3) / PEAK_HBM_BYTES, 4), "algorithmic_bytes_per_index": ALG,
              "sweep": sweep, "copy_ceiling_GBps": round(copy_gbps, 1),
              "algorithmic_frac_of_copy_ceiling": round(ALG * n_idx / (ms * 1e-3) / 1e9 / copy_gbps, 4)}
        tf = traffic_fields(traffic, name, "k_state_records8_2^24", digest) if n_idx == 1 << 24 else \
            {"traffic": None, "traffic_source": "profiled at 2^24 indices only"}
        # a bare read-modify-write of the same records (committed measurement kernel): what the memory system delivers
        # for random 32-byte records; the state kernel's share of that rate
        su["bare_record_rmw"] = dict(bare, state_kernel_frac_of_this_rate=round(bare["ms"] / ms, 4),
                                     kind="k_record_rmw: 16 bytes per lane read, one multiply-add, written back")
        su.update(tf)
        if su["traffic"] is not None:      # what the memory system moves for these random 32-byte accesses
            su["traffic_over_algorithmic"] = round(su["traffic"] / (ALG * n_idx), 3)
            su["traffic_frac_of_peak"] = round(su["traffic"] / (ms * 1e-3) / PEAK_HBM_BYTES, 4)
            su["traffic_frac_of_copy_ceiling"] = round(su["traffic"] / (ms * 1e-3) / 1e9 / copy_gbps, 4)
        su["records_of_16_floats"] = run_layout("records16", [n_max])[0]
        su["dense_arrays"] = run_layout("dense", [n_max])[0]
        out["state_update"] = su
        del perm, sums, coef, o_t1, o_t2, sws
        torch.cuda.empty_cache()

    # ---- the CPU oracle on the same workload (whole steps), on the host cores of this machine: with the threads its BLAS
    # takes by itself, and with one thread
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_info, threadpool_limits

        from oracle import fcco_step
        img64, txt64 = img32.astype(np.float64), txt32.astype(np.float64)
        tau_c = np.full(b, float(np.float32(w["tau"])))

        def oracle_steps(budget_s, max_reps):
            u1, u2 = np.zeros(b), np.zeros(b)
            reps = 0
            c0 = time.perf_counter()
            while True:
                fcco_step(img64, txt64, off, b, np.arange(b), u1, u2, version=version, gamma=gamma_at(0), eps=w["eps"],
                          rho=w["rho"], tau=tau_c[0], tau_img=tau_c, tau_txt=tau_c, tau_grad_scale=1.0 / N)
                reps += 1
                if time.perf_counter() - c0 > budget_s or reps >= max_reps:
                    break
            return (time.perf_counter() - c0) / reps, reps

        cpu_s, reps = oracle_steps(10.0, 20)
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        with threadpool_limits(limits=1):
            one_s, one_reps = oracle_steps(8.0, 5)
        try:
            usable = len(os.sched_getaffinity(0))
        except AttributeError:
            usable = os.cpu_count()
        out["cpu_baseline"] = {"value": round(b / cpu_s, 1), "unit": "anchors/s", "cores": int(os.cpu_count()),
                               "cores_usable": int(usable), "threads": int(threads), "kind": "oracle",
                               "sample": "%d full step(s) of %s (all %d anchors), fp64 numpy, %.2f s per step with the "
                                         "BLAS library's own %d threads" % (reps, name, b, cpu_s, threads),
                               "one_thread": {"value": round(b / one_s, 1), "unit": "anchors/s",
                                              "sample": "%d full step(s), %.2f s per step" % (one_reps, one_s)}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
