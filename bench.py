#!/usr/bin/env python3
"""Benchmark of the Write-Gated KV hot path on one MI355X.

A step is one new token for the whole batch through every layer of the workload:
`wgkv_decode_promote` once (victim test, page hand-out and row move of the lazy
promotion of all layers), then per layer `wgkv_decode_step` (the ring write) and
`wgkv_attend` (ragged paged GQA decode attention).  `--no-promote-ahead` leaves the
first call out: every layer's `wgkv_decode_step` then does its promotion itself.  Inputs are synthetic, seeded and already
resident in HBM when the timed region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

With `--workload llama8b_chunked_prefill_128k` a step is instead one chunk of the
batch's prompts through one layer (linear gate -> chunk attention under the
vertical-slash mask on the matrix cores -> admission), the roofline object then
describes the chunk-attention kernel against the dense bf16 MFMA peak, and the
chunks before the timed ones are the warm-up (they have to run anyway: they
fill the cache the timed chunks attend over).
"""
import argparse
import ctypes as C
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E published peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class HipEvents:
    """Raw HIP events (the library hands them to the launch of its decode attention kernel, whose begin and
    end time stamps they take, or records them before and after its prefill attention kernels)."""

    def __init__(self, n):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [C.c_void_p]
        self.hip.hipEventDestroy.argtypes = [C.c_void_p]
        self.ev = []
        for _ in range(n):
            e = C.c_void_p()
            assert self.hip.hipEventCreate(C.byref(e)) == 0
            self.ev.append(e.value)

    def elapsed_ms(self, a, b):
        ms = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b))
        assert rc == 0, rc
        return ms.value

    def destroy(self):
        for e in self.ev:
            self.hip.hipEventDestroy(C.c_void_p(e))


def attend_algorithmic_bytes(cfg, seq_len, global_len, layers):
    """Bytes one decode-attention launch must move: K and V rows of the valid
    tokens, the page-table entries that locate them, q in and out out."""
    es = 4 if cfg.dtype == "f32" else 2
    d, P, W, G = cfg.head_dim, cfg.page_size, cfg.w_local, cfg.n_q_heads // cfg.n_kv_heads
    nlp = -(-W // P)
    per_layer = []
    for l in layers:
        t = seq_len[:, l].astype(np.int64)                     # [B]
        gl = global_len[:, l, :].astype(np.int64)              # [B, H]
        tok = np.minimum(t, W)[:, None] + gl
        b = tok * 2 * d * es + 4 * (nlp + -(-gl // P)) + G * d * es + G * d * 4
        per_layer.append(int(b.sum()))
    return per_layer


def events_ok(args):
    return not args.no_kernel_events


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="llama8b_32layer_b8_128k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--event-every", type=int, default=8, metavar="N",
                    help="a pair of HIP events goes with every N-th launch of the attention kernel, rotating over the "
                         "layers (a timed launch costs a few us of GPU time more than an untimed one, which would add "
                         "several per cent to the step if every launch carried a pair)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="skip the per-kernel HIP events (roofline.achieved becomes null)")
    ap.add_argument("--ctx-scale", type=float, default=1.0, help="shrink contexts (debugging only)")
    ap.add_argument("--ctx-fixed", type=int, default=0, metavar="TOKENS",
                    help="decode workloads: every sequence gets exactly this context instead of the workload's "
                         "draw (the supplementary fixed point: 131072 for llama8b_32layer_b8_128k)")
    ap.add_argument("--gate", choices=["linear", "mlp"], default="linear",
                    help="chunked-prefill workload only: the workload's linear gate on the hidden state, or the "
                         "Write-Gate MLP (width 4*head_dim, random weights) on the keys before/after the rotary embedding")
    ap.add_argument("--select-pages", type=int, default=0,
                    help="decode workloads: read only this many pages of each head's global cache per step, picked "
                         "with key landmarks (128 pages of 16 = the 2048 KVs per query of the paper's selection run); "
                         "the step then is promotion + landmark upkeep + page scoring/selection + attention")
    ap.add_argument("--no-promote-ahead", action="store_true",
                    help="decode workloads: no wgkv_decode_promote at the start of a step (each layer's "
                         "wgkv_decode_step then decides and moves its promotions itself)")
    ap.add_argument("--no-tune", action="store_true",
                    help="decode workloads: no wgkv_tune_decode_attention before the timed steps (the split of the "
                         "tiles between the XCDs of a pair then keeps its default of 50 per mille)")
    ap.add_argument("--graph", action="store_true",
                    help="decode workloads: capture one whole step (all layers) in a HIP graph and time replays "
                         "instead of direct calls (per-kernel events are then not available)")
    ap.add_argument("--evict", action="store_true",
                    help="time the budgeted eviction (scoring from a 256-query observation window + removal of the "
                         "lowest 10 %) on one layer of the workload's batch with about 4.5K global entries per head")
    ap.add_argument("--soft-attn", type=int, default=0, metavar="TOKENS",
                    help="time the training-time Write-Gated Attention (forward + backward) of one layer on one "
                         "sequence of TOKENS tokens with the workload's head shape (the paper trains on samples of "
                         "4K to 32K tokens, batch size 1)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB read + 1 GiB write elementwise kernel (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_17452_amd as wg
    import wgkv_workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = wl.get_config(args.workload)
    if args.evict:
        return main_evict(args, cfg, torch, wg, wl, dev)
    if args.soft_attn:
        return main_soft_attn(args, cfg, torch, wg, wl, dev)
    if cfg.chunk:
        return main_prefill(args, cfg, torch, wg, wl, dev)
    B, L, Hq, Hk, d, W, P = cfg.batch, cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local, cfg.page_size
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    ctx = wl.context_lengths(cfg)
    if args.ctx_scale != 1.0:
        ctx = np.maximum((ctx * args.ctx_scale).astype(np.int64), W + 1)
    if args.ctx_fixed:
        ctx = np.full_like(ctx, max(args.ctx_fixed, W + 1))
    rates = wl.unit_rates(cfg)
    total_steps = args.steps + args.warmup
    max_ctx = int(ctx.max())

    # pool: expected admitted tokens + 10 % + room for the host's worst-case bound of one prefill call
    exp_tokens = sum(float(rates[l, h]) * int(c) for c in ctx for l in range(L) for h in range(Hk))
    exp_pages = exp_tokens / P * 1.10 + B * L * Hk * (-(-W // P) + 2 + -(-total_steps // P))
    n_pages = int(exp_pages) + Hk * (max_ctx // P + 2) + 1024
    max_gp = (max_ctx + total_steps) // P + 2
    wcfg = wg.Config(L, Hq, Hk, d, wg.F32 if cfg.dtype == "f32" else wg.BF16, P, W, B, max_gp, n_pages)
    t_setup = time.time()
    pool = wg.Pool(wcfg, max_call_seqs=B, max_call_tokens=max_ctx)
    log(f"[bench] workload {cfg.name}: B={B} L={L} ctx={ctx.tolist()} pool {n_pages} pages "
        f"({pool.pool_buf.numel() / 2**30:.1f} GiB)")

    def gen_prefill(seq, layer):
        n = int(ctx[seq])
        k = wl.draw_normal(cfg, "k", (n, Hk, d), device=dev, key=(seq, layer))
        v = wl.draw_normal(cfg, "v", (n, Hk, d), device=dev, key=(seq, layer))
        g = torch.from_numpy(wl.draw_scores(cfg, seq, layer, n, rates)).to(dev)
        return k, v, g

    for layer in range(L):
        for seq in range(B):
            k, v, g = gen_prefill(seq, layer)
            pool.prefill_admit(layer, [seq], [int(ctx[seq])], k, v, g, tau=cfg.tau)
            free, flag = pool.status()
            assert flag == 0, f"device error flag {flag}"
        if layer % 8 == 7:
            log(f"[bench] prefilled layer {layer + 1}/{L}, free pages {free}")
    del k, v, g
    seqs = list(range(B))
    # decode inputs: one K/V/Q set per layer (reused every step), fresh scores every step
    k_new = [wl.draw_normal(cfg, "dec_k", (B, Hk, d), device=dev, key=(l,)) for l in range(L)]
    v_new = [wl.draw_normal(cfg, "dec_v", (B, Hk, d), device=dev, key=(l,)) for l in range(L)]
    q_new = [wl.draw_normal(cfg, "q", (B, Hq, d), device=dev, key=(l,)) for l in range(L)]
    g_steps = np.stack([np.stack([np.concatenate([wl.draw_scores(cfg, s, l, 1, rates, purpose="dec_scores", step=st)
                                                  for s in range(B)]) for l in range(L)])
                        for st in range(total_steps)])            # [steps, L, B, Hk]
    g_new = torch.from_numpy(g_steps).to(dev)
    out = torch.empty((L, B, Hq, d), dtype=torch.float32, device=dev)
    scale = 1.0 / math.sqrt(d)
    log(f"[bench] setup {time.time() - t_setup:.1f}s")

    sel_b = args.select_pages
    promote_ahead = not args.no_promote_ahead
    if sel_b:
        lm = pool.quest_landmarks()
        pool.status()
        n_units = B * Hk
        pg_stride = int(pool.meta()["global_len"].max().item()) // P + total_steps // P + 4
        sel_scores = torch.zeros((n_units, pg_stride), dtype=torch.float32, device=dev)
        sel_pages = torch.zeros((n_units, sel_b), dtype=torch.int32, device=dev)
        sel_count = torch.zeros((n_units,), dtype=torch.int32, device=dev)
        for l in range(L):
            pool.quest_update(l, seqs, lm)
        _p, _i, _chk = wg.binding._ptr, wg.binding._ids, wg.binding._check

    def one_step(st, events=None):
        if promote_ahead:
            pool.decode_promote(seqs, tau=cfg.tau)
        for l in range(L):
            pool.decode_step(l, seqs, k_new[l], v_new[l], g_new[st, l], tau=cfg.tau)
            if sel_b:
                pool.quest_update(l, seqs, lm)
                _chk(pool.L.wgkv_quest_select(pool.h, l, B, _i(seqs), _p(q_new[l]), _p(lm), lm.numel(), sel_b,
                                              _p(sel_scores), pg_stride, _p(sel_pages), _p(sel_count),
                                              wg.binding._stream()), "wgkv_quest_select")
            if events is not None:
                if (st + l) % args.event_every == 0 and sampled[0] < n_sampled_max:
                    i = sampled[0]
                    sampled[0] += 1
                    pool.set_profile_events(events.ev[2 * i], events.ev[2 * i + 1])
                    armed[0] = True
                elif armed[0]:
                    pool.set_profile_events(None, None)
                    armed[0] = False
            if sel_b:
                pool.attend_selected(l, seqs, q_new[l], sel_pages, sel_count, out[l], scale)
            else:
                pool.attend(l, seqs, q_new[l], out[l], scale)

    for st in range(args.warmup):
        one_step(st)
    torch.cuda.synchronize()
    # the split of a launch's tiles over the XCDs, tuned to this machine on the workload's own cache (untimed
    # set-up, a few milliseconds; the cache is not changed)
    xcd_skew = None
    if not args.no_tune and not sel_b:
        xcd_skew = pool.tune_decode_attention(seqs, q_new[0], out[0], scale)
        log(f"[bench] split correction between the XCDs of a pair kept by the tuning: {xcd_skew} per mille")
    graph = None
    if args.graph:
        assert not sel_b, "--graph times the plain decode step"
        args.no_kernel_events = True
        g_static = torch.zeros_like(g_new[0])                     # [L, B, Hk] scores of the step being replayed
        graph, side = torch.cuda.CUDAGraph(), torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                if promote_ahead:
                    pool.decode_promote(seqs, tau=cfg.tau)
                for l in range(L):
                    pool.decode_step(l, seqs, k_new[l], v_new[l], g_static[l], tau=cfg.tau)
                    pool.attend(l, seqs, q_new[l], out[l], scale)
        torch.cuda.current_stream().wait_stream(side)
        pool.status()                                             # capturing ran nothing: the host counts are reset to the device's
    meta = pool.meta()
    sl0, gl0 = meta["seq_len"].cpu().numpy(), meta["global_len"].cpu().numpy()
    n_sampled_max = args.steps * L // max(args.event_every, 1) + L
    sampled, armed = [0], [False]
    events = None if args.no_kernel_events else HipEvents(2 * n_sampled_max)
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # one between every two steps
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_ev[0].record()
    for st in range(args.warmup, total_steps):
        if graph is not None:
            g_static.copy_(g_new[st])
            graph.replay()
        else:
            one_step(st, events)
        step_ev[st - args.warmup + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = step_ev[0].elapsed_time(step_ev[-1])
    step_us = np.array([step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(args.steps)]) * 1e3
    ms_per_step = max(wall_ms, gpu_ms) / args.steps
    pool.set_profile_events(None, None)
    free, flag = pool.status()
    assert flag == 0
    sl1, gl1 = meta["seq_len"].cpu().numpy(), meta["global_len"].cpu().numpy()

    bytes0 = attend_algorithmic_bytes(cfg, sl0, gl0, range(L))
    bytes1 = attend_algorithmic_bytes(cfg, sl1, gl1, range(L))
    bytes_per_launch = 0.5 * (np.mean(bytes0) + np.mean(bytes1))
    if sel_b:   # the attention kernel reads the window and at most sel_b pages per head
        capped = [attend_algorithmic_bytes(cfg, s_, np.minimum(g_, sel_b * P), range(L)) for s_, g_ in ((sl0, gl0), (sl1, gl1))]
        bytes_per_launch = 0.5 * (np.mean(capped[0]) + np.mean(capped[1]))
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                "traffic": None, "kernel": "attend_decode_kernel",
                "algorithmic_bytes_per_launch": bytes_per_launch}
    if events is not None:
        durs = np.array([events.elapsed_ms(events.ev[2 * i], events.ev[2 * i + 1]) for i in range(sampled[0])])
        avg_us = float(durs.mean() * 1e3)
        roofline.update({"achieved": bytes_per_launch / (avg_us * 1e-6) / 1e9,
                         "frac": bytes_per_launch / (avg_us * 1e-6) / 1e9 / HBM_PEAK_GBS,
                         "kernel_avg_us": avg_us, "kernel_p10_us": float(np.percentile(durs, 10) * 1e3),
                         "kernel_p50_us": float(np.percentile(durs, 50) * 1e3),
                         "kernel_p90_us": float(np.percentile(durs, 90) * 1e3), "launches": int(len(durs))})
        events.destroy()
    if args.calibrate_copy:   # known traffic: reads 2^30 bytes, writes 2^30 bytes per launch
        src = torch.zeros(2 ** 28, dtype=torch.int32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst
    # What a pure read of the same number of bytes takes on this machine, measured now: the library's
    # streaming probe over slices of the pool (fresh memory every launch), timed by its own dispatch.
    if events_ok(args) and not sel_b:
        n_probe = 12
        pe = HipEvents(2 * n_probe)
        nb = int(bytes_per_launch) // 4096 * 4096
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        span = pool.pool_buf.numel()
        for i in range(n_probe):
            off = (i * (nb + (1 << 24))) % max(span - nb, 1) // 4096 * 4096
            wg.stream_read_probe(pool.pool_buf[off:], nb, sink, pe.ev[2 * i], pe.ev[2 * i + 1])
        torch.cuda.synchronize()
        pd = np.array([pe.elapsed_ms(pe.ev[2 * i], pe.ev[2 * i + 1]) for i in range(2, n_probe)]) * 1e3
        pe.destroy()
        ceil_gbs = nb / (float(pd.mean()) * 1e-6) / 1e9
        roofline.update({"measured_read_ceiling": ceil_gbs, "measured_read_ceiling_us": float(pd.mean()),
                         "frac_of_measured_ceiling": (roofline["achieved"] / ceil_gbs) if roofline["achieved"] else None})
    # HBM bytes per launch measured with rocprofv3 counters in a run of their own; the summary names the
    # commands and the kernel source it was taken from.  It is quoted only while that source is unchanged.
    traffic_file = os.path.join("profiles", f"attend_decode_kernel_{cfg.name}_hbm_traffic.txt")
    roofline["traffic_source"] = None
    if os.path.exists(os.path.join(ROOT, traffic_file)) and not sel_b and not args.ctx_fixed and args.ctx_scale == 1.0:
        import hashlib
        src = os.path.join(ROOT, "paper_2512_17452_amd", "csrc", "attend_decode.hip")
        sha_now = hashlib.sha256(open(src, "rb").read()).hexdigest()
        traffic, sha_file, commit = None, None, None
        for line in open(os.path.join(ROOT, traffic_file)):
            if line.startswith("hbm_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
            elif line.startswith("kernel_source_sha256:"):
                sha_file = line.split(":")[1].strip()
            elif line.startswith("taken_at_commit:"):
                commit = line.split(":")[1].strip()
        if sha_file == sha_now:
            roofline["traffic"] = traffic
            roofline["traffic_source"] = f"{traffic_file} (rocprofv3 FETCH_SIZE + WRITE_SIZE runs at commit {commit}; " \
                                         f"attend_decode.hip unchanged since)"
        else:
            roofline["traffic_source"] = f"{traffic_file} is from another version of attend_decode.hip: not quoted"

    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = run_cpu_baseline(cfg, wl, ctx, rates, dev, gen_prefill, k_new[0], v_new[0], g_new[0, 0],
                                        q_new[0], scale, pool, seqs)

    res = {
        "metric": "decode_step_latency_us (all layers: lazy promotion + ragged paged GQA decode attention)" if not sel_b else
                  "decode_step_latency_us (all layers: lazy promotion + landmark upkeep + page selection + attention over window and selected pages)",
        "value": ms_per_step * 1e3, "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "layers": L, "q_heads": Hq, "kv_heads": Hk, "head_dim": d,
                   "w_local": W, "page_size": P, "tau": cfg.tau, "ctx_min": int(ctx.min()), "ctx_max": int(ctx.max()),
                   "select_pages": sel_b, "hip_graph": bool(args.graph), "promote_ahead": promote_ahead, "xcd_skew_permille": xcd_skew,
                   "mean_cached_tokens_per_head": float((np.minimum(sl1, W)[:, :, None] + gl1).mean()),
                   # the paper's x axis: cached entries of a head over the tokens it has seen, (W + G_h) / t
                   "normalized_kv_size": float(((np.minimum(sl1, W)[:, :, None] + gl1) / np.maximum(sl1, 1)[:, :, None]).mean()),
                   "step_p10_us": float(np.percentile(step_us, 10)), "step_p50_us": float(np.percentile(step_us, 50)),
                   "step_p90_us": float(np.percentile(step_us, 90)),
                   "attend_us_per_layer": roofline.get("kernel_avg_us"),
                   "gpu_ms_per_step": gpu_ms / args.steps, "host_wall_ms_per_step": wall_ms / args.steps},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(res), flush=True)


def main_evict(args, cfg, torch, wg, wl, dev):
    """One layer of the workload's batch, every head filled to a little above the paper's budget of 4096
    entries, then `--steps` rounds of scoring + removal (each round refills what was removed)."""
    B, Hq, Hk, d, W, P = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local, cfg.page_size
    n_obs, frac, target = 256, 0.1, 4500
    T = 2 * target + W                                   # scores uniform in (0,1), tau 0.5: half is admitted
    max_gp = T // P + 4
    pool = wg.Pool(wg.Config(1, Hq, Hk, d, wg.BF16, P, W, B, max_gp, B * Hk * (max_gp + -(-W // P)) + 64), B, T)
    seqs = list(range(B))
    gen = torch.Generator(device=dev).manual_seed(cfg.seed)

    def feed(n):
        for s_ in seqs:
            k = wl.draw_normal(cfg, "k", (n, Hk, d), device=dev, key=(s_, n))
            v = wl.draw_normal(cfg, "v", (n, Hk, d), device=dev, key=(s_, n))
            g = torch.rand((n, Hk), generator=gen, device=dev)
            pool.prefill_admit(0, [s_], [n], k, v, g, tau=0.5)

    feed(T)
    q_obs = wl.draw_normal(cfg, "q", (B, n_obs, Hq, d), device=dev)
    scale = 1.0 / math.sqrt(d)
    steps = min(args.steps, 16)
    t_score, t_apply, flops, removed = [], [], [], 0
    for st in range(args.warmup + steps):
        pool.status()
        gl = pool.meta()["global_len"][:, 0, :].cpu().numpy().astype(np.int64)
        stride = int(gl.max()) + 16
        raw = torch.empty((B * Hk, stride), dtype=torch.float32, device=dev)
        out = torch.empty_like(raw)
        gone = torch.zeros((B * Hk,), dtype=torch.int32, device=dev)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        wg.binding._check(pool.L.wgkv_evict_scores(pool.h, 0, B, wg.binding._ids(seqs), wg.binding._ptr(q_obs), n_obs, scale, 5,
                                                   wg.binding._ptr(raw), wg.binding._ptr(out), stride,
                                                   wg.binding._ptr(pool.workspace), pool.workspace.numel(),
                                                   wg.binding._stream()), "wgkv_evict_scores")
        ev[1].record()
        pool.evict_apply(0, seqs, out, frac, n_evicted_out=gone)
        ev[2].record()
        torch.cuda.synchronize()
        if st >= args.warmup:
            t_score.append(ev[0].elapsed_time(ev[1]))
            t_apply.append(ev[1].elapsed_time(ev[2]))
            flops.append(2.0 * 2.0 * d * n_obs * (Hq // Hk) * float(gl.sum()))      # two sweeps of Q K^T
            removed += int(gone.sum())
        feed(2 * int(frac * target))                      # grow back to about the same size
    ms = float(np.mean(t_score) + np.mean(t_apply))
    tflops = float(np.sum(flops)) / float(np.sum(t_score)) / 1e9
    res = {
        "metric": "eviction_round_latency_us (one layer: importance scores from 256 observation queries + removal of the lowest 10 %)",
        "value": ms * 1e3, "unit": "us/round", "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name + " (one layer, heads filled to ~4.5K global entries)", "batch": B, "kv_heads": Hk,
                   "q_heads": Hq, "head_dim": d, "page_size": P, "n_obs": n_obs, "pool_w": 5, "frac": frac,
                   "scores_us": float(np.mean(t_score) * 1e3), "apply_us": float(np.mean(t_apply) * 1e3),
                   "entries_removed_per_round": removed / steps},
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                     "kernel": "evict_stats_mfma_kernel + evict_weights_mfma_kernel"},
        "cpu_baseline": None,
    }
    print(json.dumps(res), flush=True)


def main_soft_attn(args, cfg, torch, wg, wl, dev):
    """One layer of training-time Write-Gated Attention: forward, then backward, on one sequence."""
    T, Hq, Hk, d, W = args.soft_attn, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local
    eps, scale = 1e-6, 1.0 / math.sqrt(d)
    rates = wl.unit_rates(cfg)
    q = wl.draw_normal(cfg, "q", (T, Hq, d), device=dev)
    k = wl.draw_normal(cfg, "k", (T, Hk, d), device=dev)
    v = wl.draw_normal(cfg, "v", (T, Hk, d), device=dev)
    dout = wl.draw_normal(cfg, "dout", (T, Hq, d), device=dev)
    g = wl.draw_scores(cfg, 0, 0, T, rates, device=dev)
    steps, warmup = min(args.steps, 16), min(args.warmup, 2)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for i in range(warmup + steps):
        if i >= warmup:
            ev[i - warmup][0].record()
        out, lse = wg.soft_attn_forward(q, k, v, g, [T], W, scale, eps)
        if i >= warmup:
            ev[i - warmup][1].record()
        grads = wg.soft_attn_backward(q, k, v, g, out, lse, dout, [T], W, scale, eps)
        if i >= warmup:
            ev[i - warmup][2].record()
    torch.cuda.synchronize()
    fwd = np.array([e[0].elapsed_time(e[1]) for e in ev])
    bwd = np.array([e[1].elapsed_time(e[2]) for e in ev])
    pairs = T * (T + 1) / 2.0 * Hq
    # the method's products per (query, key, query head): two forward, five backward, 2 d flop each;
    # the backward kernels here recompute the scores in both of them: seven products are executed
    f_fwd, f_bwd = 4.0 * d * pairs, 10.0 * d * pairs
    tf = (f_fwd + f_bwd) / ((fwd.mean() + bwd.mean()) * 1e-3) / 1e12
    log(f"[bench] soft attention T={T}: forward {fwd.mean():.2f} ms ({f_fwd / fwd.mean() / 1e9:.0f} TFLOP/s), "
        f"backward {bwd.mean():.2f} ms ({f_bwd / bwd.mean() / 1e9:.0f} TFLOP/s algorithmic)")
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import soft_attn_backward as o_bwd, soft_attn_forward as o_fwd
        Ts = min(T, 2048)
        f = lambda x: x[:Ts].float().cpu().numpy()
        t0 = time.perf_counter()
        o_fwd(f(q), f(k), f(v), f(g), W, scale, eps)
        o_bwd(f(q), f(k), f(v), f(g), f(dout), W, scale, eps)
        dt = time.perf_counter() - t0
        sample_pairs = Ts * (Ts + 1) / 2.0 * Hq
        cpu = {"value": dt * 1e3 * pairs / sample_pairs, "unit": "ms/step", "cores": min(os.cpu_count() or 1, 16),
               "kind": "oracle", "sample": f"forward + backward of the first {Ts} tokens, all heads, {dt:.1f} s "
               f"(forward: all host threads over query rows; backward: one thread per kv head, {Hk} of them); "
               f"scaled by the number of (query, key) pairs to {T} tokens (extrapolated)", "sample_seconds": dt}
    res = {
        "metric": "soft_attn_train_step_ms (one layer: Write-Gated Attention forward + backward, one sequence)",
        "value": float(fwd.mean() + bwd.mean()), "unit": "ms/step", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": float(fwd.mean() + bwd.mean()), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name} head shape, one sequence of {T} tokens", "q_heads": Hq, "kv_heads": Hk,
                   "head_dim": d, "w_local": W, "eps": eps, "tokens": T, "forward_ms": float(fwd.mean()),
                   "backward_ms": float(bwd.mean())},
        "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel": "soft_attn_fwd_kernel + soft_attn_bwd_*",
                     "algorithmic_flops": f_fwd + f_bwd, "forward_tflops": f_fwd / fwd.mean() / 1e9,
                     "backward_tflops": f_bwd / bwd.mean() / 1e9},
        "cpu_baseline": cpu,
    }
    print(json.dumps(res), flush=True)


def main_prefill(args, cfg, torch, wg, wl, dev):
    """Chunked prefill of the whole batch, one layer: the last `--steps` chunks are timed."""
    B, Hq, Hk, d, W, P, Cn, dim = (cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local,
                                   cfg.page_size, cfg.chunk, cfg.hidden_dim)
    G, N = Hq // Hk, cfg.ctx_max
    n_chunks = N // Cn
    steps = min(args.steps, n_chunks)
    first_timed = n_chunks - steps
    max_gp = N // P + 2
    pool = wg.Pool(wg.Config(1, Hq, Hk, d, wg.BF16, P, W, B, max_gp, B * Hk * (max_gp + W // P) + 64), B, B * Cn)
    gate_w = wl.draw_linear_gate(cfg, device=dev)
    mlp = wl.draw_gate_mlp(cfg, 4 * d, device=dev) if args.gate == "mlp" else None
    seqs, nt, scale = list(range(B)), [Cn] * B, 1.0 / math.sqrt(d)
    out = torch.empty((B * Cn, Hq, d), dtype=torch.float32, device=dev)
    # admitted-token prefix counts per (sequence, head): the visible pairs of a query at position p are
    # min(W, p+1) window keys plus the admitted keys at positions <= p-W (Sec. 4.2 mask)
    adm_prefix = torch.zeros((B, N + 1, Hk), dtype=torch.int64, device=dev)
    events = HipEvents(2 * steps)
    e_all = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    flops, gate_ms, admit_ms, wall0 = [], 0.0, 0.0, None
    for c in range(n_chunks):
        hidden = wl.draw_normal(cfg, "hidden", (B * Cn, dim), device=dev, key=(c,))
        k = wl.draw_normal(cfg, "k", (B * Cn, Hk, d), device=dev, key=(c,))
        v = wl.draw_normal(cfg, "v", (B * Cn, Hk, d), device=dev, key=(c,))
        q = wl.draw_normal(cfg, "q", (B * Cn, Hq, d), device=dev, key=(c,))
        timed = c >= first_timed
        if c == first_timed:
            torch.cuda.synchronize()
            wall0 = time.perf_counter()
            e_all[0].record()
        if timed:
            i = c - first_timed
            pool.set_profile_events(events.ev[2 * i], events.ev[2 * i + 1])
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record()
        if mlp is None:
            g = wg.gate_scores(hidden, gate_w)
        else:  # k stands in for the rotated keys, a second draw for the keys before the rotation
            k_pre = wl.draw_normal(cfg, "k_pre", (B * Cn, Hk, d), device=dev, key=(c,), std=1.5)
            if timed:
                ev[0].record()
            g = wg.gate_mlp_scores(k_pre, k, *mlp)
        if timed:
            ev[1].record()
        pool.attend(0, seqs, q, out, scale, n_q=nt, k_chunk=k, v_chunk=v, g_chunk=g, tau=cfg.tau)
        if timed:
            ev[2].record()
        pool.prefill_admit(0, seqs, nt, k, v, g, tau=cfg.tau)
        if timed:
            ev[3].record()
        # bookkeeping for the flop count (not part of the path; after the timed calls of this chunk)
        adm = (g >= cfg.tau).view(B, Cn, Hk).to(torch.int64)
        t0 = c * Cn
        adm_prefix[:, t0 + 1:t0 + Cn + 1] = adm_prefix[:, t0:t0 + 1] + torch.cumsum(adm, dim=1)
        if timed:
            pos = torch.arange(t0, t0 + Cn, device=dev)
            older = adm_prefix[:, torch.clamp(pos - W + 1, min=0)]          # admitted at positions <= pos-W
            pairs = (torch.clamp(pos + 1, max=W)[None, :, None] + older).sum()
            torch.cuda.synchronize()
            flops.append(4.0 * d * G * float(pairs))
            gate_ms += ev[0].elapsed_time(ev[1])
            admit_ms += ev[2].elapsed_time(ev[3])
    e_all[1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - wall0) * 1e3
    pool.set_profile_events(None, None)
    free, flag = pool.status()
    assert flag == 0
    durs = np.array([events.elapsed_ms(events.ev[2 * i], events.ev[2 * i + 1]) for i in range(steps)])
    events.destroy()
    path_ms = float(durs.sum()) + gate_ms + admit_ms   # the three calls of the path, without the input generation between them
    tflops = float(np.sum(flops)) / float(durs.sum()) / 1e9
    log(f"[bench] chunks {first_timed}..{n_chunks - 1}: attention {durs.sum():.1f} ms, gate {gate_ms:.2f} ms, "
        f"admit {admit_ms:.2f} ms, wall incl. input generation {wall_ms:.1f} ms")
    log("[bench] TFLOP/s of the attention kernel per timed chunk: "
        + " ".join(f"{f / t / 1e9:.0f}" for f, t in zip(flops, durs)))
    res = {
        "metric": "prefill_chunk_latency_us (one layer: write gate + chunk attention under the vertical-slash mask + admission)",
        "value": path_ms / steps * 1e3, "unit": "us/chunk", "n_gpus": 1, "steps": steps, "warmup": first_timed,
        "ms_per_step": path_ms / steps, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "layers": 1, "q_heads": Hq, "kv_heads": Hk, "head_dim": d,
                   "w_local": W, "page_size": P, "tau": cfg.tau, "chunk": Cn, "prompt_tokens": N,
                   "timed_chunks": [first_timed, n_chunks - 1], "gate": args.gate, "gate_us_per_chunk": gate_ms / steps * 1e3,
                   "admit_us_per_chunk": admit_ms / steps * 1e3, "attend_us_per_chunk": float(durs.mean() * 1e3),
                   "prompt_tokens_per_s": B * Cn * steps / (path_ms * 1e-3)},
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None, "kernel": "attend_prefill_kernel",
                     "algorithmic_flops": float(np.sum(flops)), "kernel_total_ms": float(durs.sum()),
                     "launches": int(steps)},
        "cpu_baseline": None,
    }
    print(json.dumps(res), flush=True)


def run_cpu_baseline(cfg, wl, ctx, rates, dev, gen_prefill, k1, v1, g1, q, scale, pool, seqs):
    """Times the CPU oracle (as it stands) on layer 0 of the same workload: one
    decode-attention call for the whole batch, (sequence, kv head) units spread
    over the host threads.  Reported per step by multiplying with the layer count."""
    import torch
    from oracle import Oracle, OracleConfig
    B, L, Hq, Hk, d, W, P = cfg.batch, cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.w_local, cfg.page_size
    t0 = time.time()
    max_gp = int(ctx.max()) // P + 8
    n_pages = B * Hk * (max_gp + W // P + 1)
    orc = Oracle(OracleConfig(1, Hq, Hk, d, P, W, B, max_gp, n_pages, True))
    chunk = 8192
    admit_s, admit_tokens = 0.0, 0
    for s in range(B):
        k, v, g = gen_prefill(s, 0)
        for a in range(0, int(ctx[s]), chunk):
            b = min(a + chunk, int(ctx[s]))
            kh, vh, gh = k[a:b].float().cpu().numpy(), v[a:b].float().cpu().numpy(), g[a:b].cpu().numpy()
            t_a = time.perf_counter()
            orc.push_tokens(0, [s], [b - a], kh, vh, gh, cfg.tau)
            admit_s += time.perf_counter() - t_a
            admit_tokens += b - a
        del k, v, g
    cpu_model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                cpu_model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    log(f"[bench] oracle state for layer 0 built in {time.time() - t0:.1f}s")
    orc.push_tokens(0, seqs, [1] * B, k1.float().cpu().numpy(), v1.float().cpu().numpy(), g1.cpu().numpy(), cfg.tau)
    qh = q.float().cpu().numpy()
    reps, best = 3, None
    for _ in range(reps):
        t1 = time.perf_counter()
        ref, threads = orc.attend_cached_batch(0, seqs, qh, scale)
        dt = time.perf_counter() - t1
        best = dt if best is None else min(best, dt)
    tokens = sum(orc.global_len(s, 0, h) + min(orc.seq_len(s, 0), W) for s in range(B) for h in range(Hk))
    return {"value": best * 1e6 * L, "unit": "us/step", "cores": int(threads), "kind": "oracle",
            "sample": f"decode attention of layer 0 only (batch {B}, {tokens} cached tokens over {B * Hk} "
                      f"(sequence, kv head) units), best of {reps}, {best * 1e3:.1f} ms per layer call, "
                      f"multiplied by {L} layers (extrapolated); promotion/paging not included",
            "layer_call_ms": best * 1e3, "cpu_model": cpu_model, "host_cpus": os.cpu_count(),
            "oracle_admission_us_per_token": admit_s / max(admit_tokens, 1) * 1e6,
            "oracle_admission_note": f"admission, paging and promotion of layer 0's prompts ({admit_tokens} tokens x {Hk} kv heads, "
                                     f"payload kept), one host thread, {admit_s:.1f} s in total"}


if __name__ == "__main__":
    main()
