#!/usr/bin/env python3
"""Benchmark of the KVBuffer GDN decode path on one MI355X.

One "step" = one chunkwise decoding step of the whole batch through one GDN layer, state
update included: either the single-kernel kvb_decode_flush(threshold = C) (--step fused,
default) or kvb_decode followed by kvb_flush(threshold = C) (--step split: the paper's
two-kernel arrangement; the flush call is issued every step and its device-side predicate
makes it a no-op until the buffer holds C records).  The headline workload is the
Qwen3-Next-shaped layer: batch 64, 16 qk + 32 v heads, d = 128, bf16 q/k/v, fp32 state,
C = 16.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="qwen3next_decode")
    ap.add_argument("--step", choices=["fused", "split"], default="fused")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph",
                    help="graph: the K timed steps are one HIP graph launch; eager: one launch per kernel")
    ap.add_argument("--batch", type=int, default=0,
                    help="override the workload's batch size (e.g. 512: 1 GiB of state, beyond the last-level cache)")
    ap.add_argument("--chunk", type=int, default=0,
                    help="override the chunk size C (and cap); 1 = the fused recurrent step, for the Fig. 3 style sweep")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--block-size", type=int, default=0,
                    help="paged record buffers: blocks of this many records dealt at random from a shared pool "
                         "(0 = the contiguous layout; bytes per step are the same)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-paths", action="store_true")
    return ap.parse_args()


class DecodeJob:
    """Device-resident workload: one store holding every layer's slots, a ring of token
    inputs, pre-marshalled calls (one per layer and ring entry)."""

    def __init__(self, w, ring=32, fused=True, block_size=0):
        import numpy as np
        import torch
        from paper_2605_19049_amd import kvb, synth
        self.w, self.torch, self.kvb, self.np = w, torch, kvb, np
        dt = kvb.BF16 if w.in_dtype == "bf16" else kvb.F32
        self.L = w.layers
        if block_size:
            mb = -(-w.cap // block_size)
            table = np.random.default_rng(w.seed + 7).permutation(w.B * self.L * mb).reshape(w.B * self.L, mb)
            self.ds = kvb.DeviceStore(w.B * self.L, w.Hk, w.Hv, w.dk, w.dv, w.cap, dt, block_size=block_size,
                                      block_table=table)
        else:
            self.ds = kvb.DeviceStore(w.B * self.L, w.Hk, w.Hv, w.dk, w.dv, w.cap, dt)
        self.sh = kvb.shape(w.B, w.Hk, w.Hv, w.dk, w.dv, w.cap, dt, 1.0)
        # many layers: each state is next read a whole model pass later -> stream it
        self.st = self.ds.c(flags=kvb.STORE_STREAM if self.L > 1 else 0)
        self.slots = [torch.arange(l * w.B, (l + 1) * w.B, dtype=torch.int32, device="cuda")
                      for l in range(self.L)]
        rng = np.random.default_rng(w.seed)
        tok = synth.token_stream(rng, w.B, ring, w.Hk, w.Hv, w.dk, w.dv, w.in_dtype)
        tdt = torch.bfloat16 if w.in_dtype == "bf16" else torch.float32
        self.ring = ring
        self.tok_np = tok
        self.tok = []
        for t in range(ring):
            self.tok.append({
                "q": torch.from_numpy(tok["q"][:, t].copy()).cuda().to(tdt),
                "k": torch.from_numpy(tok["k"][:, t].copy()).cuda().to(tdt),
                "v": torch.from_numpy(tok["v"][:, t].copy()).cuda().to(tdt),
                "g": torch.from_numpy(tok["g"][:, t].copy()).cuda(),
                "beta": torch.from_numpy(tok["beta"][:, t].copy()).cuda()})
        self.out = torch.empty((w.B, w.Hv, w.dv), dtype=torch.float32, device="cuda")
        # host mirror of every request's buffer fill (it evolves deterministically)
        self.fills = np.zeros((self.L, w.B), np.int64)
        if w.ragged:
            # independent phases: all-zero records (k = u = 0, G = 0) are a valid buffer
            self.fills = np.stack([synth.buffer_fills(rng, w.B, 0, w.C - 1) for _ in range(self.L)]).astype(np.int64)
            self.ds.fill.copy_(torch.from_numpy(self.fills.reshape(-1).astype(np.int32)))
        self.t = 0          # tokens decoded so far (selects the ring entry)
        self.fused = fused
        self._bound = {}

    def _calls(self, stream):
        if stream not in self._bound:
            kvb, w = self.kvb, self.w
            dec, fl = [], []
            for l in range(self.L):
                if self.fused:
                    dec.append([kvb.bind("kvb_decode_flush", self.sh, self.st, self.slots[l], x["q"], x["k"], x["v"],
                                         x["g"], x["beta"], self.out, w.C, stream) for x in self.tok])
                    fl.append(None)
                else:
                    dec.append([kvb.bind("kvb_decode", self.sh, self.st, self.slots[l], x["q"], x["k"], x["v"],
                                         x["g"], x["beta"], self.out, stream) for x in self.tok])
                    fl.append(kvb.bind("kvb_flush", self.sh, self.st, self.slots[l], None, w.C, stream))
            self._bound[stream] = (dec, fl)
        return self._bound[stream]

    def launch_bytes(self, fills):
        """Algorithmic bytes of one decode(-flush) launch whose requests sit at `fills`."""
        from paper_2605_19049_amd import traffic
        lay, w = traffic.KVB, self.w
        rd = lay.state + lay.token_in + fills * lay.record
        wr = lay.token_out + (lay.state if self.fused else 0) * (fills + 1 >= w.C)
        return float((rd + wr).sum()) * w.Hv

    def run(self, n, timers=None):
        """n steps (each through every layer) on the current stream; with `timers` (a list to
        fill), every decode launch carries a kvb timer, which records that kernel's own
        begin/end timestamps; the entry also notes the launch's algorithmic bytes."""
        torch = self.torch
        dec, fl = self._calls(torch.cuda.current_stream().cuda_stream)
        for _ in range(n):
            r = self.t % self.ring
            for l in range(self.L):
                if timers is not None:
                    tm = self.kvb.Timer()
                    tm.arm()
                    dec[l][r]()
                    timers.append((tm, self.launch_bytes(self.fills[l]),
                                   bool((self.fills[l] + 1 >= self.w.C).any())))
                else:
                    dec[l][r]()
                if fl[l] is not None:
                    fl[l]()
            self.fills = (self.fills + 1) % self.w.C
            self.t += 1


def time_other_paths(torch, kvb, synth, traffic, reps=20):
    """Kernel-level timings of kvb_verify, kvb_verify_tree, kvb_direct and kvb_flush at the sizes
    of the spec_verify / short_direct / qwen3next_decode workloads (context numbers only)."""
    import numpy as np
    res = {}

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    def dev_tok(tok):
        return {n: (torch.from_numpy(x).cuda().to(torch.bfloat16) if n in "qkv" else torch.from_numpy(x).cuda())
                for n, x in tok.items()}

    # verify: B=128, fill ~U(0,15), T=4
    w = synth.WORKLOADS["spec_verify"]
    rng = np.random.default_rng(w.seed)
    ds = kvb.DeviceStore(w.B, w.Hk, w.Hv, w.dk, w.dv, w.cap, kvb.BF16)
    ds.state.normal_(0, 0.5)
    ds.buf_u.normal_(0, 1.0)
    ds.buf_k.copy_(torch.nn.functional.normalize(torch.randn_like(ds.buf_k, dtype=torch.float32), dim=-1))
    ds.buf_G.copy_(-0.25 * torch.arange(1, w.cap + 1, device="cuda").float().expand_as(ds.buf_G))
    fills = synth.buffer_fills(rng, w.B, 0, w.C - 1)
    ds.fill.copy_(torch.from_numpy(fills))
    sh = kvb.shape(w.B, w.Hk, w.Hv, w.dk, w.dv, w.cap, kvb.BF16)
    st = ds.c()
    slot = torch.arange(w.B, dtype=torch.int32, device="cuda")
    tok = dev_tok(synth.token_stream(rng, w.B, w.T, w.Hk, w.Hv, w.dk, w.dv, "bf16"))
    out = torch.empty((w.B, w.T, w.Hv, w.dv), dtype=torch.float32, device="cuda")
    call = kvb.bind("kvb_verify", sh, st, slot, w.T, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"], out,
                    torch.cuda.current_stream().cuda_stream)
    sec = timed(call, reps)
    byt = sum(traffic.total(traffic.verify_rw(traffic.KVB, int(f), w.T)) for f in fills) * w.Hv
    res["kvb_verify"] = {"workload": "spec_verify B=128 T=4 fill~U(0,15)", "us": sec * 1e6,
                         "algorithmic_GBps": byt / sec / 1e9, "draft_tokens_per_s": w.B * w.T / sec}
    # the same drafts as trees (a random 4-node tree per request); same bytes
    parent = torch.from_numpy(synth.draft_trees(rng, w.B, w.T, "random")).cuda()
    call = kvb.bind("kvb_verify_tree", sh, st, slot, w.T, parent, tok["q"], tok["k"], tok["v"], tok["g"],
                    tok["beta"], out, torch.cuda.current_stream().cuda_stream)
    sec = timed(call, reps)
    res["kvb_verify_tree"] = {"workload": "spec_verify B=128, random trees of 4 drafts, fill~U(0,15)", "us": sec * 1e6,
                              "algorithmic_GBps": byt / sec / 1e9, "draft_tokens_per_s": w.B * w.T / sec}
    del ds

    # direct: B=256, L ~U(1,64)
    w = synth.WORKLOADS["short_direct"]
    rng = np.random.default_rng(w.seed)
    ds = kvb.DeviceStore(w.B, w.Hk, w.Hv, w.dk, w.dv, w.cap, kvb.BF16, with_state=False)
    lens = synth.context_lengths(rng, w.B, 1, w.Lmax)
    dl = torch.from_numpy(lens).cuda()
    sh = kvb.shape(w.B, w.Hk, w.Hv, w.dk, w.dv, w.cap, kvb.BF16)
    st = ds.c(False)
    slot = torch.arange(w.B, dtype=torch.int32, device="cuda")
    tok = dev_tok(synth.token_stream(rng, w.B, w.Lmax, w.Hk, w.Hv, w.dk, w.dv, "bf16"))
    out = torch.empty((w.B, w.Lmax, w.Hv, w.dv), dtype=torch.float32, device="cuda")
    call = kvb.bind("kvb_direct", sh, st, slot, dl, w.Lmax, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"],
                    out, torch.cuda.current_stream().cuda_stream)
    sec = timed(call, reps)
    byt = sum(traffic.total(traffic.direct_rw(traffic.KVB, int(L))) for L in lens) * w.Hv
    flop = sum(4.0 * int(L) ** 2 * w.dk for L in lens) * w.Hv
    res["kvb_direct"] = {"workload": "short_direct B=256 L~U(1,64)", "us": sec * 1e6,
                         "algorithmic_GBps": byt / sec / 1e9, "TFLOPs": flop / sec / 1e12,
                         "context_tokens_per_s": float(lens.sum()) / sec}
    del ds

    # flush as a launch of its own: every request of the layer at fill m, all of them folded.
    # The call empties the buffers, so the fill is set again before each launch and the launch
    # is timed by the library's own kernel timer.
    def flush_case(B, cap, m):
        w = synth.WORKLOADS["qwen3next_decode"]
        ds = kvb.DeviceStore(B, w.Hk, w.Hv, w.dk, w.dv, cap, kvb.BF16)
        ds.state.normal_(0, 0.5)
        ds.buf_u.normal_(0, 1.0)
        ds.buf_k.copy_(torch.nn.functional.normalize(torch.randn_like(ds.buf_k, dtype=torch.float32), dim=-1))
        ds.buf_G.copy_(-0.25 * torch.arange(1, cap + 1, device="cuda").float().expand_as(ds.buf_G))
        sh = kvb.shape(B, w.Hk, w.Hv, w.dk, w.dv, cap, kvb.BF16)
        st = ds.c()
        slot = torch.arange(B, dtype=torch.int32, device="cuda")
        call = kvb.bind("kvb_flush", sh, st, slot, None, 1, torch.cuda.current_stream().cuda_stream)
        tm = kvb.Timer()
        us = []
        for _ in range(reps + 4):
            ds.fill.fill_(m)
            tm.arm()
            call()
            us.append(tm.us())
        tm.close()
        us = sorted(us[4:])
        sec = us[len(us) // 2] * 1e-6
        byt = traffic.total(traffic.flush_rw(traffic.KVB, m)) * B * w.Hv
        return {"workload": "qwen3next layer, B=%d, every request at fill %d (cap %d)" % (B, m, cap), "us": sec * 1e6,
                "algorithmic_GBps": byt / sec / 1e9, "TFLOPs": 2.0 * m * w.dk * w.dv * B * w.Hv / sec / 1e12}

    res["kvb_flush"] = flush_case(64, 16, 16)
    res["kvb_flush_64_records"] = flush_case(128, 64, 64)
    return res


def measured_traffic(workload, fused):
    """HBM bytes per launch of the dominant kernel as the rocprofv3 FETCH_SIZE / WRITE_SIZE
    counters measured them (summary under profiles/); None for other configurations."""
    if workload != "qwen3next_decode" or not fused:
        return None
    path = os.path.join(ROOT, "profiles", "kvb_decode_flush_qwen3next_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def cpu_baseline(w, tok_np, rounds=4, steps=512):
    """The fp64 oracle, as it stands, on the host cores: same shapes, same token values.
    `rounds` consecutive calls of `steps` tokens each, the state carried from one to the next."""
    import numpy as np
    from oracle import gdn
    gdn.build_lib()
    ring = tok_np["q"].shape[1]
    n = steps - steps % ring
    S = np.zeros((w.B, w.Hv, w.dk, w.dv))
    sub = {k: np.concatenate([v] * (n // ring), axis=1) for k, v in tok_np.items()}   # the ring, replayed
    gdn.gdn_sequence(S[:1], *(sub[x][:1, :2] for x in ("q", "k", "v", "g", "beta")))   # load the library
    dt, used = 0.0, 0
    for _ in range(rounds):
        t0 = time.perf_counter()
        _, _, S, used = gdn.gdn_sequence(S, sub["q"], sub["k"], sub["v"], sub["g"], sub["beta"])
        dt += time.perf_counter() - t0
    return {"value": w.B * n * rounds / dt, "unit": "tokens/s/layer", "cores": used, "kind": "oracle",
            "sample": "all %d requests x %d decode steps of the same workload (%.1f s)" % (w.B, n * rounds, dt)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_19049_amd import kvb, synth, traffic
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    kvb.lib()   # fail loudly if the HIP library is missing
    w = synth.WORKLOADS[args.workload]
    if args.batch:
        import dataclasses
        w = dataclasses.replace(w, B=args.batch, name="%s(B=%d)" % (w.name, args.batch))
    if args.chunk:
        import dataclasses
        w = dataclasses.replace(w, C=args.chunk, cap=args.chunk, name="%s(C=%d)" % (w.name, args.chunk))
    K, W = args.steps, args.warmup

    if args.copy_calibration:
        # a plain copy kernel of known size: reads 1 GiB, writes 1 GiB per launch
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    fused = args.step == "fused"
    job = DecodeJob(w, fused=fused, block_size=args.block_size)
    L = job.L
    # untimed: build a real committed state by decoding a prompt-sized prefix, then W warm-up steps
    job.run(w.prefix + W)
    torch.cuda.synchronize()
    t_start, fills_start = job.t, job.fills.copy()
    bufs = (job.ds.state, job.ds.buf_k, job.ds.buf_u, job.ds.buf_G, job.ds.fill)

    graph = None
    if args.mode == "graph":
        snap = [x.clone() for x in bufs[1:]] if L > 1 else [x.clone() for x in bufs]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            job.run(K)
        torch.cuda.synchronize()
        # make sure the store is exactly where the captured work expects it
        for dst, src in zip(bufs[1:] if L > 1 else bufs, snap):
            dst.copy_(src)
        del snap
        job.t, job.fills = t_start, fills_start.copy()
        torch.cuda.synchronize()

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    e0.record()
    if graph is not None:
        graph.replay()
        job.t, job.fills = t_start + K, (fills_start + K) % w.C
    else:
        job.run(K)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    sec = e0.elapsed_time(e1) * 1e-3
    n_launch = K * L
    assert int(job.ds.status.sum().item()) == 0, "a buffer overflowed during the bench"

    # The same steps again, eager, every decode launch carrying a kernel timer (begin/end
    # timestamps of that kernel alone): the dominant kernel's duration, with its algorithmic
    # bytes at the fills it actually ran at.
    timers = []
    job.run(min(K, max(1, 1024 // L)), timers)
    torch.cuda.synchronize()
    units = w.B * w.Hv
    dec_us = [tm.us() for tm, _, _ in timers]
    dec_bytes = [by for _, by, _ in timers]
    for tm, _, _ in timers:
        tm.close()
    lay = traffic.KVB
    if fused:
        cycle_bytes = traffic.total(traffic.fused_cycle_rw(lay, w.C)) * units
        kname = "kvb_step_kernel<128,bf16,TM=1,W=%d,state,fused> (kvb_decode_flush)" % (16 if w.cap <= 16 else 32 if w.cap <= 32 else 64)
        step_desc = "kvb_decode_flush(threshold=C)"
    else:
        cycle_bytes = traffic.total(traffic.chunk_cycle_rw(lay, w.C)) * units
        kname = "kvb_step_kernel<128,bf16,TM=1,W=%d,state> (kvb_decode)" % (16 if w.cap <= 16 else 32 if w.cap <= 32 else 64)
        step_desc = "kvb_decode + kvb_flush(threshold=C)"
    dec_avg_us = sum(dec_us) / len(dec_us)
    achieved = sum(dec_bytes) / (sum(dec_us) * 1e-6) / 1e9
    noflush = [(u, by) for u, by, (_, _, fl_) in zip(dec_us, dec_bytes, timers) if not fl_]
    per_layer_step = sec / n_launch

    res = {
        "metric": "gdn_decode_tokens_per_s_per_layer", "value": w.B / per_layer_step, "unit": "tokens/s/layer",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": sec / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hk": w.Hk, "Hv": w.Hv, "dk": w.dk, "dv": w.dv,
                   "C": w.C, "cap": w.cap, "layers": L, "in_dtype": w.in_dtype, "state_dtype": "f32",
                   "step": step_desc + (" through each of %d layers" % L if L > 1 else ""), "launch": args.mode,
                   "state_MiB": L * units * w.dk * w.dv * 4 / 2 ** 20,
                   "records": ("blocks of %d from a shuffled pool" % args.block_size) if args.block_size else "contiguous"},
        "full_cycle": {"algorithmic_bytes_per_layer_step": cycle_bytes,
                       "algorithmic_GBps": cycle_bytes / per_layer_step / 1e9,
                       "frac_of_hbm_peak": cycle_bytes / per_layer_step / 1e9 / HBM_PEAK_GBS,
                       "us_per_layer_step": per_layer_step * 1e6,
                       "host_wall_ms_per_step": wall / K * 1e3},
        "roofline": {"bound": "hbm", "kernel": kname,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name, fused),
                     "avg_launch_us": dec_avg_us, "launches": len(dec_us),
                     "algorithmic_bytes_per_launch_avg": sum(dec_bytes) / len(dec_bytes),
                     "timing": "begin/end timestamps of each launch of this kernel (kvb timer = "
                               "hipExtLaunchKernel events), eager re-run of the same steps"},
    }
    if noflush:
        res["roofline"]["launches_without_state_update"] = {
            "avg_launch_us": sum(u for u, _ in noflush) / len(noflush),
            "achieved": sum(by for _, by in noflush) / (sum(u for u, _ in noflush) * 1e-6) / 1e9}
    if not args.no_other_paths:
        res["other_paths"] = time_other_paths(torch, kvb, synth, traffic)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, job.tok_np)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
