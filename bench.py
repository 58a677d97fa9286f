#!/usr/bin/env python3
"""Benchmark of the KVBuffer GDN decode path on one MI355X.

One "step" = one chunkwise decoding step of the whole batch through one GDN layer, state
update included: either the single-kernel kvb_decode_flush(threshold = C) (--step fused,
default) or kvb_decode followed by kvb_flush(threshold = C) (--step split: the paper's
two-kernel arrangement; the flush call is issued every step and its device-side predicate
makes it a no-op until the buffer holds C records).  The headline workload is the
Qwen3-Next-shaped layer: batch 64, 16 qk + 32 v heads, d = 128, bf16 q/k/v, fp32 state,
C = 16.  Prints ONE JSON line.

The default run also reports: the same kernel on a footprint that does not fit the 256 MB
last-level cache (`roofline_cold`), the paper's own storage regime (fp16 inputs, records and
outputs; `storage_regimes`), kernel timings of the other entry points (`other_paths`) and the
CPU oracle (`cpu_baseline`).  `--sweep chunk | verify_T | kvonly_L` prints one JSON object with
the table behind the paper's Fig. 3 / Fig. 4 / Fig. 6 quantities instead.
"""
import argparse
import dataclasses
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak
TRAFFIC_FILE = "profiles/kvb_decode_flush_qwen3next_l2_fabric_traffic.txt"


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
                    help="override the chunk size C (and cap); 1 = the fused recurrent step")
    ap.add_argument("--layers", type=int, default=0, help="override the number of stacked layers")
    ap.add_argument("--in-dtype", choices=["bf16", "f16", "f32"], default=None, help="q, k, v and buffered keys")
    ap.add_argument("--rec-dtype", choices=["f32", "bf16", "f16"], default="f32", help="buffered delta values")
    ap.add_argument("--out-dtype", choices=["f32", "bf16", "f16"], default="f32", help="outputs")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--block-size", type=int, default=0,
                    help="paged record buffers: blocks of this many records dealt at random from a shared pool "
                         "(0 = the contiguous layout; bytes per step are the same)")
    ap.add_argument("--sweep", choices=["chunk", "verify_T", "kvonly_L"], default=None,
                    help="print the table of one of the paper's kernel sweeps instead of the bench line")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-paths", action="store_true")
    ap.add_argument("--no-cold", action="store_true", help="skip the cache-defeating run")
    ap.add_argument("--no-regimes", action="store_true", help="skip the fp16 storage-regime run")
    return ap.parse_args()


def kernel_name(w, fused, types):
    win = 16 if w.cap <= 16 else 32 if w.cap <= 32 else 64
    return "kvb_step_kernel<%d,%s,rec=%s,TM=1,W=%d,state%s> (%s)" % (
        w.dk, types[0], types[1], win, ",fused" if fused else "", "kvb_decode_flush" if fused else "kvb_decode")


class DecodeJob:
    """Device-resident workload: one store holding every layer's slots, a ring of token
    inputs, pre-marshalled calls (one per layer and ring entry)."""

    def __init__(self, w, ring=32, fused=True, block_size=0, types=None):
        import numpy as np
        import torch
        from paper_2605_19049_amd import kvb, synth, traffic
        self.w, self.torch, self.kvb, self.np = w, torch, kvb, np
        self.types = types = types or (w.in_dtype, "f32", "f32")     # (inputs, records, outputs)
        code = {"f32": kvb.F32, "bf16": kvb.BF16, "f16": kvb.F16}
        dt, rdt, odt = (code[t] for t in types)
        self.lay = traffic.layout(types[0], types[1], types[2], r=w.Hv // w.Hk, dk=w.dk, dv=w.dv)
        self.L = w.layers
        if block_size:
            mb = -(-w.cap // block_size)
            table = np.random.default_rng(w.seed + 7).permutation(w.B * self.L * mb).reshape(w.B * self.L, mb)
            self.ds = kvb.DeviceStore(w.B * self.L, w.Hk, w.Hv, w.dk, w.dv, w.cap, dt, block_size=block_size,
                                      block_table=table, rec_dtype=rdt)
        else:
            self.ds = kvb.DeviceStore(w.B * self.L, w.Hk, w.Hv, w.dk, w.dv, w.cap, dt, rec_dtype=rdt)
        self.sh = kvb.shape(w.B, w.Hk, w.Hv, w.dk, w.dv, w.cap, dt, 1.0, out_dtype=odt, rec_dtype=rdt)
        # many layers: each state is next read a whole model pass later -> stream it
        self.st = self.ds.c(flags=kvb.STORE_STREAM if self.L > 1 else 0)
        self.slots = [torch.arange(l * w.B, (l + 1) * w.B, dtype=torch.int32, device="cuda")
                      for l in range(self.L)]
        rng = np.random.default_rng(w.seed)
        tok = synth.token_stream(rng, w.B, ring, w.Hk, w.Hv, w.dk, w.dv, types[0])
        tdt = kvb.torch_dtype(dt)
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
        self.out = torch.empty((w.B, w.Hv, w.dv), dtype=kvb.torch_dtype(odt), device="cuda")
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
        lay, w = self.lay, self.w
        rd = lay.state + lay.token_in + fills * lay.record
        wr = lay.token_out + (lay.state if self.fused else 0) * (fills + 1 >= w.C)
        return float((rd + wr).sum()) * w.Hv

    def cycle_bytes(self):
        """Algorithmic bytes of an average step of the whole batch through one layer."""
        from paper_2605_19049_amd import traffic
        rw = traffic.fused_cycle_rw(self.lay, self.w.C) if self.fused else traffic.chunk_cycle_rw(self.lay, self.w.C)
        return traffic.total(rw) * self.w.B * self.w.Hv

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

    def capture(self, K):
        """A HIP graph of K steps from the current position (the store is put back where the
        captured work expects it; the states only when they are cheap to copy)."""
        torch = self.torch
        bufs = (self.ds.state, self.ds.buf_k, self.ds.buf_u, self.ds.buf_G, self.ds.fill)
        keep = bufs[1:] if self.L > 1 else bufs
        t0, f0 = self.t, self.fills.copy()
        snap = [x.clone() for x in keep]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(K)
        torch.cuda.synchronize()
        for dst, src in zip(keep, snap):
            dst.copy_(src)
        del snap
        self.t, self.fills = t0, f0
        torch.cuda.synchronize()
        return graph

    def replay(self, graph, K):
        graph.replay()
        self.t, self.fills = self.t + K, (self.fills + K) % self.w.C

    def timed_replays(self, graph, K, min_ms=50.0, min_n=3, max_n=400, max_s=20.0):
        """Replays the K-step graph until at least min_ms of GPU time have been timed (and at least
        min_n replays); every replay is timed on its own, bracketed by synchronisations.  Returns
        the per-replay times in seconds."""
        torch = self.torch
        secs, t_begin = [], time.perf_counter()
        while len(secs) < max_n:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            self.replay(graph, K)
            e1.record()
            torch.cuda.synchronize()
            secs.append(e0.elapsed_time(e1) * 1e-3)
            if len(secs) >= min_n and (sum(secs) * 1e3 >= min_ms or time.perf_counter() - t_begin > max_s):
                break
        return secs

    def kernel_times(self, n_steps):
        """n_steps eager steps with a kernel timer on every decode launch: the kernel's own
        durations (us), its algorithmic bytes at the fills it ran at, and whether it folded."""
        timers = []
        self.run(n_steps, timers)
        self.torch.cuda.synchronize()
        res = [(tm.us(), by, fl_) for tm, by, fl_ in timers]
        for tm, _, _ in timers:
            tm.close()
        return res


def roofline_of(job, launches, fused, extra=None):
    us = [u for u, _, _ in launches]
    by = [b for _, b, _ in launches]
    achieved = sum(by) / (sum(us) * 1e-6) / 1e9
    res = {"bound": "hbm", "kernel": kernel_name(job.w, fused, job.types),
           "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
           "traffic": None,
           "avg_launch_us": sum(us) / len(us), "median_launch_us": statistics.median(us), "launches": len(us),
           "algorithmic_bytes_per_launch_avg": sum(by) / len(by),
           "timing": "begin/end timestamps of each launch of this kernel (kvb timer = "
                     "hipExtLaunchKernel events), eager re-run of the same steps"}
    if extra:
        res.update(extra)
    noflush = [(u, b) for u, b, f in launches if not f]
    if noflush:
        res["launches_without_state_update"] = {
            "avg_launch_us": sum(u for u, _ in noflush) / len(noflush),
            "achieved": sum(b for _, b in noflush) / (sum(u for u, _ in noflush) * 1e-6) / 1e9}
    return res


def measured_traffic(workload, fused, types, paged=False):
    """{"traffic", "traffic_source"}: bytes that left the L2 caches per launch of the dominant
    kernel (towards the last-level cache and HBM), as the rocprofv3 FETCH_SIZE / WRITE_SIZE
    counters measured them in the run summarised under profiles/ (warm and cold instance read
    the same) -- a stored figure, not one of this run; None for configurations that summary
    does not cover."""
    none = {"traffic": None, "traffic_source": None}
    if workload != "qwen3next_decode" or not fused or paged or types != ("bf16", "f32", "f32"):
        return none
    try:
        for line in open(os.path.join(ROOT, TRAFFIC_FILE)):
            if line.startswith("traffic_bytes_per_launch"):
                return {"traffic": float(line.split("=")[1]),
                        "traffic_source": TRAFFIC_FILE + " (static: rocprofv3 FETCH_SIZE/WRITE_SIZE of an earlier "
                                          "run of this workload; bytes that crossed between the L2 caches and the "
                                          "fabric, last-level-cache hits included)"}
    except OSError:
        pass
    return none


# --------------------------------------------------------------------------- other entry points
def _median_kernel_us(kvb, call, before=None, reps=20, skip=4):
    """Median of the kernel's own duration over `reps` launches (kvb timer); `before` runs ahead
    of every launch (e.g. to put the buffer fill back)."""
    tm = kvb.Timer()
    us = []
    for _ in range(reps + skip):
        if before:
            before()
        tm.arm()
        call()
        us.append(tm.us())
    tm.close()
    return statistics.median(us[skip:])


def _dev_tok(torch, kvb, tok, in_dtype):
    tdt = kvb.torch_dtype({"f32": kvb.F32, "bf16": kvb.BF16, "f16": kvb.F16}[in_dtype])
    return {n: (torch.from_numpy(x).cuda().to(tdt) if n in "qkv" else torch.from_numpy(x).cuda())
            for n, x in tok.items()}


def _filled_store(torch, kvb, B, w, cap, types, with_state=True):
    """A store with plausible contents: N(0, 0.5) state, N(0, 1) delta values, unit keys, decays
    of 0.25 per record."""
    code = {"f32": kvb.F32, "bf16": kvb.BF16, "f16": kvb.F16}
    ds = kvb.DeviceStore(B, w.Hk, w.Hv, w.dk, w.dv, cap, code[types[0]], with_state=with_state, rec_dtype=code[types[1]])
    if with_state:
        ds.state.normal_(0, 0.5)
    ds.buf_u.copy_(torch.randn(ds.buf_u.shape, device="cuda"))
    ds.buf_k.copy_(torch.nn.functional.normalize(torch.randn(ds.buf_k.shape, device="cuda"), dim=-1))
    ds.buf_G.copy_(-0.25 * torch.arange(1, cap + 1, device="cuda").float().expand_as(ds.buf_G))
    sh = kvb.shape(B, w.Hk, w.Hv, w.dk, w.dv, cap, code[types[0]], 1.0, out_dtype=code[types[2]], rec_dtype=code[types[1]])
    return ds, sh


def time_other_paths(torch, kvb, synth, traffic, reps=20):
    """Kernel-level timings of kvb_verify, kvb_verify_tree, kvb_direct and kvb_flush at the sizes
    of the spec_verify / short_direct / qwen3next_decode workloads (context numbers only)."""
    import numpy as np
    res = {}
    cs = torch.cuda.current_stream().cuda_stream
    types = ("bf16", "f32", "f32")
    lay = traffic.KVB

    # verify: B=128, fill ~U(0,15), T=4
    w = synth.WORKLOADS["spec_verify"]
    rng = np.random.default_rng(w.seed)
    ds, sh = _filled_store(torch, kvb, w.B, w, w.cap, types)
    fills = synth.buffer_fills(rng, w.B, 0, w.C - 1)
    ds.fill.copy_(torch.from_numpy(fills))
    st = ds.c()
    slot = torch.arange(w.B, dtype=torch.int32, device="cuda")
    tok = _dev_tok(torch, kvb, synth.token_stream(rng, w.B, w.T, w.Hk, w.Hv, w.dk, w.dv, "bf16"), "bf16")
    out = torch.empty((w.B, w.T, w.Hv, w.dv), dtype=torch.float32, device="cuda")
    call = kvb.bind("kvb_verify", sh, st, slot, w.T, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"], out, cs)
    sec = _median_kernel_us(kvb, call, reps=reps) * 1e-6
    byt = sum(traffic.total(traffic.verify_rw(lay, int(f), w.T)) for f in fills) * w.Hv
    res["kvb_verify"] = {"workload": "spec_verify B=128 T=4 fill~U(0,15)", "us": sec * 1e6,
                         "algorithmic_GBps": byt / sec / 1e9, "draft_tokens_per_s": w.B * w.T / sec}
    # the same drafts as trees (a random 4-node tree per request); same bytes
    parent = torch.from_numpy(synth.draft_trees(rng, w.B, w.T, "random")).cuda()
    call = kvb.bind("kvb_verify_tree", sh, st, slot, w.T, parent, tok["q"], tok["k"], tok["v"], tok["g"],
                    tok["beta"], out, cs)
    sec = _median_kernel_us(kvb, call, reps=reps) * 1e-6
    res["kvb_verify_tree"] = {"workload": "spec_verify B=128, random trees of 4 drafts, fill~U(0,15)", "us": sec * 1e6,
                              "algorithmic_GBps": byt / sec / 1e9, "draft_tokens_per_s": w.B * w.T / sec}
    del ds

    # direct: B=256, L ~U(1,64), in the default types and in the paper's fp16 regime
    w = synth.WORKLOADS["short_direct"]
    for name, ty in (("kvb_direct", types), ("kvb_direct_f16", ("f16", "f16", "f16"))):
        rng = np.random.default_rng(w.seed)
        ds, sh = _filled_store(torch, kvb, w.B, w, w.cap, ty, with_state=False)
        lens = synth.context_lengths(rng, w.B, 1, w.Lmax)
        dl = torch.from_numpy(lens).cuda()
        st = ds.c(False)
        slot = torch.arange(w.B, dtype=torch.int32, device="cuda")
        tok = _dev_tok(torch, kvb, synth.token_stream(rng, w.B, w.Lmax, w.Hk, w.Hv, w.dk, w.dv, ty[0]), ty[0])
        out = torch.empty((w.B, w.Lmax, w.Hv, w.dv), dtype=torch.float32 if ty[2] == "f32" else torch.float16,
                          device="cuda")
        call = kvb.bind("kvb_direct", sh, st, slot, dl, w.Lmax, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"],
                        out, cs)
        sec = _median_kernel_us(kvb, call, reps=reps) * 1e-6
        lay_d = traffic.layout(*ty)
        byt = sum(traffic.total(traffic.direct_rw(lay_d, int(L))) for L in lens) * w.Hv
        flop = sum(4.0 * int(L) ** 2 * w.dk for L in lens) * w.Hv
        res[name] = {"workload": "short_direct B=256 L~U(1,64), inputs/records/outputs %s/%s/%s" % ty, "us": sec * 1e6,
                     "algorithmic_GBps": byt / sec / 1e9, "TFLOPs": flop / sec / 1e12,
                     "context_tokens_per_s": float(lens.sum()) / sec}
        del ds

    # flush as a launch of its own: every request of the layer at fill m, all of them folded.
    # The call empties the buffers, so the fill is set again before each launch.
    def flush_case(B, cap, m):
        w = synth.WORKLOADS["qwen3next_decode"]
        ds, sh = _filled_store(torch, kvb, B, w, cap, types)
        st = ds.c()
        slot = torch.arange(B, dtype=torch.int32, device="cuda")
        call = kvb.bind("kvb_flush", sh, st, slot, None, 1, cs)
        sec = _median_kernel_us(kvb, call, before=lambda: ds.fill.fill_(m), reps=reps) * 1e-6
        byt = traffic.total(traffic.flush_rw(lay, m)) * B * w.Hv
        return {"workload": "qwen3next layer, B=%d, every request at fill %d (cap %d)" % (B, m, cap), "us": sec * 1e6,
                "algorithmic_GBps": byt / sec / 1e9, "TFLOPs": 2.0 * m * w.dk * w.dv * B * w.Hv / sec / 1e12}

    res["kvb_flush"] = flush_case(64, 16, 16)
    res["kvb_flush_64_records"] = flush_case(128, 64, 64)
    return res


# --------------------------------------------------------------------------- sweeps (Fig. 3 / 4 / 6 quantities)
def sweep_chunk(torch, kvb, synth, types):
    """Full-cycle decode step time against the chunk size, per batch size (the paper's Fig. 3
    quantity); C = 1 is the fused recurrent step, which reads and writes the state every token."""
    w0 = synth.WORKLOADS["qwen3next_decode"]
    rows = {}
    for B in (1, 16, 64, 256):
        row = {}
        for C in (1, 2, 4, 8, 16, 32, 64, 128):
            w = dataclasses.replace(w0, B=B, C=C, cap=C)
            job = DecodeJob(w, types=(types[0], types[1], types[2]))
            K = C * max(2, 64 // C)                      # whole cycles
            job.run(K)
            graph = job.capture(K)
            secs = job.timed_replays(graph, K, min_ms=10.0, min_n=5, max_n=50)
            row[str(C)] = statistics.median(secs) / K * 1e6
            del job, graph
        rows[str(B)] = row
    return {"sweep": "chunk", "quantity": "us per decode step, full cycle (kvb_decode_flush(threshold=C), HIP graph)",
            "types": types, "rows_batch_cols_C": rows}


def sweep_verify_T(torch, kvb, synth, types):
    """Verification of T drafts against T recurrent steps (the paper's Fig. 4 quantity): batch 128,
    empty buffer, kernel durations; the recurrent column is T launches of the fused recurrent step
    kvb_decode_flush(threshold = 1)."""
    import numpy as np
    w = synth.WORKLOADS["spec_verify"]
    B, cs = w.B, torch.cuda.current_stream().cuda_stream
    rng = np.random.default_rng(0)
    rows = []
    for T in (1, 2, 4, 8):
        ds, sh = _filled_store(torch, kvb, B, w, 16, types)
        ds.fill.zero_()
        st = ds.c()
        slot = torch.arange(B, dtype=torch.int32, device="cuda")
        tok = _dev_tok(torch, kvb, synth.token_stream(rng, B, T, w.Hk, w.Hv, w.dk, w.dv, types[0]), types[0])
        odt = kvb.torch_dtype({"f32": kvb.F32, "bf16": kvb.BF16, "f16": kvb.F16}[types[2]])
        out = torch.empty((B, T, w.Hv, w.dv), dtype=odt, device="cuda")
        acc = torch.full((B,), T, dtype=torch.int32, device="cuda")
        ver = kvb.bind("kvb_verify", sh, st, slot, T, tok["q"], tok["k"], tok["v"], tok["g"], tok["beta"], out, cs)
        t_ver = _median_kernel_us(kvb, ver)
        fl = kvb.bind("kvb_flush", sh, st, slot, acc, 1, cs)          # folds the T accepted drafts, fill back to 0
        t_fl = _median_kernel_us(kvb, fl, before=ver)
        t1 = {n: x[:, 0].contiguous() for n, x in tok.items()}
        o1 = torch.empty((B, w.Hv, w.dv), dtype=odt, device="cuda")
        rec = kvb.bind("kvb_decode_flush", sh, st, slot, t1["q"], t1["k"], t1["v"], t1["g"], t1["beta"], o1, 1, cs)
        t_rec = _median_kernel_us(kvb, rec)
        rows.append({"T": T, "kvb_verify_us": t_ver, "kvb_flush_accepted_T_us": t_fl, "sum_us": t_ver + t_fl,
                     "T_recurrent_steps_us": T * t_rec, "ratio": T * t_rec / (t_ver + t_fl)})
        del ds
    return {"sweep": "verify_T", "batch": B, "types": types, "rows": rows}


def sweep_kvonly_L(torch, kvb, synth, types_list):
    """One KV-only decode step (kvb_decode with no state) against the context length (the paper's
    Fig. 6 quantity), batch 128, next to the chunkwise (C = 16, full cycle) and recurrent steps of
    the same batch, for each storage regime."""
    import numpy as np
    w0 = synth.WORKLOADS["qwen3next_decode"]
    B, cs = 128, torch.cuda.current_stream().cuda_stream
    res = []
    for types in types_list:
        rng = np.random.default_rng(0)
        row = {"types": types, "kv_only_us": {}}
        for L in (8, 16, 32, 48, 64, 80, 96, 112, 127):
            ds, sh = _filled_store(torch, kvb, B, w0, 128, types, with_state=False)
            st = ds.c(False)
            slot = torch.arange(B, dtype=torch.int32, device="cuda")
            tok = _dev_tok(torch, kvb, synth.token_stream(rng, B, 1, w0.Hk, w0.Hv, w0.dk, w0.dv, types[0]), types[0])
            t1 = {n: x[:, 0].contiguous() for n, x in tok.items()}
            odt = kvb.torch_dtype({"f32": kvb.F32, "bf16": kvb.BF16, "f16": kvb.F16}[types[2]])
            o1 = torch.empty((B, w0.Hv, w0.dv), dtype=odt, device="cuda")
            dec = kvb.bind("kvb_decode", sh, st, slot, t1["q"], t1["k"], t1["v"], t1["g"], t1["beta"], o1, cs)
            row["kv_only_us"][str(L)] = _median_kernel_us(kvb, dec, before=lambda: ds.fill.fill_(L))
            del ds
        for name, C in (("chunkwise_C16_us", 16), ("recurrent_us", 1)):
            w = dataclasses.replace(w0, B=B, C=C, cap=C)
            job = DecodeJob(w, types=types)
            K = 64
            job.run(K)
            graph = job.capture(K)
            row[name] = statistics.median(job.timed_replays(graph, K, min_ms=10.0, min_n=5, max_n=50)) / K * 1e6
            del job, graph
        ks = sorted(int(k) for k in row["kv_only_us"])
        below = [L for L in ks if row["kv_only_us"][str(L)] <= row["chunkwise_C16_us"]]
        row["largest_L_not_slower_than_chunkwise"] = max(below) if below else None
        res.append(row)
    return {"sweep": "kvonly_L", "batch": B, "rows": res}


# --------------------------------------------------------------------------- CPU oracle
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
        w = dataclasses.replace(w, B=args.batch, name="%s(B=%d)" % (w.name, args.batch))
    if args.chunk:
        w = dataclasses.replace(w, C=args.chunk, cap=args.chunk, name="%s(C=%d)" % (w.name, args.chunk))
    if args.layers:
        w = dataclasses.replace(w, layers=args.layers, name="%s(layers=%d)" % (w.name, args.layers))
    types = (args.in_dtype or w.in_dtype, args.rec_dtype, args.out_dtype)
    K, W = args.steps, args.warmup

    if args.sweep:
        if args.sweep == "chunk":
            res = sweep_chunk(torch, kvb, synth, types)
        elif args.sweep == "verify_T":
            res = sweep_verify_T(torch, kvb, synth, types)
        else:
            regimes = [types] if (args.in_dtype or args.rec_dtype != "f32") else \
                [("bf16", "f32", "f32"), ("f16", "f16", "f16")]
            res = sweep_kvonly_L(torch, kvb, synth, regimes)
        print(json.dumps(res), flush=True)
        return

    if args.copy_calibration:
        # a plain copy kernel of known size: reads 1 GiB, writes 1 GiB per launch
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    fused = args.step == "fused"
    job = DecodeJob(w, fused=fused, block_size=args.block_size, types=types)
    L = job.L
    # untimed: build a real committed state by decoding a prompt-sized prefix, then W warm-up steps
    job.run(w.prefix + W)
    torch.cuda.synchronize()

    # The timed region is EXACTLY K steps, bracketed by synchronisations.  In graph mode it is
    # repeated until 50 ms of GPU time have been sampled and the median of the K-step times is
    # reported, so that the figure does not hang on one short sample when K is small.
    wall0 = time.perf_counter()
    if args.mode == "graph":
        graph = job.capture(K)
        wall0 = time.perf_counter()
        secs = job.timed_replays(graph, K)
    else:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        job.run(K)
        e1.record()
        torch.cuda.synchronize()
        secs = [e0.elapsed_time(e1) * 1e-3]
    wall = (time.perf_counter() - wall0) / len(secs)
    sec = statistics.median(secs)
    n_launch = K * L
    assert int(job.ds.status.sum().item()) == 0, "a buffer overflowed during the bench"

    # The same steps again, eager, every decode launch carrying a kernel timer (begin/end
    # timestamps of that kernel alone): the dominant kernel's duration, with its algorithmic
    # bytes at the fills it actually ran at.
    launches = job.kernel_times(min(max(K, 2 * w.C), max(1, 1024 // L)))
    units = w.B * w.Hv
    cycle_bytes = job.cycle_bytes()
    step_desc = "kvb_decode_flush(threshold=C)" if fused else "kvb_decode + kvb_flush(threshold=C)"
    per_layer_step = sec / n_launch
    state_mib = L * units * w.dk * w.dv * 4 / 2 ** 20

    res = {
        "metric": "gdn_decode_tokens_per_s_per_layer", "value": w.B / per_layer_step, "unit": "tokens/s/layer",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": sec / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hk": w.Hk, "Hv": w.Hv, "dk": w.dk, "dv": w.dv,
                   "C": w.C, "cap": w.cap, "layers": L, "in_dtype": types[0], "rec_dtype": types[1],
                   "out_dtype": types[2], "state_dtype": "f32", "arithmetic": "f32",
                   "step": step_desc + (" through each of %d layers" % L if L > 1 else ""), "launch": args.mode,
                   "state_MiB": state_mib,
                   "records": ("blocks of %d from a shuffled pool" % args.block_size) if args.block_size else "contiguous"},
        "timed": {"samples": len(secs), "each": "exactly %d steps, synchronised on both sides" % K,
                  "reported": "median", "min_ms_per_step": min(secs) / K * 1e3, "max_ms_per_step": max(secs) / K * 1e3},
        "full_cycle": {"algorithmic_bytes_per_layer_step": cycle_bytes,
                       "algorithmic_GBps": cycle_bytes / per_layer_step / 1e9,
                       "frac_of_hbm_peak": cycle_bytes / per_layer_step / 1e9 / HBM_PEAK_GBS,
                       "us_per_layer_step": per_layer_step * 1e6,
                       "host_wall_ms_per_step": wall / K * 1e3},
        "roofline": roofline_of(job, launches, fused, {
            **measured_traffic(w.name, fused, types, paged=bool(args.block_size)),
            "footprint": "%.0f MiB of state re-read every step: %s the 256 MB last-level cache" % (
                state_mib, "fits" if state_mib <= 256 else "exceeds")}),
    }
    del job

    if not args.no_cold and args.workload == "qwen3next_decode" and not (args.batch or args.chunk or args.layers):
        # The same kernel on a footprint the last-level cache cannot hold: the layer's shape
        # stacked 8 times (1 GiB of state), every step passing through all 8 copies, so that a
        # copy's state is next read after 1 GiB of other traffic.  Non-temporal state loads
        # (KVB_STORE_STREAM), as a model with many GDN layers would ask for.
        wc = dataclasses.replace(w, layers=8, name=w.name + " x 8 layer copies")
        cold = DecodeJob(wc, fused=fused, types=types)
        cold.run(2 * wc.C)
        torch.cuda.synchronize()
        Kc = 2 * wc.C
        g = cold.capture(Kc)
        csecs = cold.timed_replays(g, Kc, min_ms=30.0)
        cl = cold.kernel_times(2 * wc.C)
        cstep = statistics.median(csecs) / (Kc * wc.layers)
        res["roofline_cold"] = roofline_of(cold, cl, fused, {
            **measured_traffic(w.name, fused, types, paged=bool(args.block_size)),
            "workload": "%s: %d MiB of state, state loads non-temporal" % (wc.name, 8 * state_mib),
            "graph_us_per_layer_step": cstep * 1e6,
            "graph_full_cycle_GBps": cold.cycle_bytes() / cstep / 1e9,
            "graph_full_cycle_frac": cold.cycle_bytes() / cstep / 1e9 / HBM_PEAK_GBS,
            "tokens_per_s_per_layer": wc.B / cstep})
        del cold, g

    if not args.no_regimes and types == ("bf16", "f32", "f32") and args.workload == "qwen3next_decode":
        # the paper's own storage regime (Sec. 4.1): fp16 vectors and records, fp32 state
        reg = {}
        for ty in (("f16", "f16", "f16"), ("f16", "f32", "f32")):
            rj = DecodeJob(w, fused=fused, types=ty)
            rj.run(w.prefix + W)
            g = rj.capture(K)
            rsec = statistics.median(rj.timed_replays(g, K, min_ms=20.0)) / K
            reg["/".join(ty)] = {"types": "inputs/records/outputs", "us_per_step": rsec * 1e6,
                                 "tokens_per_s_per_layer": w.B / rsec,
                                 "algorithmic_bytes_per_step": rj.cycle_bytes(),
                                 "algorithmic_GBps": rj.cycle_bytes() / rsec / 1e9}
            del rj, g
        res["storage_regimes"] = reg

    if not args.no_other_paths:
        res["other_paths"] = time_other_paths(torch, kvb, synth, traffic)
    if not args.no_cpu_baseline:
        import numpy as np
        tok_np = synth.token_stream(np.random.default_rng(w.seed), w.B, 32, w.Hk, w.Hv, w.dk, w.dv, types[0])
        res["cpu_baseline"] = cpu_baseline(w, tok_np)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
