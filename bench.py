#!/usr/bin/env python3
"""Benchmark of the CacheCard hot path on one MI355X.

One step = one handoff over synthetic Llama-3.1-8B-shaped KV already resident in HBM:
scores -> widths -> planned card (qkv_assign_plan), K/V rows -> card (qkv_card_fill), card -> dense
fp16 cache (qkv_unpack_dequant).  Prints ONE JSON line: whole-job throughput in GB/s of fp16 KV
bytes per handoff, the HBM roofline of the slowest kernel, the same figures for the other
benchmark configurations (`workloads`), and the CPU oracle timed on the same tensors.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu] [--no-workloads]
"""
import argparse
import hashlib
import json
import math
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import qkv_synth  # noqa: E402

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak
MALL_BYTES = 256 << 20    # memory-side cache: a working set below this is served from it, not from HBM

# Bytes between L2 and the memory fabric per launch, from the FETCH_SIZE and WRITE_SIZE counters scaled by
# what a plain 512 MiB copy reads on them.  They describe the kernels as they were when the profile was
# taken: `sources` is a digest of the kernel sources at that time, and the figures are reported only while
# the sources still have that digest (else `traffic` is null and says why).
MEASURED_TRAFFIC = {
    "llama8b_8k_b3": {"pack": 1341416838, "unpack": 1346860972, "sources": "0f70b0a498685514",
                      "profile": "profiles/pack_unpack_llama8b_8k_b3_hbm_traffic.txt"},
}
KERNEL_SOURCES = ["pack.hip", "unpack.hip", "qkv_encode.h", "qkv_decode.h", "qkv_common.h"]

# The attention kernel is bound by instruction issue, not by memory: its roofline block is priced against the
# vector pipes.  One compute unit has 4 SIMDs, each of which starts one vector instruction (64 lanes wide, 16
# lanes a cycle) every 4 cycles: 256 CUs x 4 x 2.4 GHz = 614.4 G vector instructions/s, or 39.3 T lane
# operations/s (the published 157.3 TFLOP/s of fp32 is this figure times 2 flops of an FMA times 2 values of a
# packed instruction).  The kernel's vector instructions per launch come from the SQ_INSTS_VALU counter
# (matrix instructions included), with the digest of the sources they were counted for.
VECTOR_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
MEASURED_ATTEND = {
    "llama8b_8k_b3": {"valu_instructions": 24405761, "mfma_instructions": 3182592, "lds_instructions": 2981888,
                      "lds_active_cycles": 18725549, "lds_bank_conflict_cycles": 10719405, "sources": "884543a9d0931eac",
                      "profile": "profiles/card_attend_llama8b_8k_b3.txt"},
}
ATTEND_SOURCES = ["attend.hip", "qkv_decode.h", "qkv_common.h"]


def kernel_sources_digest(names=KERNEL_SOURCES):
    h = hashlib.sha256()
    for name in names:
        with open(os.path.join(ROOT, "paper_2605_03884_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def pct_of_peak(nbytes, ms):
    return round(100.0 * nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)


class Handoff:
    """One benchmark configuration resident in HBM: inputs, widths, and rotating sets of cards and outputs."""

    def __init__(self, qkv, name, dev, kv=None, want_sets=3, hop=0, src=None):
        self.qkv, self.name, self.dev = qkv, name, dev
        cfg = self.cfg = qkv_synth.CONFIGS[name]
        L, H, T, D, G = cfg["layers"], cfg["kv_heads"], cfg["tokens"], cfg["head_dim"], cfg["group_size"]
        self.shape = (L, H, T, D, G)
        self.desc = qkv.Desc.make(L, H, T, D, G, model_id=0x11A3A8B, sender_id=1)
        if src is not None:
            K, V = src
        elif kv is not None:
            K, V = kv
        else:
            K, V = qkv_synth.make_kv(L, H, T, D, cfg["data_seed"], cfg["kind"], device=dev)
        self.kv_bytes = K.numel() * 2 + V.numel() * 2
        kind = cfg["bits"][0]
        self.kc = bool(cfg.get("keys_per_channel"))
        self.scores, self.budget, self.score_seed = None, None, None
        if kind == "budget":
            self.score_seed, self.budget = cfg["bits"][1], cfg["bits"][2]
        elif kind == "hops":
            self.score_seed, self.budget = cfg["bits"][1][hop], cfg["bits"][2][hop]
        if self.score_seed is not None:
            self.scores = qkv_synth.make_scores(T, self.score_seed, dev)
            self.counts = qkv.budget_counts(T, self.budget)
            self.bits = torch.empty(T, dtype=torch.uint8, device=dev)
        else:
            self.bits = (qkv_synth.make_bits_uniform_choice(T, cfg["bits"][1], dev) if kind == "choice"
                         else qkv_synth.make_bits_constant(T, cfg["bits"][1], dev))
            self.counts = qkv.count_bits(self.bits)
        self.card_bytes = qkv.card_bytes(self.desc, self.counts)
        self.moved = self.kv_bytes + self.card_bytes          # algorithmic bytes of either direction
        # Rotation: a card must never be written over its own copy still sitting in the memory-side cache, and
        # small inputs must not be served from that cache either, so small workloads rotate their inputs too.
        need = max(want_sets, 1)
        if want_sets > 1 and self.moved * want_sets < 3 * MALL_BYTES:
            need = min(8, max(want_sets, -(-3 * MALL_BYTES // self.moved)))
        self.nsets = need
        self.inputs = [(K, V)]
        if need > want_sets or (want_sets > 1 and self.kv_bytes < 2 * MALL_BYTES):
            self.inputs += [(K.clone(), V.clone()) for _ in range(need - 1)]
        self.cards = [torch.empty(self.card_bytes, dtype=torch.uint8, device=dev) for _ in range(need)]
        self.outs = [(torch.empty_like(K), torch.empty_like(V)) for _ in range(need)]
        self.turn = 0
        self.stage_names = (["assign_plan", "card_fill", "unpack_dequant"] if self.scores is not None and not self.kc
                            else ["quantize_pack", "unpack_dequant"] if self.kc
                            else ["card_plan", "card_fill", "unpack_dequant"])

    def working_set_bytes(self):
        return self.nsets * (self.card_bytes + self.kv_bytes) + len(self.inputs) * self.kv_bytes

    def step(self, events=None):
        """One handoff.  `events`: len(stage_names) + 1 HIP events recorded around the stages on the launch stream."""
        qkv = self.qkv
        i = self.turn % self.nsets
        self.turn += 1
        K, V = self.inputs[i % len(self.inputs)]
        card, (K_out, V_out) = self.cards[i], self.outs[i]
        n = 0

        def mark():
            nonlocal n
            if events is not None:
                events[n].record()
            n += 1

        mark()
        if self.kc:
            qkv.quantize_pack_kc(self.desc, K, V, self.bits, self.counts, card)
            mark()
            qkv.unpack_dequant_kc(card, self.desc, K_out, V_out)
            mark()
            return
        if self.scores is not None:
            qkv.assign_plan(self.desc, self.scores, self.budget, card, bits=self.bits)
        else:
            qkv.card_plan(self.desc, self.bits, self.counts, card)
        mark()
        qkv.card_fill(self.desc, K, V, self.counts, card)
        mark()
        qkv.unpack_dequant(card, self.desc, K_out, V_out)
        mark()

    def last(self):
        i = (self.turn - 1) % self.nsets
        return self.inputs[i % len(self.inputs)], self.cards[i], self.outs[i]

    def wall_ms(self, steps, warmup):
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def event_ms(self, steps):
        """The same steps with HIP events between the launches: per stage the list of per-step times."""
        ns = len(self.stage_names)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(ns + 1)] for _ in range(steps)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in evs:
            self.step(e)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps * 1e3
        return {name: [e[k].elapsed_time(e[k + 1]) for e in evs] for k, name in enumerate(self.stage_names)}, wall


def parity_sample(h):
    """Layer 0 of the card and of the rebuilt cache that the timed buffers hold, byte for byte against the CPU oracle
    (the oracle builds the one-layer card of the same tokens and widths; the planes of a layer are the same rows
    in either card).  Returns a short record; raises on a mismatch."""
    import numpy as np
    from oracle import ref
    L, H, T, D, G = h.shape
    (K, V), card, (K_out, V_out) = h.last()
    torch.cuda.synchronize()
    bits = h.bits.cpu().numpy()
    t0 = time.perf_counter()
    if h.scores is not None:
        want_bits, want_counts = ref.assign_bits(qkv_synth.make_scores(T, h.score_seed).numpy(), h.budget)
        assert np.array_equal(bits, want_bits), "widths differ from the oracle's"
        assert h.counts == want_counts.tolist()
    d1 = ref.make_desc(1, H, T, D, G, 0x11A3A8B, 1, 0)
    dL = ref.make_desc(L, H, T, D, G, 0x11A3A8B, 1, 0)
    k0, v0 = K[:1].cpu().numpy(), V[:1].cpu().numpy()
    pack = ref.quantize_pack_kc if h.kc else ref.quantize_pack
    unpack = ref.unpack_dequant_kc if h.kc else ref.unpack_dequant
    small = pack(d1, k0, v0, bits, h.counts)
    o1, oL = ref.card_offsets(d1, h.counts), ref.card_offsets(dL, h.counts)
    compared = 0

    def same(lo_big, lo_small, n, what):
        nonlocal compared
        if n == 0:
            return
        got = card[lo_big:lo_big + n].cpu().numpy()
        assert np.array_equal(got, small[lo_small:lo_small + n]), "card differs from the oracle's in " + what
        compared += n

    same(oL["bits"], o1["bits"], o1["codes2"] - o1["bits"], "the bits / slot / order tables")
    for c, w in enumerate((2, 4, 8, 16)):
        n_c = h.counts[c]
        secs = [("fp16", D * 2)] if w == 16 else [("codes%d" % w, D * w // 8), ("meta%d" % w, (D // G) * 4)]
        for sec, row in secs:
            same(oL[sec], o1[sec], H * n_c * row, sec + " of the key planes")                       # K planes 0 .. H-1
            same(oL[sec] + L * H * n_c * row, o1[sec] + H * n_c * row, H * n_c * row, sec + " of the value planes")
    wk, wv = unpack(small, d1)
    assert np.array_equal(K_out[0].cpu().numpy().view(np.uint16), wk[0]), "rebuilt keys differ from the oracle's"
    assert np.array_equal(V_out[0].cpu().numpy().view(np.uint16), wv[0]), "rebuilt values differ from the oracle's"
    return {"against": "oracle", "planes": "layer 0 (%d key and %d value planes), all tokens" % (H, H),
            "card_bytes_compared": compared, "cache_bytes_compared": 2 * H * T * D * 2, "equal": True,
            "seconds": round(time.perf_counter() - t0, 2)}


def mean(v):
    return sum(v) / len(v)


def workload_record(h, steps, warmup, check):
    """Short run of one configuration: microseconds per stage by HIP events, GB/s, % of the HBM peak."""
    wall = h.wall_ms(steps, warmup)
    stages, _ = h.event_ms(steps)
    rec = {"workload": h.name, "tokens": h.shape[2], "group_size": h.shape[4], "counts_2_4_8_16": h.counts,
           "card_bytes": h.card_bytes, "kv_bytes": h.kv_bytes, "bytes_moved_per_direction": h.moved,
           "buffer_sets": h.nsets, "input_sets": len(h.inputs), "steps": steps,
           "us": {k: round(mean(v) * 1e3, 2) for k, v in stages.items()}, "us_per_handoff": round(wall * 1e3, 2),
           "kv_gbs_per_handoff": round(h.kv_bytes / (wall * 1e-3) / 1e9, 1)}
    create = sum(mean(stages[k]) for k in h.stage_names[:-1])
    unpack = mean(stages["unpack_dequant"])
    rec["pct_hbm_peak"] = {"creation (all launches before the card is complete)": pct_of_peak(h.moved, create),
                           "unpack_dequant": pct_of_peak(h.moved, unpack),
                           "unpack_dequant, fp16 bytes written only": pct_of_peak(h.kv_bytes, unpack)}
    if "card_fill" in stages:
        rec["pct_hbm_peak"]["card_fill"] = pct_of_peak(h.moved, mean(stages["card_fill"]))
    if h.working_set_bytes() < 2 * MALL_BYTES:
        rec["note"] = "working set below the 256 MB memory-side cache: launch-bound, not an HBM figure"
    if check:
        rec["parity_before_timing"] = check
    return rec


def cpu_baseline(h, layers):
    """The oracle, unchanged and single-threaded, on the first `layers` layers of the same tensors."""
    import numpy as np
    from oracle import ref
    L, H, T, D, G = h.shape
    (K_dev, V_dev), _, _ = h.last()
    K = K_dev[:layers].cpu().numpy()
    V = V_dev[:layers].cpu().numpy()
    bits_host = h.bits.cpu().numpy()
    d = ref.make_desc(layers, H, T, D, G)
    t0 = time.perf_counter()
    if h.scores is not None:
        bits, counts = ref.assign_bits(qkv_synth.make_scores(T, h.score_seed).numpy(), h.budget)
        assert np.array_equal(bits, bits_host)
    else:
        bits = bits_host
        counts = ref.count_bits(bits)
    card = ref.quantize_pack(d, K, V, bits, counts)
    ref.unpack_dequant(card, d)
    dt = time.perf_counter() - t0
    return 2 * layers * H * T * D * 2 / dt / 1e9, dt


def cpu_baseline_threads(h, layers, threads):
    """The same unchanged oracle on disjoint layers in `threads` host threads (the planes of different layers are
    independent given the widths): the widths once, then every thread builds and unpacks the one-layer cards of
    its layers."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import ref
    L, H, T, D, G = h.shape
    (K_dev, V_dev), _, _ = h.last()
    K = K_dev[:layers].cpu().numpy()
    V = V_dev[:layers].cpu().numpy()
    d1 = ref.make_desc(1, H, T, D, G)
    ref.lib()
    t0 = time.perf_counter()
    if h.scores is not None:
        bits, counts = ref.assign_bits(qkv_synth.make_scores(T, h.score_seed).numpy(), h.budget)
    else:
        bits = h.bits.cpu().numpy()
        counts = ref.count_bits(bits)

    def one(l):
        card = ref.quantize_pack(d1, K[l:l + 1], V[l:l + 1], bits, counts)
        ref.unpack_dequant(card, d1)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        list(pool.map(one, range(layers)))
    dt = time.perf_counter() - t0
    return 2 * layers * H * T * D * 2 / dt / 1e9, dt


def hop_report(qkv, name, K, V, dev, steps, check):
    """The multi-hop workload: every hop quantizes what the previous hop's receiver rebuilt, at that hop's budget
    (paper Sec. 3.2, challenge 3: error accumulates across hops).  Per hop: the workload record (stage times by HIP
    events, % of peak), the signal-to-noise ratio of the rebuilt cache against the original one, and the same hop
    taken card to card."""
    cfg = qkv_synth.CONFIGS[name]
    out = []
    src = (K, V)
    prev = None

    def snr_db(ref_t, got_t):
        num = den = 0.0
        for l in range(ref_t.shape[0]):                # layer by layer: no 4 GiB temporaries
            r = ref_t[l].float()
            num += float((r * r).sum(dtype=torch.float64))
            den += float(((got_t[l].float() - r) ** 2).sum(dtype=torch.float64))
        return round(10.0 * math.log10(num / den), 2) if den > 0 else float("inf")

    for hop, budget in enumerate(cfg["bits"][2]):
        h = Handoff(qkv, name, dev, want_sets=1, hop=hop, src=src)
        h.step()
        verdict = parity_sample(h) if check else None
        rec = workload_record(h, steps, 2, verdict)
        rec["hop"], rec["budget"] = hop + 1, budget
        _, card, (k_out, v_out) = h.last()
        rec["snr_db_k"], rec["snr_db_v"] = snr_db(K, k_out), snr_db(V, v_out)
        if prev is not None:                            # the same hop card to card, without the dense cache
            prev_card, prev_desc = prev
            direct = torch.empty_like(card)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            for _ in range(3):
                ev[0].record()
                qkv.requantize(prev_card, prev_desc, h.bits, h.counts, direct)
                ev[1].record()
                torch.cuda.synchronize()
            rec["requantize"] = {"ms": round(ev[0].elapsed_time(ev[1]), 4), "equals_chain_card": bool(torch.equal(direct, card))}
            del direct
        prev = (card, h.desc)
        src = (k_out, v_out)
        out.append(rec)
    return out


def device_state(dev):
    """Name, unit counts and clocks of the GPU the run used: the limits HIP reports, and the levels the
    driver's sysfs files show as active at the end of the run (absent where the files are not readable)."""
    import glob
    pr = torch.cuda.get_device_properties(dev)
    st = {"name": pr.name, "arch": getattr(pr, "gcnArchName", None), "compute_units": pr.multi_processor_count,
          "hbm_bytes": pr.total_memory}
    for key in ("clock_rate", "memory_clock_rate", "L2_cache_size"):
        if hasattr(pr, key):
            st[key + ("_khz" if key.endswith("rate") else "")] = getattr(pr, key)
    try:
        want = "%04x:%02x:%02x" % (pr.pci_domain_id, pr.pci_bus_id, pr.pci_device_id)
        for card in sorted(glob.glob("/sys/class/drm/card*/device")):
            if not os.path.basename(os.path.realpath(card)).startswith(want):
                continue
            for name, key in (("pp_dpm_sclk", "sclk_active"), ("pp_dpm_mclk", "mclk_active"),
                              ("power_dpm_force_performance_level", "performance_level")):
                try:
                    with open(os.path.join(card, name)) as f:
                        lines = [ln.strip() for ln in f.read().splitlines() if ln.strip()]
                except OSError:
                    continue
                active = [ln for ln in lines if ln.endswith("*")]
                st[key] = (active[0].rstrip("* ") if active else lines[0]) if lines else None
    except (AttributeError, OSError):
        pass
    return st


def timed_calls(fn, n, warm=3):
    for _ in range(warm):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(n):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama8b_8k_b3", choices=sorted(qkv_synth.CONFIGS))
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle legs (timing and parity sample)")
    ap.add_argument("--no-workloads", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--buffer-sets", type=int, default=3,
                    help="card / output buffer sets rotated over the steps, so that a card is never written over "
                         "its own copy still sitting in the 256 MB memory-side cache (that would hide its HBM "
                         "write-back: 223 instead of 244 us for quantize_pack at 8K with a single set)")
    ap.add_argument("--inject-layout", default="separate", choices=["separate", "pool", "dense"],
                    help="where the per-layer injection writes: one allocation per layer tensor with room for a 64-token "
                         "prefix (as frameworks keep their caches), views of one pooled allocation, or the dense output "
                         "tensors of the handoff itself (same addresses as qkv_unpack_dequant)")
    ap.add_argument("--beside-forward", action="store_true",
                    help="also time layer-by-layer injection on a second stream beside a stand-in for the receiver's "
                         "forward pass over its prefix (library GEMMs), against running the two one after the other")
    ap.add_argument("--handoff-only", action="store_true",
                    help="time the handoff alone and skip everything around it (other workloads, attention, injection, "
                         "requantization, controller, CPU legs): for profiles in which every launch of a kernel belongs "
                         "to the timed step")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a captured graph (reported beside the eager figure)")
    ap.add_argument("--cpu-layers", type=int, default=0,
                    help="layers of the workload the CPU oracle is timed on (0: about 8192*32 token-layers)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (a card is built and unpacked per GPU, planes shard without exchange); "
              "run with --gpus 1", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU path", file=sys.stderr)
        return 3

    import paper_2605_03884_amd as qkv
    import bench_probe
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.handoff_only:
        args.no_cpu = args.no_workloads = True
    is_hops = qkv_synth.CONFIGS[args.workload]["bits"][0] == "hops"
    h = Handoff(qkv, args.workload, dev, want_sets=1 if is_hops else max(1, args.buffer_sets))
    L, H, T, D, G = h.shape
    desc, kv_bytes, card_bytes, moved, counts = h.desc, h.kv_bytes, h.card_bytes, h.moved, h.counts
    K, V = h.inputs[0]

    # before any timing: the buffers the timed steps use hold what the oracle computes
    h.step()
    parity = None if args.no_cpu else parity_sample(h)
    _, c2, avg_bits, status = qkv.card_peek(h.last()[1])
    assert status == 0 and c2 == counts, (status, c2, counts)

    for _ in range(args.warmup):
        h.step()
    # timed region: exactly K steps, nothing else on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        h.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3

    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            h.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        # one graph holds one step per buffer set, so that a replay rotates the sets as the eager loop does
        h.turn = 0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(h.nsets):
                h.step()
        replays = max(1, args.steps // h.nsets)
        for _ in range(max(1, args.warmup // h.nsets)):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) / (replays * h.nsets) * 1e3

    # the same K steps again with HIP events between the launches (the events cost a few microseconds per
    # step themselves, which is why the figure above is taken without them)
    stages, ms_per_step_events = h.event_ms(args.steps)
    stage_avg = {k: mean(v) for k, v in stages.items()}

    def spread(v):
        v = sorted(v)
        return {"median": round(v[len(v) // 2], 4), "min": round(v[0], 4), "max": round(v[-1], 4)}

    unpack_ms = stage_avg["unpack_dequant"]
    fill_ms = stage_avg.get("card_fill", stage_avg.get("quantize_pack"))
    create_ms = sum(stage_avg[k] for k in h.stage_names[:-1])
    (_, _), card, (K_out, V_out) = h.last()

    # the three-launch path the one-launch planning replaces (qkv_assign_bits, then qkv_quantize_pack = plan + fill)
    three_launch = None
    if h.scores is not None and not h.kc and not args.handoff_only:
        n3 = max(10, args.steps // 4)
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(3 + n3)]
        torch.cuda.synchronize()
        for it, e in enumerate(ev):
            c3 = h.cards[it % h.nsets]
            e[0].record()
            qkv.assign_bits(h.scores, h.budget, bits=h.bits)
            e[1].record()
            qkv.quantize_pack(desc, K, V, h.bits, counts, c3)
            e[2].record()
            qkv.unpack_dequant(c3, desc, *h.outs[it % h.nsets])
        torch.cuda.synchronize()
        a_ms, q_ms = mean([e[0].elapsed_time(e[1]) for e in ev[3:]]), mean([e[1].elapsed_time(e[2]) for e in ev[3:]])
        three_launch = {"assign_bits_ms": round(a_ms, 4), "quantize_pack_ms": round(q_ms, 4),
                        "pct_hbm_peak_quantize_pack": pct_of_peak(moved, q_ms),
                        "pct_hbm_peak_assign_bits+quantize_pack": pct_of_peak(moved, a_ms + q_ms)}

    # beyond the handoff itself: one decode step's attention taken directly over the card
    # (32 query heads on 8 kv heads as in Llama-3.1-8B), timed on its own
    attend = None
    if D == 128 and not args.handoff_only:
        rep = 4
        qv = qkv_synth.normal(h.cfg["data_seed"] + 17, 9, 0, L * H * rep * D, dev).view(L, H * rep, D).to(torch.float16)
        a_out = torch.empty((L, H * rep, D), dtype=torch.float32, device=dev)
        a_lse = torch.empty((L, H * rep), dtype=torch.float32, device=dev)
        ws = torch.empty(qkv.card_attend_workspace(desc, H * rep), dtype=torch.uint8, device=dev)
        n_att = max(10, args.steps // 4)
        attend_call = qkv.card_attend_kc if h.kc else qkv.card_attend      # by the grouping of the card's keys
        att_ms = timed_calls(lambda: attend_call(card, desc, qv, D ** -0.5, a_out, lse=a_lse, workspace=ws), n_att,
                             warm=max(3, args.warmup // 4))
        att_bytes = card_bytes + qv.numel() * 2 + a_out.numel() * 4 + a_lse.numel() * 4
        attend = {"call": "qkv_card_attend_kc" if h.kc else "qkv_card_attend", "q_heads": H * rep, "avg_ms": round(att_ms, 4), "calls": n_att,
                  "algorithmic_bytes": att_bytes, "achieved_gbs": round(att_bytes / (att_ms * 1e-3) / 1e9, 1),
                  "frac_hbm_peak": round(att_bytes / (att_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "dense_cache_gbs_equivalent": round(kv_bytes / (att_ms * 1e-3) / 1e9, 1)}
        # what bounds it: the vector pipes (the whole call is timed, merging kernel included)
        meas, att_digest = MEASURED_ATTEND.get(args.workload), kernel_sources_digest(ATTEND_SOURCES)
        if meas is not None and meas["sources"] == att_digest:
            tlane = meas["valu_instructions"] * 64 / (att_ms * 1e-3) / 1e12
            attend["roofline"] = {"bound": "alu", "achieved": round(tlane, 2), "peak": round(VECTOR_PEAK_TLANEOPS, 1),
                                  "unit": "T lane-op/s", "frac": round(tlane / VECTOR_PEAK_TLANEOPS, 4),
                                  "vector_instructions_per_launch": meas["valu_instructions"],
                                  "of_which_matrix": meas["mfma_instructions"], "profile": meas["profile"],
                                  "kernel_sources_digest": att_digest}
        else:
            attend["roofline"] = {"bound": "alu", "achieved": None, "peak": round(VECTOR_PEAK_TLANEOPS, 1), "unit": "T lane-op/s",
                                  "frac": None, "kernel_sources_digest": att_digest,
                                  "note": "no instruction count on file for this workload and these sources"}

    # injection into per-layer caches (one key and one value tensor per layer, room for a prefix), with and
    # without realigning the keys, in one call and layer by layer
    inject = None
    if L <= 64 and not h.kc and not args.handoff_only:
        prefix, cap = 64, T + 64
        if args.inject_layout == "dense":
            prefix, cap = 0, T
            per_layer = [(K_out[l], V_out[l]) for l in range(L)]
        elif args.inject_layout == "pool":
            pool = torch.empty((L, 2, H, cap, D), dtype=torch.float16, device=dev)
            per_layer = [(pool[l, 0], pool[l, 1]) for l in range(L)]
        else:
            per_layer = [(torch.empty((H, cap, D), dtype=torch.float16, device=dev), torch.empty((H, cap, D), dtype=torch.float16, device=dev))
                         for _ in range(L)]
        kls = [k[:, prefix:prefix + T] for k, _ in per_layer]
        vls = [v[:, prefix:prefix + T] for _, v in per_layer]
        n_inj = max(10, args.steps // 4)
        dense_ms = timed_calls(lambda: qkv.unpack_dequant(card, desc, K_out, V_out), n_inj)     # same loop, for comparison
        plain_ms = timed_calls(lambda: qkv.inject_layers(card, desc, kls, vls, 0), n_inj)
        rope_ms = timed_calls(lambda: qkv.inject_layers(card, desc, kls, vls, 0, rope_base=500000.0, rope_delta=prefix), n_inj)

        def by_layer():
            for l in range(L):
                qkv.inject_layers(card, desc, kls[l:l + 1], vls[l:l + 1], l, rope_base=500000.0, rope_delta=prefix)

        layer_ms = timed_calls(by_layer, n_inj)

        # Layer-at-a-time injection beside the receiver's own forward pass (Sec. 4.2.2: the receiver prefills its
        # prefix while the foreign cache arrives).  The forward pass is a stand-in: the dense projections of one
        # Llama-3.1-8B layer (hidden 4096, 14336 wide MLP, bf16, library GEMMs) over the prefix tokens, the same
        # weights for every layer; layer l of it waits for layer l of the injection, which runs on a second stream.
        overlap = None
        if args.beside_forward and args.workload.startswith("llama8b") and prefix > 0:
            hid, ffn = 4096, 14336
            gen = torch.Generator(device=dev).manual_seed(h.cfg["data_seed"] + 41)
            mk = lambda *shape: (torch.randn(*shape, device=dev, generator=gen, dtype=torch.float32) * 0.02).to(torch.bfloat16)
            w_qkv, w_o, w_gu, w_d = mk(hid, hid + 2 * H * D), mk(hid, hid), mk(hid, 2 * ffn), mk(ffn, hid)
            x0 = mk(prefix, hid)

            def layer_forward(x):
                x = x + (x @ w_qkv)[:, :hid] @ w_o
                gu = x @ w_gu
                return x + (torch.nn.functional.silu(gu[:, :ffn]) * gu[:, ffn:]) @ w_d

            def forward_alone():
                x = x0
                for _ in range(L):
                    x = layer_forward(x)

            def serial():
                by_layer()
                forward_alone()

            side = torch.cuda.Stream()
            main_stream = torch.cuda.current_stream()
            ready = [torch.cuda.Event() for _ in range(L)]

            def overlapped():
                side.wait_stream(main_stream)
                with torch.cuda.stream(side):
                    for l in range(L):
                        qkv.inject_layers(card, desc, kls[l:l + 1], vls[l:l + 1], l, rope_base=500000.0, rope_delta=prefix)
                        ready[l].record(side)
                x = x0
                for l in range(L):
                    main_stream.wait_event(ready[l])
                    x = layer_forward(x)
                main_stream.wait_stream(side)

            overlap = {"receiver_forward_stand_in": "dense projections of %d Llama-3.1-8B layers over %d prefix tokens, bf16" % (L, prefix),
                       "forward_alone_ms": round(timed_calls(forward_alone, n_inj), 4),
                       "injection_then_forward_ms": round(timed_calls(serial, n_inj), 4),
                       "injection_beside_forward_ms": round(timed_calls(overlapped, n_inj), 4)}
            del w_qkv, w_o, w_gu, w_d
        inject = {"call": "qkv_inject_layers", "layers": L, "calls": n_inj, "layout": args.inject_layout,
                  "unpack_dequant_same_loop_ms": round(dense_ms, 4), "one_call_ms": round(plain_ms, 4), "one_call_realigned_ms": round(rope_ms, 4),
                  "layer_by_layer_realigned_ms": round(layer_ms, 4),
                  "frac_hbm_peak": round(moved / (plain_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "frac_hbm_peak_realigned": round(moved / (rope_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "beside_receiver_forward": overlap}
        del per_layer, kls, vls

    # forwarding the card at a lower budget, card to card (one hop of a chain), against the chain it replaces
    requant = None
    if h.scores is not None and not h.kc and not args.handoff_only and not is_hops:
        b2, c2 = qkv.assign_bits(qkv_synth.make_scores(T, h.cfg["data_seed"] + 31, dev), max(2.0, h.budget - 0.5))
        nxt = torch.empty(qkv.card_bytes(desc, c2), dtype=torch.uint8, device=dev)
        nxt2 = torch.empty_like(nxt)
        n_rq = max(10, args.steps // 4)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
        rq_ms = chain_ms = 0.0
        for it in range(3 + n_rq):
            ev[0].record()
            qkv.requantize(card, desc, b2, c2, nxt)
            ev[1].record()
            qkv.unpack_dequant(card, desc, K_out, V_out)
            qkv.quantize_pack(desc, K_out, V_out, b2, c2, nxt2)
            ev[2].record()
            torch.cuda.synchronize()
            if it >= 3:
                rq_ms += ev[0].elapsed_time(ev[1]) / n_rq
                chain_ms += ev[1].elapsed_time(ev[2]) / n_rq
        requant = {"call": "qkv_requantize", "to_budget": max(2.0, h.budget - 0.5), "ms": round(rq_ms, 4),
                   "chain_unpack_then_pack_ms": round(chain_ms, 4), "equal": bool(torch.equal(nxt, nxt2)),
                   "card_bytes_in_out": [card_bytes, nxt.numel()]}
        del nxt, nxt2

    # the controller in front of the handoff: features -> scores -> widths (objective-greedy), timed on its own
    controller = None
    if not args.handoff_only:
        feats = qkv_synth.make_features(T, h.cfg["data_seed"] + 23, dev)
        params = qkv.Controller.make(*[a.cpu() for a in qkv_synth.make_controller(h.cfg["data_seed"] + 24)])
        c_scores = torch.empty(T, dtype=torch.float32, device=dev)
        c_bits = torch.empty(T, dtype=torch.uint8, device=dev)
        c_counts = torch.empty(4, dtype=torch.int64, device=dev)
        n_ctl = max(10, args.steps // 4)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ctl_ms = [0.0, 0.0]
        for it in range(3 + n_ctl):
            ev[0].record()
            qkv.controller_scores(feats, params, c_scores)
            ev[1].record()
            qkv.assign_bits_greedy(c_scores, h.budget if h.budget is not None else 4.0, c_bits, c_counts)
            ev[2].record()
            torch.cuda.synchronize()
            if it >= 3:
                ctl_ms[0] += ev[0].elapsed_time(ev[1]) / n_ctl
                ctl_ms[1] += ev[1].elapsed_time(ev[2]) / n_ctl
        controller = {"controller_scores_ms": round(ctl_ms[0], 4), "assign_bits_greedy_ms": round(ctl_ms[1], 4),
                      "calls": n_ctl, "greedy_counts_2_4_8_16": c_counts.cpu().tolist()}

    # plain device copy of the same fp16 bytes: what this machine's HBM gives a kernel with no arithmetic
    copy_ms = timed_calls(lambda: K_out.copy_(K), 10)
    copy_gbs = 2 * K.numel() * 2 / (copy_ms * 1e-3) / 1e9

    # the handoff's memory traffic without its arithmetic, in the same rotation of buffer sets: 8 KiB read and
    # 2 KiB written per unit where card creation reads fp16 rows and writes a card of a quarter their size, then the
    # reverse for injection; the same cache policies (rows streamed, the card kept in the memory-side cache)
    ceiling = None
    if 0.22 <= card_bytes / kv_bytes <= 0.28 and not args.handoff_only:
        nsets = h.nsets
        src = torch.empty(kv_bytes, dtype=torch.uint8, device=dev)
        src[:kv_bytes // 2].copy_(K.view(torch.uint8).reshape(-1))
        src[kv_bytes // 2:].copy_(V.view(torch.uint8).reshape(-1))
        small = [torch.empty(kv_bytes // 4, dtype=torch.uint8, device=dev) for _ in range(nsets)]
        big = [torch.empty(kv_bytes, dtype=torch.uint8, device=dev) for _ in range(nsets)]
        n_pr = max(10, args.steps // 4)
        pev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(3 + n_pr)]
        torch.cuda.synchronize()
        for it in range(3 + n_pr):                    # queued back to back, like the event-timed steps above
            i = it % nsets
            pev[it][0].record()
            bench_probe.stream_probe(src, small[i], 8, 2, nontemporal=1)
            pev[it][1].record()
            bench_probe.stream_probe(small[i], big[i], 2, 8, nontemporal=2)
            pev[it][2].record()
        torch.cuda.synchronize()
        pr_ms = [sum(e[0].elapsed_time(e[1]) for e in pev[3:]) / n_pr, sum(e[1].elapsed_time(e[2]) for e in pev[3:]) / n_pr]
        ceiling = {"call": "qkv_stream_probe (bench_probe/)", "bytes_per_direction": kv_bytes + kv_bytes // 4,
                   "creation_like_ms": round(pr_ms[0], 4), "injection_like_ms": round(pr_ms[1], 4),
                   "creation_like_gbs": round((kv_bytes + kv_bytes // 4) / (pr_ms[0] * 1e-3) / 1e9, 1),
                   "injection_like_gbs": round((kv_bytes + kv_bytes // 4) / (pr_ms[1] * 1e-3) / 1e9, 1),
                   "pack_kernel_time_over_probe": round(fill_ms / pr_ms[0], 3),
                   "unpack_kernel_time_over_probe": round(unpack_ms / pr_ms[1], 3)}
        del src, small, big

    digest = kernel_sources_digest()

    def roof(name, ms, leg):
        a = moved / (ms * 1e-3) / 1e9
        meas = MEASURED_TRAFFIC.get(args.workload)
        traffic, note = None, "no counter profile for this workload"
        if meas is not None:
            if meas["sources"] == digest:
                traffic, note = meas[leg], meas["profile"]
            else:
                note = "the kernel sources changed since %s was taken" % meas["profile"]
        return {"kernel": name, "bound": "hbm", "achieved": round(a, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(a / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": note,
                "avg_ms": round(ms, 4), "algorithmic_bytes": moved, "kv_gbs": round(kv_bytes / (ms * 1e-3) / 1e9, 1)}

    legs = [roof("pack_kernel<%d> (qkv_card_fill)" % G, fill_ms, "pack"),
            roof("unpack_kernel<%d> (qkv_unpack_dequant)" % G, unpack_ms, "unpack")]
    dominant = max(legs, key=lambda r: r["avg_ms"])

    out = {
        "metric": "quantize+pack & unpack+dequant GB/s (fp16 KV bytes), % HBM peak, Llama8B-8K",
        "value": round(kv_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GB/s of fp16 KV bytes per handoff (%s)" % " + ".join(h.stage_names),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "buffer_sets": h.nsets, "layers": L, "kv_heads": H, "tokens": T, "head_dim": D,
                   "group_size": G, "storage_dtype": "f16 K/V and scale/zero pairs, u8 codes; arithmetic in f32",
                   "counts_2_4_8_16": counts, "avg_code_bits": round(avg_bits, 4), "kv_bytes": kv_bytes, "card_bytes": card_bytes,
                   "kernel_sources_digest": digest},
        "roofline": dominant,
        "roofline_all": legs,
        "parity_before_timing": parity,
        "stages_ms": {k: round(v, 4) for k, v in stage_avg.items()},
        "creation_ms": round(create_ms, 4),
        "pct_hbm_peak": {"creation: " + " + ".join(h.stage_names[:-1]): pct_of_peak(moved, create_ms),
                         "card_fill": pct_of_peak(moved, fill_ms),
                         "unpack_dequant": pct_of_peak(moved, unpack_ms),
                         "unpack_dequant, fp16 bytes written only (the card comes out of the memory-side cache)":
                             pct_of_peak(kv_bytes, unpack_ms)},
        "stages_ms_spread": {k: spread(v) for k, v in stages.items()},
        "three_launch_path": three_launch,
        "ms_per_step_with_events": round(ms_per_step_events, 4),
        "ms_per_step_graph_replay": None if graph_ms is None else round(graph_ms, 4),
        "copy_ceiling_gbs": round(copy_gbs, 1),
        "traffic_ceiling": ceiling,
        "device": device_state(dev),
        "card_attend": attend,
        "controller": controller,
        "inject_layers": inject,
        "requantize": requant,
    }
    if not args.no_cpu:
        layers = args.cpu_layers if args.cpu_layers > 0 else (L * 8192) // max(T, 8192)
        layers = max(1, min(layers, L))
        model = cpu_model()
        v, secs = cpu_baseline(h, layers)
        unit = "GB/s of fp16 KV bytes per handoff (assign_bits + quantize_pack + unpack_dequant)"
        out["cpu_baseline"] = {"value": round(v, 4), "unit": unit, "cores": 1, "cpu": model, "kind": "oracle",
                               "sample": "first %d of %d layers of the same tensors, all tokens, same widths; %.1f s"
                                         % (layers, L, secs)}
        threads = max(1, min(16, os.cpu_count() or 1, layers))
        v2, secs2 = cpu_baseline_threads(h, layers, threads)
        out["cpu_baseline_all_cores"] = {"value": round(v2, 4), "unit": unit, "cores": threads, "cpu": model, "kind": "oracle",
                                         "sample": "the same %d layers: assign_bits once, then one layer per task "
                                                   "(quantize_pack + unpack_dequant); %.1f s" % (layers, secs2)}
    if is_hops and not args.handoff_only:
        out["hops"] = hop_report(qkv, args.workload, K, V, dev, max(3, args.steps // 20), not args.no_cpu)

    # the other benchmark configurations, a short run each: microseconds per stage, GB/s, % of the HBM peak
    if not args.no_workloads:
        del h
        K = V = K_out = V_out = card = None
        torch.cuda.empty_cache()
        recs = []
        shared_kv = {}
        n_w = max(20, args.steps // 4)
        for name in ("tiny", "llama8b_1k_b5", "llama8b_1k_b4", "llama8b_8k_b3", "llama8b_8k_u4_g64", "llama8b_8k_u2_g64"):
            if name == args.workload:
                continue
            cfg = qkv_synth.CONFIGS[name]
            key = (cfg["layers"], cfg["kv_heads"], cfg["tokens"], cfg["head_dim"], cfg["data_seed"], cfg["kind"])
            if key not in shared_kv:
                shared_kv.clear()
                torch.cuda.empty_cache()
                shared_kv[key] = qkv_synth.make_kv(*key, device=dev)
            w = Handoff(qkv, name, dev, kv=shared_kv[key], want_sets=3)
            w.step()
            recs.append(workload_record(w, n_w, 5, None if args.no_cpu else parity_sample(w)))
            del w
        shared_kv.clear()
        torch.cuda.empty_cache()
        if args.workload != "llama8b_32k_hops":
            cfg = qkv_synth.CONFIGS["llama8b_32k_hops"]
            K32, V32 = qkv_synth.make_kv(cfg["layers"], cfg["kv_heads"], cfg["tokens"], cfg["head_dim"], cfg["data_seed"],
                                         cfg["kind"], device=dev)
            recs += hop_report(qkv, "llama8b_32k_hops", K32, V32, dev, 5, not args.no_cpu)
            del K32, V32
        out["workloads"] = recs
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
