#!/usr/bin/env python3
"""Benchmark of the decode + routing-tail path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

One "step" is one pass of the whole hot path (embedding, all decoder layers over the KV cache, routing tail)
over one batch. The headline workload is the 0.5B-class bf16 small model at 64 concurrent sequences with
prompt lengths uniform on [128, 1024] and a contiguous per-sequence cache; the same run also reports the
batch-1 decode and the isolated routing tail at 256 rows. Inputs are seeded and synthetic and are resident in
HBM when the timed region starts. Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

SEED = 7878
HBM_PEAK_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kv_bytes_per_token(s):
    return 2 * s.n_layers * s.n_kv_heads * s.head_dim * 2   # K and V, bf16


def weight_bytes_per_step(s):
    d, qw, kvw, F = s.d_model, s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim, s.d_ffn
    per_layer = d * qw + 2 * d * kvw + qw * d + 3 * d * F
    head = s.vocab * d
    router = s.router_hidden * d + s.router_hidden if s.router_hidden else 0
    return 2 * (s.n_layers * per_layer + head + router)


FAMILY_ID = None   # kernel family name -> TR_KERNEL_* (filled from the binding)


def family_times(model, slots, tokens_per_step, out, families):
    """Average duration of one launch of each kernel family inside real decode steps: per family a short run of steps with one
    launch of the family per step bracketed by events (the family's launches take turns, so every layer is sampled). The
    sequences are rolled back afterwards. Returns {family: (net us, bracketed us, empty-pair us, launches per step, samples)}."""
    import torch
    base = [model.seq_len(sl) for sl in slots]
    res = {}
    for fam, per_step in families.items():
        model.profile_select(FAMILY_ID[fam])
        model.profile_enable(True)
        n = max(8, per_step)                                 # every launch of the family is sampled at least once
        for i in range(n):
            model.decode_step(slots, tokens_per_step[i % len(tokens_per_step)], out)
        torch.cuda.synchronize()
        ms, gap, cnt = model.profile_read()
        model.profile_enable(False)
        for sl, b in zip(slots, base):
            model.seq_truncate(sl, b)
        if cnt:
            res[fam] = ((ms - gap) / cnt * 1e3, ms / cnt * 1e3, gap / cnt * 1e3, per_step, cnt)
    model.profile_select(FAMILY_ID["lmhead"])
    # the same steps with nothing bracketed: what is left of the step time after the kernels' own durations is the cost of
    # getting from the end of one kernel to the start of the next, shared equally by the launches
    n = 24
    for i in range(4):
        model.decode_step(slots, tokens_per_step[i % len(tokens_per_step)], out)
    for sl, b in zip(slots, base):
        model.seq_truncate(sl, b)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        model.decode_step(slots, tokens_per_step[i % len(tokens_per_step)], out)
    torch.cuda.synchronize()
    step_us = (time.perf_counter() - t0) / n * 1e6
    for sl, b in zip(slots, base):
        model.seq_truncate(sl, b)
    launches = sum(v[3] for v in res.values())
    res["_step_us"] = step_us
    res["_gap_us"] = max(0.0, (step_us - sum(v[0] * v[3] for v in res.values() if isinstance(v, tuple))) / max(launches, 1))
    return res


def time_decode(model, slots, tokens_per_step, steps, warmup, out, family="lmhead"):
    """Warm up, roll the sequences back, then time `steps` decode steps; one launch of `family` per step is bracketed by events.
    Returns seconds, the bracketed kernel time, ..."""
    import torch
    base = [model.seq_len(sl) for sl in slots]
    for i in range(warmup):
        model.decode_step(slots, tokens_per_step[i % len(tokens_per_step)], out)
    torch.cuda.synchronize()
    for sl, n in zip(slots, base):
        model.seq_truncate(sl, n)
    model.profile_select(FAMILY_ID[family])
    model.profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    room = min(model.cfg.max_seq - n for n in base)          # steps that fit before the longest sequence fills its cache
    for i in range(steps):
        if i and i % room == 0:                          # more steps asked for than the cache holds: start over from the prompts (host bookkeeping only)
            for sl, n in zip(slots, base):
                model.seq_truncate(sl, n)
        model.decode_step(slots, tokens_per_step[i % len(tokens_per_step)], out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms, gap_ms, launches = model.profile_read()
    model.profile_enable(False)
    # kernel duration = bracketed interval minus the empty event interval recorded right behind it on the same stream
    return dt, ms - gap_ms, launches, base, (ms, gap_ms)


def cpu_baseline(s, weights, seconds_budget=12.0, max_steps=600):
    """The oracle, as it stands, on the host cores: decode steps of a few sequences over a synthetic cache, for about
    `seconds_budget` seconds."""
    from oracle import tro
    from paper_2504_07878_amd import synth
    n_seq, ctx = 2, 576
    o = tro.Model(s.asdict(), weights, n_seq, ctx + max_steps)
    for b in range(n_seq):
        k, v = synth.kv_fill(SEED, f"cpu.kv{b}", s, ctx)
        o.load_kv(b, synth.bf16_bits_to_f32(k), synth.bf16_bits_to_f32(v))
    toks = synth.prompt_tokens(SEED, "cpu.toks", 64 * n_seq, s.vocab).reshape(64, n_seq)
    done, t0 = 0, time.perf_counter()
    while done < max_steps and time.perf_counter() - t0 < seconds_budget:
        o.decode_step(list(range(n_seq)), toks[done % len(toks)])
        done += 1
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": n_seq * done / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"{done} decode steps of {n_seq} sequences from context {ctx} on a synthetic cache, {dt:.1f} s (0.5B-class bf16 weights, fp32 oracle)"}


def counters_workload(s):
    """A plain copy kernel of known size, then the routing tail at 64 rows (and at 256 rows, for the matrix-core counters)."""
    import torch
    from paper_2504_07878_amd import synth, tokroute
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)                       # 1 GiB read + 1 GiB written
    torch.cuda.synchronize()
    one = s.with_(n_layers=1)
    w = synth.make_weights(one, SEED, workers=8)
    m = tokroute.Model(one.asdict(), w, 64, 8)
    x = torch.from_numpy(synth.hidden_rows(SEED, "counters.x", 64, s.d_model, False)).cuda()
    out = m.outputs(64)
    for _ in range(5):
        m.tail(x, out)
    torch.cuda.synchronize()
    m256 = tokroute.Model(one.asdict(), m.dev, 256, 8)
    x256 = torch.from_numpy(synth.hidden_rows(SEED, "counters.x256", 256, s.d_model, False)).cuda()
    out256 = m256.outputs(256)
    for _ in range(3):
        m256.tail(x256, out256)
    torch.cuda.synchronize()
    # decode steps of 64 ragged sequences (the headline workload's prompts) on a 2-layer model of the same shapes: the per-layer
    # kernels (attention over the caches, gate/up, down, q|k|v, output projection, the residual + norm kernel) at their real sizes
    two = s.with_(n_layers=2)
    w2 = synth.make_weights(two, SEED, workers=8)
    B = 64
    md = tokroute.Model(two.asdict(), w2, B, 1536)
    lens = synth.prompt_lengths(SEED, "cfg3.lens", B, 128, 1024)
    prompts = [synth.prompt_tokens(SEED, f"cfg3.prompt{b}", int(n), s.vocab) for b, n in enumerate(lens)]
    od = md.outputs(B)
    md.prefill(list(range(B)), prompts, od)
    toks = synth.prompt_tokens(SEED, "cfg3.steps", 4 * B, s.vocab).reshape(4, B)
    for i in range(4):
        md.decode_step(list(range(B)), toks[i], od)
    torch.cuda.synchronize()
    log(f"counters workload done: 1 copy of 1 GiB, 5 tail calls at 64 rows, 3 tail calls at 256 rows, 4 decode steps of 64 sequences on 2 layers "
        f"(cached tokens at the first step: {int(lens.sum())}, i.e. {(int(lens.sum()) + B) * 512} bytes of keys and values per attention launch)")


def floor_workload():
    """Chains of dependent do-nothing kernels (one 4-byte store per thread) of 1, 64 and 256 workgroups: what a launch costs
    whatever it does, the floor under a step that is a chain of ~170 dependent kernels. Prints one JSON line."""
    import torch
    from paper_2504_07878_amd import tokroute
    lib = tokroute.load_library()
    buf = torch.zeros(256 * 256, dtype=torch.int32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    rows = []
    for wgs in (1, 64, 256):
        assert lib.tr_profile_chain(st, buf.data_ptr(), wgs, 300) == 0
        torch.cuda.synchronize()
        n = 3000
        t0 = time.perf_counter()
        assert lib.tr_profile_chain(st, buf.data_ptr(), wgs, n) == 0
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        row = {"workgroups": wgs, "launches": n, "us_per_launch": (t2 - t0) / n * 1e6, "host_enqueue_us_per_launch": (t1 - t0) / n * 1e6}
        # the same chain replayed from a captured graph: no host enqueue in the way, what is left is the GPU's own cost per launch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                assert lib.tr_profile_chain(torch.cuda.current_stream().cuda_stream, buf.data_ptr(), wgs, 1000) == 0
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                graph.replay()
            torch.cuda.synchronize()
            row["graph_replay_us_per_launch"] = (time.perf_counter() - t0) / 5000 * 1e6
        torch.cuda.current_stream().wait_stream(side)
        rows.append(row)
    print(json.dumps({"metric": "cost of one launch in a chain of dependent do-nothing kernels", "unit": "us", "chains": rows,
                      "note": "wall clock over the whole chain; a kernel trace of this command gives the start-to-start spacing on the GPU"}), flush=True)


def gpu_drawn_weights(L, seed):
    """Weights of a large model drawn on the GPU (N(0, 0.02), seeded): drawing 7.6 G values on the host takes minutes."""
    import torch
    from paper_2504_07878_amd import synth, tokroute
    torch.manual_seed(seed)
    one = synth.make_weights(L.with_(n_layers=1, vocab=64), seed)
    draw = lambda shape: torch.randn(shape, device="cuda").mul_(0.02).to(torch.bfloat16)
    lw = {}
    for k, v in one.items():
        if k.startswith("l0."):
            for l in range(L.n_layers):
                lw[f"l{l}." + k[3:]] = draw(v.shape) if v.ndim == 2 else tokroute.to_device(v, L.dtype)
        elif k in ("tok_emb", "lm_head"):
            lw[k] = draw((L.vocab, L.d_model))
        else:
            lw[k] = draw(v.shape) if v.ndim == 2 else tokroute.to_device(v, L.dtype)
    return lw


def llm7b_workload(steps, warmup, as_dict=False, shares=(0.07,)):
    """Large-model decode on the routed subset: 32 sequences with 2048 cached positions, each flagged with probability 0.07 per step.

    The caches hold synthetic N(0, 1) values (one seeded fill, loaded into every slot). Two schedules over the same flags:
    the host picks the flagged sequences and calls the decode step on them (a step with no flagged sequence costs nothing);
    and tr_decode_step_active, which reads the flags on the device (launches sized for 8 rows, no host round trip).
    Prints one JSON line of its own, or returns it as a dict.
    """
    import numpy as np
    import torch
    from paper_2504_07878_amd import synth, tokroute
    L = synth.LLM_7B
    B, CTX, N_MAX = 32, 2048, 8
    total = warmup + steps
    llm = tokroute.Model(L.asdict(), gpu_drawn_weights(L, SEED), B, CTX + 2 * len(shares) * total + 8)
    k, v = synth.kv_fill(SEED, "cfg5.kv", L, CTX)
    k, v = tokroute.to_device(k, L.kv_dtype), tokroute.to_device(v, L.kv_dtype)
    for b in range(B):
        llm.load_kv(b, k, v)
    del k, v
    toks = synth.prompt_tokens(SEED, "cfg5.toks", total * B, L.vocab).reshape(-1, B)
    outs = {n: llm.outputs(n) for n in range(1, B + 1)}
    wb = 2 * (L.n_layers * (2 * L.d_model * L.n_q_heads * L.head_dim + 2 * L.d_model * L.n_kv_heads * L.head_dim + 3 * L.d_model * L.d_ffn)
              + L.vocab * L.d_model)
    kvb = 2 * L.n_layers * L.n_kv_heads * L.head_dim * 2
    res = None
    by_share = []
    for p in shares:
        flags = synth.bernoulli_flags(SEED, f"cfg5.flags{p:g}" if p != 0.07 else "cfg5.flags", (total, B), p)
        lens = np.array([llm.seq_len(b) for b in range(B)], np.int64)
        # (a) the host picks the subset
        routed = nbytes = 0
        hist = {}
        t0 = 0.0
        for i in range(total):
            if i == warmup:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            act = [b for b in range(B) if flags[i, b]]
            if not act:
                if i >= warmup:
                    hist[0] = hist.get(0, 0) + 1
                continue
            llm.decode_step(act, toks[i, act], outs[len(act)])
            if i >= warmup:
                routed += len(act)
                nbytes += wb + int(lens[act].sum() + len(act)) * kvb
                hist[len(act)] = hist.get(len(act), 0) + 1
            lens[act] += 1
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # (b) the device picks the subset from flags in device memory
        dflags = torch.from_numpy(flags.astype(np.int32)).cuda()
        dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
        active = torch.zeros(2 + N_MAX, dtype=torch.int32, device="cuda")
        nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
        taken = torch.zeros(1, dtype=torch.int64, device="cuda")
        slots = list(range(B))
        for i in range(total):
            if i == warmup:
                torch.cuda.synchronize()
                taken.zero_()
                t0 = time.perf_counter()
            llm.decode_step_active(slots, dflags[i], dtoks[i], N_MAX, active, nxt, outs[N_MAX])
            taken += active[0]
        torch.cuda.synchronize()
        dt_dev = time.perf_counter() - t0
        entry = {"flag_probability": p, "host_selected": {"ms_per_step": dt / steps * 1e3, "routed_tokens_per_s": routed / dt, "routed_tokens": routed},
                 "device_selected": {"ms_per_step": dt_dev / steps * 1e3, "routed_tokens_per_s": int(taken.item()) / dt_dev, "routed_tokens": int(taken.item()),
                                     "n_max": N_MAX}}
        by_share.append(entry)
        if p == 0.07:
            res = {"metric": "large-model decode on the routed subset, routed tokens/s", "value": routed / dt, "unit": "tokens/s", "n_gpus": 1,
                   "steps": steps, "warmup": warmup, "ms_per_step": dt / steps * 1e3, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
                   "config": {"workload": "7B-class bf16 decoder, 32 sequences with 2048 cached positions (synthetic cache), each flagged with "
                                          "probability 0.07 per step, decode on the flagged ones",
                              "routed_tokens": routed, "steps_by_rows": {str(n): c for n, c in sorted(hist.items())},
                              "ms_per_nonempty_step": dt / max(1, steps - hist.get(0, 0)) * 1e3,
                              "algorithmic_GB_per_s": nbytes / dt / 1e9, "fraction_of_hbm_roofline": nbytes / dt / 1e9 / HBM_PEAK_GBPS}}
    res = res or {}
    res["subset_selected_on_host_vs_device"] = by_share
    del llm, outs
    torch.cuda.empty_cache()
    if as_dict:
        return res
    print(json.dumps(res), flush=True)


def joint_workload(s, new_tokens=32, B=64, quantiles=(0.0, 0.02, 0.07, 0.2)):
    """Joint decoding of B sequences: 0.5B-class small model + router, 7B-class large model called on the flagged positions.

    The router of a random-weight model knows nothing, so each threshold is a quantile of its scores on a plain
    small-model run: 0.07 routes about 7 % of the positions (the paper's operating point, abstract), the others show how
    the rate moves with the routed share (the shape of the paper's Table 1). Prints one JSON line per threshold.
    """
    import numpy as np
    import torch
    from paper_2504_07878_amd import joint, synth, tokroute
    L = synth.LLM_7B
    max_seq = 128
    weights = synth.make_weights(s, SEED, workers=8)
    slm = tokroute.Model(s.asdict(), weights, B, max_seq)
    llm = tokroute.Model(L.asdict(), gpu_drawn_weights(L, SEED), B, max_seq)
    prompts = [synth.prompt_tokens(SEED, f"joint.p{b}", 32, s.vocab) for b in range(B)]
    # scores of a plain small-model run fix the thresholds
    slm.set_mode(1)
    out = slm.prefill(list(range(B)), prompts).cpu()
    scores = [out.score.copy()]
    for _ in range(8):
        out = slm.decode_step(list(range(B)), out.token).cpu()
        scores.append(out.score.copy())
    scores = np.concatenate(scores)
    slm.set_mode(0)
    # cost of the one host round trip per step (synchronise + copy tokens, scores and flags back), for comparison with the step time
    dev_out = slm.decode_step(list(range(B)), out.token)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        dev_out.cpu(joint.NEEDED)
    round_trip_us = (time.perf_counter() - t0) / 20 * 1e6
    for q in quantiles:
        tau = float(np.quantile(scores, q)) if q > 0 else 0.0
        slm.set_threshold(tau)
        joint.generate(slm, llm, prompts, 4)              # warm-up (every run starts with a prefill, which overwrites the caches)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tokens, routed = joint.generate(slm, llm, prompts, new_tokens)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # the same decoding with the large model on a stream of its own: flagged sequences wait for it, the others go on
        joint.generate_overlapped(slm, llm, prompts, 4)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tokens2, routed2 = joint.generate_overlapped(slm, llm, prompts, new_tokens)
        torch.cuda.synchronize()
        dt2 = time.perf_counter() - t0
        print(json.dumps({"metric": "joint decoding tokens/s (0.5B-class small model + router, 7B-class large model on the routed positions)",
                          "value": B * new_tokens / dt, "unit": "tokens/s", "n_gpus": 1, "data": "synthetic", "dtype": "bf16",
                          "config": {"workload": f"{B} sequences, 32-token prompts, {new_tokens} new tokens each, threshold at the {q:g} quantile of the router scores",
                                     "threshold": tau, "routed_fraction": float(routed.mean()), "seconds": dt,
                                     "host_round_trip_us_per_step": round_trip_us,
                                     "overlapped_schedule": {"tokens_per_s": B * new_tokens / dt2, "seconds": dt2,
                                                             "sequences_with_identical_output": int((tokens == tokens2).all(axis=1).sum()),
                                                             "what": "flagged sequences wait for the large model on a second stream while the others keep decoding"},
                                     "note": "prefill of both models is inside the timed region"}}), flush=True)


def measured_traffic(family):
    """HBM traffic (bytes read + written per launch) of a kernel family from hardware counters, valid only for the kernel
    sources it was taken on; None otherwise."""
    import hashlib
    t = TRAFFIC.get(family)
    if not t:
        return None
    h = hashlib.sha256()
    for name in ("mfma_kernels.hip", "tr_internal.h"):
        path = os.path.join(ROOT, "paper_2504_07878_amd", "csrc", name)
        if not os.path.exists(path):
            return None
        h.update(open(path, "rb").read())
    return t["fetch_bytes"] + t["write_bytes"] if h.hexdigest() == t["source_sha256"] else None


# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on `bench.py --workload counters`, scaled by the 1 GiB copy kernel of the same
# run (see profiles/); bytes per launch, per kernel family, with the hash of the kernel sources they were taken on.
TRAFFIC = {
    "attention": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 20754989, "write_bytes": 1660144},
    "gateup": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 19572731, "write_bytes": 1245184},
    "down": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 19317768, "write_bytes": 1376256},
    "qkv": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 6232760, "write_bytes": 507904},
    "oproj": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 5444322, "write_bytes": 516096},
    "prep": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 946608, "write_bytes": 809562},
    "lmhead": {"source_sha256": "3c3c251f49f4dae610eb9c84ca2080ead685e0ede0a9a81077ff54542a8f159d", "fetch_bytes": 274908243, "write_bytes": 322567},
}


# kernel families of a decode step of the 0.5B-class model at 64 rows: launches per step, and the kernels behind them
B64_FAMILIES = {"setup": 1, "prep": 25, "qkv": 24, "attention": 24, "oproj": 24, "gateup": 24, "down": 24, "lmhead": 1, "tail_merge": 1}
B1_FAMILIES = {"setup": 1, "qkv_attention": 24, "oproj": 24, "gateup": 24, "down": 24, "prep": 1, "lmhead": 1, "tail_merge": 1}
B1_KERNELS = {"setup": "setup_embed_kernel", "qkv_attention": "qkv_attn_kernel", "oproj": "residual_gemv_kernel<1,StageAttn>", "gateup": "gateup_kernel<1>",
              "down": "residual_splitk_kernel<3,1>", "prep": "prep_kernel (final norm)", "lmhead": "gemm22_kernel<28,EpiLmHead>", "tail_merge": "tail_final_kernel"}
B64_KERNELS = {"setup": "setup_embed_kernel", "prep": "prep_kernel", "qkv": "gemm_kernel<2,14,EpiQkv>", "attention": "attn_rows_kernel<64>",
               "oproj": "gemm_kernel<2,14,EpiResidualNorm>", "gateup": "gemm22_kernel<28,EpiSwiglu>", "down": "gemm22_kernel<28,EpiPartial>",
               "lmhead": "gemm22_kernel<28,EpiLmHead>", "tail_merge": "tail_final_kernel"}


def family_bytes(s, rows, attention_bytes):
    """Algorithmic bytes of ONE launch of each kernel family: each weight matrix once, each sequence's keys and values of one
    layer once (attention_bytes, given), new keys/values written; activations count as on-chip (0 for the kernels that only move them)."""
    d, qw, kvw, F = s.d_model, s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim, s.d_ffn
    return {"setup": 0, "prep": 0, "tail_merge": 0,
            "qkv": 2 * (qw + 2 * kvw) * d + rows * 2 * kvw * 2, "attention": attention_bytes, "oproj": 2 * d * qw,
            "gateup": 2 * 2 * F * d, "down": 2 * d * F, "lmhead": 2 * (s.vocab + s.router_hidden) * d,
            "qkv_attention": 2 * (qw + 2 * kvw) * d + rows * 2 * kvw * 2 + attention_bytes}


def kernel_table(s, fam, kernels, rows, attention_bytes):
    """One entry per kernel family: launches per step, average duration, algorithmic bytes per launch, fraction of the HBM peak."""
    fb = family_bytes(s, rows, attention_bytes)
    step_us, launch_gap = fam["_step_us"], fam["_gap_us"]
    table = []
    for name, v in fam.items():
        if not isinstance(v, tuple):
            continue
        net, raw, gap, per_step, cnt = v
        b = fb[name]
        dur = net + launch_gap        # what one launch of the family costs the step: its own duration and its share of the time between kernels
        table.append({"family": name, "kernel": kernels[name], "launches_per_step": per_step, "avg_us": dur, "kernel_us": net, "launch_gap_us": launch_gap,
                      "event_pair_avg_us": raw, "empty_event_pair_avg_us": gap, "samples": cnt, "us_per_step": dur * per_step,
                      "share_of_step": dur * per_step / step_us, "algorithmic_bytes_per_launch": b,
                      "achieved_GB_per_s": b / dur / 1e3 if b else None, "frac": b / dur / 1e3 / HBM_PEAK_GBPS if b else None,
                      "frac_of_kernel_time_alone": b / net / 1e3 / HBM_PEAK_GBPS if b else None})
    return table


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=512)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="b64", choices=["b64", "counters", "joint", "llm7b", "floor"],
                    help="b64: the benchmark; counters: one 1 GiB device copy (calibration) and a few routing-tail calls at 64 rows, "
                         "short enough for a hardware-counter pass of rocprofv3; joint: the two-model routing loop end to end at several routed shares; "
                         "llm7b: the large model's decode steps on a randomly flagged subset of 32 sequences; "
                         "floor: chains of dependent do-nothing kernels of 1, 64 and 256 workgroups")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: the library runs on ONE GPU (no collectives, no sharding); --gpus must be 1")
        sys.exit(2)

    import torch
    from paper_2504_07878_amd import synth, tokroute

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; there is no CPU path")
        sys.exit(2)
    tokroute.load_library()
    global FAMILY_ID
    FAMILY_ID = {name: i for i, name in enumerate(tokroute.KERNEL_FAMILIES)}
    s = synth.SLM_0P5B
    if args.workload == "counters":
        counters_workload(s)
        return
    if args.workload == "floor":
        floor_workload()
        return
    if args.workload == "joint":
        joint_workload(s)
        return
    if args.workload == "llm7b":
        llm7b_workload(min(args.steps, 256), args.warmup, shares=(0.07, 0.02, 0.0))
        return
    t0 = time.perf_counter()
    weights = synth.make_weights(s, SEED, workers=8)
    log(f"weights drawn in {time.perf_counter() - t0:.1f}s")

    B, MAX_SEQ = 64, 1536
    steps = max(1, args.steps)
    model = tokroute.Model(s.asdict(), weights, B, MAX_SEQ)
    lens = synth.prompt_lengths(SEED, "cfg3.lens", B, 128, 1024)
    prompts = [synth.prompt_tokens(SEED, f"cfg3.prompt{b}", int(n), s.vocab) for b, n in enumerate(lens)]
    slots = list(range(B))
    out = model.outputs(B)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    model.prefill(slots, prompts, out)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    log(f"prefill of {int(lens.sum())} tokens: {prefill_s:.3f}s")

    toks = synth.prompt_tokens(SEED, "cfg3.steps", 512 * B, s.vocab).reshape(512, B)
    kvb = kv_bytes_per_token(s)
    base0 = [model.seq_len(sl) for sl in slots]
    # 1. where the time of a step goes: every kernel family of the step, timed inside real steps (at the prompts' contexts)
    fam = family_times(model, slots, toks, out, B64_FAMILIES)
    by_kernel = kernel_table(s, fam, B64_KERNELS, B, (sum(base0) + B) * kvb / s.n_layers)
    dominant = max(by_kernel, key=lambda r: r["us_per_step"])["family"] if by_kernel else "lmhead"
    log("per-kernel table: " + "; ".join(f"{r['family']} {r['launches_per_step']} x {r['avg_us']:.2f} us" for r in by_kernel)
        + f"; {fam['_gap_us']:.2f} us of that between kernels -> dominant: {dominant}")
    # 2. the timed steps, with one launch per step of the dominant family bracketed by events
    dt, k_ms, k_n, base, k_raw = time_decode(model, slots, toks, steps, args.warmup, out, dominant)
    ms_per_step = dt / steps * 1e3
    tok_s = B * steps / dt
    # algorithmic bytes of the timed steps: weights once per step, each sequence's cache once, new K/V written
    room = min(MAX_SEQ - int(n) for n in base)           # time_decode starts over from the prompts every `room` steps
    ctx_sum = sum(int(n) + i % room for n in base for i in range(steps))        # sum over steps and sequences of cached tokens read
    step_bytes = weight_bytes_per_step(s) + (ctx_sum + B * steps) * kvb / steps
    roof_tok_s = B / (step_bytes / (HBM_PEAK_GBPS * 1e9))
    # bytes of one launch of the dominant family, averaged over the timed steps (attention: the caches of all 64 sequences, one layer)
    k_bytes = family_bytes(s, B, (ctx_sum + B * steps) / steps * kvb / s.n_layers)[dominant]
    launch_gap_us = fam["_gap_us"]
    k_net_us = k_ms * 1e3 / max(k_n, 1)
    k_avg_s = (k_net_us + launch_gap_us) / 1e6     # duration of a launch as the step sees it: the kernel and its share of the time between kernels
    share = B64_FAMILIES[dominant] * k_avg_s * 1e3 / ms_per_step
    result = {
        # the metric names three figures: value is the batch-64 one (the workload below); batch 1 and the isolated tail are in extras
        "metric": "SLM decode tokens/s at B=1/64 + fused routing-tail GB/s, % of HBM roofline", "value": tok_s, "unit": "tokens/s",
        "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "0.5B-class bf16 decoder + router, 64 concurrent sequences, prompts U[128,1024], contiguous KV cache, "
                               f"{steps} decode steps after prefill",
                   "batch": B, "max_seq": MAX_SEQ, "seed": SEED, "prefill_seconds": prefill_s,
                   "algorithmic_bytes_per_step": step_bytes, "hbm_roofline_tokens_per_s": roof_tok_s,
                   "fraction_of_hbm_roofline": tok_s / roof_tok_s},
        # the kernel family with the largest share of the step's time
        "roofline": {"bound": "hbm", "kernel": f"{B64_KERNELS[dominant]} ({dominant}, {B64_FAMILIES[dominant]} launches per step, 64 rows)",
                     "achieved": k_bytes / k_avg_s / 1e9 if k_n and k_bytes else None,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": (k_bytes / k_avg_s / 1e9 / HBM_PEAK_GBPS) if k_n and k_bytes else None,
                     "traffic": measured_traffic(dominant), "launches": k_n, "avg_us": k_avg_s * 1e6, "algorithmic_bytes_per_launch": k_bytes,
                     "share_of_step_time": share, "kernel_us": k_net_us, "launch_gap_us": launch_gap_us,
                     "frac_of_kernel_time_alone": (k_bytes / k_net_us / 1e3 / HBM_PEAK_GBPS) if k_n and k_bytes else None,
                     "event_pair_avg_us": k_raw[0] / max(k_n, 1) * 1e3, "empty_event_pair_avg_us": k_raw[1] / max(k_n, 1) * 1e3,
                     "how": "avg_us = event-bracketed duration of the kernel inside the timed steps (bracketed interval minus the empty event pair behind it) "
                            "+ the per-launch share of the step time that lies between kernels; the profiler's begin-to-end durations (profiles/) include that share too"},
        "roofline_by_kernel": by_kernel,
    }

    if not args.no_extras:
        extras = {}
        # catch-up step: every one of the 64 sequences ingests 14 tokens that another model produced (at ~7 % routing
        # about 14 small-model tokens lie between two routed ones); one call, the sequences one after the other
        seg = synth.prompt_tokens(SEED, "ext.seg", 14 * B, s.vocab).reshape(B, 14)
        for sl, n in zip(slots, base):                   # back to the prompts: room for the segments
            model.seq_truncate(sl, n)
        lens0 = list(base)
        reps = 3
        t0 = 0.0
        for r in range(reps + 1):            # first round is the warm-up
            if r == 1:
                torch.cuda.synchronize()
                t0 = time.perf_counter()
            model.extend(slots, list(seg), out)
            for sl, n in zip(slots, lens0):
                model.seq_truncate(sl, n)
        torch.cuda.synchronize()
        dte = (time.perf_counter() - t0) / reps
        extras["extend_k14"] = {"ingested_tokens_per_s": B * 14 / dte, "us_per_sequence": dte / B * 1e6, "ms_per_call_64_sequences": dte * 1e3,
                                "ms_of_14_decode_steps_at_batch_64": 14 * ms_per_step}
        # batch 1: 256-token prompt, 256 steps
        model.seq_truncate(0, 0)
        p1 = synth.prompt_tokens(SEED, "cfg2.prompt", 256, s.vocab)
        out1 = model.outputs(1)
        model.prefill([0], [p1], out1)
        n1 = min(steps, 256)
        fam1 = family_times(model, [0], toks[:, :1], out1, B1_FAMILIES)
        dt1, ms1, l1, _, _ = time_decode(model, [0], toks[:, :1], n1, args.warmup, out1)
        b1_bytes = weight_bytes_per_step(s) + (256 + (n1 - 1) / 2 + 1) * kvb
        extras["b1_decode"] = {"tokens_per_s": n1 / dt1, "ms_per_step": dt1 / n1 * 1e3, "steps": n1,
                               "hbm_roofline_tokens_per_s": HBM_PEAK_GBPS * 1e9 / b1_bytes,
                               "fraction_of_hbm_roofline": (n1 / dt1) / (HBM_PEAK_GBPS * 1e9 / b1_bytes),
                               "lmhead_avg_us": ms1 / max(l1, 1) * 1e3,
                               "roofline_by_kernel": kernel_table(s, fam1, B1_KERNELS, 1, 257 * kvb / s.n_layers)}
        # free-running greedy generation of one sequence: each step's token read back by the host and passed in again, against
        # the steps chained on the device (tr_decode_step_dev: the token output of a step is the next step's input)
        model.seq_truncate(0, 256)
        nf = min(steps, 256)
        o1 = model.decode_step([0], toks[0, :1], out1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nf):
            o1 = model.decode_step([0], o1.cpu(("token",)).token, out1)
        torch.cuda.synchronize()
        dt_host = time.perf_counter() - t0
        model.seq_truncate(0, 257)
        t0 = time.perf_counter()
        for _ in range(nf):
            model.decode_step_dev([0], out1.token, out1)
        torch.cuda.synchronize()
        dt_dev = time.perf_counter() - t0
        extras["b1_free_running"] = {"host_fed_tokens_per_s": nf / dt_host, "device_fed_tokens_per_s": nf / dt_dev,
                                     "host_fed_ms_per_step": dt_host / nf * 1e3, "device_fed_ms_per_step": dt_dev / nf * 1e3, "steps": nf}
        # the same 64 sequences on the paged cache (pages of 64 positions from a pool): what the page lookups cost
        paged = tokroute.Model(s.asdict(), model.dev, B, MAX_SEQ, kv_page=64)
        outp = paged.outputs(B)
        paged.prefill(slots, prompts, outp)
        np_steps = min(steps, 256)
        dtp, _, _, _, _ = time_decode(paged, slots, toks, np_steps, args.warmup, outp)
        extras["b64_paged_cache"] = {"tokens_per_s": B * np_steps / dtp, "ms_per_step": dtp / np_steps * 1e3, "steps": np_steps, "kv_page": 64}
        del paged, outp
        paged_done = True
        # isolated routing tail, 256 rows
        tail_model = tokroute.Model(s.asdict(), model.dev, 256, 8)
        x = torch.from_numpy(synth.hidden_rows(SEED, "cfg4.x", 256, s.d_model, True)).cuda()
        outt = tail_model.outputs(256)
        for _ in range(3):
            tail_model.tail(x, outt)
        torch.cuda.synchronize()
        reps = 20
        t0 = time.perf_counter()
        for _ in range(reps):
            tail_model.tail(x, outt)
        torch.cuda.synchronize()
        dtt = (time.perf_counter() - t0) / reps
        lm_bytes = 2 * (s.vocab + s.router_hidden) * s.d_model   # the head matrix and, in the same launch, the rows of the router's first layer
        tail_bytes = lm_bytes + 256 * s.d_model * 4 + 2 * 2 * s.router_hidden + 256 * 16   # head + router layer 1 (in lm_bytes), rows in, router biases and output unit, results out
        # at 256 rows the head is a 256 x 151936 x 896 product with exact (hi + lo bf16) activations: twice the flops of a plain bf16 product
        tail_flops = 2 * 2.0 * 256 * s.vocab * s.d_model
        extras["tail_b256"] = {"GB_per_s": tail_bytes / dtt / 1e9, "us_per_call": dtt * 1e6, "algorithmic_bytes": tail_bytes,
                               "fraction_of_hbm_roofline": tail_bytes / dtt / 1e9 / HBM_PEAK_GBPS,
                               "mfma_TFLOP_per_s": tail_flops / dtt / 1e12, "fraction_of_bf16_mfma_peak": tail_flops / dtt / 1e12 / 2500.0}
        # the roofs of the 256-row tail: bytes once at the HBM peak; the products of exact (hi + lo) activations at the bf16 matrix peak
        extras["tail_b256"]["hbm_roof_us"] = tail_bytes / (HBM_PEAK_GBPS * 1e9) * 1e6
        extras["tail_b256"]["mfma_roof_us"] = tail_flops / 2500e12 * 1e6
        del tail_model, outt, paged_done
        torch.cuda.empty_cache()
        # large model on the routed subset (7B-class shapes, 32 sequences at context 2048, flags Bernoulli(0.07))
        extras["llm7b_routed_subset"] = llm7b_workload(min(max(steps, 64), 256), args.warmup, as_dict=True)
        result["extras"] = extras

    if not args.no_cpu_baseline:
        del model
        torch.cuda.empty_cache()
        result["cpu_baseline"] = cpu_baseline(s, weights)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
