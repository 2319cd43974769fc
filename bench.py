#!/usr/bin/env python3
"""Benchmark of the TiDAR decode step on one MI355X.

A "step" is one pass of the whole hot path (row assembly .. next-draft select) over one batch of synthetic
input: 8B-shaped model (36 layers, d 4096, 32 q / 8 kv heads, head_dim 128, ffn 12288, vocab 151936),
bf16, batch 1, block length k = 16 (272 rows), prompt of 4096 random tokens already in the paged cache.

The timed steps are the workload as named: random-init weights, the step's own next drafts fed back as the
next step's drafts, greedy.  Trained weights do not exist here, so the drafts of an untrained diffusion head are
almost never accepted: `value` is the measured decode rate at that natural acceptance (about one token per
step); the hardware statement is `ms_per_step` and `tidar_over_ar_latency`, which do not depend on what is
accepted.  Reported beside it under their own keys: the same step driven with drafts that are correct up to a
seeded acceptance length whose mean is the paper's tokens-per-forward for the 8B model (Table 2: 8.25) -
verification, KV commit and draft selection run for real, the drafts come from a reference continuation - and
with fully correct drafts (upper bound, k tokens per step).

Prints ONE JSON line (see the keys below).  Also reported: the 1-token AR step on the same state, the sampled
(temperature 1) step, the roofline of the dominant kernel (the weight-streaming skinny GEMM) from HIP events
recorded by the library on the launch stream, and the CPU oracle timed on one full-depth step.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--k", type=int, default=16)
    ap.add_argument("--prefix", type=int, default=4096)
    ap.add_argument("--layers", type=int, default=36)
    ap.add_argument("--shape", default="8b-shape")
    ap.add_argument("--mean-accept", type=float, default=8.25)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel from the host instead of replaying "
                    "a captured HIP graph of the step")
    ap.add_argument("--attn-bench", action="store_true",
                    help="time the hybrid-mask attention call alone (TiDAR shape and 1-row AR shape) at --prefix/--k")
    ap.add_argument("--sweep", action="store_true",
                    help="latency table instead of the headline line: TiDAR step vs 1-token AR step for batch in "
                         "--sweep-batches and k in --sweep-ks at a synthetic cache of --prefix tokens per sequence "
                         "(one JSON line per point on stdout)")
    ap.add_argument("--sweep-batches", type=str, default="1,4,8,16,32")
    ap.add_argument("--sweep-ks", type=str, default="4,8,16")
    ap.add_argument("--sweep-tokens", type=int, default=256,
                    help="tokens every sequence of a sweep point generates (natural acceptance: one step per token)")
    ap.add_argument("--score-bench", action="store_true",
                    help="time the many-row entry points on a --prefix-token text: tidar_prefill, tidar_score with the "
                         "causal section only (AR-mode likelihood) and with the mask section (training layout, block "
                         "length --k), with the per-kernel-class split of each")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain device copy of 1 GiB ten times (known traffic: 1 GiB read + 1 GiB written "
                         "per launch) so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    ap.add_argument("--traffic-kib", type=str, default=None,
                    help="FETCH_SIZE,WRITE_SIZE per gemm launch (KiB, already scaled) measured with rocprofv3 --pmc")
    return ap.parse_args()


def cpu_baseline(shape, k, L):
    """Times the oracle as it stands on ONE TiDAR step of the benchmark's workload at full depth (after one untimed
    step that starts the thread pool and pages the weights in): the same seeded bf16 weights as the device run,
    generated on the GPU and copied to the host, fp32 accumulation with the bf16 rounding points, a synthetic cache of
    L tokens.  About ten seconds of CPU work at the 8B shape; tokens/s at the natural acceptance of that step."""
    import torch
    import tidar_inputs as TI
    from oracle import tidar_oracle as O

    w = TI.make_weights(shape, seed=4, dtype=torch.bfloat16, device="cuda:0")
    w_cpu = TI.weights_to(w, device="cpu")
    del w
    torch.cuda.empty_cache()
    model = O.OracleModel(shape, w_cpu, dtype=torch.float32, bf16_faithful=True)
    del w_cpu
    st = model.new_state(L + 3 * k)
    for l in range(shape.n_layers):
        st.k[l][:L] = TI.make_normal((L, shape.n_kv_heads, shape.head_dim), 500 + l, torch.bfloat16).float()
        st.v[l][:L] = TI.make_normal((L, shape.n_kv_heads, shape.head_dim), 600 + l, torch.bfloat16).float()
    st.L = L
    drafts = [int(t) for t in TI.make_drafts(shape, k, seed=9)[0]]
    _, _, drafts, _ = model.tidar_step(st, drafts)
    t0 = time.perf_counter()
    a, _, drafts, _ = model.tidar_step(st, drafts)
    dt = time.perf_counter() - t0
    return {"value": a / dt, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"one oracle TiDAR step of the full {shape.n_layers}-layer {shape.name} model (k={k}, prefix {L}, "
                      f"fp32 accumulation, bf16 rounding points) after one untimed step: {dt:.2f} s, {a} token(s) "
                      f"accepted (random-init weights)",
            "step_s": dt}


def gemm_source_digest():
    """Digest of the sources the GEMM launches are built from: a traffic summary measured on another build does not
    describe this one."""
    import hashlib
    h = hashlib.sha256()
    for name in ("kernels_gemm.hip", "tidar_internal.h"):
        with open(os.path.join(ROOT, "paper_2511_08923_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_traffic_summary(shape_name, k, prefix):
    """HBM bytes per GEMM launch measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy of
    known size): counters cannot be collected from inside this process, so the figure comes from the committed
    summary of those runs for this workload (lines 'traffic_bytes_per_launch: N' and 'gemm_source_digest: H').  It is
    null when there is no summary or when the summary was measured on other GEMM sources than the ones built here."""
    rel = os.path.join("profiles", f"gemm_traffic_{shape_name}_k{k}_prefix{prefix}_pmc.md")
    traffic, digest = None, None
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    traffic = float(line.split(":")[1])
                if line.startswith("gemm_source_digest:"):
                    digest = line.split(":")[1].strip()
    except OSError:
        return None, "no committed pmc summary for this workload"
    if traffic is None:
        return None, f"{rel} holds no traffic_bytes_per_launch line"
    if digest != gemm_source_digest():
        return None, f"{rel} was measured on other GEMM sources (digest {digest}, built {gemm_source_digest()}): stale"
    return traffic, rel


def attention_microbench(args, torch, T, TI, dev):
    """The hybrid-mask attention call alone at the 8B head geometry: 32 query / 8 kv heads, head_dim 128, a prefix
    of --prefix tokens in shuffled 16-token pages, k = --k (TiDAR shape, k(k+1) rows) and the 1-row AR shape.
    Sixteen distinct caches are rotated so that K/V comes from HBM, not from a cache level."""
    sh = TI.SHAPE_8B.with_layers(1)
    L, n_q, n_kv, hd = args.prefix, sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    ctx = T.tidar_create(T.make_config(sh, T.TIDAR_BF16, max_k=max(args.k, 1), max_batch=1))
    pps = (L + args.k + 15) // 16 + 1
    nbuf = 16
    g = torch.Generator(device=dev)
    g.manual_seed(42)
    kps = [torch.randn(1, pps, n_kv, 16 * hd, device=dev, generator=g).bfloat16() for _ in range(nbuf)]
    vps = [torch.randn(1, pps, n_kv, 16 * hd, device=dev, generator=g).bfloat16() for _ in range(nbuf)]
    table = torch.randperm(pps, device=dev, generator=g).int().view(1, pps)
    plen = torch.tensor([L], dtype=torch.int32, device=dev)
    ws = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    out = {}
    for name, (nc, nb, bl, cond0) in (("tidar", (args.k, args.k, args.k, 1)), ("ar", (1, 0, 1, 1))):
        R = nc + nb * bl
        q = torch.randn(1, R, n_q, hd, device=dev, generator=g).bfloat16()
        kn = torch.randn(1, R, n_kv, hd, device=dev, generator=g).bfloat16()
        vn = torch.randn(1, R, n_kv, hd, device=dev, generator=g).bfloat16()
        o = torch.empty(1, R, n_q, hd, dtype=torch.bfloat16, device=dev)

        def call(i):
            kv = T.tidar_kv_cache(kps[i % nbuf].data_ptr(), vps[i % nbuf].data_ptr(), table.data_ptr(), pps, pps)
            T.tidar_hybrid_attention(ctx, kv, 0, 1, plen, q, kn, vn, nc, nb, bl, cond0, o, L, ws)

        for i in range(args.warmup):
            call(i)
        torch.cuda.synchronize()
        T.tidar_profile_reset(ctx)
        T.tidar_profile_enable(ctx, True)
        for i in range(args.steps):
            call(i)
        torch.cuda.synchronize()
        pr = T.tidar_profile_read(ctx)
        T.tidar_profile_enable(ctx, False)
        us = {n: pr[n]["ms"] / pr[n]["launches"] * 1e3 for n in ("place_kv", "attention", "attention_combine") if n in pr}
        allowed_new = nc * (nc + 1) // 2 + nb * bl * (cond0 - 1) + nb * bl * (nb + 1) // 2 + nb * bl * bl
        flops = 4.0 * n_q * hd * (R * L + allowed_new)
        kv_bytes = 2.0 * L * n_kv * hd * 2
        t = us["attention"] + us.get("attention_combine", 0.0)
        out[name] = {"rows": R, "prefix_len": L, "kernel_us": us, "attention_plus_combine_us": t,
                     "tflops": flops / t / 1e6, "mfma_frac": flops / t / 1e6 / MFMA_BF16_PEAK_TFLOPS,
                     "kv_GBs": kv_bytes / t / 1e3, "hbm_frac": kv_bytes / t / 1e3 / HBM_PEAK_GBS}
    T.tidar_destroy(ctx)
    print(json.dumps({"attention_microbench": out, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16",
                      "data": "synthetic N(0,1) Q/K/V, 16 rotating caches, shuffled page table"}))


def score_bench(args, shape, torch, T, TI, dev):
    """Prefill, AR-mode scoring and the training-layout forward over one synthetic text of --prefix tokens: whole-call
    wall time between two synchronisations (second of two calls) and the HIP-event time per kernel class."""
    S, k = args.prefix, args.k
    w = TI.make_weights(shape, seed=4, dtype=torch.bfloat16, device=dev)
    eng = T.Engine(shape, w, dtype=T.TIDAR_BF16, max_k=k, max_batch=1, max_seq_len=S + 4 * k, device=dev,
                   free_source=True)
    del w
    text = TI.make_prompt(shape, S, seed=5).to(dev)
    out = {}
    calls = (("prefill", lambda: eng.prefill(text, k)),
             ("score_causal", lambda: eng.score(text, block_len=0)),
             ("score_training_layout", lambda: eng.score(text, block_len=k)))
    for name, call in calls:
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            res = call()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
        T.tidar_profile_reset(eng.ctx)
        T.tidar_profile_enable(eng.ctx, True)
        call()
        torch.cuda.synchronize()
        pr = T.tidar_profile_read(eng.ctx)
        T.tidar_profile_enable(eng.ctx, False)
        out[name] = {"ms": dt * 1e3, "tokens_per_s": S / dt,
                     "kernel_class_ms": {n: round(v["ms"], 2) for n, v in sorted(pr.items(), key=lambda kv: -kv[1]["ms"])}}
        if name != "prefill":
            out[name]["loss"] = float(res[2][0])
    print(json.dumps({"score_bench": out, "tokens": S, "block_len": k, "shape": shape.name, "layers": shape.n_layers,
                      "dtype": "bf16", "data": "synthetic uniform token ids, random-init weights"}))


def sweep(args, shape, torch, T, TI, dev):
    """TiDAR-step vs AR-step latency over batch and block length (the free-slot regime and its crossover): every
    point generates --sweep-tokens tokens per sequence from a context of --prefix tokens, the step's own drafts fed
    back (random-init weights accept about one token per step, so that is one step per token; the prefix grows as
    it would in a decode loop), and the 1-token AR step generates as many.  The cache is filled synthetically
    (N(0,1) K/V, as in the attention micro-benchmark): step latency does not depend on token values, and a real
    prefill of batch x prefix tokens would only lengthen the set-up."""
    batches = [int(x) for x in args.sweep_batches.split(",")]
    ks = [int(x) for x in args.sweep_ks.split(",")]
    P, n_tok = args.prefix, args.sweep_tokens
    bmax, kmax = max(batches), max(ks)
    w = TI.make_weights(shape, seed=4, dtype=torch.bfloat16, device=dev)
    max_seq = P + n_tok * kmax + 4 * kmax                   # every step could accept k tokens
    eng = T.Engine(shape, w, dtype=T.TIDAR_BF16, max_k=kmax, max_batch=bmax, max_seq_len=max_seq, device=dev,
                   free_source=True)
    del w
    torch.cuda.empty_cache()
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    for l in range(shape.n_layers):                       # page by page would be the same bytes: fill whole layers
        eng.k_pages[l].normal_(0.0, 1.0, generator=g)
        eng.v_pages[l].normal_(0.0, 1.0, generator=g)
    mode = T.make_mode()
    wbytes = eng.weight_bytes_per_step()
    kv_per_tok = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2

    def graphed(body):
        if args.no_graph:
            return body
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            body()
        torch.cuda.current_stream().wait_stream(side)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            body()
        return gr.replay

    def generate(fn, B, reset):
        """n_tok steps from the reset state (a step accepts at least one token per sequence); ms per step and the
        tokens the sequences really advanced by."""
        reset()
        for _ in range(min(args.warmup, 5)):
            fn()
        reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_tok):
            fn()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        return dt / n_tok * 1e3, int((eng.prefix_len[:B] - P).sum()), dt

    for B in batches:
        tok0 = TI.make_drafts(shape, 1, seed=11, batch=B).to(dev).view(B).contiguous()
        tok_buf = tok0.clone()
        tok_out = torch.empty(B, dtype=torch.int32, device=dev)

        def ar_body():
            eng.ar_step(tok_buf, hint=P + n_tok, mode=mode, out=tok_out)
            tok_buf.copy_(tok_out)

        def ar_reset():
            eng.prefix_len[:B].fill_(P)
            tok_buf.copy_(tok0)

        ar_ms, ar_tokens, ar_dt = generate(graphed(ar_body), B, ar_reset)
        for k in ks:
            R = k * (k + 1)
            d0 = TI.make_drafts(shape, k, seed=12, batch=B).to(dev)
            drafts = d0.clone()
            out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, k, dtype=torch.int32, device=dev),
                   torch.empty(B, k, dtype=torch.int32, device=dev))

            # bound on the prefix length for the whole run (the library cuts its attention splits from it): random-init
            # weights accept about one token per step; the bound is checked after the run
            bound = P + 2 * n_tok + k

            def td_body():
                eng.step(drafts, k, hint=bound, mode=mode, out=out)
                drafts.copy_(out[2])

            def td_reset():
                eng.prefix_len[:B].fill_(P)
                drafts.copy_(d0)

            td_ms, td_tokens, td_dt = generate(graphed(td_body), B, td_reset)
            if int(eng.prefix_len[:B].max()) > bound:
                raise RuntimeError("a sequence outgrew the length bound given to tidar_step")
            L_mid = P + n_tok // 2
            flops = 2.0 * B * R * (wbytes / 2) + 4.0 * shape.n_layers * shape.n_q_heads * B * R * L_mid * shape.head_dim
            row = {"sweep": True, "batch": B, "k": k, "rows": B * R, "prefix_len": P, "steps": n_tok,
                   "tokens_generated_per_sequence": td_tokens / B, "tidar_step_ms": td_ms,
                   "ar_step_ms": ar_ms, "tidar_over_ar_latency": td_ms / ar_ms,
                   "tidar_tokens_per_s_natural": td_tokens / td_dt, "ar_tokens_per_s": ar_tokens / ar_dt,
                   "tidar_step_hbm_GBs": (wbytes + B * kv_per_tok * L_mid) / (td_ms * 1e-3) / 1e9,
                   "ar_step_hbm_GBs": (wbytes + B * kv_per_tok * L_mid) / (ar_ms * 1e-3) / 1e9,
                   "ar_step_hbm_frac": (wbytes + B * kv_per_tok * L_mid) / (ar_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "tidar_step_tflops": flops / (td_ms * 1e-3) / 1e12,
                   "tidar_step_mfma_frac": flops / (td_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                   "layers": shape.n_layers, "shape": shape.name}
            print(json.dumps(row), flush=True)
    eng.close()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2511_08923_amd as T
    import tidar_inputs as TI

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.zeros(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 10}}))
        return
    shape = TI.SHAPES[args.shape]
    if args.layers != shape.n_layers:
        shape = shape.with_layers(args.layers)
    if args.attn_bench:
        return attention_microbench(args, torch, T, TI, dev)
    if args.sweep:
        return sweep(args, shape, torch, T, TI, dev)
    if args.score_bench:
        return score_bench(args, shape, torch, T, TI, dev)
    k, P, V = args.k, args.prefix, shape.vocab
    R = k * (k + 1)
    n_timed = args.steps + args.warmup

    # ---- acceptance lengths forced on the timed steps (host-known, so the token bound below is exact)
    acc_len = TI.make_acceptance_lengths(k, n_timed, args.mean_accept, seed=6)
    # the seeded draws average close to the requested mean; nudge single steps by one until the timed window
    # carries exactly round(mean * steps) tokens, so that the token count does not depend on --steps
    want_total = int(round(args.mean_accept * args.steps))
    i = 0
    while int(acc_len[args.warmup:].sum()) != want_total and i < 64 * n_timed:
        j = args.warmup + i % args.steps
        d = 1 if int(acc_len[args.warmup:].sum()) < want_total else -1
        if 1 <= int(acc_len[j]) + d <= k:
            acc_len[j] += d
        i += 1
    n_full = min(args.steps, 20)                       # steps of the full-acceptance phase
    ref_tokens = max(int(acc_len.sum()), (n_full + 4) * k) + 2 * k   # reference continuation every phase fits in
    # One bound on the prefix length for every call of this run: the library derives the key partition of its
    # attention splits from this bound, so the reference pass and the replays group every row's keys alike and
    # a row's logits come out bit-identical whenever its context is the same.
    hint_all = P + ref_tokens + k
    max_seq = P + 2 * ref_tokens + 4 * k

    w = TI.make_weights(shape, seed=4, dtype=torch.bfloat16, device=dev)
    eng = T.Engine(shape, w, dtype=T.TIDAR_BF16, max_k=k, max_batch=1, max_seq_len=max_seq, device=dev,
                   free_source=True)
    del w
    torch.cuda.empty_cache()
    prompt = TI.make_prompt(shape, P, seed=5).to(dev)
    mode = T.make_mode()

    # ---- untimed set-up: prefill, then the reference continuation by natural TiDAR steps (also a warm-up)
    drafts, _ = eng.prefill(prompt, k, mode)
    first_drafts = drafts.clone()
    out = (torch.empty(1, dtype=torch.int32, device=dev), torch.empty(1, k, dtype=torch.int32, device=dev),
           torch.empty(1, k, dtype=torch.int32, device=dev))
    stream = torch.zeros(ref_tokens + 2 * k, dtype=torch.int32, device=dev)
    n_ref, nat_steps = 0, 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while n_ref < ref_tokens:
        a, acc, nxt, _ = eng.step(drafts, k, hint=hint_all, mode=mode, out=out)
        na = int(a[0])                                  # host read: this loop is set-up, not the timed region
        stream[n_ref:n_ref + na] = acc[0, :na]
        n_ref += na
        nat_steps += 1
        drafts = nxt.clone()
    torch.cuda.synchronize()
    natural_tok_s = n_ref / (time.perf_counter() - t0)
    stream[n_ref:n_ref + k] = nxt[0]                    # slot 0 is final, the rest only pads the gather below

    # ---- forced-acceptance drafts built on the device from the reference continuation
    acc_len = acc_len.to(dev)
    ar = torch.arange(k, device=dev, dtype=torch.int64)

    # Device-side step state, so that one step (draft synthesis + tidar_step) is a fixed launch sequence that
    # can be captured once into a HIP graph and replayed: the step counter, the running token count and the
    # drafts buffer live in HBM; nothing crosses to the host inside the timed region.
    step_no = torch.zeros(1, dtype=torch.int64, device=dev)
    tok_count = torch.zeros(1, dtype=torch.int64, device=dev)
    drafts_buf = torch.zeros(1, k, dtype=torch.int32, device=dev)
    one = torch.ones(1, dtype=torch.int64, device=dev)

    def one_step(full):
        if full == "natural":                               # the step's own next drafts, as a decode loop feeds them
            drafts_buf.copy_(out[2])
            eng.step(drafts_buf, k, hint=hint_all, mode=step_mode[0], out=out)
            return
        base = eng.prefix_len[:1].long() - P
        tok = stream[base + ar]
        if full:
            drafts_buf.copy_(tok.view(1, k))
        else:
            wrong = (tok + 1) % (V - 1)
            want = acc_len[step_no].long()                  # acceptance length forced for this step
            drafts_buf.copy_(torch.where(ar < want, tok, wrong).to(torch.int32).view(1, k))
        eng.step(drafts_buf, k, hint=hint_all, mode=mode, out=out)
        tok_count.add_(out[0].long())
        step_no.add_(one)

    graphs = {}

    def stepper(full):
        """Returns a callable that runs one step: a graph replay unless --no-graph."""
        if args.no_graph:
            return lambda: one_step(full)
        if full not in graphs:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):                   # warm up on the side stream before capture
                one_step(full)
            torch.cuda.current_stream().wait_stream(side)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                one_step(full)
            graphs[full] = g
        return graphs[full].replay

    def reset(first_idx=0):
        eng.prefix_len.fill_(P)
        step_no.fill_(first_idx)
        tok_count.zero_()

    def run_steps(n, first_idx, full=False, count=None):
        fn = stepper(full)
        reset_needed = int(step_no[0]) != first_idx
        if reset_needed:
            step_no.fill_(first_idx)
        for i in range(n):
            fn()
            if count is not None:
                count[i] = out[0][0]

    # ---- timed: the workload as named (random-init weights, the step's own drafts fed back, greedy)
    step_mode = [mode]
    stepper(False)
    stepper(True)
    stepper("natural")

    def natural_run(n_warm, n):
        reset()
        out[2].copy_(first_drafts)
        run_steps(n_warm, 0, full="natural")
        c = torch.zeros(n, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run_steps(n, n_warm, full="natural", count=c)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, int(c.sum())

    t_tidar, tokens = natural_run(args.warmup, args.steps)
    step_ms = t_tidar / args.steps * 1e3

    # ---- the same step at the paper's acceptance mix: drafts from the reference continuation, correct up to a
    # seeded length (a projection of what trained weights would accept, with real verification)
    reset()
    run_steps(args.warmup, 0)
    counts = torch.zeros(args.steps, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(args.steps, args.warmup, count=counts)
    torch.cuda.synchronize()
    t_forced = time.perf_counter() - t0
    tokens_forced = int(counts.sum())
    forced_ok = bool((counts == acc_len[args.warmup:args.warmup + args.steps]).all())

    # ---- the sampled step (temperature 1, seeded): the Gumbel noise is added in the LM head's epilogue
    if not args.no_graph:
        graphs.pop("natural")
    step_mode[0] = T.make_mode(sample=True, temperature=1.0, seed=2024)
    t_sampled, _ = natural_run(min(args.warmup, 3), min(args.steps, 20))
    sampled_step_ms = t_sampled / min(args.steps, 20) * 1e3
    step_mode[0] = mode
    if not args.no_graph:
        graphs.pop("natural")

    # ---- per-step latency spread: the same steps once more, an event pair around each replay (kept out of the
    # timed region above so that the headline number has no events inside it)
    reset()
    run_steps(args.warmup, 0)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    fn = stepper(False)
    for e0, e1 in evs:
        e0.record()
        fn()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    step_pcts = {"p10": pct(0.10), "p50": pct(0.50), "p90": pct(0.90)}

    # ---- full acceptance (drafts = the true continuation): upper bound k tokens per step
    reset()
    run_steps(min(args.warmup, 3), 0, full=True)
    cfull = torch.zeros(n_full, dtype=torch.int32, device=dev)
    reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(n_full, 0, full=True, count=cfull)
    torch.cuda.synchronize()
    full_tok_s = int(cfull.sum()) / (time.perf_counter() - t0)

    # ---- the 1-token AR step on the same state
    reset()
    tok_out = torch.empty(1, dtype=torch.int32, device=dev)

    tin_buf = torch.zeros(1, dtype=torch.int32, device=dev)

    tin_buf.copy_(stream[:1])

    def one_ar():
        # ordinary one-token decoding: each step's token is the next step's input (one copy, no host work)
        eng.ar_step(tin_buf, hint=hint_all, mode=mode, out=tok_out)
        tin_buf.copy_(tok_out)

    if args.no_graph:
        ar_fn = one_ar
    else:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            one_ar()
        torch.cuda.current_stream().wait_stream(side)
        ar_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(ar_graph):
            one_ar()
        ar_fn = ar_graph.replay
        reset()

    def run_ar(n):
        for i in range(n):
            ar_fn()

    run_ar(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_ar(args.steps)
    torch.cuda.synchronize()
    ar_ms = (time.perf_counter() - t0) / args.steps * 1e3

    # ---- per-kernel HIP-event timing on the launch stream (separate from the timed region above)
    def profile(fn, n):
        T.tidar_profile_reset(eng.ctx)
        T.tidar_profile_enable(eng.ctx, True)
        fn(n)
        torch.cuda.synchronize()
        prof = T.tidar_profile_read(eng.ctx)
        T.tidar_profile_enable(eng.ctx, False)
        return prof

    reset()
    n_prof = min(10, args.steps)

    def eager_steps(n):
        for _ in range(n):
            one_step(False)

    def eager_ar(n):
        for _ in range(n):
            one_ar()

    prof_tidar = profile(eager_steps, n_prof)
    reset()
    prof_ar = profile(eager_ar, n_prof)

    wbytes = eng.weight_bytes_per_step()
    gemm = prof_tidar["gemm"]
    gemm_ms_per_step = gemm["ms"] / n_prof
    gemm_launch_ms = gemm["ms"] / gemm["launches"]
    launches_per_step = gemm["launches"] // n_prof
    bytes_per_launch = wbytes / launches_per_step
    achieved = bytes_per_launch / (gemm_launch_ms * 1e-3) / 1e9
    gemm_flops = 2.0 * R * (wbytes / 2)
    traffic, traffic_source = None, None
    if args.traffic_kib:
        f, wr = [float(x) for x in args.traffic_kib.split(",")]
        traffic, traffic_source = (f + wr) * 1024.0, "--traffic-kib"
    else:
        traffic, traffic_source = read_traffic_summary(shape.name, k, P)
    roofline = {"bound": "hbm", "kernel": "gemm_bf16_kernel (all projections + LM head)", "achieved": achieved,
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                "traffic_source": traffic_source,
                "bytes_per_launch": bytes_per_launch, "avg_launch_ms": gemm_launch_ms,
                "launches_per_step": launches_per_step,
                "mfma_tflops": gemm_flops / (gemm_ms_per_step * 1e-3) / 1e12,
                "mfma_frac": gemm_flops / (gemm_ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS}
    ar_gemm = prof_ar["gemm"]
    kv_bytes = 2 * shape.n_layers * shape.n_kv_heads * shape.head_dim * 2 * P
    res = {
        "metric": "tidar_decode_tokens_per_sec", "value": tokens / t_tidar, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": step_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "launch": "host launches" if args.no_graph else "HIP graph replay of the captured step",
        "config": {"workload": f"{shape.name} TiDAR decode, batch 1, k={k} ({R} rows/step), prompt {P} random tokens, "
                               f"random-init weights, greedy, the step's own drafts fed back (natural acceptance)",
                   "k": k, "prefix_len": P, "batch": 1, "layers": shape.n_layers},
        "value_note": "tokens/s at the natural acceptance of random-init weights (about one token per step: an "
                      "untrained diffusion head drafts nothing the causal logits accept); the step latency does not "
                      "depend on acceptance, see paper_acceptance_projection for the same step at the paper's mix",
        "tidar_step_ms": step_ms, "tidar_step_ms_percentiles": step_pcts, "ar_step_ms": ar_ms,
        "tidar_over_ar_latency": step_ms / ar_ms, "tidar_over_ar_latency_target": 1.3,
        "ar_tokens_per_s": 1e3 / ar_ms, "tokens_per_step": tokens / args.steps,
        "sampled_step_ms": sampled_step_ms, "sampled_over_greedy_step": sampled_step_ms / step_ms,
        "paper_acceptance_projection": {
            "what": f"the same step fed drafts from a reference continuation that are correct up to a seeded length "
                    f"(mean {args.mean_accept} = the paper's Table 2 tokens per forward, trained 8B model); verification, "
                    f"commit and draft selection run for real",
            "tokens_per_s": tokens_forced / t_forced, "tokens_per_step": tokens_forced / args.steps,
            "ms_per_step": t_forced / args.steps * 1e3, "forced_acceptance_reproduced": forced_ok,
            "speedup_vs_ar_tokens_per_s": (tokens_forced / t_forced) / (1e3 / ar_ms)},
        "full_acceptance_tokens_per_s": full_tok_s,
        "step_hbm_GBs": (wbytes + kv_bytes) / (step_ms * 1e-3) / 1e9,
        "ar_step_hbm_GBs": (wbytes + kv_bytes) / (ar_ms * 1e-3) / 1e9,
        "ar_step_hbm_frac": (wbytes + kv_bytes) / (ar_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "ar_step_hbm_frac_target": 0.70,
        "roofline": roofline,
        "ar_gemm_GBs": wbytes / (ar_gemm["ms"] / n_prof * 1e-3) / 1e9,
        "kernel_ms_per_tidar_step": {n: v["ms"] / n_prof for n, v in prof_tidar.items()},
        "kernel_ms_per_ar_step": {n: v["ms"] / n_prof for n, v in prof_ar.items()},
        "parity_note": "logit tolerance: 2e-2 absolute holds on the small test models; at the full 28/36-layer depth "
                       "with N(0, 0.02) weights no bf16 implementation can hold it (the oracle with fp32 accumulation is "
                       "0.15 max / 0.024 rms away from the same oracle with fp64 accumulation at the 8B shape): the "
                       "full-depth tests allow 1.5x that measured floor and compare tokens under a near-tie rule",
        "paper_context": "paper reports 5.91x tokens/s over AR for its 8B model on one H100 (Figure 4); other "
                         "hardware, trained weights: context only",
    }
    eng.close()
    del eng
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(shape, k, P)
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


if __name__ == "__main__":
    main()
