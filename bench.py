"""Benchmark: speculative rounds per second on one MI355X, 7B-shaped layer + LM head (bf16).

A step is one full round through the C ABI: drafter pass over 1 pending + K=32 [MASK] rows against a
2048-token KV cache -> LM head -> token lattice (top-8) -> path search (beam 4) -> verifier pass over 33
causal rows + LM head + greedy acceptance -> host read-back of the accepted length -> draft-length update.
Inputs (weights, KV caches, proxy table) are resident in HBM before the timed region.

Prints ONE JSON line (the fields are described in the README).
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

HBM_PEAK_GBS = 8000.0
PREFIX, K_DRAFT, M_MAX, BEAM, LAM = 2048, 32, 8, 4, 0.5


def algorithmic_bytes(cfg, rows_prefix):
    """Bytes the method must move per stage (weights once + KV once); activations and logits excluded."""
    from paper_2510_02358_amd import synth
    layer = synth.layer_param_count(cfg) * 2
    head = cfg.vocab * cfg.d_model * 2
    kv = (rows_prefix + K_DRAFT + 1) * 2 * cfg.n_kv * cfg.head_dim * 2
    return {"draft": layer + kv, "lm_head": head, "verify": layer + kv + head,
            "round": 2 * (layer + kv) + 2 * head}


def traffic_from_profiles():
    """HBM bytes per LM-head launch measured with rocprofv3 --pmc (committed summary), or None."""
    path = os.path.join(ROOT, "profiles", "lm_head_gemm_cfg1_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def run_stress(args) -> int:
    """cfg3: the lattice and the path search on their own (no model): float32 logits [16, K, 152064] drawn as g / T
    (g ~ N(0, 1), one T ~ U[0.5, 2] per row), K in {8, 16, 32, 64}, top-16 lattice, beam 8.  Reports the lattice's
    achieved GB/s against 4 bytes per logit and the path search's time."""
    import numpy as np
    import torch

    from paper_2510_02358_amd import binding as ds
    from paper_2510_02358_amd import synth
    from paper_2510_02358_amd import round as rnd

    vocab, batch, m_max, beam, lam = 152064, 16, 16, 8, 0.5
    eos_id = vocab - 2
    table = rnd.upload(synth.make_ngram_table(3))
    proxy = ds.ds_ngram_create(table, synth.NGRAM_LOG2_SIZE)
    res = {}
    for k in (8, 16, 32, 64):
        rows = batch * k
        gen = torch.Generator(device="cuda")
        gen.manual_seed(100 + k)
        logits = torch.randn(rows, vocab, generator=gen, device="cuda", dtype=torch.float32)
        logits /= torch.empty(rows, 1, device="cuda").uniform_(0.5, 2.0, generator=gen)
        i32, f32 = torch.int32, torch.float32
        cand_id = torch.empty(rows, m_max, dtype=i32, device="cuda")
        cand_logp = torch.empty(rows, m_max, dtype=f32, device="cuda")
        cand_cnt = torch.empty(rows, dtype=i32, device="cuda")
        eos_logp = torch.empty(rows, dtype=f32, device="cuda")
        lse = torch.empty(rows, dtype=f32, device="cuda")
        lat_ws = torch.empty(ds.ds_lattice_workspace_bytes(rows, vocab, m_max), dtype=torch.uint8, device="cuda")
        cps_ws = torch.empty(ds.ds_cps_workspace_bytes(batch, k, m_max), dtype=torch.uint8, device="cuda")
        ctx = rnd.upload(synth.make_contexts(vocab, batch, 7))
        path = torch.empty(batch, k, dtype=i32, device="cuda")
        plen = torch.empty(batch, dtype=i32, device="cuda")
        score = torch.empty(batch, dtype=f32, device="cuda")
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        lat_us, cps_us = [], []
        for rep in range(12):
            ev[0].record()
            ds.ds_build_lattice(logits, rows, vocab, m_max, 0.8, eos_id, cand_id, cand_logp, cand_cnt, eos_logp, lse,
                                lat_ws)
            ev[1].record()
            ds.ds_cps_path(cand_id, cand_logp, cand_cnt, eos_logp, batch, k, m_max, beam, lam, proxy, ctx, eos_id, path,
                           plen, score, cps_ws)
            ev[2].record()
            torch.cuda.synchronize()
            if rep >= 2:
                lat_us.append(ev[0].elapsed_time(ev[1]) * 1e3)
                cps_us.append(ev[1].elapsed_time(ev[2]) * 1e3)
        lat = float(np.median(lat_us))
        res[f"K={k}"] = {"rows": rows, "lattice_us": round(lat, 1),
                         "lattice_GBps": round(rows * vocab * 4 / (lat * 1e-6) / 1e9, 1),
                         "lattice_hbm_frac": round(rows * vocab * 4 / (lat * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                         "cps_us": round(float(np.median(cps_us)), 1)}
        del logits
    ds.ds_ngram_destroy(proxy)
    k64 = res["K=64"]
    out = {"metric": "lattice_GBps", "value": k64["lattice_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": 10, "warmup": 2,
           "ms_per_step": round(k64["lattice_us"] / 1e3, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "cfg3: float32 logits [16, K, 152064], K in {8, 16, 32, 64}, top-16 lattice with mass "
                                  "pruning 0.8, beam 8, hashed 3-gram proxy"},
           "roofline": {"bound": "hbm", "kernel": "scan_rows_kernel<softmax> + lattice_merge_kernel (K = 64)",
                        "achieved": k64["lattice_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": k64["lattice_hbm_frac"], "traffic": None},
           "sizes": res, "cpu_baseline": None}
    print(json.dumps(out))
    return 0


def run_deep(args) -> int:
    """Full-depth pairs (extra evidence beside the default workload; weights are drawn on the device, no CPU leg).

    cfg2: 28-layer drafter + 28-layer verifier (7B-shaped), prefix 1024, 64 rounds, draft length adapted in
          [4, 64] from k_1 = 16.
    cfg4: 28-layer 7B-shaped drafter + 64-layer 32B-shaped verifier, prefix 16384, K = 64 fixed, 16 rounds.
    Two variants each: natural (independent random models accept nothing) and synthetic acceptance injected
    from the verifier's greedy stream.
    """
    import numpy as np
    import torch

    from paper_2510_02358_amd import round as rnd
    from paper_2510_02358_amd import synth

    d_cfg = synth.with_layers(synth.CFG_7B_LAYER, 28)
    if args.workload == "cfg2":
        v_cfg, n_rounds, prefix_len, k1, k_min, k_max = d_cfg, 64, 1024, 16, 4, 64
        name = ("cfg2: 28-layer 7B-shaped drafter + 28-layer verifier, prefix 1024, ADL k in [4, 64] from 16, "
                "64 rounds, top-8 lattice, beam 4, batch 1")
    else:
        v_cfg, n_rounds, prefix_len, k1, k_min, k_max = synth.with_layers(synth.CFG_32B_LAYER, 64), 16, 16384, 64, 64, 64
        name = ("cfg4: 28-layer 7B-shaped drafter + 64-layer 32B-shaped verifier (d=5120, 40q/8kv x128, FFN 27648), "
                "prefix 16384, K=64, 16 rounds, top-8 lattice, beam 4, batch 1")
    t0 = time.time()
    prefix = synth.make_prefix(d_cfg, prefix_len, 2)
    table = synth.make_ngram_table(3)
    cap = prefix_len + 1024
    dm = rnd.DeviceModel(d_cfg, rnd.device_weights(d_cfg, 0), cap)
    vm = rnd.DeviceModel(v_cfg, rnd.device_weights(v_cfg, 1), cap)
    params = rnd.RoundParams(m_max=M_MAX, beam=BEAM, lam=LAM, k_min=k_min, k_max=k_max, delta=10.0, rho=0.5)

    def model_bytes(c):
        return c.n_layers * synth.layer_param_count(c) * 2 + c.vocab * c.d_model * 2

    def kv_bytes(c, n):
        return c.n_layers * 2 * c.n_kv * c.head_dim * 2 * n

    round_bytes = model_bytes(d_cfg) + model_bytes(v_cfg) + kv_bytes(d_cfg, prefix_len) + kv_bytes(v_cfg, prefix_len)
    res = {"algorithmic_bytes_per_round": round_bytes}
    for variant in ("natural", "synthetic_acceptance"):
        dec = rnd.SpecDecoder(dm, vm, table, synth.NGRAM_LOG2_SIZE, params, k_cap=64)
        stream = stream_dev = None
        if variant == "synthetic_acceptance":
            ar_t = {}
            stream = rnd.ar_greedy(vm, prefix, n_rounds * 9 + 72, timing=ar_t)
            stream_dev = rnd.upload(np.asarray(stream, dtype=np.int32))
            res["ar_greedy_tokens_per_s"] = round(ar_t["steps"] / (ar_t["decode_ms"] * 1e-3), 1)
            res["ar_greedy_hbm_frac"] = round((model_bytes(v_cfg) + kv_bytes(v_cfg, prefix_len)) /
                                              (ar_t["decode_ms"] * 1e-3 / ar_t["steps"]) / 1e9 / HBM_PEAK_GBS, 4)
        dec.start(prefix)
        rng = np.random.default_rng(5)
        k, ks, n_tok, n_acc_sum = k1, [], 0, 0
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(n_rounds):
            inject = None
            if stream is not None:
                done = len(dec.tokens) - len(prefix)
                a = int(min(k, rng.geometric(1.0 / 7.0) - 1))
                inject = (stream_dev[done:done + a], a)
            got = dec.round(k, inject=inject)
            ks.append(k)
            n_tok += got["n_accept"] + 1
            n_acc_sum += got["n_accept"]
            k = got["k_next"]
        torch.cuda.synchronize()
        el = time.perf_counter() - c0
        res[variant] = {"rounds_per_s": round(n_rounds / el, 2), "ms_per_round": round(el * 1e3 / n_rounds, 3),
                        "tokens_per_s": round(n_tok / el, 1), "mean_accepted": round(n_acc_sum / n_rounds, 2),
                        "mean_k": round(float(np.mean(ks)), 1), "k_last": ks[-1],
                        "round_hbm_frac": round(round_bytes / (el / n_rounds) / 1e9 / HBM_PEAK_GBS, 4)}
        if stream is not None:
            res[variant]["committed_stream_equals_ar_greedy"] = bool(
                dec.tokens[len(prefix):] == stream[:len(dec.tokens) - len(prefix)])
            res[variant]["speedup_vs_ar_greedy"] = round(res[variant]["tokens_per_s"] / res["ar_greedy_tokens_per_s"], 3)
        dec.close()
    nat = res["natural"]
    out = {"metric": "spec_rounds_per_s", "value": nat["rounds_per_s"], "unit": "rounds/s", "n_gpus": 1,
           "steps": n_rounds, "warmup": 0, "ms_per_step": nat["ms_per_round"], "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic (weights drawn on the device)",
           "config": {"workload": name}, "variants": res, "setup_s": round(time.time() - t0, 1), "roofline": None,
           "cpu_baseline": None}
    print(json.dumps(out))
    dm.close()
    vm.close()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", choices=["cfg1", "cfg2", "cfg3", "cfg4"], default="cfg1",
                    help="cfg1 (default): the benchmark workload.  cfg2: full 28-layer 7B-shaped drafter + verifier, "
                         "prefix 1024, draft length adapted in [4, 64] over 64 rounds.  cfg4: that drafter + 64-layer "
                         "32B-shaped verifier, prefix 16384, K=64 (both: extra evidence, no CPU leg)")
    ap.add_argument("--core-only", action="store_true",
                    help="only the timed rounds and the per-stage pass (skips the synthetic-acceptance loop, the "
                         "round variants and the CPU baseline): keeps profiler runs short")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for rocprofv3 --pmc byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2510_02358_amd import binding as ds
    from paper_2510_02358_amd import round as rnd
    from paper_2510_02358_amd import synth

    ds.load()  # raises if the HIP library is missing: there is no fallback
    torch.cuda.set_device(0)
    if args.workload == "cfg3":
        return run_stress(args)
    if args.workload != "cfg1":
        return run_deep(args)
    cfg = synth.CFG_7B_LAYER
    t0 = time.time()
    dw, vw = synth.make_weights(cfg, 0), synth.make_weights(cfg, 1)
    prefix = synth.make_prefix(cfg, PREFIX, 2)
    table = synth.make_ngram_table(3)
    cap = PREFIX + 1024
    dm, vm = rnd.DeviceModel(cfg, dw, cap), rnd.DeviceModel(cfg, vw, cap)
    dec = rnd.SpecDecoder(dm, vm, table, synth.NGRAM_LOG2_SIZE,
                          rnd.RoundParams(m_max=M_MAX, beam=BEAM, lam=LAM), k_cap=K_DRAFT)
    dec.start(prefix)
    dec.stage_inputs()
    torch.cuda.synchronize()
    if args.calibrate:  # known traffic: reads 1 GiB, writes 1 GiB
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    setup_s = time.time() - t0
    p0 = PREFIX

    # the LM-head GEMM is bracketed by two events on every EV_EVERY-th timed round (an event pair costs the round
    # about 5 us of stream time, so timing every round would tax the quantity being measured)
    EV_EVERY = 4
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    ev_used = [i for i in range(args.steps) if i % EV_EVERY == 0]
    acc_tokens = 0
    k_next = K_DRAFT

    def one_round(i_timed):
        nonlocal acc_tokens, k_next
        dm.set_kv_len(p0)
        vm.set_kv_len(p0)
        p = dec.p
        dec.arm_verdict()
        ds.ds_draft_block(dm.handle, dec.pending_dev, 1, K_DRAFT, dec.mask_id, dec.hidden, dm.ws)
        timed_lm = i_timed >= 0 and i_timed % EV_EVERY == 0
        if timed_lm:
            ev[i_timed][0].record()
        ds.ds_lm_head_tiles(dm.handle, None, K_DRAFT, dec.eos_id, None, dm.ws)     # the logits stay on chip
        if timed_lm:
            ev[i_timed][1].record()
        ds.ds_lattice_from_tiles(dm.handle, K_DRAFT, p.m_max, p.tau, dec.eos_id, dec.cand_id, dec.cand_logp,
                                 dec.cand_cnt, dec.eos_logp, dec.lse, dm.ws)
        ds.ds_cps_path(dec.cand_id, dec.cand_logp, dec.cand_cnt, dec.eos_logp, 1, K_DRAFT, p.m_max, p.beam, p.lam,
                       dec.proxy, dec.ctx, dec.eos_id, dec.block[1:], dec.path_len, dec.path_score, dec.cps_ws)
        ds.ds_verify_block(vm.handle, dec.block, K_DRAFT, dec.path_len, dec.eos_id, dec.result[0:1],
                           dec.result[1:2], dec.argmax, dec.result[2:3], None, vm.ws)
        dec.wait_verdict()                             # the round's one host crossing: poll the pinned verdict
        n_acc = int(dec.result_np[0])                  # written by the acceptance kernel into pinned host memory
        k_next = ds.ds_adl_update(dec.adl, K_DRAFT, 0, n_acc)
        if i_timed >= 0:
            acc_tokens += n_acc + 1

    for _ in range(args.warmup):
        one_round(-1)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        one_round(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t1
    ms_per_step = elapsed * 1e3 / args.steps
    rounds_per_s = args.steps / elapsed

    lm_ms = sum(ev[i][0].elapsed_time(ev[i][1]) for i in ev_used) / len(ev_used)
    ab = algorithmic_bytes(cfg, PREFIX)
    achieved = ab["lm_head"] / (lm_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "gemm_bf16_kernel (LM head 152064x3584, 32 rows)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic_from_profiles(),
                "avg_launch_us": round(lm_ms * 1e3, 2), "algorithmic_bytes": ab["lm_head"]}

    # per-stage times (separate untimed pass, events between the calls)
    stages = {}
    names = ["draft", "lm_head", "lattice", "cps", "verify"]
    n_rep = 20
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(n_rep)]
    for r in range(n_rep):
        dm.set_kv_len(p0)
        vm.set_kv_len(p0)
        p = dec.p
        marks[r][0].record()
        ds.ds_draft_block(dm.handle, dec.pending_dev, 1, K_DRAFT, dec.mask_id, dec.hidden, dm.ws)
        marks[r][1].record()
        ds.ds_lm_head_tiles(dm.handle, None, K_DRAFT, dec.eos_id, None, dm.ws)
        marks[r][2].record()
        ds.ds_lattice_from_tiles(dm.handle, K_DRAFT, p.m_max, p.tau, dec.eos_id, dec.cand_id, dec.cand_logp,
                                 dec.cand_cnt, dec.eos_logp, dec.lse, dm.ws)
        marks[r][3].record()
        ds.ds_cps_path(dec.cand_id, dec.cand_logp, dec.cand_cnt, dec.eos_logp, 1, K_DRAFT, p.m_max, p.beam, p.lam,
                       dec.proxy, dec.ctx, dec.eos_id, dec.block[1:], dec.path_len, dec.path_score, dec.cps_ws)
        marks[r][4].record()
        ds.ds_verify_block(vm.handle, dec.block, K_DRAFT, dec.path_len, dec.eos_id, dec.result[0:1],
                           dec.result[1:2], dec.argmax, dec.result[2:3], None, vm.ws)
        marks[r][5].record()
        torch.cuda.synchronize()
    for i, nm in enumerate(names):
        us = float(np.median([marks[r][i].elapsed_time(marks[r][i + 1]) for r in range(n_rep)])) * 1e3
        st = {"us": round(us, 1)}
        if nm in ab:
            st["hbm_frac"] = round(ab[nm] / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)
        stages[nm] = st

    out = {
        "metric": "spec_rounds_per_s", "value": round(rounds_per_s, 2), "unit": "rounds/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg1: 7B-shaped decoder layer + LM head (d=3584, 28q/4kv x128, FFN 18944, "
                               "vocab 152064), drafter + verifier, prefix 2048, K=32, top-8 lattice, beam 4, "
                               "33 verify rows, batch 1"},
        "accepted_tokens_per_s": round(acc_tokens / elapsed, 2),
        "round_hbm_frac": round(ab["round"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "roofline": roofline, "stages": stages, "setup_s": round(setup_s, 1),
    }

    if args.core_only:
        print(json.dumps(out))
        dec.close(); dm.close(); vm.close()
        return 0

    # Synthetic acceptance (labelled as such): independent random-init models accept nothing, so to exercise
    # the loop at the paper's acceptance level (mean accepted tokens about 6-7 per round, Table 1) the first
    # a_t searched tokens are overwritten with the verifier's own greedy continuation, a_t ~ geometric, mean 6.
    # The plain one-token-per-step greedy decode of the verifier on this GPU is the speed-up's denominator.
    n_rounds_inj = 64
    ar_t = {}
    stream = rnd.ar_greedy(vm, prefix, n_rounds_inj * 8 + K_DRAFT + 8, timing=ar_t)
    ar_tok_s = ar_t["steps"] / (ar_t["decode_ms"] * 1e-3)
    stream_dev = rnd.upload(np.asarray(stream, dtype=np.int32))
    def injected_loop():
        dec.start(prefix)
        rng = np.random.default_rng(5)
        torch.cuda.synchronize()
        i0 = time.perf_counter()
        n_tok, n_acc_sum, n_done = 0, 0, 0
        for _ in range(n_rounds_inj):
            done = len(dec.tokens) - len(prefix)
            if done + K_DRAFT + 1 >= len(stream):
                break
            a = int(min(K_DRAFT, rng.geometric(1.0 / 7.0) - 1))
            got = dec.round(K_DRAFT, inject=(stream_dev[done:done + a], a))
            n_tok += got["n_accept"] + 1
            n_acc_sum += got["n_accept"]
            n_done += 1
        torch.cuda.synchronize()
        return n_tok, n_acc_sum, n_done, time.perf_counter() - i0

    injected_loop()  # untimed pass: the pending-row counts of this loop launch kernel variants not loaded so far
    n_tok, n_acc_sum, n_done, inj_el = injected_loop()
    lossless = dec.tokens[len(prefix):] == stream[:len(dec.tokens) - len(prefix)]
    out["synthetic_acceptance"] = {
        "rounds": n_done, "mean_accepted_per_round": round(n_acc_sum / max(n_done, 1), 2),
        "tokens_per_s": round(n_tok / inj_el, 1), "rounds_per_s": round(n_done / inj_el, 1),
        "ar_greedy_tokens_per_s": round(ar_tok_s, 1), "speedup_vs_ar_greedy": round(n_tok / inj_el / ar_tok_s, 3),
        "committed_stream_equals_ar_greedy": bool(lossless),
        "note": "acceptance injected from the verifier's greedy stream (geometric, mean 6); K fixed at 32"}

    # Variants of the round beyond the default (same workload, same timing protocol, 20 repetitions each):
    # S drafter passes with the confidence-ranked refinement update, and the stochastic acceptance rule.
    def time_variant(steps, uniforms):
        dec.p.refine_steps = steps
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for rep in range(23):
            if rep == 3:
                e0.record()
            dm.set_kv_len(p0)
            vm.set_kv_len(p0)
            dec.enqueue_round(K_DRAFT, uniforms=uniforms)
            torch.cuda.current_stream().synchronize()
        e1.record()
        torch.cuda.synchronize()
        dec.p.refine_steps = 1
        return e0.elapsed_time(e1) / 20.0

    dec.start(prefix)
    dec.stage_inputs()
    dec.u[:K_DRAFT + 1].copy_(torch.from_numpy(np.random.default_rng(6).random(K_DRAFT + 1).astype(np.float32)))
    variants = {}
    for steps in (2, 4):
        ms = time_variant(steps, None)
        variants[f"refine_steps_{steps}"] = {"ms_per_round": round(ms, 4), "rounds_per_s": round(1e3 / ms, 1)}
    ms = time_variant(1, dec.u)
    variants["stochastic_verify"] = {"ms_per_round": round(ms, 4), "rounds_per_s": round(1e3 / ms, 1)}
    out["variants"] = variants

    if not args.no_cpu_baseline:
        from oracle import round as o_round
        try:
            from threadpoolctl import threadpool_info
            cores = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
        except Exception:
            cores = len(os.sched_getaffinity(0))
        st = o_round.SpecState(cfg, dw, cfg, vw, prefix)     # oracle prefill, untimed like the GPU's
        c0 = time.perf_counter()
        o_round.spec_round(st, K_DRAFT, M_MAX, 1.0, BEAM, LAM, table, synth.NGRAM_LOG2_SIZE)
        c_el = time.perf_counter() - c0
        out["cpu_baseline"] = {"value": round(1.0 / c_el, 4), "unit": "rounds/s", "cores": int(cores),
                               "kind": "oracle", "sample": "1 full round of the same workload (same weights, "
                               "prefix and parameters; float64 numpy oracle), prefill untimed"}
    print(json.dumps(out))
    dec.close(); dm.close(); vm.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
