#!/usr/bin/env python3
"""Learner-throughput benchmark on one MI355X.

A step = one pass of the whole hot path on one synthetic minibatch:
tj_sample (staleness mask, prefix sum, uniform select, gather from the
device-resident ring) followed by tj_learner_step (three forward passes,
double-DQN TD target, Huber loss, backward, Adam, periodic target update).
By default the gather of the observation rows is folded into the update: the
sampler gathers the scalar fields and hands over indices, and the learner's
first kernels read the sampled rows where they lie in the ring (the indirect
minibatch of the C ABI); --copy-minibatch makes the sampler write dense copies
that the learner then reads.  The stand-alone gather kernel is timed after the
loop in either case, for its own roofline figure.
The ring is filled on the device before the timed region starts.

Prints ONE JSON line: transitions consumed per second, the roofline figure of
the dominant kernel (the MFMA GEMM) from HIP events recorded inside the timed
region, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM traffic of the contraction launches of one step (c3, c5), from two rocprofv3 --pmc runs of
# this script each (FETCH_SIZE, WRITE_SIZE; see profiles/c3_gemm_counters.md), scaled by what the
# same counters read for a streaming kernel of known size in the same runs (adam_update: FETCH_SIZE
# reads half the bytes, WRITE_SIZE all of them).  Valid for the sources it was taken with: the contraction
# kernels and the learner that decides which of them a step launches.
GEMM_SOURCES = ("tj_gemm.h", "tj_gemm.hip", "tj_conv_first.hip", "tj_conv_wgrad.hip", "tj_conv.h", "tj_learner.hip")
GEMM_TRAFFIC = {"c3": {"bytes_per_step": 738.6e6, "gemm_source_sha256_16": "db2a35045902baea"},
                "c5": {"bytes_per_step": 1354.0e6, "gemm_source_sha256_16": "db2a35045902baea"}}
PEAK_HBM_GBS = 8000.0
PEAK_TFLOPS = {"bf16": 2500.0, "fp32": 157.3}


def adam_slice_traffic(dims, precision, B, P):
    """Bytes the optimizer kernel of an MLP moves on top of the algorithmic ones: it adds the S
    slices of the split weight-gradient contraction (S more gradient reads, one gradient write).
    dims: (in, out) per layer.  On a bf16 network of three layers or more whose first and last
    layers take the transposing-read contractions (the library's conditions), the slices of the
    layers between them are summed by blocks that ride in the last weight-gradient launch, and
    the optimizer kernel only has the first layer's and the head's slices left."""
    S = max(1, min(8, B // (1024 if precision == "bf16" else 64)))
    ends = [dims[0], dims[-1]]
    n_ends = sum(i * o + o for i, o in ends)
    S_ends = S      # the first layer's and the head's gradients take more slices on a large batch
    if precision == "bf16" and len(dims) >= 3 and (dims[0][0] * dims[0][1] + dims[0][1]) % 4 == 0 and (P - dims[-1][0] * dims[-1][1] - dims[-1][1]) % 4 == 0:
        tiles = sum(((i + 255) // 256) * ((o + 127) // 128) for i, o in ends)
        S_ends = max(S, min(B // 1024, 256 // tiles))
    early = (precision == "bf16" and len(dims) >= 3 and S > 1 and B % 32 == 0
             and all(i % 8 == 0 and o % 8 == 0 for i, o in ends) and S_ends >= 1)
    extra = 4 * S_ends * n_ends if S_ends > 1 else 0
    if not early and S > 1:
        extra += 4 * S * (P - n_ends)
    return extra


def gemm_flops_per_step(wl, synth, head_in_td_phase):
    """Algorithmic flops of the dense contractions of one step: three forward
    passes (2*B*W each), weight gradients (2*B*W) and input gradients for every
    layer but the first (2*B*W_l).  Where the head layer's forward runs fused
    with the TD kernel (bf16, at most 32 actions) its flops are left out, since
    its time falls into the TD phase, not the GEMM phases; so are those of the
    head's input gradient where that kernel writes it (the layer below is linear)."""
    shapes = synth.layer_shapes(wl.layers, wl.in_chw)
    per_sample = []
    for kind, ws, fin, fout, out_chw in shapes:
        w = 1
        for x in ws:
            w *= x
        per_sample.append(2 * w * (out_chw[1] * out_chw[2] if kind == synth.CONV else 1))
    fwd = sum(per_sample[:-1] if head_in_td_phase else per_sample)
    bwd = sum(per_sample) + sum(per_sample[1:])
    if head_in_td_phase and len(shapes) >= 2 and shapes[-2][0] != synth.CONV:
        bwd -= per_sample[-1]      # the TD kernel also writes the head's input gradient
    return wl.batch * (3 * fwd + bwd)


def gemm_traffic(cfg, n_launch):
    """Counter-measured HBM bytes per GEMM launch, or None when there is no measurement for this
    workload or a source of the contraction kernels has changed since it was taken."""
    import hashlib

    rec = GEMM_TRAFFIC.get(cfg)
    if rec is None:
        return None
    h = hashlib.sha256()
    try:
        for name in GEMM_SOURCES:
            h.update(open(os.path.join(ROOT, "paper_2502_20190_amd", "csrc", name), "rb").read())
    except OSError:
        return None
    sha = h.hexdigest()[:16]
    return rec["bytes_per_step"] / n_launch if sha == rec["gemm_source_sha256_16"] else None


def fill_ring(tj, synth, wl, chunk_rows):
    import torch

    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    versions = []
    c = 0
    for start in range(0, wl.capacity, chunk_rows):
        n = min(chunk_rows, wl.capacity - start)
        rows = synth.make_chunk_device(wl, synth.MASTER_SEED, c, n)
        buf.insert(rows["obs"], rows["next_obs"], rows["action"], rows["reward"], rows["done"],
                   rows["version"])
        versions.append(rows["version"].cpu())
        c += 1
    torch.cuda.synchronize()
    return buf, torch.cat(versions).numpy()


def fill_frame_ring(tj, synth, wl, chunk_rows):
    import torch

    buf = tj.FrameBuffer(wl.capacity, wl.obs_shape[1] * wl.obs_shape[2], wl.obs_shape[0])
    c = 0
    for start in range(0, wl.capacity, chunk_rows):
        n = min(chunk_rows, wl.capacity - start)
        rows = synth.make_frame_stream_device(wl, synth.MASTER_SEED, c, n, start)
        st = buf.insert(rows["frame"], rows["action"], rows["reward"], rows["done"], rows["version"])
        assert st == tj.TJ_OK
        c += 1
    torch.cuda.synchronize()
    return buf, None


def cpu_baseline(wl, synth, buf, versions, theta, target, budget_rows):
    """The CPU oracle on a bounded sample: sampling over the full tag array with
    the full batch, then one learner step on `budget_rows` rows (copied from the
    device ring, copy untimed); the learner time is scaled to the full batch."""
    import numpy as np
    import torch

    from oracle import orc

    t0 = time.perf_counter()
    st, idx, K = orc.sample(versions, wl.capacity, wl.current_version, wl.max_staleness, 1, wl.batch)
    t_sample = time.perf_counter() - t0
    sel = torch.from_numpy(idx[:budget_rows].astype(np.int64)).cuda()
    rows = {f: buf.field(f)[sel].cpu().numpy() for f in ("obs", "next_obs", "action", "reward", "done")}
    o = orc.Learner(wl.layers, wl.in_chw, obs_dtype=wl.obs_dtype, gamma=wl.gamma, kappa=wl.kappa, lr=wl.lr,
                    beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, target_interval=wl.target_interval)
    o.set_state(orc.PARAMS, theta.astype(np.float64))
    o.set_state(orc.TARGET, target.astype(np.float64))
    t0 = time.perf_counter()
    o.step(**rows)
    t_learn = time.perf_counter() - t0
    full = t_sample + t_learn * wl.batch / budget_rows
    return {
        "value": wl.batch / full, "unit": "transitions/s", "cores": orc.num_threads(), "kind": "oracle",
        "sample": (f"sampling over all {wl.capacity} tags at batch {wl.batch} ({t_sample * 1e3:.1f} ms) + one "
                   f"fp64 learner step on {budget_rows} of the {wl.batch} rows ({t_learn:.2f} s), learner "
                   f"time scaled by {wl.batch}/{budget_rows}"),
    }


def library_gemm_reference(batch_cols, width, batch):
    """torch.matmul (vendor GEMM) in bf16 on the three shapes of a width x width layer: forward over
    batch_cols stacked rows, input gradient and weight gradient over batch rows.  Events on torch's
    current stream, 50 calls each."""
    import torch

    out = {}
    for name, (M, N, K) in {"forward": (batch_cols, width, width), "input_gradient": (batch, width, width),
                            "weight_gradient": (width, width, batch)}.items():
        a = torch.randn(M, K, device="cuda", dtype=torch.bfloat16)
        b = torch.randn(N, K, device="cuda", dtype=torch.bfloat16)
        for _ in range(5):
            a @ b.t()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(50):
            a @ b.t()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 50 * 1e3
        out[name] = {"M": M, "N": N, "K": K, "us": us, "TFLOP/s": 2.0 * M * N * K / us / 1e6}
    return out


def bench_ppo(args):
    """On-policy workload: a step is advantage estimation over the whole rollout buffer (tj_gae)
    plus one clipped actor-critic update on it (tj_ppo_step), batch = buffer."""
    import numpy as np
    import torch

    from paper_2502_20190_amd import binding as tj, synth

    name, D, hidden, A, n_env, T, precision = synth.PPO_WORKLOADS[args.config]
    torch.cuda.set_device(0)
    B = n_env * T
    layers = synth.ppo_layers(hidden, A)
    theta = synth.xavier_init(layers, (D, 1, 1), 1)
    H = synth.PPO_HYPER
    lrn = tj.PpoLearner(D, hidden, A, precision, B, theta, lr=H["lr"], beta1=H["beta1"], beta2=H["beta2"],
                        eps=H["eps"], clip=0.2, c_v=0.5, c_e=0.01)
    ro = synth.make_rollouts(D, A, n_env, T, seed=1)
    dev = {k: torch.from_numpy(v).cuda() for k, v in ro.items()}
    L = tj.lib()

    def one_step():
        adv, ret = tj.gae(dev["reward"], dev["value"], dev["done"], H["gamma"], H["lam"])
        rc = lrn.step(dev["obs"], dev["action"], dev["old_logp"], adv.view(-1), ret.view(-1))
        if rc != tj.TJ_OK:
            raise tj.TjError(rc, "bench step")

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    K = args.steps
    every = max(1, args.event_every)
    sampled = list(range(0, K, every))
    lev = [tj.HipEvents(5) for _ in sampled]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        if i % every == 0:
            L.tj_learner_set_phase_events(lrn.h, lev[i // every].ev, 5)
        elif i % every == 1:
            L.tj_learner_set_phase_events(lrn.h, None, 0)
        one_step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    L.tj_learner_set_phase_events(lrn.h, None, 0)
    stats = lrn.read_stats()
    assert stats[4] == args.warmup + K and np.isfinite(stats[3])

    # advantage estimation alone (the learner's events start after its input cast)
    t1 = time.perf_counter()
    for _ in range(200):
        tj.gae(dev["reward"], dev["value"], dev["done"], H["gamma"], H["lam"])
    torch.cuda.synchronize()
    gae_ms = (time.perf_counter() - t1) / 200 * 1e3

    ms = lambda evs, a, b: sum(e.elapsed_ms(a, b) for e in evs) / len(evs)
    ph = {"gae_ms_standalone": gae_ms, "forward_gemm_ms": ms(lev, 0, 1), "objective_ms": ms(lev, 1, 2),
          "backward_gemm_ms": ms(lev, 2, 3), "adam_ms": ms(lev, 3, 4)}
    shapes = synth.layer_shapes(layers, (D, 1, 1))
    per_sample = [2 * int(np.prod(ws)) for _, ws, _, _, _ in shapes]
    n_layers = len(layers)
    # bf16 with at most 32 head outputs: the head's forward runs inside the objective kernel, so its
    # flops are left out of the GEMM phases, as for the Q-learner's fused head
    fused_head = precision == "bf16" and A + 1 <= 32 and n_layers >= 2
    # ... and the head's input gradient too where the layer below takes it row-major (the library's conditions)
    fused_dx = (fused_head and n_layers >= 3 and hidden[-1] % 32 == 0 and hidden[-1] <= 1024 and hidden[-2] % 8 == 0
                and B % 32 == 0)
    fwd = sum(per_sample[:-1] if fused_head else per_sample)
    bwd = sum(per_sample) + sum(per_sample[1:]) - (per_sample[-1] if fused_dx else 0)
    flops = B * (fwd + bwd)     # forward, weight and input gradients
    n_launch = ((n_layers - (1 if fused_head else 0)) + (n_layers if precision == "bf16" else 2 * n_layers - 1)
                - (1 if fused_dx else 0))
    gemm_ms = ph["forward_gemm_ms"] + ph["backward_gemm_ms"]
    achieved = flops / (gemm_ms * 1e-3) / 1e12
    P = synth.num_params(layers, (D, 1, 1))
    adam_bytes = (30 if precision == "bf16" else 28) * P               # algorithmic; the kernel also reads gradient slices
    widths = [D] + [l[1] for l in layers]
    adam_extra = adam_slice_traffic(list(zip(widths[:-1], widths[1:])), precision, B, P)
    gae_bytes = n_env * T * (4 + 4 + 1 + 4 + 4) + n_env * 4      # reward, value, done in; adv, ret out
    out = {
        "metric": "learner transitions consumed/sec at 1 MI355X",
        "value": B * K / wall, "unit": "transitions/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": precision, "data": "synthetic",
        "config": {"workload": name, "n_env": n_env, "rollout": T, "batch": B, "obs_elems": D,
                   "layers": [l[1] for l in layers], "params": P},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_TFLOPS[precision], "unit": "TFLOP/s",
                     "frac": achieved / PEAK_TFLOPS[precision], "traffic": None,
                     "kernel": "gemm_bf16_dlds + gemm_bf16_dlds_pair + gemm_bf16_dlds_pair_sum (its blocks that add gradient slices included)" if precision == "bf16" else "gemm_pq<float>",
                     "launches_per_step": n_launch, "flops_per_launch": flops / n_launch,
                     "avg_launch_ms": gemm_ms / n_launch},
        "phases_ms": ph, "phase_events_on_steps": len(sampled),
        "gae": {"bound": "hbm", "achieved": gae_bytes / (gae_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "bytes": gae_bytes, "frac": gae_bytes / (gae_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "adam": {"bound": "hbm", "achieved": adam_bytes / (ph["adam_ms"] * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                 "unit": "GB/s", "bytes": adam_bytes, "kernel_traffic_bytes": adam_bytes + adam_extra,
                 "frac": adam_bytes / (ph["adam_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS},
        "loss": stats[3],
    }
    if args.library_gemm and precision == "bf16":
        out["library_gemm_reference"] = library_gemm_reference(B, max(hidden), B)
    if not args.no_cpu_baseline:
        from oracle import orc

        rows = args.cpu_rows or max(8, min(B, int(3e11 / (flops / B))))
        t1 = time.perf_counter()
        adv, ret = orc.gae(ro["reward"], ro["value"], ro["done"], H["gamma"], H["lam"])
        t_gae = time.perf_counter() - t1
        o = orc.Learner(layers, (D, 1, 1), lr=H["lr"], eps=H["eps"])
        o.set_state(orc.PARAMS, theta.astype(np.float64))
        t1 = time.perf_counter()
        o.ppo_step(ro["obs"][:rows], ro["action"][:rows], ro["old_logp"][:rows], adv.ravel()[:rows],
                   ret.ravel()[:rows])
        t_learn = time.perf_counter() - t1
        out["cpu_baseline"] = {
            "value": B / (t_gae + t_learn * B / rows), "unit": "transitions/s", "cores": orc.num_threads(),
            "kind": "oracle",
            "sample": (f"advantage estimation over all {n_env} x {T} steps ({t_gae * 1e3:.1f} ms) + one fp64 "
                       f"update on {rows} of the {B} rows ({t_learn:.2f} s), update time scaled by {B}/{rows}"),
        }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="c3", help="workload: c1 ... c5 (replay + double-DQN), p1, p2 (on-policy)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--max-staleness", type=int, default=None,
                    help="override the workload's staleness gate (config 5 names a sweep over 1, 4, 16, 64)")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows of the oracle's learner step (0 = auto)")
    ap.add_argument("--insert-rows", type=int, default=0,
                    help="also push this many new transitions per step into the ring on a second stream "
                         "(tj_buffer_insert_concurrent) while the learner loops")
    ap.add_argument("--frame-ring", action="store_true",
                    help="pixel workloads: keep the replay ring as one frame per slot (tj_frame_buffer); the "
                         "learner reads the frames of each stack through their slots (with --copy-minibatch the "
                         "gather rebuilds dense stacks)")
    ap.add_argument("--actor-rows", type=int, default=0,
                    help="after the learner loop, also time epsilon-greedy policy inference (tj_actor_act) "
                         "on this many observations per call (at most twice the batch)")
    ap.add_argument("--copy-minibatch", action="store_true",
                    help="tj_sample writes dense copies of the sampled observation rows and the learner reads "
                         "those, instead of the learner reading the rows out of the ring through the indices")
    ap.add_argument("--overlap", action="store_true",
                    help="run the sample of step i+1 on a second stream while step i learns (double-buffered "
                         "minibatches) instead of one stream, strictly one after the other; measured: no "
                         "gain, the GEMM kernels leave no registers for a second kernel's waves")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the vendor GEMM behind torch.matmul on this workload's largest forward, "
                         "input-gradient and weight-gradient shapes (plain products, no fused epilogue): a "
                         "reference point for the roofline figures, not part of the step")
    ap.add_argument("--no-second-workload", action="store_true",
                    help="default run only: skip the nested c5 record (the pixel workload with the 231 MB gather)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="record the per-phase HIP events on every n-th timed step (each event costs "
                         "about 5 us of stream time, so recording them on every step slows the loop)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no collectives are part of it)",
              file=sys.stderr)
        sys.exit(2)

    if args.config.startswith("p"):
        if args.insert_rows or args.frame_ring or args.actor_rows:
            print("bench.py: the on-policy workloads take none of the replay-ring options", file=sys.stderr)
            sys.exit(2)
        return bench_ppo(args)

    out = bench_replay(args, args.config, args.steps, args.warmup, not args.no_cpu_baseline)
    if args.config == "c3" and not (args.insert_rows or args.frame_ring or args.actor_rows or args.overlap or
                                    args.library_gemm or args.max_staleness is not None or args.no_second_workload):
        # the configuration the gather target is judged on (231 MB per gather), in the same invocation
        c5 = bench_replay(args, "c5", max(10, min(args.steps, 60)), 10, False)
        out["c5"] = {k: c5[k] for k in ("value", "unit", "ms_per_step", "steps", "warmup", "dtype", "config", "roofline",
                                        "phases_ms", "gather", "adam")}
    print(json.dumps(out))


def bench_replay(args, cfg, steps, warmup, with_cpu_baseline):
    """One replay workload (c1 ... c5): returns the result record."""
    import numpy as np
    import torch

    from paper_2502_20190_amd import binding as tj, synth

    wl = synth.WORKLOADS[cfg]
    if args.max_staleness is not None:
        from dataclasses import replace

        wl = replace(wl, max_staleness=args.max_staleness)
    torch.cuda.set_device(0)
    if args.frame_ring:
        if wl.obs_dtype != "u8" or args.insert_rows:
            print("bench.py: --frame-ring needs a pixel workload and no --insert-rows", file=sys.stderr)
            sys.exit(2)
        with_cpu_baseline = False            # the baseline leg samples from the two-stack ring
        buf, versions = fill_frame_ring(tj, synth, wl, 65_536)
    else:
        buf, versions = fill_ring(tj, synth, wl, 65_536 if wl.obs_dtype == "f32" else 16_384)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 1)
    target = synth.xavier_init(wl.layers, wl.in_chw, 2)
    lrn = tj.learner_for_workload(wl, theta, target)
    L = tj.lib()
    overlap = args.overlap
    # Buffer loop and learner loop run asynchronously (Section 3.1): the sampler fills minibatch
    # i % 2 on its own stream while the learner consumes the other one.  Two events per minibatch
    # order the hand-over in both directions; every step still samples and learns once.
    indirect = not args.copy_minibatch
    mbs = [tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=buf if indirect else None)
           for _ in range(2 if overlap else 1)]
    s_sample = torch.cuda.Stream() if overlap else None
    s_learn = torch.cuda.Stream() if overlap else None
    filled = [torch.cuda.Event() for _ in mbs]
    consumed = [torch.cuda.Event() for _ in mbs]

    side = torch.cuda.Stream() if args.insert_rows else None
    fresh = synth.make_chunk_device(wl, synth.MASTER_SEED, 10_000, args.insert_rows) if args.insert_rows else None
    n_issued = [0]

    def one_step(i):
        if fresh is not None:
            buf.insert_concurrent(fresh["obs"], fresh["next_obs"], fresh["action"], fresh["reward"],
                                  fresh["done"], fresh["version"], side)
        k = n_issued[0] % len(mbs)
        if overlap:
            if n_issued[0] >= len(mbs):
                s_sample.wait_event(consumed[k])
            rc = buf.sample(mbs[k], wl.current_version, wl.max_staleness, i, stream=s_sample)
            filled[k].record(s_sample)
            s_learn.wait_event(filled[k])
            rc = rc or lrn.step(mbs[k], stream=s_learn)
            consumed[k].record(s_learn)
        else:
            rc = buf.sample(mbs[k], wl.current_version, wl.max_staleness, i)
            rc = rc or lrn.step(mbs[k])
        if indirect and fresh is not None:      # the next insert may overwrite rows this update reads
            buf.reads_done(stream=s_learn)
        n_issued[0] += 1
        if rc != tj.TJ_OK:
            raise tj.TjError(rc, "bench step")

    for i in range(warmup):
        one_step(i)
    torch.cuda.synchronize()

    set_buf_events = L.tj_frame_buffer_set_phase_events if args.frame_ring else L.tj_buffer_set_phase_events
    K = steps
    every = max(1, args.event_every)
    sampled = list(range(0, K, every))
    bev = [tj.HipEvents(3) for _ in sampled]
    lev = [tj.HipEvents(5) for _ in sampled]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        if i % every == 0:
            set_buf_events(buf.h, bev[i // every].ev, 3)
            L.tj_learner_set_phase_events(lrn.h, lev[i // every].ev, 5)
        elif i % every == 1:
            set_buf_events(buf.h, None, 0)
            L.tj_learner_set_phase_events(lrn.h, None, 0)
        one_step(warmup + i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    set_buf_events(buf.h, None, 0)
    L.tj_learner_set_phase_events(lrn.h, None, 0)
    st, info = buf.status()
    loss, t = lrn.read_stats()
    assert st == tj.TJ_OK and t == warmup + K and np.isfinite(loss)

    ms = lambda evs, a, b: sum(e.elapsed_ms(a, b) for e in evs) / len(evs)
    gather_ms = ms(bev, 1, 2)
    if indirect:
        # no gather kernel ran in the loop: time the stand-alone one (dense destination) on its own
        dense = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype)
        gev = [tj.HipEvents(3) for _ in range(12)]
        for j in range(len(gev) + 3):
            if j >= 3:
                set_buf_events(buf.h, gev[j - 3].ev, 3)
            rc = buf.sample(dense, wl.current_version, wl.max_staleness, 10_000 + j)
            assert rc == tj.TJ_OK
        torch.cuda.synchronize()
        set_buf_events(buf.h, None, 0)
        gather_ms = ms(gev, 1, 2)
        del dense
    ph = {
        "mask_scan_select_ms": ms(bev, 0, 1),
        ("gather_ms_standalone" if indirect else "gather_ms"): gather_ms,
        "forward_gemm_ms": ms(lev, 0, 1),
        ("head_td_ms" if wl.precision == "bf16" and wl.layers[-1][1] <= 32 else "td_huber_ms"): ms(lev, 1, 2), "backward_gemm_ms": ms(lev, 2, 3),
        "adam_ms": ms(lev, 3, 4),
    }
    n_layers = len(wl.layers)
    n_conv = sum(1 for l in wl.layers if l[0] == synth.CONV)
    # forward: one grouped launch per linear layer, two (online, target) per convolution;
    # backward: a weight-gradient GEMM per layer and an input-gradient GEMM per layer but the first
    fused_head = wl.precision == "bf16" and wl.layers[-1][1] <= 32
    if wl.precision == "bf16" and n_conv == 0:
        # forward: hidden layers (the head runs in the TD kernel where fused); backward: weight and input
        # gradient of a layer share one launch; with the fused head its weight gradient rides with the first
        # layer's and its input gradient is written by the TD kernel
        n_gemm_launch = (n_layers - 1) + (n_layers - 1) if fused_head else 2 * n_layers
    elif n_conv == 0:
        # fp32 MLP: the two gradients of a layer share a launch where both problems are small (the
        # library's thresholds: fewer than 128 tiles of 128 x 128 and fewer than 256 of 64 x 64)
        S = max(1, min(8, wl.batch // 64))
        cdiv = lambda a, b: -(-a // b)
        small = lambda I, J, z: cdiv(I, 128) * cdiv(J, 128) * z < 128 and cdiv(I, 64) * cdiv(J, 64) * z < 256
        widths = [wl.obs_elems] + [l[1] for l in wl.layers]
        n_gemm_launch = n_layers + n_layers + (n_layers - 1)
        for l in range(1, n_layers):       # layer l + 1 of the network: its weight and input gradient
            if small(widths[l], widths[l + 1], S) and small(widths[l], wl.batch, 1):
                n_gemm_launch -= 1
    else:
        n_gemm_launch = (n_layers + n_conv - (1 if fused_head else 0)) + n_layers + (n_layers - 1)
        first = wl.layers[0]
        if wl.precision == "bf16" and wl.in_chw[0] == 4 and first[1] == 32 and first[2] in (4, 8) and first[3] % 2 == 0:
            n_gemm_launch -= 1   # the fused first convolution multiplies with both networks' weights
        if wl.precision == "bf16":
            # later convolutions on the gathered-operand kernel (32 / 64 channels, patch length a multiple
            # of 64): the online and the target pass share one launch
            c_in = first[1]
            for kind, out, k, _ in wl.layers[1:]:
                if kind != synth.CONV:
                    break
                if out in (32, 64) and (k * k * c_in) % 64 == 0:
                    n_gemm_launch -= 1
                c_in = out
            # a linear layer's weight and input gradient share a launch where both fit the direct-to-LDS
            # kernel (the input gradient contracts over the layer's padded width: whole 64-element stages)
            for li, (kind, out, _, _) in enumerate(wl.layers):
                if kind == synth.LIN and li > 0 and (-(-out // 8) * 8) % 64 == 0 and wl.batch % 64 == 0:
                    n_gemm_launch -= 1
            # the fused TD kernel writes the head's input gradient where the layer below it is linear
            if fused_head and n_layers >= 2 and wl.layers[-2][0] == synth.LIN:
                n_gemm_launch -= 1

    flops = gemm_flops_per_step(wl, synth, fused_head)
    # the kernels behind the forward and backward phases (their launches share the MFMA roofline)
    if wl.precision != "bf16":
        gemm_kernel_name = "gemm_pq<float>"
    elif n_conv == 0:
        gemm_kernel_name = "gemm_bf16_dlds + gemm_bf16_dlds_pair + gemm_bf16_dlds_pair_sum (its blocks that add gradient slices included)"
    else:
        gemm_kernel_name = "gemm_bf16_dlds (gathered operands) + conv_first_u8c4 + conv_wgrad_bf16"
    gemm_ms = ph["forward_gemm_ms"] + ph["backward_gemm_ms"]
    achieved = flops / (gemm_ms * 1e-3) / 1e12
    peak = PEAK_TFLOPS[wl.precision]
    P = synth.num_params(wl.layers, wl.in_chw)
    # algorithmic bytes of the update: theta, m, v, g read, theta, m, v written (+ the bf16 weight copy)
    adam_bytes = (30 if wl.precision == "bf16" else 28) * P
    adam_kernel_traffic = adam_bytes
    if n_conv == 0:
        # MLPs: the kernel also sums slices of the split weight-gradient contraction: traffic of the
        # kernel, not of the algorithm
        widths = [wl.obs_elems] + [l[1] for l in wl.layers]
        adam_kernel_traffic += adam_slice_traffic(list(zip(widths[:-1], widths[1:])), wl.precision, wl.batch, P)
    gather_bytes = 2 * wl.batch * wl.record_bytes
    if args.frame_ring:   # k + 1 distinct frames read, 2k planes written, plus the scalars
        k, fe = wl.obs_shape[0], wl.obs_shape[1] * wl.obs_shape[2]
        gather_bytes = wl.batch * ((k + 1) * fe + 2 * k * fe + 2 * 9)
    out = {
        "metric": "learner transitions consumed/sec at 1 MI355X",
        "value": wl.batch * K / wall, "unit": "transitions/s", "n_gpus": 1, "steps": K,
        "warmup": warmup, "ms_per_step": wall / K * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": wl.precision, "data": "synthetic",
        "config": {"workload": wl.name + ("+frame-ring" if args.frame_ring else ""), "ring_slots": wl.capacity, "obs_elems": wl.obs_elems,
                   "batch": wl.batch, "max_staleness": wl.max_staleness, "n_eligible": int(info.last_n_eligible),
                   "layers": [l[1] for l in wl.layers], "params": P,
                   "minibatch": ("indirect: the learner reads the sampled ring rows through the indices" if indirect
                                 else "dense copy written by the sampler")},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
                     "frac": achieved / peak, "traffic": gemm_traffic(wl.name.split("-")[0], n_gemm_launch),
                     "traffic_source": "rocprofv3 counters in profiles/ (null when the kernel sources have changed since)",
                     "kernel": gemm_kernel_name, "launches_per_step": n_gemm_launch,
                     "flops_per_launch": flops / n_gemm_launch, "avg_launch_ms": gemm_ms / n_gemm_launch},
        "phases_ms": ph, "phase_events_on_steps": len(sampled),
        "sample_learn_overlap": overlap,
        "gather": {"bound": "hbm", "achieved": gather_bytes / (gather_ms * 1e-3) / 1e9,
                   "peak": PEAK_HBM_GBS, "unit": "GB/s", "bytes": gather_bytes,
                   "timed": ("stand-alone after the loop (dense destination); inside the loop the rows are read "
                             "by the learner's first kernels" if indirect else "inside the loop")},
        "adam": {"bound": "hbm", "achieved": adam_bytes / (ph["adam_ms"] * 1e-3) / 1e9,
                 "peak": PEAK_HBM_GBS, "unit": "GB/s", "bytes": adam_bytes, "kernel_traffic_bytes": adam_kernel_traffic},
        "loss": loss,
    }
    if args.insert_rows:
        ins_bytes = args.insert_rows * (wl.record_bytes + 4)
        out["concurrent_insert"] = {"rows_per_step": args.insert_rows, "rows_per_s": args.insert_rows * K / wall,
                                    "GB_per_s_written": ins_bytes * K / wall / 1e9,
                                    "last_excluded_len": int(info.last_excluded_len)}
    out["gather"]["frac"] = out["gather"]["achieved"] / PEAK_HBM_GBS
    out["adam"]["frac"] = out["adam"]["achieved"] / PEAK_HBM_GBS
    if args.actor_rows:
        rows = synth.make_chunk_device(wl, synth.MASTER_SEED, 20_000, args.actor_rows)
        for i in range(5):
            lrn.act(rows["obs"], 0.05, i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(50):
            lrn.act(rows["obs"], 0.05, 100 + i)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 50
        out["actor_inference"] = {"rows_per_call": args.actor_rows, "ms_per_call": dt * 1e3,
                                  "actions_per_s": args.actor_rows / dt, "epsilon": 0.05}
    if args.library_gemm and wl.precision == "bf16" and n_conv == 0:
        width = max(l[1] for l in wl.layers)
        out["library_gemm_reference"] = library_gemm_reference(3 * wl.batch, width, wl.batch)
    if with_cpu_baseline:
        rows = args.cpu_rows or max(8, min(wl.batch, int(3e11 / (gemm_flops_per_step(wl, synth, False) / wl.batch))))
        out["cpu_baseline"] = cpu_baseline(wl, synth, buf, versions, theta, target, rows)
    del buf, lrn, mbs
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
