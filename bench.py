"""Benchmark of the Pro-GRPO pruned-sampling hot path on one MI355X.

One "step" = one whole pass of the hot path over one batch: init group, T x (network evaluation on
every active trajectory, prune at the checkpoints, fused update + log-prob), final rewards and
advantages.  Metric: trajectory-steps/s (network evaluations of one trajectory at one step) and
seconds per group.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0       # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
PEAK_VALU_LANE_OPS = 256 * 64 * 2.4e9       # vector-ALU issue roofline: 256 compute units x 64 lanes x 2.4 GHz
# Vector-ALU instructions per latent element of the two kernels that the Philox / Box-Muller arithmetic bounds, as
# the SQ_INSTS_VALU counter reads them (profiles/attention_and_streaming_kernels_issue_counters.txt)
VALU_OPS_PER_ELEMENT = {"init_latents": 20.81, "sde_step_bf16": 33.94}

DESCRIPTIONS = {
    "cfg1": "tiny flow group 8->4, DiT 64 tok x 128 x 2 blocks",
    "cfg2": "diffusion-shaped group N=24->12 @ step 5 of 20 (DDIM eta=1), latent 4x64x64, DiT 1024 tok x 768 x 12 blocks, 77x768 cross-attention",
    "cfg3": "flow-shaped group N=48->32->16 @ steps 2,4 of 10, latent 16x64x64, DiT (1024+154) tok x 1536 x 24 blocks, joint attention",
    "cfg4": "8 prompts x N=48 (ragged 48->32->16, one group unpruned), cfg3 network, one packed batch",
    "cfg3_mmdit": "cfg3 with dual-stream blocks (per-stream weights, RMS-normalised queries / keys): N=48->32->16 @ steps 2,4 of 10",
    "paper_std": "the paper's standard flow schedule N=48->24->12 @ steps 5,7 of 10 on the cfg3 network",
    "paper_flash": "the paper's efficiency schedule N=24->16->12 @ steps 5,7 of 10 on the cfg3 network",
}


def progress(msg):
    """Stage marker on stderr (stdout carries the one JSON line): a long run must show that it is alive."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(cfg, w, inp, seed, budget_traj):
    """The oracle, as it stands, on a bounded sample: `budget_traj` trajectories of the first group for
    one whole step (network evaluation, preview + proxy reward, OVF over the sample, update + log-prob)."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import dit, philox, sampler, ovf
    s = cfg["sampler"]
    tables = (sampler.flow_sde_tables(cfg["T"], s["a"]) if s["kind"] == "flow"
              else sampler.ddim_sde_tables(cfg["T"], s["eta"], s["beta0"], s["beta1"], s["T_train"]))
    n, d = budget_traj, cfg["d"]
    t0 = time.perf_counter()
    x = np.stack([philox.normals(seed, philox.STREAM_INIT, i, 0, d) for i in range(n)])
    ctx = inp["ctx"][0] if inp.get("ctx") is not None else None
    u = dit.forward(w, cfg, x, tables["t_in"][0], inp["y"][0], ctx)
    r = sampler.linear_reward(sampler.preview(x, u, tables["P"][0], tables["Q"][0]), inp["probe_w"], inp["probe_b"])
    ovf.ovf_select(r.astype(np.float32), max(1, n // 2))
    xi = np.stack([philox.normals(seed, philox.STREAM_STEP, i, 0, d) for i in range(n)])
    xn, mean = sampler.sde_step(x, u, tables["A"][0], tables["B"][0], tables["C"][0], xi)
    sampler.gaussian_logprob(xn, mean, tables["C"][0])
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return dict(value=n / dt, unit="trajectory-steps/s", cores=int(threads), kind="oracle",
                sample=f"{n} trajectories of group 0, one full step (network + preview/OVF + update/log-prob) in {dt:.1f} s",
                s_per_group_extrapolated=workloads_evals(cfg) / (n / dt) / cfg["P"],
                note="s_per_group_extrapolated = this sample's rate applied to all trajectory-steps of a group-batch; "
                     "the oracle did not run a whole group")


def stream_kernels_at_stress_shape(pg, torch, n=1024, d=16 * 128 * 128, reps=10):
    """Fused update + log-prob, preview + reward and survivor compaction on 1024 x (16x128x128) fp32 latents:
    algorithmic bytes / event-timed duration against the 8 TB/s HBM peak."""
    dev = "cuda:0"
    g = torch.Generator(device=dev); g.manual_seed(251215347)
    x = torch.randn(n, d, device=dev, generator=g); u = torch.randn(n, d, device=dev, generator=g)
    xo = torch.empty(n, d, device=dev)
    w = torch.randn(d, device=dev, generator=g) / d ** 0.5
    ids = torch.arange(n, dtype=torch.int32, device=dev)
    r = torch.zeros(n, device=dev)
    part = torch.zeros(pg.pg_step_scratch_floats(n, d), device=dev)
    src = torch.arange(0, n, 2, dtype=torch.int32, device=dev)
    res = {}

    def timed(fn, nbytes):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        us = 1e3 * e0.elapsed_time(e1) / reps
        gbs = nbytes / us / 1e3
        return dict(us=round(us, 1), gbs=round(gbs, 1), frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 4))

    res["sde_step_logprob_1024x16x128x128"] = timed(
        lambda: pg.pg_sde_step_logprob(x, u, xo, None, None, None, None, ids, n, d, 0.93, -0.1, 0.38, 7, 3, part), 12.0 * n * d)
    res["preview_reward_1024x16x128x128"] = timed(
        lambda: pg.pg_preview_reward(x, u, w, r, n, d, 1.0, -0.7, 0.1, part), 8.0 * n * d)
    res["compact_gather_1024_to_512"] = timed(lambda: pg.pg_compact_gather(x, xo, src, n // 2, d), 8.0 * (n // 2) * d)
    xb = x.to(torch.bfloat16).view(torch.int16); ub = u.to(torch.bfloat16).view(torch.int16)
    xob = torch.empty(n, d, dtype=torch.int16, device=dev)
    res["sde_step_logprob_bf16_storage_1024x16x128x128"] = timed(
        lambda: pg.pg_sde_step_logprob_bf16(xb, ub, xob, None, None, None, None, ids, n, d, 0.93, -0.1, 0.38, 7, 3, part), 6.0 * n * d)
    res["init_latents_1024x16x128x128"] = timed(lambda: pg.pg_init_latents(xo, ids, 7), 4.0 * n * d)
    # these two issue vector-ALU instructions in (nearly) every cycle: their roofline is the ALU's, not the memory's
    for key, name in (("init_latents_1024x16x128x128", "init_latents"), ("sde_step_logprob_bf16_storage_1024x16x128x128", "sde_step_bf16")):
        ops = VALU_OPS_PER_ELEMENT[name]
        res[key].update(bound="alu", valu_ops_per_element=ops,
                        alu_frac=round(ops * n * d / (res[key]["us"] * 1e-6) / PEAK_VALU_LANE_OPS, 4))
    # the plain copy above is the practical ceiling for a kernel that reads and writes in equal parts
    res["sde_step_vs_copy_ceiling"] = round(res["sde_step_logprob_1024x16x128x128"]["gbs"] / res["compact_gather_1024_to_512"]["gbs"], 3)
    return res


def group_kernels_at_stress_shape(pg, torch, np, workloads, reps=10):
    """Variance-maximising selection 64 -> 16 and group advantages over many clustered-reward groups: these are
    issue/latency bound (4 bytes per reward), so the figure is groups per second, not a bandwidth fraction."""
    dev = "cuda:0"
    res = {}
    for n_groups in (4096, 1 << 20):
        n, k = 64, 16
        if n_groups == 4096:
            r = torch.from_numpy(workloads.stress_rewards(n_groups, n)).to(dev).reshape(-1)
        else:  # same distribution drawn on the device (the host recipe would take seconds at this size)
            g = torch.Generator(device=dev); g.manual_seed(251215347)
            cl = torch.rand(n_groups * n, device=dev, generator=g) < 0.8
            r = torch.where(cl, torch.randn(n_groups * n, device=dev, generator=g) * 0.05,
                            torch.rand(n_groups * n, device=dev, generator=g) * 2 - 1)
        offs = torch.arange(0, (n_groups + 1) * n, n, dtype=torch.int32, device=dev)
        kk = torch.full((n_groups,), k, dtype=torch.int32, device=dev)
        masks = torch.zeros(n_groups, dtype=torch.int64, device=dev)
        sel = torch.zeros(n_groups * k, dtype=torch.int32, device=dev)
        noffs = torch.zeros(n_groups + 1, dtype=torch.int32, device=dev)
        status = torch.zeros(4, dtype=torch.int32, device=dev)
        scratch = torch.zeros(pg.pg_ovf_scratch_ints(n_groups), dtype=torch.int32, device=dev)
        adv = torch.zeros(n_groups * n, device=dev)

        def timed(fn):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            us = 1e3 * e0.elapsed_time(e1) / reps
            return dict(us=round(us, 1), groups_per_s=round(n_groups / us * 1e6, 0))

        res[f"ovf_select_{n_groups}x64_to_16"] = timed(
            lambda: pg.pg_ovf_select(r, offs, kk, n_groups, masks, sel, noffs, status, scratch))
        res[f"group_advantages_{n_groups}x64"] = timed(lambda: pg.pg_group_advantages(r, offs, n_groups, 1e-6, adv))
    return res


def comparison_arms(pg, torch, workloads, cfg, w, inp, seed, inloop_ctx, inloop_buf):
    """Within-group reward spread of the paper's comparison arms (Sec. 4.1-4.2) on this workload: the full
    expanded group, a uniform k-subset, OVF applied once after sampling, and the in-loop pruned survivors.
    sigma_G and the share of members within one sigma of the mean, averaged over groups, plus the wall time
    of sampling the full group (what the static arms pay) next to the pruned loop."""
    import copy
    import time
    P = cfg["P"]
    k_final = [sched[-1][1] if sched else cfg["N"] for sched in cfg["schedule"]]
    full = copy.deepcopy(cfg)
    full["schedule"] = [[] for _ in range(P)]
    c, keep = pg.make_config(full, probe_bias=inp["probe_b"])
    ctx = pg.pg_create(c)
    buf = pg.Buffers(ctx, full, inputs=inp, weights_flat=pg.pack_weights(ctx, full, w))
    pg.pg_bind(ctx, buf)
    sig = torch.zeros(P, device="cuda:0"); share = torch.zeros(P, device="cuda:0")

    def stats(b):
        pg.pg_group_stats(b.rewards, b.group_offsets, P, 1.0, sig, share)
        torch.cuda.synchronize()
        return dict(sigma_G=round(float(sig.mean()), 6), share_within_1_sigma=round(float(share.mean()), 4))

    out = {}
    pg.pg_sample_group(ctx, seed)                       # warm-up of this context
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pg.pg_sample_group(ctx, seed)
    torch.cuda.synchronize()
    out["full_group_s_per_group"] = round((time.perf_counter() - t0) / P, 6)
    out["full_group"] = dict(members=cfg["N"], **stats(buf))
    pg.pg_select_final(ctx, pg.SELECT_UNIFORM, k_final, 0)
    out["uniform_subset"] = dict(members=k_final[0], **stats(buf))
    pg.pg_sample_group(ctx, seed)
    pg.pg_select_final(ctx, pg.SELECT_OVF, k_final, 0)
    out["ovf_after_sampling"] = dict(members=k_final[0], **stats(buf))
    pg.pg_check(ctx)
    pg.pg_destroy(ctx)
    pg.pg_sample_group(inloop_ctx, seed)
    out["ovf_in_loop"] = dict(members=k_final[0], **stats(inloop_buf))
    pg.pg_check(inloop_ctx)
    return out


def policy_ratio_pass(pg, torch, cfg, w, inp, seed):
    """The forward part of the policy update (Eq. 19 and the clipped term of Eq. 20) on a finished run: sampling
    with the trajectory record kept, then the survivors' T transitions re-evaluated under the same weights.
    Seconds per group for each; the ratio pass costs T network evaluations of the K survivors."""
    import time
    P, T = cfg["P"], cfg["T"]
    c, keep = pg.make_config(cfg, probe_bias=inp["probe_b"])
    ctx = pg.pg_create(c)
    buf = pg.Buffers(ctx, cfg, inputs=inp, weights_flat=pg.pack_weights(ctx, cfg, w), keep_history=True)
    pg.pg_bind(ctx, buf)
    M0 = P * cfg["N"]
    logp_new = torch.zeros(T, M0, device="cuda:0"); ratio = torch.zeros(T, M0, device="cuda:0"); J = torch.zeros(P, device="cuda:0")
    out = {}
    for rep in range(2):                                # the second repetition is the timed one
        torch.cuda.synchronize(); t0 = time.perf_counter()
        pg.pg_sample_group(ctx, seed)
        torch.cuda.synchronize(); t1 = time.perf_counter()
        pg.pg_policy_ratio(ctx, buf.weights, 0.2, logp_new, ratio, J)
        torch.cuda.synchronize(); t2 = time.perf_counter()
        out = dict(sampling_with_record_s_per_group=round((t1 - t0) / P, 6), ratio_pass_s_per_group=round((t2 - t1) / P, 6))
    st = pg.pg_state(ctx, P)
    out["survivor_steps_per_group_batch"] = st["M"] * T
    pg.pg_check(ctx)
    pg.pg_destroy(ctx)
    return out


class PowerMeter:
    """Socket power from the driver's hwmon file (microwatts), polled from a host thread at about 50 Hz while a
    phase runs.  The part has a package power limit (hwmon power1_cap); a dense MFMA load on random operands runs
    into it, and then throughput is set by energy per flop, not by cycles."""

    def __init__(self):
        import glob
        files = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")
        self.path = files[0] if files else None
        caps = glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap")
        self.cap_w = None
        if caps:
            try:
                self.cap_w = int(open(caps[0]).read()) / 1e6
            except (OSError, ValueError):
                pass
        self.samples = []
        self._stop = False
        self._thread = None

    def _poll(self):
        while not self._stop:
            try:
                self.samples.append((time.perf_counter(), int(open(self.path).read()) / 1e6))
            except (OSError, ValueError):
                pass
            time.sleep(0.02)

    def start(self):
        if self.path is None:
            return
        import threading
        self._stop = False
        self._thread = threading.Thread(target=self._poll, daemon=True)
        self._thread.start()

    def stop(self):
        if self._thread is not None:
            self._stop = True
            self._thread.join()
            self._thread = None

    def window(self, t0, t1):
        """Mean and maximum power between two perf_counter readings (the first fifth of the window is left out:
        the power controller takes that long to settle), or None without telemetry."""
        w = [p for (t, p) in self.samples if t0 + 0.2 * (t1 - t0) <= t <= t1]
        if not w:
            return None
        return dict(mean_w=round(sum(w) / len(w), 1), max_w=round(max(w), 1), samples=len(w))


def sustained(pg, torch, meter, fn, flops_per_call, seconds=2.0):
    """fn() queued back to back for about `seconds`: TFLOP/s and the socket power meanwhile."""
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(10):
            fn()
        n += 10
        torch.cuda.synchronize()
    t1 = time.perf_counter()
    out = dict(tflops=round(flops_per_call * n / (t1 - t0) / 1e12, 1))
    pw = meter.window(t0, t1)
    if pw:
        out.update(power_mean_w=pw["mean_w"], power_max_w=pw["max_w"])
    time.sleep(0.5)
    return out


def mfma_register_loop(pg, torch, reps=3):
    """A loop of bf16 MFMAs on registers alone (no LDS, no memory): what the matrix pipes of this part sustain with
    all-zero and with random operands.  The published peak assumes the nominal clock; under a dense MFMA load the
    part runs below it, the more so the more operand bits toggle."""
    out = torch.zeros(512 * 256, device="cuda:0")
    res = {}
    for name, scale in (("zeros", 0.0), ("random", 1.0)):
        best = 0.0
        for _ in range(reps):
            pg.pg_mfma_probe(512, 2000, scale, out)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = pg.pg_mfma_probe(512, 20000, scale, out)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        res[name + "_tflops"] = round(best, 1)
    return res


def power_legs(pg, torch, meter, shapes):
    """Sustained (about 2 s each) runs with the socket power beside them: the register-only MFMA loop with zero and
    with random operands, and the GEMM entry point alone with zero / small-integer / N(0, 1) operands."""
    res = {}
    out = torch.zeros(512 * 256, device="cuda:0")
    fl = 512 * 4.0 * 20000 * 8 * 32768.0
    res["mfma_register_loop_zeros"] = sustained(pg, torch, meter, lambda: pg.pg_mfma_probe(512, 20000, 0.0, out), fl)
    res["mfma_register_loop_random"] = sustained(pg, torch, meter, lambda: pg.pg_mfma_probe(512, 20000, 1.0, out), fl)
    for (M, N, K) in shapes:
        kinds = ("random", "ints", "zeros") if (M, N, K) == shapes[0] else ("random",)
        for kind in kinds:
            if kind == "random":
                A = torch.randn(M, K, device="cuda"); W = torch.randn(N, K, device="cuda") * 0.02
            elif kind == "ints":
                A = torch.randint(-2, 3, (M, K), device="cuda").float(); W = torch.randint(-2, 3, (N, K), device="cuda").float()
            else:
                A = torch.zeros(M, K, device="cuda"); W = torch.zeros(N, K, device="cuda")
            A = A.to(torch.bfloat16).view(torch.int16); W = W.to(torch.bfloat16).view(torch.int16)
            Cm = torch.empty(M, N, device="cuda")
            res[f"gemm_{M}x{N}x{K}_{kind}"] = sustained(
                pg, torch, meter, lambda: pg.pg_gemm_bf16(A, K, W, K, None, Cm, N, M, N, K), 2.0 * M * N * K)
            del A, W, Cm
    x = torch.randn(1024, 1 << 18, device="cuda"); y = torch.empty_like(x)
    src = torch.arange(0, 1024, dtype=torch.int32, device="cuda")
    res["copy_2GiB_of_traffic"] = sustained(pg, torch, meter, lambda: pg.pg_compact_gather(x, y, src, 1024, 1 << 18), 0.0)
    res["copy_2GiB_of_traffic"].pop("tflops")
    return res


def recorded_gemm_traffic(workload):
    """HBM bytes per GEMM launch from the committed counter summary, or None when there is none for this
    workload or the kernel source has changed since the counters were taken."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", f"gemm_kernel_{workload}_loop_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    m_t = re.search(r"^traffic_bytes_per_launch=(\d+)", text, re.M)
    m_h = re.search(r"^source_sha256=([0-9a-f]+)", text, re.M)
    if not (m_t and m_h):
        return None
    h = hashlib.sha256()
    for fn in ("gemm.hip", "gemm.hpp"):
        h.update(open(os.path.join(ROOT, "paper_2512_15347_amd", "csrc", fn), "rb").read())
    return int(m_t.group(1)) if h.hexdigest() == m_h.group(1) else None


def gemm_algorithmic_bytes(cfg):
    """Bytes a GEMM launch of the network must move at least (each operand read once, the output written once, the
    residual stream read and written by the launches that add into it), averaged over the launches of one group-batch:
    the figure the counter-measured roofline.traffic stands beside.  Returns (bytes per launch, launches)."""
    D, C, L_i, Lc, kind = cfg["D"], cfg["C"], cfg["Li"], cfg["Lc"], cfg["kind"]
    Kp = (4 * C + 63) // 64 * 64
    joint = kind in ("joint", "mmdit")
    total = 0.0
    launches = 0

    def gemm(rows, n, k, out_bytes_per_elem):
        nonlocal total, launches
        total += 2.0 * rows * k + 2.0 * n * k + out_bytes_per_elem * rows * n
        launches += 1

    active = [cfg["N"]] * cfg["P"]
    for s_ in range(cfg["T"]):
        M = sum(active)
        Ri = M * L_i
        streams = [M * (L_i + (Lc if joint else 0))] if kind != "mmdit" else [Ri, M * Lc]
        gemm(Ri, D, Kp, 4)                                    # patch embedding into the fp32 residual stream
        for _ in range(cfg["blocks"]):
            for R in streams:
                gemm(R, 3 * D, D, 2)                          # q | k | v
                gemm(R, D, D, 8)                              # output projection, residual read + write
                if kind == "cross":
                    gemm(R, D, D, 2)                          # cross-attention queries
                    gemm(R, D, D, 8)                          # cross-attention output, residual read + write
                gemm(R, 4 * D, D, 2)                          # MLP up, GELU
                gemm(R, D, 4 * D, 8)                          # MLP down, residual read + write
        gemm(Ri, 4 * C, D, 4)                                 # final projection into the latent layout
        for g in range(cfg["P"]):
            active[g] = dict(cfg["schedule"][g]).get(s_, active[g])
    return total / launches, launches


def workloads_evals(cfg):
    from paper_2512_15347_amd import workloads
    return workloads.network_evals(cfg)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg4", choices=sorted(DESCRIPTIONS),
                    help="cfg4 (the largest configuration, 8 prompts x 48 trajectories on the 1536-wide network) is the headline")
    ap.add_argument("--bracket-batches", type=int, default=3,
                    help="group-batches of the second pass in which every heavy launch is bracketed by events")
    ap.add_argument("--power-legs", action="store_true",
                    help="also run, for about 2 s each with the socket power beside them, the register-only MFMA loop and the "
                         "GEMM entry point alone (8192^3 with zero / integer / normal operands, two shapes of the 1536-wide network)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-arms", action="store_true", help="skip the comparison arms (full group, uniform subset, static OVF)")
    ap.add_argument("--cpu-sample", type=int, default=0, help="trajectories in the oracle sample (0 = auto)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("this library runs on ONE GPU: the path has no inter-GPU part (groups are independent and would "
                 "shard by prompt); run with --gpus 1")

    progress("importing torch and loading the library")
    import numpy as np
    import torch
    from paper_2512_15347_amd.build import ensure_built
    ensure_built()
    from paper_2512_15347_amd import binding as pg, workloads

    cfg = workloads.get_config(args.workload)
    seed = workloads.MASTER_SEED
    progress(f"workload {args.workload}: drawing the synthetic network weights and inputs")
    w = workloads.make_weights(cfg)
    inp = workloads.make_inputs(cfg, w)
    c, keep = pg.make_config(cfg, probe_bias=inp["probe_b"])
    ctx = pg.pg_create(c)
    progress(f"packing {pg.pg_weights_numel(ctx) / 1e6:.0f} M weights, workspace {pg.pg_workspace_bytes(ctx) / 2**30:.2f} GiB")
    buf = pg.Buffers(ctx, cfg, inputs=inp, weights_flat=pg.pack_weights(ctx, cfg, w))
    pg.pg_bind(ctx, buf)
    evals = workloads.network_evals(cfg)

    for i in range(args.warmup):
        pg.pg_sample_group(ctx, seed + i)
        pg.pg_check(ctx)
        progress(f"warm-up group-batch {i + 1} of {args.warmup} done")
    torch.cuda.synchronize()

    # timed region: K whole group-batches, nothing but the library's own launches on the stream
    # (a host thread reads the socket power from sysfs meanwhile; it touches neither the GPU nor the stream)
    meter = PowerMeter()
    meter.start()
    torch.cuda.synchronize()
    done = [torch.cuda.Event() for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        pg.pg_sample_group(ctx, seed + 100 + i)
        done[i].record()                               # queued behind the batch: the host does not wait here
    for i in range(args.steps):                        # everything is queued; report each batch as it completes
        done[i].synchronize()
        progress(f"timed group-batch {i + 1} of {args.steps} done")
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    power = meter.window(t0, t0 + dt)
    pg.pg_check(ctx)
    st = pg.pg_state(ctx, cfg["P"])
    assert st["evals"] == evals, (st, evals)

    # the same K group-batches once more with every heavy launch bracketed by HIP events on its stream
    # (the brackets cost about a tenth of the loop's wall time, so they stay out of `value`)
    progress(f"timed region: {dt:.1f} s; event-bracketed pass")
    n_br = max(1, min(args.steps, args.bracket_batches))
    pg.pg_profile_begin(1 << 18)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(n_br):
        pg.pg_sample_group(ctx, seed + 100 + i)
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t1
    prof = {k: pg.pg_profile_read(i) for i, k in enumerate(("gemm", "attention", "sde_step", "preview"))}
    pg.pg_profile_end()
    pg.pg_check(ctx)

    g = prof["gemm"]
    gemm_tflops = g["work"] / (g["ms"] * 1e-3) / 1e12 if g["ms"] > 0 else 0.0
    a = prof["attention"]
    s = prof["sde_step"]
    roofline = dict(bound="mfma", kernel="gemm_kernel (bf16 MFMA GEMM, all epilogues)", achieved=round(gemm_tflops, 2),
                    peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=round(gemm_tflops / PEAK_BF16_TFLOPS, 4),
                    traffic=recorded_gemm_traffic(args.workload),
                    traffic_algorithmic=round(gemm_algorithmic_bytes(cfg)[0]),
                    launches=g["launches"], avg_launch_us=round(1e3 * g["ms"] / max(g["launches"], 1), 2),
                    share_of_step_time=round(g["ms"] * 1e-3 / dt_prof, 4), bracketed_batches=n_br,
                    bracketed_pass_ms_per_step=round(1e3 * dt_prof / n_br, 3))
    # the same figure against what a loop of MFMAs alone sustains on this part with random operands
    reg = mfma_register_loop(pg, torch)
    roofline["mfma_register_loop"] = reg
    roofline["frac_of_register_loop_random"] = round(gemm_tflops / reg["random_tflops"], 4) if reg["random_tflops"] > 0 else None
    roofline["note"] = ("with N(0,1)-like operands this GEMM draws the socket power cap at every shape and the clock drops with MFMA activity: "
                        "the figure is set by energy per flop, see profiles/power_telemetry_cfg3_loop_and_gemm_alone.txt and the `power` object")
    others = dict(
        attention=dict(tflops=round(a["work"] / (a["ms"] * 1e-3) / 1e12, 2) if a["ms"] > 0 else None,
                       share_of_step_time=round(a["ms"] * 1e-3 / dt_prof, 4), launches=a["launches"]),
        sde_step=dict(gbs=round(s["work"] / (s["ms"] * 1e-3) / 1e9, 1) if s["ms"] > 0 else None,
                      frac_of_hbm_peak=round(s["work"] / (s["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4) if s["ms"] > 0 else None,
                      share_of_step_time=round(s["ms"] * 1e-3 / dt_prof, 4), launches=s["launches"]))

    # the HBM-bound kernels at the stress shape (1024 trajectories of 16x128x128 fp32), outside the timed region
    progress("streaming and selection kernels at the stress shapes")
    others.update(stream_kernels_at_stress_shape(pg, torch))
    others.update(group_kernels_at_stress_shape(pg, torch, np, workloads))

    out = dict(metric="trajectory-steps/s and s per group (N->k pruned sampling), 1 GPU",
               value=round(evals * args.steps / dt, 3), unit="trajectory-steps/s", n_gpus=1, steps=args.steps,
               warmup=args.warmup, ms_per_step=round(1e3 * dt / args.steps, 3),
               s_per_group=round(dt / args.steps / cfg["P"], 6), higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="bf16", data="synthetic",
               config=dict(workload=f"{args.workload}: {DESCRIPTIONS[args.workload]}",
                           trajectory_steps_per_group_batch=evals, groups=cfg["P"]),
               roofline=roofline, other_kernels=others)
    if not args.no_arms:
        progress("comparison arms (full groups, uniform subset, selection after sampling)")
        out["comparison_arms"] = comparison_arms(pg, torch, workloads, cfg, w, inp, seed, ctx, buf)
        progress("importance-ratio pass")
        out["policy_ratio"] = policy_ratio_pass(pg, torch, cfg, w, inp, seed)
    if power:
        out["power"] = dict(socket_cap_w=meter.cap_w, timed_region_mean_w=power["mean_w"], timed_region_max_w=power["max_w"],
                            source="hwmon power1_input polled at 50 Hz by a host thread")
    if args.power_legs:
        progress("sustained legs with socket power")
        out["power_legs"] = power_legs(pg, torch, meter, [(8192, 8192, 8192), (56544, 4608, 1536), (56544, 1536, 6144)])
    meter.stop()
    if not args.no_cpu_baseline:
        budget = args.cpu_sample or {"cfg1": 8, "cfg2": 8}.get(args.workload, 1)
        progress(f"oracle on the host cores: {budget} trajectory(ies), one whole step")
        out["cpu_baseline"] = cpu_baseline(cfg, w, inp, seed, budget)
    pg.pg_destroy(ctx)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
