"""Seeded synthetic workloads: configurations and input tensors.

This module holds NO arithmetic of the method.  It only names the workload
shapes and draws the random tensors (network weights, prompt vectors, context
tokens, reward probe, stress-test rewards) that both the HIP library and the
CPU checker receive as inputs.  Trained backbones, prompt sets and reward
models of the paper's experiments (Sec. 6.1) are not available offline; these
tensors stand in for them with the same shapes.
"""
import copy
import numpy as np

MASTER_SEED = 251215347


def bf16_round(a):
    """Round fp32 values to the nearest bf16 (ties to even); returns fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(a):
    """fp32 array holding bf16-representable values -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _flow(a=0.7):
    return dict(kind="flow", a=a)


def _ddim(eta=1.0, beta0=1e-4, beta1=0.02, T_train=1000):
    return dict(kind="ddim", eta=eta, beta0=beta0, beta1=beta1, T_train=T_train)


CONFIGS = {
    # the five benchmark configurations
    "cfg1": dict(P=1, N=8, C=4, H=16, W=16, T=10, sampler=_flow(), kind="adaln",
                 D=128, blocks=2, heads=4, Lc=0, Dc=0, schedule=[[(4, 4)]]),
    "cfg2": dict(P=1, N=24, C=4, H=64, W=64, T=20, sampler=_ddim(), kind="cross",
                 D=768, blocks=12, heads=12, Lc=77, Dc=768, schedule=[[(5, 12)]]),
    "cfg3": dict(P=1, N=48, C=16, H=64, W=64, T=10, sampler=_flow(), kind="joint",
                 D=1536, blocks=24, heads=24, Lc=154, Dc=1536, schedule=[[(2, 32), (4, 16)]]),
    "cfg4": dict(P=8, N=48, C=16, H=64, W=64, T=10, sampler=_flow(), kind="joint",
                 D=1536, blocks=24, heads=24, Lc=154, Dc=1536,
                 schedule=[[(2, 32), (4, 16)]] * 7 + [[]]),
    # reduced shapes of the same structure that the CPU checker finishes in seconds;
    # token counts are chosen to leave ragged tiles (90 = 64 + 26 tokens, 13 context tokens)
    "cfg2_small": dict(P=1, N=6, C=4, H=16, W=16, T=5, sampler=_ddim(), kind="cross",
                       D=128, blocks=2, heads=2, Lc=13, Dc=128, schedule=[[(2, 3)]]),
    "cfg3_small": dict(P=1, N=12, C=4, H=16, W=16, T=6, sampler=_flow(), kind="joint",
                       D=128, blocks=2, heads=2, Lc=26, Dc=128, schedule=[[(1, 8), (3, 4)]]),
    "cfg4_small": dict(P=3, N=12, C=4, H=16, W=16, T=6, sampler=_flow(), kind="joint",
                       D=128, blocks=2, heads=2, Lc=26, Dc=128,
                       schedule=[[(1, 8), (3, 4)], [(1, 7), (3, 5)], []]),
    # dual-stream blocks with normalised queries / keys (the block structure of the flow model the paper trains)
    "cfg3_mmdit_small": dict(P=2, N=6, C=4, H=16, W=16, T=4, sampler=_flow(), kind="mmdit",
                             D=128, blocks=2, heads=2, Lc=26, Dc=128, schedule=[[(1, 3)], [(2, 4)]]),
    "cfg3_mmdit": dict(P=1, N=48, C=16, H=64, W=64, T=10, sampler=_flow(), kind="mmdit",
                       D=1536, blocks=24, heads=24, Lc=154, Dc=1536, schedule=[[(2, 32), (4, 16)]]),
    # the paper's own schedules (Sec. 6.1, experimental settings) on the small network
    "paper_std_small": dict(P=1, N=48, C=4, H=16, W=16, T=10, sampler=_flow(), kind="adaln",
                            D=128, blocks=2, heads=4, Lc=0, Dc=0, schedule=[[(5, 24), (7, 12)]]),
    # efficiency variant: 24 -> 16 -> 12 (the checkpoint steps are taken to be those of the standard variant)
    "paper_flash_small": dict(P=1, N=24, C=4, H=16, W=16, T=10, sampler=_flow(), kind="joint",
                              D=128, blocks=2, heads=2, Lc=26, Dc=128, schedule=[[(5, 16), (7, 12)]]),
    # diffusion-model schedule: 48 -> 32 -> 8 at steps 30 and 40 of T = 50
    "paper_diffusion_small": dict(P=1, N=48, C=4, H=8, W=8, T=50, sampler=_ddim(), kind="cross",
                                  D=64, blocks=1, heads=1, Lc=13, Dc=64, schedule=[[(30, 32), (40, 8)]]),
    # group-size ablation (Sec. 6.3): 32, 48 and 64 expanded trajectories pruned to 8; the intermediate size
    # halves at the standard checkpoints (the paper prints only the two ends)
    "paper_ablation32_small": dict(P=1, N=32, C=4, H=16, W=16, T=10, sampler=_flow(), kind="adaln",
                                   D=128, blocks=2, heads=4, Lc=0, Dc=0, schedule=[[(5, 16), (7, 8)]]),
    "paper_ablation48_small": dict(P=1, N=48, C=4, H=16, W=16, T=10, sampler=_flow(), kind="adaln",
                                   D=128, blocks=2, heads=4, Lc=0, Dc=0, schedule=[[(5, 24), (7, 8)]]),
    "paper_ablation64_small": dict(P=1, N=64, C=4, H=16, W=16, T=10, sampler=_flow(), kind="adaln",
                                   D=128, blocks=2, heads=4, Lc=0, Dc=0, schedule=[[(5, 32), (7, 8)]]),
    # the same schedules at the size of the flow-model benchmark network (bench.py workloads)
    "paper_std": dict(P=1, N=48, C=16, H=64, W=64, T=10, sampler=_flow(), kind="joint",
                      D=1536, blocks=24, heads=24, Lc=154, Dc=1536, schedule=[[(5, 24), (7, 12)]]),
    "paper_flash": dict(P=1, N=24, C=16, H=64, W=64, T=10, sampler=_flow(), kind="joint",
                        D=1536, blocks=24, heads=24, Lc=154, Dc=1536, schedule=[[(5, 16), (7, 12)]]),
}


def get_config(name):
    cfg = copy.deepcopy(CONFIGS[name])
    cfg["name"] = name
    cfg["d"] = cfg["C"] * cfg["H"] * cfg["W"]
    cfg["Li"] = (cfg["H"] // 2) * (cfg["W"] // 2)
    return cfg


def network_evals(cfg):
    """Trajectory-steps of a configuration: sum over steps of active trajectories."""
    total = 0
    for g in range(cfg["P"]):
        n = cfg["N"]
        sched = dict(cfg["schedule"][g])
        for s in range(cfg["T"]):
            total += n                     # evaluation happens before the prune of step s
            n = sched.get(s, n)
    return total


def _normal(seed_words, shape, std):
    rng = np.random.default_rng(seed_words)
    return bf16_round(rng.standard_normal(shape, dtype=np.float32) * np.float32(std))


# tensor name -> (index used in the seed, shape as a function of the config)
def weight_shapes(cfg):
    D, C, Li, Dc = cfg["D"], cfg["C"], cfg["Li"], cfg["Dc"]
    top = dict(pe_w=(D, 4 * C), pe_b=(D,), pos=(Li, D), t_w1=(D, 256), t_b1=(D,),
               t_w2=(D, D), t_b2=(D,), fmod_w=(2 * D, D), fmod_b=(2 * D,),
               f_w=(4 * C, D), f_b=(4 * C,))
    if cfg["kind"] in ("joint", "mmdit"):
        top.update(ctx_w=(D, Dc), ctx_b=(D,))
    blk = dict(mod_w=(6 * D, D), mod_b=(6 * D,), qkv_w=(3 * D, D), qkv_b=(3 * D,),
               o_w=(D, D), o_b=(D,), fc1_w=(4 * D, D), fc1_b=(4 * D,),
               fc2_w=(D, 4 * D), fc2_b=(D,))
    if cfg["kind"] == "cross":
        blk.update(cq_w=(D, D), cq_b=(D,), ckv_w=(2 * D, Dc), ckv_b=(2 * D,),
                   co_w=(D, D), co_b=(D,))
    if cfg["kind"] == "mmdit":
        hd = D // cfg["heads"]
        blk.update({"c_" + k: v for k, v in list(blk.items())})          # the context stream's own copy
        blk.update(qn_g=(hd,), kn_g=(hd,), c_qn_g=(hd,), c_kn_g=(hd,))    # per-channel scales of the query / key norms
    return top, blk


def make_weights(cfg, seed=MASTER_SEED, std=0.02):
    """All network tensors ~ N(0, std^2) (norm scales: 1 + N(0, std^2)), rounded to bf16 once, returned as fp32."""
    top, blk = weight_shapes(cfg)
    w = {}
    for i, (name, shape) in enumerate(sorted(top.items())):
        w[name] = _normal([seed, 1000, i], shape, std)
    w["blocks"] = []
    for b in range(cfg["blocks"]):
        w["blocks"].append({name: (bf16_round(1.0 + _normal([seed, b, i], shape, std)) if name.endswith("_g")
                                   else _normal([seed, b, i], shape, std))
                            for i, (name, shape) in enumerate(sorted(blk.items()))})
    return w


def make_inputs(cfg, weights, seed=MASTER_SEED):
    """Prompt vectors y [P, D], context tokens ctx [P, Lc, Dc] (bf16-rounded) and
    the linear reward probe (dense w [d] fp32, bias)."""
    P, D, C, H, W, Li = cfg["P"], cfg["D"], cfg["C"], cfg["H"], cfg["W"], cfg["Li"]
    rng = np.random.default_rng([seed, 2000])
    inp = dict(y=bf16_round(rng.standard_normal((P, D), dtype=np.float32)))
    inp["ctx"] = (bf16_round(rng.standard_normal((P, cfg["Lc"], cfg["Dc"]), dtype=np.float32))
                  if cfg["Lc"] > 0 else None)
    # probe: a random width-D direction pulled back through the patch embedding and
    # mean-pooled over tokens, i.e. a dense linear functional of the latent, unit norm
    direction = rng.standard_normal(D).astype(np.float64)
    per_patch = direction @ weights["pe_w"].astype(np.float64)        # [4C], index c*4+dy*2+dx
    wp = np.tile(per_patch.reshape(C, 1, 2, 1, 2), (1, H // 2, 1, W // 2, 1)).reshape(C * H * W)
    wp = wp / np.linalg.norm(wp)
    inp["probe_w"] = wp.astype(np.float32)
    inp["probe_b"] = float(np.float32(rng.standard_normal() * 0.1))
    return inp


def stress_rewards(n_groups, n, seed=MASTER_SEED, offset=0.0):
    """Reward-clustering stress input: each entry is N(0, 0.05^2) with probability
    0.8 (the cluster at the group mean, cf. the clustering figure of Sec. 4.1), else
    U(-1, 1); optional constant offset (reward models score around 20+)."""
    rng = np.random.default_rng([seed, 3000])
    clustered = rng.random((n_groups, n)) < 0.8
    vals = np.where(clustered, rng.standard_normal((n_groups, n)) * 0.05,
                    rng.uniform(-1.0, 1.0, (n_groups, n)))
    return (vals + offset).astype(np.float32)


def stress_latents(n_traj, d, seed=MASTER_SEED):
    """x, u ~ N(0, 1) fp32 for the fused update / log-prob stress case."""
    rng = np.random.default_rng([seed, 4000])
    x = rng.standard_normal((n_traj, d), dtype=np.float32)
    u = rng.standard_normal((n_traj, d), dtype=np.float32)
    return x, u


def stress_latent_rows(rows, d, seed=MASTER_SEED, stream=4100):
    """Rows of the large fused-update stress tensor, each drawn from its own seed so that any
    sample of rows can be regenerated without the rest: fp32 ~ N(0, 1)."""
    out = np.empty((len(rows), d), dtype=np.float32)
    for i, r in enumerate(rows):
        out[i] = np.random.default_rng([seed, stream, int(r)]).standard_normal(d, dtype=np.float32)
    return out


def perturbed_weights(weights, rel=0.02, seed=MASTER_SEED + 17):
    """A nearby weight set (every tensor plus rel * std-0.02 noise, rounded to bf16 again): stands in for
    the policy after a small update when the stored transitions are re-evaluated."""
    rng = np.random.default_rng([seed, 5000])
    bump = lambda a: bf16_round(a + rel * 0.02 * rng.standard_normal(a.shape, dtype=np.float32))
    out = {k: bump(v) for k, v in weights.items() if k != "blocks"}
    out["blocks"] = [{k: bump(v) for k, v in blk.items()} for blk in weights["blocks"]]
    return out
