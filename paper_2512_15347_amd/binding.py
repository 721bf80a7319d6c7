"""ctypes binding of libprogrpo.so: same names as the C ABI, argument marshalling only.

PyTorch appears here for device memory and streams; every step of the sampling path runs inside
the HIP library.  There is no CPU fallback: importing this module without the built library
raises.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PROGRPO_LIB", os.path.join(_HERE, "libprogrpo.so"))

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
        "(there is no fallback path)")

_lib = C.CDLL(LIB_PATH)

PG_OK, PG_EINVAL, PG_ESHAPE, PG_ENAN, PG_ESCHED, PG_EWORKSPACE, PG_EHIP = range(7)
STATUS_NAMES = ["PG_OK", "PG_EINVAL", "PG_ESHAPE", "PG_ENAN", "PG_ESCHED", "PG_EWORKSPACE", "PG_EHIP"]
PG_SAMPLER_FLOW, PG_SAMPLER_DDIM, PG_SAMPLER_TABLE = 0, 1, 2
PG_NET_NONE, PG_NET_ADALN, PG_NET_CROSS, PG_NET_JOINT, PG_NET_MMDIT = 0, 1, 2, 3, 4

WEIGHT_IDS = ["pe_w", "pe_b", "pos", "t_w1", "t_b1", "t_w2", "t_b2", "ctx_w", "ctx_b", "fmod_w", "fmod_b",
              "f_w", "f_b", "mod_w", "mod_b", "qkv_w", "qkv_b", "o_w", "o_b", "fc1_w", "fc1_b", "fc2_w",
              "fc2_b", "cq_w", "cq_b", "ckv_w", "ckv_b", "co_w", "co_b",
              "c_mod_w", "c_mod_b", "c_qkv_w", "c_qkv_b", "c_o_w", "c_o_b", "c_fc1_w", "c_fc1_b", "c_fc2_w", "c_fc2_b",
              "qn_g", "kn_g", "c_qn_g", "c_kn_g"]
FIRST_BLOCK_ID = WEIGHT_IDS.index("mod_w")

_dp = C.POINTER(C.c_double)
_ip = C.POINTER(C.c_int32)


class pg_config(C.Structure):
    _fields_ = [("P", C.c_int32), ("N", C.c_int32), ("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32),
                ("T", C.c_int32), ("sampler_kind", C.c_int32), ("noise_level", C.c_double),
                ("eta", C.c_double), ("beta0", C.c_double), ("beta1", C.c_double), ("T_train", C.c_int32),
                ("tab_A", _dp), ("tab_B", _dp), ("tab_C", _dp), ("tab_P", _dp), ("tab_Q", _dp), ("tab_tin", _dp),
                ("net_kind", C.c_int32), ("D", C.c_int32), ("blocks", C.c_int32), ("heads", C.c_int32),
                ("Lc", C.c_int32), ("Dc", C.c_int32), ("n_sched", C.c_int32),
                ("sched_group", _ip), ("sched_step", _ip), ("sched_k", _ip),
                ("probe_bias", C.c_double), ("adv_eps", C.c_double)]


class pg_buffers(C.Structure):
    _fields_ = [("x", C.c_void_p * 2), ("u", C.c_void_p), ("orig_id", C.c_void_p * 2),
                ("group_offsets", C.c_void_p), ("group_of", C.c_void_p), ("rewards", C.c_void_p),
                ("masks", C.c_void_p), ("sel_idx", C.c_void_p), ("logp_hist", C.c_void_p),
                ("logp_sum", C.c_void_p), ("adv", C.c_void_p), ("probe_w", C.c_void_p),
                ("weights", C.c_void_p), ("ctx", C.c_void_p), ("y", C.c_void_p), ("status", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("x_hist", C.c_void_p)]


class PgError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 7 else status}: {message}")
        self.status = status


_vp, _i32, _i64, _u64, _u32, _f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_uint32, C.c_double
_SIGNATURES = {
    "pg_last_error": (C.c_char_p, []),
    "pg_create": (_i32, [C.POINTER(pg_config), C.POINTER(_vp)]),
    "pg_destroy": (None, [_vp]),
    "pg_workspace_bytes": (C.c_size_t, [_vp]),
    "pg_weights_numel": (_i64, [_vp]),
    "pg_weight_slot": (_i32, [_vp, _i32, _i32, C.POINTER(_i64), _ip, _ip, _ip]),
    "pg_get_tables": (_i32, [_vp, _dp, _dp, _dp, _dp, _dp, _dp]),
    "pg_get_schedule": (_i32, [_vp, _i32, _ip, _ip]),
    "pg_bind": (_i32, [_vp, C.POINTER(pg_buffers)]),
    "pg_state": (_i32, [_vp, _ip, _ip, _ip, _ip, C.POINTER(_i64), C.POINTER(_i64)]),
    "pg_init_group": (_i32, [_vp, _u64, _vp]),
    "pg_net_forward": (_i32, [_vp, _i32, _vp]),
    "pg_prune": (_i32, [_vp, _i32, _vp]),
    "pg_prune_forced": (_i32, [_vp, _i32, C.POINTER(_u64), _vp, _vp]),
    "pg_step": (_i32, [_vp, _i32, _vp]),
    "pg_advantages": (_i32, [_vp, _vp]),
    "pg_sample_group": (_i32, [_vp, _u64, _vp]),
    "pg_check": (_i32, [_vp, _vp]),
    "pg_policy_ratio": (_i32, [_vp, _vp, _f64, _vp, _vp, _vp, _vp]),
    "pg_select_final": (_i32, [_vp, _i32, _ip, _u32, _vp]),
    "pg_init_latents": (_i32, [_vp, _vp, _i64, _i64, _u64, _vp]),
    "pg_step_scratch_floats": (_i64, [_i64, _i64]),
    "pg_sde_step_logprob": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _f64, _f64, _f64, _u64,
                                    _u32, _vp, _vp]),
    "pg_sde_step_logprob_bf16": (_i32, [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i64, _i64, _f64, _f64, _f64, _u64,
                                         _u32, _vp, _vp]),
    "pg_preview_reward": (_i32, [_vp, _vp, _vp, _vp, _i64, _i64, _f64, _f64, _f64, _vp, _vp]),
    "pg_ovf_scratch_ints": (_i64, [_i64]),
    "pg_ovf_select": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pg_ovf_select_noalloc": (_i32, [_vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "pg_ovf_select_large": (_i32, [_vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pg_uniform_select": (_i32, [_vp, _vp, _i32, _u64, _u32, _vp, _vp, _vp, _vp, _vp, _vp]),
    "pg_group_stats": (_i32, [_vp, _vp, _i32, _f64, _vp, _vp, _vp]),
    "pg_compact_gather": (_i32, [_vp, _vp, _vp, _i64, _i64, _vp]),
    "pg_group_advantages": (_i32, [_vp, _vp, _i32, _f64, _vp, _vp]),
    "pg_gemm_bf16": (_i32, [_vp, _i64, _vp, _i64, _vp, _vp, _i64, _i64, _i64, _i64, _vp]),
    "pg_attention_bf16": (_i32, [_vp, _vp, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp]),
    "pg_mfma_probe": (_i32, [_i32, _i32, C.c_float, _vp, _dp, _vp]),
    "pg_profile_begin": (_i32, [_i32]),
    "pg_profile_read": (_i32, [_i32, _dp, _dp, C.POINTER(_i64)]),
    "pg_profile_end": (_i32, []),
}
EXPORTS = sorted(_SIGNATURES)
for _name, (_res, _args) in _SIGNATURES.items():
    _fn = getattr(_lib, _name)          # AttributeError here = symbol missing from the library
    _fn.restype = _res
    _fn.argtypes = _args


def pg_last_error():
    return _lib.pg_last_error().decode()


def _check(status):
    if status != PG_OK:
        raise PgError(status, pg_last_error())


def _ptr(t):
    """Device (or host) address of a torch tensor / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "the C ABI takes contiguous buffers"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


# ---------------------------------------------------------------- context-level calls

def make_config(cfg, probe_bias=0.0, adv_eps=1e-6, net=True, tables=None):
    """workloads-style dict -> (pg_config, keep-alive list)."""
    keep = []
    c = pg_config()
    for f in ("P", "N", "C", "H", "W", "T"):
        setattr(c, f, int(cfg[f]))
    s = cfg["sampler"]
    if tables is not None:
        c.sampler_kind = PG_SAMPLER_TABLE
        for name, key in (("tab_A", "A"), ("tab_B", "B"), ("tab_C", "C"), ("tab_P", "P"), ("tab_Q", "Q"),
                          ("tab_tin", "t_in")):
            arr = (C.c_double * cfg["T"])(*[float(v) for v in tables[key]])
            keep.append(arr)
            setattr(c, name, C.cast(arr, _dp))
    elif s["kind"] == "flow":
        c.sampler_kind = PG_SAMPLER_FLOW
        c.noise_level = float(s["a"])
    else:
        c.sampler_kind = PG_SAMPLER_DDIM
        c.eta, c.beta0, c.beta1, c.T_train = float(s["eta"]), float(s["beta0"]), float(s["beta1"]), int(s["T_train"])
    if net:
        c.net_kind = {"adaln": PG_NET_ADALN, "cross": PG_NET_CROSS, "joint": PG_NET_JOINT,
                      "mmdit": PG_NET_MMDIT}[cfg["kind"]]
        c.D, c.blocks, c.heads, c.Lc, c.Dc = (int(cfg[k]) for k in ("D", "blocks", "heads", "Lc", "Dc"))
    else:
        c.net_kind = PG_NET_NONE
    entries = [(g, st, k) for g, lst in enumerate(cfg["schedule"]) for (st, k) in lst]
    c.n_sched = len(entries)
    if entries:
        for name, col in (("sched_group", 0), ("sched_step", 1), ("sched_k", 2)):
            arr = (C.c_int32 * len(entries))(*[int(e[col]) for e in entries])
            keep.append(arr)
            setattr(c, name, C.cast(arr, _ip))
    c.probe_bias = float(probe_bias)
    c.adv_eps = float(adv_eps)
    return c, keep


def pg_create(config):
    out = _vp()
    _check(_lib.pg_create(C.byref(config), C.byref(out)))
    return out


def pg_destroy(ctx):
    _lib.pg_destroy(ctx)


def pg_workspace_bytes(ctx):
    return int(_lib.pg_workspace_bytes(ctx))


def pg_weights_numel(ctx):
    return int(_lib.pg_weights_numel(ctx))


def pg_weight_slot(ctx, wid, block=0):
    off, rows, cols, ld = _i64(), _i32(), _i32(), _i32()
    _check(_lib.pg_weight_slot(ctx, wid, block, C.byref(off), C.byref(rows), C.byref(cols), C.byref(ld)))
    return off.value, rows.value, cols.value, ld.value


def pg_get_tables(ctx, T):
    arrs = [(C.c_double * T)() for _ in range(6)]
    _check(_lib.pg_get_tables(ctx, *arrs))
    return {k: np.array(a[:]) for k, a in zip(("A", "B", "C", "P", "Q", "t_in"), arrs)}


def pg_get_schedule(ctx, step, P):
    k, off = (C.c_int32 * P)(), (C.c_int32 * (P + 1))()
    _check(_lib.pg_get_schedule(ctx, step, k, off))
    return list(k), list(off)


def pack_weights(ctx, cfg, weights):
    """Lay the network tensors out as the library asks (uint16 bf16 bit patterns, host array)."""
    from .workloads import bf16_bits
    flat = np.zeros(pg_weights_numel(ctx), dtype=np.uint16)

    def put(wid, block, arr):
        off, rows, cols, ld = pg_weight_slot(ctx, wid, block)
        a = np.asarray(arr, dtype=np.float32).reshape(rows, cols)
        view = flat[off:off + rows * ld].reshape(rows, ld)
        view[:, :cols] = bf16_bits(a)

    for wid, name in enumerate(WEIGHT_IDS):
        if wid < FIRST_BLOCK_ID:
            if name in weights:
                put(wid, 0, weights[name])
        else:
            for b, blk in enumerate(weights["blocks"]):
                if name in blk:
                    put(wid, b, blk[name])
    return flat


class Buffers:
    """Device tensors for one context (torch owns the memory) + the filled pg_buffers."""

    def __init__(self, ctx, cfg, inputs=None, weights_flat=None, device="cuda:0", keep_history=False):
        import torch
        P, N, T, d = cfg["P"], cfg["N"], cfg["T"], cfg["d"]
        M0 = P * N
        dev = torch.device(device)
        z = lambda *shape, dtype=torch.float32: torch.zeros(*shape, dtype=dtype, device=dev)
        self.x = [z(M0, d), z(M0, d)]
        self.u = z(M0, d)
        self.orig_id = [z(M0, dtype=torch.int32), z(M0, dtype=torch.int32)]
        self.group_offsets = z(P + 1, dtype=torch.int32)
        self.group_of = z(M0, dtype=torch.int32)
        self.rewards = z(M0)
        self.masks = z(P, dtype=torch.int64)
        self.sel_idx = z(M0, dtype=torch.int32)
        self.logp_hist = z(T, M0)
        self.logp_sum = z(M0)
        self.adv = z(M0)
        self.status = z(4, dtype=torch.int32)
        self.probe_w = (torch.from_numpy(np.ascontiguousarray(inputs["probe_w"], dtype=np.float32)).to(dev)
                        if inputs is not None else z(d))
        self.weights = self.ctx_tok = self.y = None
        if weights_flat is not None:
            self.weights = torch.from_numpy(weights_flat.view(np.int16)).to(dev)
            self.y = torch.from_numpy(np.ascontiguousarray(inputs["y"], dtype=np.float32)).to(dev)
            if inputs.get("ctx") is not None:
                from .workloads import bf16_bits
                self.ctx_tok = torch.from_numpy(bf16_bits(inputs["ctx"]).view(np.int16)).to(dev)
        nbytes = pg_workspace_bytes(ctx)
        self.workspace = torch.empty(max(nbytes, 256) + 256, dtype=torch.uint8, device=dev)
        ws_ptr = (self.workspace.data_ptr() + 255) & ~255
        b = pg_buffers()
        b.x[0], b.x[1] = self.x[0].data_ptr(), self.x[1].data_ptr()
        b.u = self.u.data_ptr()
        b.orig_id[0], b.orig_id[1] = self.orig_id[0].data_ptr(), self.orig_id[1].data_ptr()
        for name in ("group_offsets", "group_of", "rewards", "masks", "sel_idx", "logp_hist", "logp_sum", "adv",
                     "probe_w", "status"):
            setattr(b, name, getattr(self, name).data_ptr())
        b.weights = _ptr(self.weights)
        b.ctx = _ptr(self.ctx_tok)
        b.y = _ptr(self.y)
        b.workspace = ws_ptr
        b.workspace_bytes = nbytes
        self.x_hist = z(T + 1, M0, d) if keep_history else None
        b.x_hist = _ptr(self.x_hist)
        self.c = b


def pg_bind(ctx, buffers):
    _check(_lib.pg_bind(ctx, C.byref(buffers.c if isinstance(buffers, Buffers) else buffers)))


def pg_state(ctx, P):
    M, cx, ci, ev, up = _i32(), _i32(), _i32(), _i64(), _i64()
    off = (C.c_int32 * (P + 1))()
    _check(_lib.pg_state(ctx, C.byref(M), C.byref(cx), C.byref(ci), off, C.byref(ev), C.byref(up)))
    return dict(M=M.value, cur_x=cx.value, cur_id=ci.value, offsets=list(off), evals=ev.value, updates=up.value)


def pg_init_group(ctx, seed, stream=None):
    _check(_lib.pg_init_group(ctx, seed, _stream(stream)))


def pg_net_forward(ctx, step, stream=None):
    _check(_lib.pg_net_forward(ctx, step, _stream(stream)))


def pg_prune(ctx, step, stream=None):
    _check(_lib.pg_prune(ctx, step, _stream(stream)))


def pg_prune_forced(ctx, step, masks, ovf_masks_out=None, stream=None):
    arr = (C.c_uint64 * len(masks))(*[int(m) for m in masks])
    _check(_lib.pg_prune_forced(ctx, step, arr, _ptr(ovf_masks_out), _stream(stream)))


def pg_step(ctx, step, stream=None):
    _check(_lib.pg_step(ctx, step, _stream(stream)))


def pg_advantages(ctx, stream=None):
    _check(_lib.pg_advantages(ctx, _stream(stream)))


def pg_sample_group(ctx, seed, stream=None):
    _check(_lib.pg_sample_group(ctx, seed, _stream(stream)))


SELECT_OVF, SELECT_UNIFORM = 0, 1


def pg_select_final(ctx, mode, k_per_group, draw=0, stream=None):
    k = (C.c_int32 * len(k_per_group))(*[int(v) for v in k_per_group])
    _check(_lib.pg_select_final(ctx, mode, k, draw, _stream(stream)))


def pg_policy_ratio(ctx, weights_new, clip_eps, logp_new, ratio, J, stream=None):
    _check(_lib.pg_policy_ratio(ctx, _ptr(weights_new), clip_eps, _ptr(logp_new), _ptr(ratio), _ptr(J), _stream(stream)))


def pg_check(ctx, stream=None):
    _check(_lib.pg_check(ctx, _stream(stream)))


# ---------------------------------------------------------------- kernel-level calls

def pg_init_latents(x, orig_id, seed, stream=None):
    n, d = x.shape
    _check(_lib.pg_init_latents(_ptr(x), _ptr(orig_id), n, d, seed, _stream(stream)))


def pg_step_scratch_floats(n_traj, d):
    return int(_lib.pg_step_scratch_floats(n_traj, d))


def pg_sde_step_logprob(x, u, x_out, logp, logp_hist, logp_sum, src, orig_id, n_traj, d, A, B, Cc, seed, step,
                        partials, stream=None):
    _check(_lib.pg_sde_step_logprob(_ptr(x), _ptr(u), _ptr(x_out), _ptr(logp), _ptr(logp_hist), _ptr(logp_sum),
                                    _ptr(src), _ptr(orig_id), n_traj, d, A, B, Cc, seed, step, _ptr(partials),
                                    _stream(stream)))


def pg_sde_step_logprob_bf16(x, u, x_out, logp, logp_hist, logp_sum, src, orig_id, n_traj, d, A, B, Cc, seed, step,
                             partials, stream=None):
    _check(_lib.pg_sde_step_logprob_bf16(_ptr(x), _ptr(u), _ptr(x_out), _ptr(logp), _ptr(logp_hist), _ptr(logp_sum),
                                         _ptr(src), _ptr(orig_id), n_traj, d, A, B, Cc, seed, step, _ptr(partials),
                                         _stream(stream)))


def pg_preview_reward(x, u, w, rewards, n_traj, d, Pc, Qc, bias, partials, stream=None):
    _check(_lib.pg_preview_reward(_ptr(x), _ptr(u), _ptr(w), _ptr(rewards), n_traj, d, Pc, Qc, bias,
                                  _ptr(partials), _stream(stream)))


def pg_ovf_scratch_ints(n_groups):
    return int(_lib.pg_ovf_scratch_ints(n_groups))


def pg_ovf_select(rewards, group_offsets, k, n_groups, masks, sel_idx, new_offsets, status, scratch, stream=None):
    _check(_lib.pg_ovf_select(_ptr(rewards), _ptr(group_offsets), _ptr(k), n_groups, _ptr(masks), _ptr(sel_idx),
                              _ptr(new_offsets), _ptr(status), _ptr(scratch), _stream(stream)))


PG_OVF_NOALLOC_MAX_GROUPS = 4194304


def pg_ovf_select_noalloc(rewards, group_offsets, k, n_groups, masks, sel_idx, new_offsets, status, stream=None):
    _check(_lib.pg_ovf_select_noalloc(_ptr(rewards), _ptr(group_offsets), _ptr(k), n_groups, _ptr(masks), _ptr(sel_idx),
                                      _ptr(new_offsets), _ptr(status), _stream(stream)))


def pg_ovf_select_large(rewards, group_offsets, k, n_groups, mask_words, masks, sel_idx, new_offsets, status, scratch,
                        stream=None):
    _check(_lib.pg_ovf_select_large(_ptr(rewards), _ptr(group_offsets), _ptr(k), n_groups, mask_words, _ptr(masks),
                                    _ptr(sel_idx), _ptr(new_offsets), _ptr(status), _ptr(scratch), _stream(stream)))


def pg_uniform_select(group_offsets, k, n_groups, seed, draw, masks, sel_idx, new_offsets, status, scratch, stream=None):
    _check(_lib.pg_uniform_select(_ptr(group_offsets), _ptr(k), n_groups, seed, draw, _ptr(masks), _ptr(sel_idx),
                                  _ptr(new_offsets), _ptr(status), _ptr(scratch), _stream(stream)))


def pg_group_stats(rewards, group_offsets, n_groups, delta, sigma, clustered_share, stream=None):
    _check(_lib.pg_group_stats(_ptr(rewards), _ptr(group_offsets), n_groups, delta, _ptr(sigma), _ptr(clustered_share),
                               _stream(stream)))


def pg_compact_gather(x, out, src, n_out, d, stream=None):
    _check(_lib.pg_compact_gather(_ptr(x), _ptr(out), _ptr(src), n_out, d, _stream(stream)))


def pg_group_advantages(rewards, group_offsets, n_groups, eps, adv, stream=None):
    _check(_lib.pg_group_advantages(_ptr(rewards), _ptr(group_offsets), n_groups, eps, _ptr(adv), _stream(stream)))


def pg_gemm_bf16(A, lda, W, ldw, bias, Cout, ldc, M, N, K, stream=None):
    _check(_lib.pg_gemm_bf16(_ptr(A), lda, _ptr(W), ldw, _ptr(bias), _ptr(Cout), ldc, M, N, K, _stream(stream)))


def pg_attention_bf16(q, k, vt, out, B, Lq, Lk, heads, hd, stream=None):
    _check(_lib.pg_attention_bf16(_ptr(q), _ptr(k), _ptr(vt), _ptr(out), B, Lq, Lk, heads, hd, _stream(stream)))


def pg_mfma_probe(blocks, iters, operand_scale, out, stream=None):
    flops = C.c_double()
    _check(_lib.pg_mfma_probe(blocks, iters, operand_scale, _ptr(out), C.byref(flops), _stream(stream)))
    return flops.value


def pg_profile_begin(max_records=1 << 16):
    _check(_lib.pg_profile_begin(max_records))


def pg_profile_read(kind):
    ms, work, n = C.c_double(), C.c_double(), _i64()
    _check(_lib.pg_profile_read(kind, C.byref(ms), C.byref(work), C.byref(n)))
    return dict(ms=ms.value, work=work.value, launches=n.value)


def pg_profile_end():
    _check(_lib.pg_profile_end())
