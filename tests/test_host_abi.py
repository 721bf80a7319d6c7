"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, validates its
arguments on the host, and builds the same per-step tables as the oracle."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import sampler
from paper_2512_15347_amd import binding as pg, workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    text = open(os.path.join(ROOT, "include", "progrpo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(pg_[a-z0-9_]+)\s*\(", text))
    assert declared == set(pg.EXPORTS), declared ^ set(pg.EXPORTS)
    lib = C.CDLL(pg.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_header_is_plain_c_and_matches_the_binding_structs(tmp_path):
    """include/progrpo.h compiles as C99 and as C++17, and the struct sizes the binding marshals are the
    compiler's."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no host C compiler")
    src = tmp_path / "abi.c"
    src.write_text('#include <stdio.h>\n#include "progrpo.h"\n'
                   'int main(void) { printf("%zu %zu %d\\n", sizeof(pg_config), sizeof(pg_buffers), (int)PG_W_COUNT); return 0; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.check_call([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, str(src), "-o", str(tmp_path / "abi")])
    out = subprocess.check_output([str(tmp_path / "abi")]).decode().split()
    assert int(out[0]) == C.sizeof(pg.pg_config) and int(out[1]) == C.sizeof(pg.pg_buffers)
    assert int(out[2]) == len(pg.WEIGHT_IDS)
    gxx = shutil.which("g++")
    if gxx:
        subprocess.check_call([gxx, "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)])


def _ctx(name, **kw):
    cfg = workloads.get_config(name)
    c, keep = pg.make_config(cfg, **kw)
    return cfg, c, keep


def test_tables_match_oracle_flow_and_ddim():
    for name in ("cfg1", "cfg3", "cfg2", "cfg2_small"):
        cfg, c, keep = _ctx(name)
        ctx = pg.pg_create(c)
        got = pg.pg_get_tables(ctx, cfg["T"])
        s = cfg["sampler"]
        want = (sampler.flow_sde_tables(cfg["T"], s["a"]) if s["kind"] == "flow"
                else sampler.ddim_sde_tables(cfg["T"], s["eta"], s["beta0"], s["beta1"], s["T_train"]))
        for key in ("A", "B", "C", "P", "Q", "t_in"):
            np.testing.assert_allclose(got[key], want[key], rtol=1e-12, atol=1e-14, err_msg=f"{name} {key}")
        pg.pg_destroy(ctx)


def test_explicit_tables_roundtrip():
    cfg = workloads.get_config("cfg1")
    t = sampler.flow_sde_tables(cfg["T"], 0.3)
    c, keep = pg.make_config(cfg, tables=t)
    ctx = pg.pg_create(c)
    got = pg.pg_get_tables(ctx, cfg["T"])
    np.testing.assert_array_equal(got["A"], t["A"])
    np.testing.assert_array_equal(got["t_in"], t["t_in"])
    pg.pg_destroy(ctx)


@pytest.mark.parametrize("mutate,status", [
    (lambda c: setattr(c, "N", 65), pg.PG_ESHAPE),
    (lambda c: setattr(c, "N", 0), pg.PG_EINVAL),
    (lambda c: setattr(c, "H", 15), pg.PG_ESHAPE),
    (lambda c: setattr(c, "T", 0), pg.PG_EINVAL),
    (lambda c: setattr(c, "noise_level", 0.0), pg.PG_EINVAL),
    (lambda c: setattr(c, "adv_eps", 0.0), pg.PG_EINVAL),
    (lambda c: setattr(c, "D", 100), pg.PG_ESHAPE),
    (lambda c: setattr(c, "heads", 1), pg.PG_ESHAPE),          # head width 128
    (lambda c: setattr(c, "Lc", 5), pg.PG_EINVAL),             # adaLN-only network with context
    (lambda c: setattr(c, "sampler_kind", 7), pg.PG_EINVAL),
    (lambda c: setattr(c, "net_kind", 9), pg.PG_EINVAL),
])
def test_create_rejects_bad_config(mutate, status):
    cfg, c, keep = _ctx("cfg1")
    mutate(c)
    with pytest.raises(pg.PgError) as e:
        pg.pg_create(c)
    assert e.value.status == status and len(str(e.value)) > 10


def test_create_rejects_bad_schedules():
    for sched in ([[(4, 8)]], [[(4, 9)]], [[(4, 0)]], [[(10, 4)]], [[(2, 4), (5, 4)]], [[(2, 4), (2, 3)]],
                  [[(5, 4), (2, 3)]]):
        cfg = workloads.get_config("cfg1")
        cfg["schedule"] = sched
        c, keep = pg.make_config(cfg)
        with pytest.raises(pg.PgError) as e:
            pg.pg_create(c)
        assert e.value.status == pg.PG_ESCHED, sched
    cfg = workloads.get_config("cfg1")
    cfg["schedule"] = [[(2, 6), (5, 3)]]
    c, keep = pg.make_config(cfg)
    pg.pg_destroy(pg.pg_create(c))
    c.n_sched = 1
    c.sched_group[0] = 3                                         # group out of range
    with pytest.raises(pg.PgError):
        pg.pg_create(c)


def test_schedule_table_is_the_funnel():
    """The counts / offsets a prune uses come from a table built once from the schedule (Sec. 5.2): every row is
    the funnel's state at that step, also for ragged groups and for a group that is never pruned."""
    for name in ("cfg1", "cfg3", "cfg4", "cfg4_small", "paper_diffusion_small"):
        cfg, c, keep = _ctx(name)
        ctx = pg.pg_create(c)
        P, N = cfg["P"], cfg["N"]
        size = [N] * P
        for s in range(cfg["T"]):
            k, off = pg.pg_get_schedule(ctx, s, P)
            want = [dict(cfg["schedule"][g]).get(s, size[g]) for g in range(P)]
            assert k == want, (name, s)
            assert off == np.concatenate([[0], np.cumsum(want)]).tolist()
            size = want
        final = [cfg["schedule"][g][-1][1] if cfg["schedule"][g] else N for g in range(P)]
        assert size == final
        with pytest.raises(pg.PgError):
            pg.pg_get_schedule(ctx, cfg["T"], P)
        pg.pg_destroy(ctx)


def test_ddim_needs_enough_training_steps_and_eta():
    cfg, c, keep = _ctx("cfg2_small")
    c.T_train = cfg["T"]
    with pytest.raises(pg.PgError):
        pg.pg_create(c)
    cfg, c, keep = _ctx("cfg2_small")
    c.eta = 0.0
    with pytest.raises(pg.PgError):
        pg.pg_create(c)


def test_weight_layout_is_disjoint_and_covers_all_tensors():
    for name in ("cfg1", "cfg2_small", "cfg3_small", "cfg3_mmdit_small"):
        cfg, c, keep = _ctx(name)
        ctx = pg.pg_create(c)
        top, blk = workloads.weight_shapes(cfg)
        spans = []
        for wid, wname in enumerate(pg.WEIGHT_IDS):
            shapes = top if wid < pg.FIRST_BLOCK_ID else blk
            for b in range(cfg["blocks"] if wid >= pg.FIRST_BLOCK_ID else 1):
                if wname not in shapes:
                    with pytest.raises(pg.PgError):
                        pg.pg_weight_slot(ctx, wid, b)
                    continue
                off, rows, cols, ld = pg.pg_weight_slot(ctx, wid, b)
                shp = shapes[wname]
                assert (rows, cols) == (shp if len(shp) == 2 else (1, shp[0]))
                assert ld >= cols and off % 8 == 0 and (rows == 1 or ld % 64 == 0)
                spans.append((off, off + rows * ld))
        spans.sort()
        assert all(a[1] <= b[0] for a, b in zip(spans[:-1], spans[1:]))
        assert spans[-1][1] <= pg.pg_weights_numel(ctx)
        w = workloads.make_weights(cfg)
        flat = pg.pack_weights(ctx, cfg, w)
        off, rows, cols, ld = pg.pg_weight_slot(ctx, pg.WEIGHT_IDS.index("qkv_w"), 1)
        got = flat[off:off + rows * ld].reshape(rows, ld)[:, :cols]
        np.testing.assert_array_equal(got, workloads.bf16_bits(w["blocks"][1]["qkv_w"]))
        assert pg.pg_workspace_bytes(ctx) > 0
        pg.pg_destroy(ctx)


def test_context_free_argument_checks_need_no_gpu():
    # rejected on the host before any launch
    assert pg._lib.pg_sde_step_logprob(None, None, None, None, None, None, None, None, 4, 10, 1.0, 1.0, 1.0, 0, 0,
                                       None, None) == pg.PG_ESHAPE          # d not a multiple of 4
    assert pg._lib.pg_sde_step_logprob(None, None, None, None, None, None, None, None, 4, 16, 1.0, 1.0, 1.0, 0, 0,
                                       None, None) == pg.PG_EINVAL          # null pointers
    assert pg._lib.pg_ovf_select(None, None, None, -1, None, None, None, None, None, None) == pg.PG_EINVAL
    assert pg._lib.pg_ovf_select(None, None, None, 0, None, None, None, None, None, None) == pg.PG_OK
    assert pg._lib.pg_ovf_select_noalloc(None, None, None, pg.PG_OVF_NOALLOC_MAX_GROUPS + 1, None, None, None, None,
                                         None) == pg.PG_ESHAPE              # beyond the built-in scratch
    assert "at most" in pg.pg_last_error()
    assert pg._lib.pg_compact_gather(None, None, None, 0, 16, None) == pg.PG_OK      # empty input
    assert pg._lib.pg_group_advantages(None, None, 3, -1.0, None, None) == pg.PG_EINVAL
    assert pg.pg_step_scratch_floats(1024, 262144) == 1024 * 64
    assert "null" in pg.pg_last_error().lower() or len(pg.pg_last_error()) > 0
