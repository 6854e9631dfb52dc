"""The library's host-side evaluator against the paper's printed figures and
against the exact-rational closed forms of oracle/placement.py."""
import random
import re
import os

import pytest

import paper_2601_02311_amd as ps
from oracle import placement as pl
from synth import WORKLOADS

GB = 10 ** 9
MODE = {"R": ps.PS_R, "S": ps.PS_S, "S*": ps.PS_SG, "M": ps.PS_M, "O": ps.PS_O}


def test_printed_figures(golden):
    P, N = int(golden["P_70b"]), int(golden["N_example"])
    dp = ps.ps_cost_eval(ps.ps_spec_preset("dp", N, 0, P))
    z3 = ps.ps_cost_eval(ps.ps_spec_preset("zero3", N, 0, P))
    assert dp.theta_bytes == int(golden["theta_GB"]) * GB
    assert dp.grad_bytes == int(golden["grad_GB"]) * GB
    assert dp.omega_bytes == (int(golden["master_GB"]) + int(golden["adam_mv_GB"])) * GB
    assert dp.peak_total == int(golden["model_state_GB"]) * GB == int(golden["bytes_per_param"]) * P
    assert z3.peak_total == int(golden["zero3_per_device_GB"]) * GB
    assert dp.peak_total == int(golden["memory_reduction"]) * z3.peak_total
    assert dp.comm_total_bytes == float(golden["dp_comm_P_times"]) * P
    assert z3.comm_total_bytes == float(golden["zero3_comm_P_times"]) * P
    assert round(dp.comm_total_bytes / GB) == int(golden["dp_comm_GB_approx"])
    assert round(z3.comm_total_bytes / GB) == int(golden["zero3_comm_GB_approx"])
    # exactly 3/2 on the integer fields
    assert 2 * (z3.comm_grad_sync_xN + z3.comm_param_gather_xN) == 3 * dp.comm_grad_sync_xN


def test_table2_presets_match_closed_forms():
    P, N = 70 * 10 ** 9, 8
    for name, modes in pl.STRATEGIES.items():
        spec = ps.ps_spec_preset(name, N, 3, P)
        assert (spec.theta, spec.omega, spec.grad, spec.act) == tuple(MODE[m] for m in modes)
        c = ps.ps_cost_eval(spec)
        assert c.peak_total == pl.memory(modes, P, N)
        assert c.comm_grad_sync_xN + c.comm_param_gather_xN == pl.communication(modes, P, N) * N
    # values derived (not printed) from the paper's rules at 70B, N = 8
    assert ps.ps_cost_eval(ps.ps_spec_preset("zero1", N, 0, P)).peak_total == 385 * GB
    z2 = ps.ps_cost_eval(ps.ps_spec_preset("zero2", N, 0, P))
    assert z2.peak_total == 262.5 * GB and z2.comm_total_bytes == 122.5 * GB
    assert z2.implied_update_gather_xN == 7 * 140 * GB      # reported, never added in
    assert ps.ps_cost_eval(ps.ps_spec_preset("zero_offload", N, 0, P)).peak_total == 17.5 * GB
    assert ps.ps_cost_eval(ps.ps_spec_preset("fsdp", N, 0, P)).peak_total == 140 * GB
    with pytest.raises(ps.PsError) as e:
        ps.ps_spec_preset("zero9", N, 0, P)
    assert e.value.status == ps.PS_EINVAL


def test_random_specs_match_closed_forms():
    rnd = random.Random(5)
    modes = list(MODE)
    for _ in range(300):
        N = rnd.choice([1, 2, 3, 4, 6, 8, 16, 64])
        P = N * rnd.randrange(1, 10 ** 9)
        m = [rnd.choice(modes) for _ in range(4)]
        s_unit = rnd.choice([0, 12 * 8192 * 8192 * 2])
        act = N * rnd.randrange(0, 10 ** 9)
        spec = ps.ps_spec_t(MODE[m[0]], MODE[m[1]], MODE[m[2]], MODE[m[3]], N, rnd.randrange(N),
                            P, 0, 0, s_unit, act)
        c = ps.ps_cost_eval(spec)
        assert c.peak_total == pl.memory(tuple(m), P, N, s_unit, act)
        assert c.persistent_total + c.transient_bytes == c.peak_total
        assert c.comm_grad_sync_xN + c.comm_param_gather_xN == pl.communication(tuple(m), P, N) * N
        assert (c.psi_padded, c.shard_offset, c.shard_len, c.valid_len) == \
            pl.shard_geometry(P, N, spec.shard_index)


def test_shard_geometry_with_padding_and_workloads():
    for psi, N, a in [(25, 4, 8), (1535, 6, 256), (1537, 6, 256), (13_015_864_320 - 1001, 6, 256)]:
        for i in range(N):
            spec = ps.ps_spec_preset("zero3", N, i, psi, align_elems=a)
            c = ps.ps_cost_eval(spec)
            assert (c.psi_padded, c.shard_offset, c.shard_len, c.valid_len) == \
                pl.shard_geometry(psi, N, i, a)
    for w in WORKLOADS.values():
        c = ps.ps_cost_eval(ps.ps_spec_preset(w.strategy, w.n_devices, w.shard_index, w.psi,
                                               align_elems=w.align_elems))
        assert (c.psi_padded, c.shard_offset, c.shard_len, c.valid_len) == \
            (w.psi_padded, w.shard_offset, w.shard_len, w.valid_len)
    # the sizes the workload descriptions quote
    assert WORKLOADS["tiny"].shard_len == 262_144
    assert WORKLOADS["gpt2s"].shard_len == 15_554_976
    assert WORKLOADS["7b_zero2"].shard_len == 842_301_952
    assert WORKLOADS["70b_zero3"].shard_len == 8_750_000_000
    assert WORKLOADS["13b_clip"].shard_len == 2_169_310_720
    z = ps.ps_cost_eval(ps.ps_spec_preset("zero2", 8, 0, WORKLOADS["7b_zero2"].psi))
    assert round(z.omega_bytes / GB, 1) == 10.1
    z = ps.ps_cost_eval(ps.ps_spec_preset("zero3", 8, 7, WORKLOADS["70b_zero3"].psi))
    assert z.omega_bytes == 105 * GB and z.theta_bytes == 17.5 * GB


def test_errors():
    def status(fn):
        with pytest.raises(ps.PsError) as e:
            fn()
        return e.value.status
    assert status(lambda: ps.ps_cost_eval(None)) == ps.PS_EINVAL
    assert status(lambda: ps.ps_cost_eval(ps.ps_spec_preset("dp", 0, 0, 8))) == ps.PS_EINVAL
    assert status(lambda: ps.ps_cost_eval(ps.ps_spec_preset("dp", 4, 4, 8))) == ps.PS_ERANGE
    assert status(lambda: ps.ps_cost_eval(ps.ps_spec_preset("zero3", 4, 0, 10))) == ps.PS_ERANGE
    bad = ps.ps_spec_preset("dp", 4, 0, 8)
    bad.theta = 7
    assert status(lambda: ps.ps_cost_eval(bad)) == ps.PS_EINVAL
    assert status(lambda: ps.ps_cost_eval(ps.ps_spec_preset("dp", 4, 0, 2 ** 62))) == ps.PS_ERANGE
    assert "overflow" in ps.ps_last_error()
    assert ps.ps_cost_eval(ps.ps_spec_preset("zero3", 4, 0, 10, align_elems=2)).psi_padded == 16


def test_header_symbols_are_exported_and_bound():
    """Every function include/ps_step.h declares is exported by the built library."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    text = open(os.path.join(root, "include", "ps_step.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(ps_[a-z_0-9]+)\s*\(", text))
    assert declared == set(ps.EXPORTED_SYMBOLS)
    L = ps.library()
    for name in declared:
        assert getattr(L, name) is not None
    assert ps.ps_abi_version() == ps.ABI_VERSION == int(re.search(r'#define PS_ABI_VERSION (\d+)u', text).group(1))
    assert ps.ps_status_string(ps.PS_EALIGN).startswith("pointer")


def test_clip_coef_against_the_oracle():
    import math
    from oracle import step as orc
    for ss, others, mx in [(4.0, 12.0, 1.0), (1e-9, 0.0, 1.0), (3.7, 5 * 3.7, 0.5), (0.0, 0.0, 1.0),
                           (1e30, 1e30, 1e-3)]:
        assert ps.ps_clip_coef(ss, others, mx) == orc.clip_coef(ss, others, mx)
    assert ps.ps_clip_coef(4.0, 12.0, 1.0) == 1.0 / (4.0 + 1e-6)
    assert ps.ps_clip_coef(1e-12, 0.0, 1.0) == 1.0
    for bad in [(math.inf, 0.0, 1.0), (math.nan, 0.0, 1.0), (-1.0, 0.0, 1.0), (1.0, 1.0, 0.0)]:
        assert math.isnan(ps.ps_clip_coef(*bad))


def test_strategy_selection_against_the_oracle():
    rnd = random.Random(11)
    GBy = 10 ** 9
    cases = [(70 * GBy, 80 * GBy, 8, 30 * GBy, True), (70 * GBy, 80 * GBy, 8, 30 * GBy, False),
             (70 * GBy, 80 * GBy, 8, 20 * GBy, True), (1 * GBy, 80 * GBy, 8, 0, False),
             (7 * GBy, 80 * GBy, 8, 0, True), (7, 160, 8, 0, False), (7, 161, 8, 0, False),
             (7 * GBy, 288 * GBy, 8, 0, False), (70 * GBy, 288 * GBy, 8, 0, False),
             (2 ** 60, 2 ** 62, 3, 2 ** 61, True)]
    for _ in range(300):
        cases.append((rnd.randrange(1, 10 ** 12), rnd.randrange(1, 10 ** 12), rnd.choice([1, 2, 8, 64]),
                      rnd.randrange(0, 10 ** 12), rnd.random() < 0.5))
    for P, M, N, L, fast in cases:
        want_modes, want_tp = pl.select_strategy(P, M, N, L, fast)
        spec, fits, tp = ps.ps_select_strategy(P, M, N, L, fast)
        assert (spec.theta, spec.omega, spec.grad, spec.act) == tuple(MODE[m] for m in want_modes)
        assert tp == want_tp and (spec.n_devices, spec.psi) == (N, P)
        per_device = 16 * P if want_modes == pl.STRATEGIES["dp"] else 16 * P / N
        assert fits == (per_device * 10 < 7 * M if isinstance(per_device, int) else 160 * P < 7 * M * N)
    spec, fits, tp = ps.ps_select_strategy(70 * GBy, 80 * GBy, 8, 30 * GBy, True)
    assert (not fits) and tp                       # the paper's 70B on 80 GB devices: ZeRO-3 + TP
    with pytest.raises(ps.PsError):
        ps.ps_select_strategy(1, 1, 0)


def test_composition_index_against_the_oracle(golden):
    for A, B in [(4, 2), (1, 8), (8, 1), (3, 5), (2, 2)]:
        tp, dp = pl.tp_dp_groups(A, B)
        stages, pipes = pl.pp_dp_groups(B, A)      # pipeline x data: inner = replicas per stage
        for d in range(A * B):
            ig, ir, og, orank = ps.ps_compose_index(A, B, d)
            assert tp[ig][ir] == d and dp[og][orank] == d
            assert stages[ig][ir] == d and pipes[og][orank] == d
    T, D = int(golden["fig2_tp_degree"]), int(golden["fig2_dp_degree"])
    assert ps.ps_compose_index(T, D, 6) == (1, 2, 2, 1)     # Figure 2: device 6 = TP group 1, syncs with 2
    with pytest.raises(ps.PsError) as e:
        ps.ps_compose_index(4, 2, 8)
    assert e.value.status == ps.PS_ERANGE
    with pytest.raises(ps.PsError) as e:
        ps.ps_compose_index(0, 2, 0)
    assert e.value.status == ps.PS_EINVAL


def test_composed_cost_per_device_and_per_group(golden):
    """Definition 5 / Theorems 6-7: the outer data-parallel family rules act on the 1/inner
    share an inner strategy leaves each device, among the D devices holding that share."""
    P = int(golden["P_70b"])
    T, D = int(golden["fig2_tp_degree"]), int(golden["fig2_dp_degree"])       # Figure 2: TP(4) x DP(2)
    c = ps.ps_compose_cost(ps.ps_spec_preset("dp", D, 0, P), T)
    assert c.peak_total == 16 * P // T == 280 * GB                             # a quarter of 1120 GB
    assert c.comm_grad_sync_xN == 2 * (D - 1) * (2 * P // T) and c.comm_total_bytes == 35 * GB
    z3 = ps.ps_compose_cost(ps.ps_spec_preset("zero3", D, 0, P), T)
    assert z3.peak_total == 16 * P // (T * D) == 140 * GB                      # same bytes as ZeRO-3 over 8
    assert 2 * (z3.comm_grad_sync_xN + z3.comm_param_gather_xN) == 3 * c.comm_grad_sync_xN   # 1.5x inside the group
    # against the exact closed forms, including the three-way case inner = T * K
    for name, modes in pl.STRATEGIES.items():
        for inner, Dg in [(1, 8), (4, 2), (2, 4), (8, 4), (16, 1), (7, 5)]:
            Pm = 70 * 10 ** 9 // (7 * 16 * 5 * 8) * (7 * 16 * 5 * 8)
            got = ps.ps_compose_cost(ps.ps_spec_preset(name, Dg, 0, Pm), inner)
            mem, comm = pl.composed_cost(modes, Pm, inner, Dg)
            assert got.peak_total == mem, (name, inner, Dg)
            assert got.comm_grad_sync_xN + got.comm_param_gather_xN == comm * Dg
            assert got.psi_padded == Pm // inner
    # inner = 1 is the outer strategy itself; one outer device means no data-parallel traffic
    spec = ps.ps_spec_preset("zero2", 8, 3, P)
    a, b = ps.ps_cost_eval(spec), ps.ps_compose_cost(spec, 1)
    assert bytes(a) == bytes(b)
    assert ps.ps_compose_cost(ps.ps_spec_preset("dp", 1, 0, P), 8).comm_total_bytes == 0.0
    with pytest.raises(ps.PsError) as e:
        ps.ps_compose_cost(spec, 0)
    assert e.value.status == ps.PS_EINVAL
    with pytest.raises(ps.PsError) as e:
        ps.ps_compose_cost(spec, 3)            # 70e9 is not a multiple of 3
    assert e.value.status == ps.PS_ERANGE


def test_corollary1_on_the_library():
    """Corollary 1 on the evaluator's integer fields, for several N and sizes: sharding Omega
    leaves communication alone and saves (N-1)/N of 12 psi; sharding G halves gradient
    synchronisation; S* for Theta adds exactly two All-Gathers of |Theta|."""
    rnd = random.Random(11)
    for _ in range(50):
        N = rnd.choice([2, 3, 4, 6, 8, 16, 64, 512])
        P = N * rnd.randrange(1, 10 ** 9)
        dp, z1, z2, z3 = (ps.ps_cost_eval(ps.ps_spec_preset(k, N, 0, P)) for k in ("dp", "zero1", "zero2", "zero3"))
        total = lambda c: c.comm_grad_sync_xN + c.comm_param_gather_xN
        assert total(z1) == total(dp)
        assert (dp.peak_total - z1.peak_total) * N == 12 * P * (N - 1)
        assert 2 * total(z2) == total(z1)
        assert total(z3) - total(z2) == 2 * (N - 1) * 2 * P
        assert z3.peak_total * N == 16 * P and z2.peak_total * N == 2 * P * N + 14 * P


def test_a_library_built_from_other_sources_counts_as_stale(tmp_path, monkeypatch):
    """The binding rebuilds (or refuses to load) a library whose recorded source hash differs
    from the sources on disk, whatever the time stamps say."""
    from paper_2601_02311_amd import build
    assert not build.stale()                              # the library in the tree matches its sources
    monkeypatch.setattr(build, "BUILD_ID", str(tmp_path / "id"))
    assert build.stale()                                  # no record of what it was built from
    (tmp_path / "id").write_text("0" * 64 + "\n")
    assert build.stale()                                  # built from something else
    (tmp_path / "id").write_text(build.source_id() + "\n")
    assert not build.stale()


def test_public_header_is_plain_c():
    """include/ps_step.h is the boundary: it must compile as C11 and as C++17 on its own,
    with no HIP, torch or library-internal type in sight."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hdr = os.path.join(root, "include", "ps_step.h")
    for cmd in (["gcc", "-std=c11", "-x", "c"], ["g++", "-std=c++17", "-x", "c++"]):
        p = subprocess.run(cmd + ["-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", hdr],
                           stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert p.returncode == 0, p.stdout
    text = open(hdr).read()
    assert "hip/" not in text and "torch" not in text
