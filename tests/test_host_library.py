"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side logic (decision rule, shortlist legality, cache file) behaves as specified.
No kernel is launched here."""
import os
import re

import numpy as np
import pytest

import oracle
from paper_2511_17594_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def ab():
    from paper_2511_17594_amd import binding
    return binding


@pytest.fixture()
def host(ab):
    h = ab.Handle(-1)
    yield h
    h.close()


def test_library_exports_every_declared_symbol(ab):
    header = open(os.path.join(ROOT, "include", "autosage.h")).read()
    declared = set(re.findall(r"\b(autosage_[a-z_0-9]+)\s*\(", header))
    declared -= {"autosage_ctx"}
    assert len(declared) >= 20
    import ctypes
    lib = ctypes.CDLL(ab.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), name
    assert set(ab.EXPORTED) == declared


def test_host_only_handle_refuses_compute(ab, host):
    with pytest.raises(ab.AutosageError) as ei:
        host.spmm(4, 4, None, None, None, None, None, 8, nnz=0, stream=0)
    assert ei.value.status == ab.ERR_UNSUPPORTED
    assert ab.status_string(ab.ERR_WORKSPACE_TOO_SMALL).startswith("workspace")


def test_decision_rule_matches_oracle_and_never_regresses(ab):
    rng = np.random.default_rng(1)
    for _ in range(3000):
        k = int(rng.integers(0, 6))
        t = np.round(rng.uniform(0.1, 2.0, k), 1)          # coarse values -> many exact ties
        tb = float(np.round(rng.uniform(0.1, 2.0), 1))
        alpha = float(rng.choice([0.5, 0.9, 0.95, 0.98, 1.0]))
        c = ab.decide_from_times(t, tb, alpha)
        assert c == oracle.decide(t, tb, alpha)
        assert (tb if c < 0 else t[c]) <= tb               # Proposition 1
    assert ab.decide_from_times([1.0, 1.0], 2.0, 0.95) == 0
    assert ab.decide_from_times([0.95], 1.0, 0.95) == 0
    assert ab.decide_from_times([], 1.0, 0.95) == -1


def test_params_and_baseline(ab, host):
    assert host.get_param("alpha") == pytest.approx(0.95)
    assert host.get_param("probe_frac") == pytest.approx(0.02)
    assert host.get_param("probe_min_rows") == 16384
    host.set_param("alpha", 0.98)
    assert host.get_param("alpha") == pytest.approx(0.98)
    for bad in (("alpha", 0.0), ("probe_frac", 1.5), ("probe_iters", 0), ("no_such_param", 1.0)):
        with pytest.raises(ab.AutosageError):
            host.set_param(*bad)
    b = ab.baseline_schedule()
    assert b.mapping == ab.MAP_PLAIN and b.hub_t == 0 and b.f_tile == 64
    # defaults and round trips of the later parameters
    assert host.get_param("baseline_bound") == 1 and host.get_param("softmax_group") == 0
    for name, value in (("baseline_bound", 0), ("softmax_group", 16), ("softmax_group", -1)):
        host.set_param(name, value)
        assert host.get_param(name) == value


def test_stream_probe_argument_checks_need_no_device(ab, host):
    """The probe's argument checks come before the device check; a host-only handle then refuses the launch."""
    assert host.stream_probe_dst_bytes() % 4 == 0 and host.stream_probe_dst_bytes() > 0
    import ctypes
    buf = (ctypes.c_char * 64)()
    aligned = (ctypes.addressof(buf) + 15) & ~15

    class FakeTensor:                                   # what the binding needs of a tensor: a pointer
        def __init__(self, ptr):
            self._ptr = ptr

        def data_ptr(self):
            return self._ptr

    good = FakeTensor(aligned)
    for args, status in (((ab.STREAM_COPY, good, good, 24), ab.ERR_INVALID_ARG),          # not a multiple of 16
                         ((ab.STREAM_COPY, FakeTensor(aligned + 4), good, 16), ab.ERR_INVALID_ARG),
                         ((9, good, good, 16), ab.ERR_INVALID_ARG),
                         ((ab.STREAM_COPY, good, good, 16), ab.ERR_UNSUPPORTED)):          # valid, but no device
        with pytest.raises(ab.AutosageError) as ei:
            host.stream_probe(*args, stream=0)
        assert ei.value.status == status


def test_workspace_bytes(ab, host):
    s = ab.Schedule()
    assert host.workspace_bytes(ab.OP_SPMM, 1000, 50000, 64, 1, s) == 256          # no hub split: minimum
    s.hub_t = 1024
    w1 = host.workspace_bytes(ab.OP_SPMM, 262144, 8388608, 64, 1, s)
    assert w1 >= (8388608 // 1024) * 64 * 4                                       # at least one partial row per chunk
    assert host.workspace_bytes(ab.OP_SPMM, 262144, 8388608, 64, 1, None) >= w1     # the selector bound covers it
    assert host.workspace_bytes(ab.OP_ATTENTION, 1000, 50000, 64, 8, None) >= 50000 * 8 * 4
    s.hub_t = 7
    with pytest.raises(ab.AutosageError):
        host.workspace_bytes(ab.OP_SPMM, 1000, 50000, 64, 1, s)


def hist_of(A):
    hist, mx = oracle.degree_histogram(A.rowptr)
    return hist.tolist(), mx


def test_shortlist_only_proposes_legal_vector_widths(ab, host):
    A = W.config2_powerlaw(n=20000, mean_deg=16.0, dmax=4096, seed=1)
    hist, mx = hist_of(A)
    # F = 602 is even but not a multiple of 4: 16-byte loads are illegal, 8-byte ones are fine
    c = host.shortlist(ab.OP_SPMM, A.n_rows, A.n_cols, A.nnz, hist, mx, 602, ab.F32, 16)
    assert c and all(s.vec_bytes in (4, 8) for s, _ in c) and any(s.vec_bytes == 8 for s, _ in c)
    # operands only 4-byte aligned: nothing wider than 4 bytes
    c = host.shortlist(ab.OP_SPMM, A.n_rows, A.n_cols, A.nnz, hist, mx, 64, ab.F32, 4)
    assert c and all(s.vec_bytes == 4 for s, _ in c)
    # aligned F = 64 ranks a 16-byte schedule first, estimates ascend, hub thresholds stay below the max degree
    c = host.shortlist(ab.OP_SPMM, A.n_rows, A.n_cols, A.nnz, hist, mx, 64, ab.F32, 16)
    assert c[0][0].vec_bytes == 16
    est = [e for _, e in c]
    assert est == sorted(est) and all(e > 0 for e in est)
    assert all(s.hub_t <= mx for s, _ in c)
    assert any(s.hub_t > 0 for s, _ in c[:6])             # a skewed graph gets hub candidates near the top
    # multi-row needs the dense row to fit half a wavefront: never offered at F = 256
    c = host.shortlist(ab.OP_SPMM, A.n_rows, A.n_cols, A.nnz, hist, mx, 256, ab.F32, 16)
    assert all(s.mapping == ab.MAP_WAVE_ROW for s, _ in c)
    # a regular graph without heavy rows gets no hub candidates at all
    B, _, _, _ = W.config1_tiny()
    hist, mx = hist_of(B)
    c = host.shortlist(ab.OP_SDDMM, B.n_rows, B.n_cols, B.nnz, hist, mx, 32, ab.F32, 16)
    assert c and all(s.hub_t == 0 for s, _ in c)


def test_cache_round_trip_and_corrupt_file(ab, host, tmp_path):
    s = ab.Schedule()
    s.mapping, s.vec_bytes, s.hub_t, s.hub_chunk, s.unroll, s.waves_per_wg = ab.MAP_WAVE_ROW, 16, 1024, 512, 4, 4
    host.cache_insert(0xDEADBEEF12345678, 64, ab.OP_SPMM, ab.F32, s)
    host.cache_insert(42, 128, ab.OP_SDDMM, ab.BF16, ab.baseline_schedule())
    fused = ab.Schedule(mapping=ab.MAP_FUSED, hub_t=512, hub_chunk=512, waves_per_wg=4)
    host.cache_insert(42, 64, ab.OP_ATTENTION, ab.BF16, fused, H=8)
    assert host.cache_lookup(42, 64, ab.OP_ATTENTION, ab.BF16, H=8).mapping == ab.MAP_FUSED
    assert host.cache_lookup(42, 64, ab.OP_ATTENTION, ab.BF16, H=4) is None         # heads are part of the key
    assert host.cache_lookup(0xDEADBEEF12345678, 64, ab.OP_SPMM, ab.F32).as_dict() == s.as_dict()
    assert host.cache_lookup(0xDEADBEEF12345678, 64, ab.OP_SDDMM, ab.F32) is None   # op is part of the key
    assert host.cache_lookup(0xDEADBEEF12345678, 32, ab.OP_SPMM, ab.F32) is None    # so is F
    path = str(tmp_path / "cache.txt")
    host.cache_save(path)
    assert not os.path.exists(path + ".tmp")
    h2 = ab.Handle(-1)
    h2.cache_load(path)
    assert h2.cache_lookup(0xDEADBEEF12345678, 64, ab.OP_SPMM, ab.F32).as_dict() == s.as_dict()
    assert h2.cache_lookup(42, 128, ab.OP_SDDMM, ab.BF16).mapping == ab.MAP_PLAIN
    assert h2.cache_lookup(42, 64, ab.OP_ATTENTION, ab.BF16, H=8).as_dict() == fused.as_dict()
    # records of another device signature, truncated and garbage lines are skipped, good lines still load
    lines = open(path).read().splitlines()
    with open(path, "w") as f:
        f.write("garbage line\n")
        f.write(lines[0][: len(lines[0]) // 2] + "\n")
        f.write(lines[0].replace(" host ", " some_other_gpu ") + "\n")
        f.write(lines[1] + "\n")
        f.write(lines[1].replace("autosage-cache-v3", "autosage-cache-v2") + "\n")      # records of an older schema are skipped
    h3 = ab.Handle(-1)
    h3.cache_load(path)
    found = [h3.cache_lookup(0xDEADBEEF12345678, 64, ab.OP_SPMM, ab.F32), h3.cache_lookup(42, 128, ab.OP_SDDMM, ab.BF16)]
    assert sum(x is not None for x in found) == 1
    with pytest.raises(ab.AutosageError) as ei:
        h3.cache_load(str(tmp_path / "missing.txt"))
    assert ei.value.status == ab.ERR_IO
    h3.cache_clear()
    assert h3.cache_lookup(42, 128, ab.OP_SDDMM, ab.BF16) is None
    h2.close()
    h3.close()


def test_env_toggles_are_read_at_creation(ab, monkeypatch, tmp_path):
    path = str(tmp_path / "auto_cache.txt")
    monkeypatch.setenv("AUTOSAGE_ALPHA", "0.9")
    monkeypatch.setenv("AUTOSAGE_PROBE_FRAC", "0.03")
    monkeypatch.setenv("AUTOSAGE_REPLAY_ONLY", "1")
    monkeypatch.setenv("AUTOSAGE_HUB_T", "2048")
    monkeypatch.setenv("AUTOSAGE_CACHE", path)
    h = ab.Handle(-1)
    assert h.get_param("alpha") == pytest.approx(0.9)
    assert h.get_param("probe_frac") == pytest.approx(0.03)
    assert h.get_param("replay_only") == 1
    assert h.get_param("force_hub_t") == 2048
    A = W.config2_powerlaw(n=20000, mean_deg=16.0, dmax=4096, seed=1)
    hist, mx = hist_of(A)
    c = h.shortlist(ab.OP_SPMM, A.n_rows, A.n_cols, A.nnz, hist, mx, 64, ab.F32, 16)
    assert c and all(s.hub_t == 2048 for s, _ in c)
    h.cache_insert(7, 64, ab.OP_SPMM, ab.F32, ab.baseline_schedule())
    h.close()                                               # AUTOSAGE_CACHE is written on destroy
    assert os.path.exists(path) and "autosage-cache-v3" in open(path).read()


def test_size_limits_are_checked_before_anything_else(ab, host):
    """nnz and n_rows up to 2^31 - 2^20 pass the argument check (the host-only handle then refuses to compute);
    one more is an invalid argument.  A hub chunk longer than 2^20 is refused, a threshold above it is not."""
    header = open(os.path.join(ROOT, "include", "autosage.h")).read()
    limit = int(re.search(r"#define AUTOSAGE_MAX_NNZ (\d+)LL", header).group(1))
    assert limit == (1 << 31) - (1 << 20)
    for nnz, status in ((limit, ab.ERR_UNSUPPORTED), (limit + 1, ab.ERR_INVALID_ARG)):
        with pytest.raises(ab.AutosageError) as ei:
            host.spmm(4, 4, None, None, None, None, None, 8, nnz=nnz, stream=0)
        assert ei.value.status == status
    with pytest.raises(ab.AutosageError) as ei:
        host.spmm(limit + 1, 4, None, None, None, None, None, 8, nnz=0, stream=0)
    assert ei.value.status == ab.ERR_INVALID_ARG
    s = ab.Schedule(hub_t=1 << 21)
    assert host.workspace_bytes(ab.OP_SPMM, 1000, 50000, 64, 1, s) >= 256
    s.hub_chunk = (1 << 20) + 1
    with pytest.raises(ab.AutosageError):
        host.workspace_bytes(ab.OP_SPMM, 1000, 50000, 64, 1, s)
    s.hub_chunk = 1 << 20
    assert host.workspace_bytes(ab.OP_SPMM, 1000, 50000, 64, 1, s) >= 256
