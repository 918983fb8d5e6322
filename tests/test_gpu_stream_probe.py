"""The bandwidth-probe kernels move exactly the bytes they claim: read sums every element once, copy
reproduces the source, the in-place pass halves every element, the gather reads every indexed row once; ragged
sizes and bad arguments included."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def ab():
    from paper_2511_17594_amd import binding
    return binding


@pytest.mark.parametrize("n_floats", [0, 4, 1 << 10, (1 << 22) + 4 * 37, 3 * 256 * 2048 * 4 * 4])
def test_stream_probe_moves_every_byte_once(torch, ab, n_floats):
    h = ab.Handle(0)
    try:
        rng = np.random.default_rng(n_floats % 1000)
        host = rng.integers(-8, 9, size=n_floats).astype(np.float32)          # small integers: fp32 sums are exact
        src = torch.from_numpy(host).cuda()
        sums = torch.full((h.stream_probe_dst_bytes() // 4,), float("nan"), device="cuda")
        h.stream_probe(ab.STREAM_READ, src, sums, n_floats * 4)
        assert float(sums.double().sum()) == float(host.astype(np.float64).sum())
        dst = torch.full((n_floats + 8,), -1.0, device="cuda")
        h.stream_probe(ab.STREAM_COPY, src, dst, n_floats * 4)
        assert torch.equal(dst[:n_floats], src) and bool((dst[n_floats:] == -1.0).all())
        h.stream_probe(ab.STREAM_INPLACE, None, dst, n_floats * 4)
        assert torch.equal(dst[:n_floats], 0.5 * src) and bool((dst[n_floats:] == -1.0).all())
    finally:
        h.close()


def test_stream_probe_rejects_bad_arguments(torch, ab):
    h = ab.Handle(0)
    try:
        buf = torch.zeros(1024, device="cuda")
        for args in ((ab.STREAM_COPY, buf, buf[1:], 64), (ab.STREAM_COPY, buf, buf, 60), (ab.STREAM_COPY, None, buf, 64),
                     (7, buf, buf, 64), (ab.STREAM_READ, buf, None, 64)):
            with pytest.raises(ab.AutosageError) as e:
                h.stream_probe(*args)
            assert e.value.status == ab.ERR_INVALID_ARG
    finally:
        h.close()


@pytest.mark.parametrize("row_bytes", [16, 32, 64, 128, 256, 512, 1024])
@pytest.mark.parametrize("n_idx", [0, 1, 63, 64, 4096 + 17, 300001])
def test_gather_probe_reads_every_indexed_row_once(torch, ab, row_bytes, n_idx):
    h = ab.Handle(0)
    try:
        n_rows, w = 3001, row_bytes // 4
        rng = np.random.default_rng(row_bytes + n_idx)
        host = rng.integers(-4, 5, size=(n_rows, w)).astype(np.float32)      # small integers: fp32 sums are exact
        idx = rng.integers(0, n_rows, size=n_idx).astype(np.int32)
        if n_idx > 2:
            idx[0], idx[-1] = -5, n_rows + 9                                   # out-of-table values are clamped
        table = torch.from_numpy(host).cuda()
        d_idx = torch.from_numpy(idx).cuda()
        sums = torch.full((h.stream_probe_dst_bytes() // 4,), float("nan"), device="cuda")
        h.gather_probe(table, n_rows, row_bytes, d_idx, sums, n_idx=n_idx)
        want = float(host[np.clip(idx, 0, n_rows - 1)].astype(np.float64).sum())
        assert float(sums.double().sum()) == want
    finally:
        h.close()


def test_gather_probe_rejects_bad_arguments(torch, ab):
    h = ab.Handle(0)
    try:
        table = torch.zeros((16, 32), device="cuda")
        idx = torch.zeros(8, dtype=torch.int32, device="cuda")
        sums = torch.zeros(h.stream_probe_dst_bytes() // 4, device="cuda")
        for args in ((table, 16, 48, idx, sums), (table, 16, 2048, idx, sums), (table, 16, 8, idx, sums),
                     (table.view(-1)[1:], 15, 128, idx, sums), (table, 0, 128, idx, sums), (table, 16, 128, idx, None),
                     (None, 16, 128, idx, sums)):
            with pytest.raises(ab.AutosageError) as e:
                h.gather_probe(*args)
            assert e.value.status == ab.ERR_INVALID_ARG
    finally:
        h.close()
