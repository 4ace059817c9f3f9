"""The two instrumentation kernels of the library.  bns_probe_gather, the bare access pattern of the
aggregate used by bench.py as this machine's ceiling: every wavefront's row must be the plain sum of
the table rows its indices name.  bns_probe_mfma, the bare matrix instruction of the update: its
checksum must be what that many products add up to."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,per_wave,n_idx", [(128, 22, 100_003), (16, 7, 5000), (256, 300, 70_001), (64, 64, 64 * 50), (32, 1, 999)])
def test_probe_sums_the_rows_it_is_told_to(d, per_wave, n_idx):
    import torch
    import paper_2203_10983_amd as pkg
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(d + per_wave)
    n_rows = 4099
    table = rng.standard_normal((n_rows, d)).astype(np.float32)
    idx = rng.integers(0, n_rows, size=n_idx).astype(np.int32)
    waves = (n_idx + per_wave - 1) // per_wave
    out = torch.full((waves + 1, d), 7.0, dtype=torch.float32, device=dev)
    pkg.probe_gather(torch.from_numpy(table).to(dev), torch.from_numpy(idx).to(dev), per_wave, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    pad = waves * per_wave - n_idx
    rows = table.astype(np.float64)[np.concatenate([idx, np.zeros(pad, np.int32)])]
    rows[n_idx:] = 0.0
    want = rows.reshape(waves, per_wave, d).sum(axis=1)
    abs_sum = np.abs(rows).reshape(waves, per_wave, d).sum(axis=1)
    assert np.all(np.abs(got[:waves] - want) <= 1e-4 * np.maximum(np.abs(want), 1e-6) + 4 * 2.0 ** -24 * np.sqrt(per_wave) * abs_sum)
    assert np.all(got[waves] == 7.0), "the row past the last wavefront must stay untouched"


def test_probe_rejects_bad_arguments():
    import torch
    import paper_2203_10983_amd as pkg
    dev = torch.device("cuda:0")
    t = torch.zeros(8, 100, dtype=torch.float32, device=dev)      # width 100 is not one the probe runs at
    i = torch.zeros(8, dtype=torch.int32, device=dev)
    o = torch.zeros(8, 100, dtype=torch.float32, device=dev)
    with pytest.raises(pkg.BnsError):
        pkg.probe_gather(t, i, 4, o)
    with pytest.raises(pkg.BnsError):
        pkg.probe_gather(torch.zeros(8, 128, dtype=torch.float32, device=dev), i, 0, o)


@pytest.mark.parametrize("n_acc,waves,iters", [(1, 4, 1), (4, 16, 3), (6, 8, 2), (2, 1, 5)])
def test_mfma_probe_adds_up(n_acc, waves, iters):
    """Every product adds sum_k A[i][k] B[k][j] with A[i][k] = 1 + 1e-6 * (lane i + 32 k) and B = 0.5 to
    C[i][j]; thread 0 of a workgroup holds C[8 (r / 4) + r % 4][0] in register r and stores the sum
    over its registers and accumulators."""
    import torch
    import paper_2203_10983_amd as pkg
    dev = torch.device("cuda:0")
    blocks = 5
    out = torch.full((blocks + 1,), 7.0, dtype=torch.float32, device=dev)
    pkg.probe_mfma(n_acc, waves, blocks, iters, out)
    torch.cuda.synchronize()
    a = lambda lane: 1.0 + 1e-6 * lane  # noqa: E731
    per_product = sum(0.5 * (a(8 * (r // 4) + r % 4) + a(8 * (r // 4) + r % 4 + 32)) for r in range(16))
    want = n_acc * 8 * iters * per_product
    got = out.cpu().numpy()
    assert np.allclose(got[:blocks], want, rtol=1e-5), (got, want)
    assert got[blocks] == 7.0


def test_mfma_probe_rejects_bad_arguments():
    import torch
    import paper_2203_10983_amd as pkg
    out = torch.zeros(4, dtype=torch.float32, device="cuda:0")
    for args in ((5, 4, 1, 1), (4, 17, 1, 1), (4, 0, 1, 1), (4, 4, 0, 1), (4, 4, 1, -1)):
        with pytest.raises(pkg.BnsError):
            pkg.probe_mfma(*args, out)
