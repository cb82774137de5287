"""GPU: the skinny GEMM path against a float64 matrix product on the same inputs."""
import numpy as np
import pytest

import paper_2407_19947_amd as pkg
import synth_inputs as si
from oracle import stairs_oracle as so

pytestmark = pytest.mark.gpu


def _ref(W, X):
    Wr = so._decode(W, np.float64)
    return X.astype(np.float64) @ Wr.T


# (N, K): tiles that end in the middle of a work-group, odd number of 256-wide k units (ragged
# last split-K slice), the benchmark shapes of the 125M model, one 7B shape
BF16_SHAPES = [(16, 256), (48, 768), (2304, 768), (6144, 768), (768, 3072), (32000, 768), (4096, 11008)]


@pytest.mark.parametrize("N,K", BF16_SHAPES)
@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 16, 17, 32])
def test_gemm_bf16(N, K, M):
    print(f"gemm bf16 N={N} K={K} M={M}", flush=True)
    rng = np.random.default_rng([N, K, M])
    W = si.bf16_round(rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02))
    X = rng.standard_normal((M, K), dtype=np.float32)
    Y = pkg.stairs_gemm_host(W, X)
    ref = _ref(W, X)
    # x is carried as bf16 hi + lo (~16 mantissa bits), products accumulate in fp32
    tol = 4e-5 * np.sqrt(K) * 0.02 * 4 + 1e-6
    assert np.max(np.abs(Y - ref)) < tol, np.max(np.abs(Y - ref))


@pytest.mark.parametrize("N,K", [(4, 4), (1024, 256), (768, 1024), (1024, 1028)])
@pytest.mark.parametrize("M", [1, 4, 5, 17, 32])
def test_gemm_fp32(N, K, M):
    print(f"gemm fp32 N={N} K={K} M={M}", flush=True)
    rng = np.random.default_rng([N, K, M, 1])
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    X = rng.standard_normal((M, K), dtype=np.float32)
    Y = pkg.stairs_gemm_host(W, X)
    assert np.max(np.abs(Y - _ref(W, X))) < 2e-6 * np.sqrt(K)


def test_gemm_rows_do_not_depend_on_batch():
    """Row i computed in a batch of M rows is bit-identical to row i computed alone."""
    rng = np.random.default_rng(5)
    for dt in ("bf16", "fp32"):
        W = rng.standard_normal((512, 768), dtype=np.float32) * np.float32(0.02)
        W = si.bf16_round(W) if dt == "bf16" else W
        X = rng.standard_normal((17, 768), dtype=np.float32)
        full = pkg.stairs_gemm_host(W, X)
        for i in (0, 3, 16):
            assert np.array_equal(pkg.stairs_gemm_host(W, X[i:i + 1])[0], full[i])
        assert np.array_equal(pkg.stairs_gemm_host(W, X[:5]), full[:5])


@pytest.mark.parametrize("K", [256, 768, 4096, 8192])
def test_both_bf16_gemm_kernels_give_the_same_bits(K):
    """Up to 4 rows take the kernel that keeps the whole activation block in LDS (when it fits: at K = 8192 only
    1 and 2 rows do), more rows the split-K kernel: the first m rows of a 16-row and of a 32-row batch must equal
    the m-row result bit for bit, whichever kernel computed it."""
    rng = np.random.default_rng([7, K])
    W = si.bf16_round(rng.standard_normal((272, K), dtype=np.float32) * np.float32(0.02))
    X = rng.standard_normal((32, K), dtype=np.float32)
    wide = pkg.stairs_gemm_host(W, X)
    mid = pkg.stairs_gemm_host(W, X[:16])
    assert np.array_equal(mid, wide[:16])
    for m in (1, 2, 3, 4, 5):
        assert np.array_equal(pkg.stairs_gemm_host(W, X[:m]), wide[:m]), m
    assert np.array_equal(pkg.stairs_gemm_host(W, X[7:10]), wide[7:10])


@pytest.mark.parametrize("M", [1, 3, 5, 17])
def test_activation_split_keeps_sixteen_bits(M):
    """The bf16 kernels carry an activation as a bf16 high part plus the bf16 of the remainder.  Against an identity
    matrix the product returns that pair's sum: exact for values of at most 16 significant bits (ties of the first
    rounding, both signs, a subnormal and a large value among them), within 2^-17 relative otherwise.  A dropped low
    part or a rounding that is not to nearest shows as an error of 2^-9."""
    print(f"activation split M={M}", flush=True)
    K = 256
    W = si.bf16_round(np.eye(K, dtype=np.float32))
    rng = np.random.default_rng([11, M])
    X = rng.standard_normal((M, K), dtype=np.float32) * np.float32(3.0)
    exact = X.copy()
    exact.view(np.uint32)[...] &= np.uint32(0xFFFFFF00)          # 16 significant bits
    special = np.array([1 + 2.0 ** -8, -(1 + 2.0 ** -8), 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -7 + 2.0 ** -15, 2.0 ** -130,
                        -3.0 * 2.0 ** 100, 0.0, 255.5], np.float32)
    exact[0, :special.size] = special
    assert np.array_equal(pkg.stairs_gemm_host(W, exact), exact)
    Y = pkg.stairs_gemm_host(W, X)
    assert np.all(np.abs(Y.astype(np.float64) - X) <= np.abs(X).astype(np.float64) * 2.0 ** -17)


@pytest.mark.parametrize("name", ["cfg1_tiny_fp32", "cfg2_125m"])
def test_timing_probes_run_on_both_dtypes(name):
    """Every mode of stairs_time_kernel returns a positive duration and the bytes it states, on an fp32 and a bf16
    pair (the benchmark calls them on whatever workload it is given), and leaves the context usable."""
    w = si.scaled_workload(name, target=dict(n_layers=2), draft=dict(kind="prefix", n_layers=1), P=40, G=8)
    target, draft = si.make_pair(w)
    prompt = si.make_prompt(w)
    with pkg.Stairs(target, draft, k_max=4, max_seq=128) as s:
        base, _ = s.generate(prompt, 8, 2)
        for which in range(11):
            ms, by = s.time_kernel(which, 3, 64, 4)
            assert ms > 0 and (by > 0 or which == 9), which
        again, _ = s.generate(prompt, 8, 2)
        assert np.array_equal(base, again)
