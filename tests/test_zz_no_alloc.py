"""GPU: stairs_gemm_device, the allocation-free variant of stairs_gemm_host (fixed scratch array inside the library),
against stairs_gemm_host on the same inputs: same kernels, same bits.  Two calls in a row on the same GPU, the second
with a smaller input (the array keeps the first call's contents), both dtypes, all three bf16 kernel paths (up to 4
rows, split-K, hand-off-free), limits rejected."""
import numpy as np
import pytest

import paper_2407_19947_amd as pkg
import synth_inputs as si

pytestmark = pytest.mark.gpu


def _device_gemm(W, X):
    """Inputs and output live in device memory the CALLER allocates (torch here); the library allocates nothing."""
    import torch
    dev = torch.device("cuda:0")
    if W.dtype == np.uint16:
        Wd = torch.from_numpy(W.view(np.int16)).to(dev)
        dt = 1
    else:
        Wd = torch.from_numpy(W).to(dev)
        dt = 0
    Xd = torch.from_numpy(X).to(dev)
    (N, K), M = W.shape, X.shape[0]
    Yd = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream().cuda_stream
    pkg.stairs_gemm_device(dt, Wd.data_ptr(), Xd.data_ptr(), Yd.data_ptr(), M, N, K, stream)
    torch.cuda.synchronize()
    return Yd.cpu().numpy()


def _inputs(N, K, M, bf16, seed):
    rng = np.random.default_rng([N, K, M, seed])
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    W = si.bf16_round(W) if bf16 else W
    X = rng.standard_normal((M, K), dtype=np.float32)
    return W, X


@pytest.mark.parametrize("bf16", [True, False])
def test_two_calls_in_a_row_match_the_allocating_entry_point(bf16):
    # first a large input, then a smaller one of every kernel path: leftovers of the first call must not show
    shapes = [(1024, 2048, 32), (272, 768, 3), (528, 512, 9), (8192, 256, 17), (3072, 512, 9), (2048, 256, 17), (16, 256, 1)] if bf16 else \
             [(1024, 1024, 32), (260, 516, 5), (4, 4, 1)]
    for i, (N, K, M) in enumerate(shapes):
        print(f"gemm_device bf16={bf16} N={N} K={K} M={M}", flush=True)
        W, X = _inputs(N, K, M, bf16, i)
        want = pkg.stairs_gemm_host(W, X)
        got = _device_gemm(W, X)
        assert np.array_equal(got, want), (N, K, M, float(np.max(np.abs(got - want))))
    # and the same input twice gives the same bits twice
    W, X = _inputs(512, 1024, 16, bf16, 99)
    a = _device_gemm(W, X)
    assert np.array_equal(a, _device_gemm(W, X))
    assert np.array_equal(a, pkg.stairs_gemm_host(W, X))


def test_shapes_beyond_the_fixed_scratch_are_rejected():
    import torch
    dev = torch.device("cuda:0")
    buf = torch.zeros(1 << 20, dtype=torch.float32, device=dev)
    p = buf.data_ptr()
    for dt, M, N, K in ((1, 1, 4096, 1024),        # bf16 weights of 8 MiB
                        (1, 32, 8192, 256),        # bf16 weights fit, 1 * 32 * 8192 * 4 partial sums = 1 MiB: accepted shape ...
                        (0, 32, 65536, 4),         # fp32 partial sums of 8 MiB
                        (1, 1, 16, 8448)):         # K beyond the fragment region
        if (dt, M, N, K) == (1, 32, 8192, 256):
            continue
        with pytest.raises(pkg.StairsError) as ei:
            pkg.stairs_gemm_device(dt, p, p, p, M, N, K, None)
        assert ei.value.code == -2, (dt, M, N, K)
    with pytest.raises(pkg.StairsError) as ei:
        pkg.stairs_gemm_device(1, p, p, p, 33, 16, 256, None)       # shape rules as stairs_gemm_host
    assert ei.value.code == -1
