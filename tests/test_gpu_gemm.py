"""The projection GEMM kernel against a float64 product of the same half-
precision inputs, for every tile configuration, K split and output mode, on shapes that
span several tiles with ragged edges in M, N and K."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _ref(A, W):
    return A.double().cpu().numpy() @ W.double().cpu().numpy().T


@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (37, 344, 128), (200, 1000, 344), (256, 1536, 1536),
                                   (300, 2048, 1000), (130, 520, 8960),
                                   (5000, 1100, 512),    # more than 8 row tiles: the super-tile block map
                                   (8192, 1536, 640)])   # 192 tiles of 256 x 256: a partly filled last round
def test_gemm_all_configs(M, N, K):
    NO_SWIGLU = (22, 23, 25)  # one 32-column panel per wave: no gate/up pair in a wave
    ADD_ONLY = (24,)          # pieces of a tile add into C with atomics: the residual-add mode only
    import torch
    from paper_2505_24298_amd import binding
    L = binding.lib()
    g = torch.Generator(device="cuda").manual_seed(M * 7 + N)
    A = torch.randn((M, K), generator=g, device="cuda").to(torch.float16)
    W0 = (torch.randn((N, K), generator=g, device="cuda") * 0.05).to(torch.float16)
    W1 = (torch.randn((N, K), generator=g, device="cuda") * 0.05).to(torch.float16)
    ref0, ref1 = _ref(A, W0), _ref(A, W1)
    scale = np.abs(ref0).max()
    for cfg in list(range(L.areal_op_gemm_num_configs())) + [-1]:
        if cfg >= 7 and K % 64:
            # the direct-to-LDS configurations take whole 64-wide K slabs only
            with pytest.raises(binding.ArealError):
                binding.op_gemm(A, W0, None, torch.zeros((M, N), device="cuda"), 0, cfg, 1)
            continue
        for splits in (1, 3, -1):
            C = torch.zeros((M, N), device="cuda")
            if cfg in ADD_ONLY:
                with pytest.raises(binding.ArealError):
                    binding.op_gemm(A, W0, None, C, 0, cfg, splits)
            else:
                binding.op_gemm(A, W0, None, C, 0, cfg, splits)
                assert np.abs(C.cpu().numpy() - ref0).max() <= 2e-5 * scale * (K ** 0.5), (cfg, splits)
            base = torch.randn((M, N), generator=g, device="cuda")
            C = base.clone()
            binding.op_gemm(A, W0, None, C, 1, cfg, splits)
            assert np.abs(C.cpu().numpy() - (base.cpu().numpy() + ref0)).max() <= 2e-5 * scale * (K ** 0.5)
        Cb = torch.zeros((M, N), device="cuda", dtype=torch.float16)
        if cfg in NO_SWIGLU or cfg in ADD_ONLY:
            with pytest.raises(binding.ArealError):
                binding.op_gemm(A, W0, W1, Cb, 2, cfg, 1)
            continue
        binding.op_gemm(A, W0, W1, Cb, 2, cfg, 1)
        want = ref0 / (1.0 + np.exp(-ref0)) * ref1
        got = Cb.float().cpu().numpy()
        assert np.abs(got - want).max() <= 2 ** -10 * np.abs(want).max() + 1e-6, cfg


def test_stream_read_calibration_launch():
    """The read-only calibration kernel: runs over whole and ragged sizes without touching anything
    (the sink stays as it was), and refuses sizes that are not a multiple of 16 bytes."""
    import torch
    from paper_2505_24298_amd import binding
    buf = torch.empty(3 << 20, dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_()
    keep = buf.clone()
    sink = torch.full((16,), 7, dtype=torch.uint8, device="cuda")
    for off, n in ((0, 3 << 20), (4096, 65536 + 16), (16, 48), (0, 16)):
        binding.op_stream_read(buf, off, n, sink)
    torch.cuda.synchronize()
    assert torch.equal(buf, keep) and bool((sink == 7).all())
    with pytest.raises(binding.ArealError):
        binding.op_stream_read(buf, 0, 40, sink)
    with pytest.raises(binding.ArealError):
        binding.op_stream_read(buf, 0, 0, sink)
