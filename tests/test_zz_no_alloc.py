"""The entry point that allocates nothing, kg_op_linear_static, against kg_op_linear: same product,
bit-identical results, on two calls in a row that share the library's static staging array, the
second with a smaller input (fewer rows, shorter K, a K that leaves half of the last activation tile
unwritten), for bf16 and fp32 weights.  Also its limits: K beyond the static array is refused."""
import numpy as np
import pytest

from paper_2404_18911_amd import inputs as I

pytestmark = pytest.mark.gpu


def _pair(L, B, torch, dev, dtype, N, K, M, seed):
    """(y of kg_op_linear, y of kg_op_linear_static) for one seeded case."""
    rng = np.random.default_rng(seed)
    Wf = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    Wh = I.f32_to_bf16_bits(Wf) if dtype == 1 else Wf
    x = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32)).to(dev)
    w = torch.from_numpy(Wh.view(np.int16) if dtype else Wh).to(dev)
    packed = torch.empty(L.kg_op_packed_bytes(dtype, N, K), dtype=torch.uint8, device=dev)
    work = torch.empty(L.kg_op_work_bytes(K), dtype=torch.uint8, device=dev)
    s = torch.cuda.current_stream(dev).cuda_stream
    assert L.kg_op_pack(dtype, w.data_ptr(), N, K, packed.data_ptr(), s) == B.KG_OK
    y0 = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    y1 = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    assert L.kg_op_linear(dtype, packed.data_ptr(), N, K, x.data_ptr(), M, y0.data_ptr(), work.data_ptr(), s) == B.KG_OK
    assert L.kg_op_linear_static(dtype, packed.data_ptr(), N, K, x.data_ptr(), M, y1.data_ptr(), s) == B.KG_OK
    torch.cuda.synchronize(dev)
    return y0.cpu().numpy(), y1.cpu().numpy(), Wh, x.cpu().numpy()


@pytest.mark.parametrize("dtype", [1, 0])
def test_static_scratch_entry_point_equals_workspace_entry_point(dtype):
    import torch
    from paper_2404_18911_amd import binding as B
    L = B.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    # first call: the largest K the static array takes, 8 rows; second call: smaller in every way,
    # K = 1040 = 32 * 32 + 16 (the upper half of its last activation tile is never written)
    for N, K, M, seed in ((1024, 16384, 8, 5), (272, 1040, 3, 6)):
        y0, y1, Wh, x = _pair(L, B, torch, dev, dtype, N, K, M, seed)
        assert np.isfinite(y0).all() and np.isfinite(y1).all()
        assert np.array_equal(y0, y1), float(np.abs(y0 - y1).max())
        # and both are the product: fp64 reference within the projection kernel's bound
        W64 = (I.bf16_bits_to_f32(Wh) if dtype else Wh).astype(np.float64)
        ref = x.astype(np.float64) @ W64.T
        bound = (np.abs(x.astype(np.float64)) @ np.abs(W64).T) * 2.0 ** -15 + 1e-6
        assert np.all(np.abs(y1 - ref) <= bound)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2404_18911_amd import binding as B
    L = B.lib()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    t = torch.zeros(1 << 20, dtype=torch.uint8, device=dev)
    s = torch.cuda.current_stream(dev).cuda_stream
    assert L.kg_op_linear_static(1, t.data_ptr(), 16, 16384 + 32, t.data_ptr(), 1, t.data_ptr(), s) == B.KG_ENOSPC
    assert L.kg_op_linear_static(1, t.data_ptr(), 16, 64, t.data_ptr(), 9, t.data_ptr(), s) == B.KG_EINVAL
    assert L.kg_op_linear_static(1, None, 16, 64, t.data_ptr(), 1, t.data_ptr(), s) == B.KG_EINVAL
    torch.cuda.synchronize(dev)
