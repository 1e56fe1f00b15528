"""e2eg_layer_transform_noalloc (scratch memory in a static device array, nothing allocated) against
e2eg_layer_transform (caller's workspace): the same results bit for bit, through the C ABI, on two
calls in a row of which the second is smaller (it must not see what the first left in the array),
and a clear error past the array's size."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_20564_amd import binding
    binding.load_library()
    return binding


def case(n, fin, fout, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    P = torch.randn(n, fin, device="cuda", generator=g).to(torch.bfloat16)
    W = (torch.randn(fin, fout, device="cuda", generator=g) / fin ** 0.5).to(torch.bfloat16)
    gH = torch.randn(n, fout, device="cuda", generator=g).to(torch.bfloat16)
    return P, W, gH


def run_both(B, n, fin, fout, relu, seed):
    P, W, gH = case(n, fin, fout, seed)
    stream = torch.cuda.current_stream().cuda_stream
    out = {}
    for name in ("workspace", "noalloc"):
        H = torch.full((n, fout), float("nan"), device="cuda", dtype=torch.bfloat16)
        gP = torch.full((n, fin), float("nan"), device="cuda", dtype=torch.bfloat16)
        gW = torch.full((fin, fout), float("nan"), device="cuda", dtype=torch.float32)
        if name == "workspace":
            for mode in (B.E2EG_TRANSFORM_FWD, B.E2EG_TRANSFORM_BWD):
                ws = torch.empty(max(B.e2eg_layer_transform_workspace_bytes(mode, n, fin, fout, B.E2EG_BF16), 256),
                                 dtype=torch.uint8, device="cuda")
                B.e2eg_layer_transform(mode, n, fin, fout, B.E2EG_BF16, int(relu), P, W, H, gH, gP, gW, ws, None, stream)
        else:
            for mode in (B.E2EG_TRANSFORM_FWD, B.E2EG_TRANSFORM_BWD):
                B.e2eg_layer_transform_noalloc(mode, n, fin, fout, B.E2EG_BF16, int(relu), P, W, H, gH, gP, gW, stream)
        torch.cuda.synchronize()
        out[name] = (H, gP, gW)
    for a, b, what in zip(out["workspace"], out["noalloc"], ("H", "dP", "dW")):
        assert not bool(torch.isnan(a.float()).any()), what
        assert torch.equal(a, b), f"{what} differs for n={n}, {fin}x{fout}, relu={relu}"
    return out["noalloc"]


def test_noalloc_matches_the_workspace_call_twice_in_a_row(B):
    # a large call first, then a smaller one that reuses the front of the same static array
    big = run_both(B, 150_001, 128, 128, True, seed=1)
    small = run_both(B, 3_333, 128, 128, True, seed=2)
    # the small case again after another large one with other shapes: still the same bits
    run_both(B, 8_000, 256, 256, False, seed=3)
    again = run_both(B, 3_333, 128, 128, True, seed=2)
    for a, b in zip(small, again):
        assert torch.equal(a, b)
    run_both(B, 1, 64, 32, True, seed=4)        # a single row
    del big


def test_noalloc_refuses_what_the_static_array_cannot_hold(B):
    n, f = 100_000, 256      # 256 x 256 partial matrices of more than 64 workgroups pass 16 MiB
    assert B.e2eg_layer_transform_workspace_bytes(B.E2EG_TRANSFORM_BWD, n, f, f, B.E2EG_BF16) > 16 << 20
    P, W, gH = case(n, f, f, 5)
    H = torch.empty(n, f, device="cuda", dtype=torch.bfloat16)
    gP = torch.empty_like(P)
    gW = torch.empty(f, f, device="cuda", dtype=torch.float32)
    stream = torch.cuda.current_stream().cuda_stream
    B.e2eg_layer_transform_noalloc(B.E2EG_TRANSFORM_FWD, n, f, f, B.E2EG_BF16, 1, P, W, H, None, None, None, stream)
    with pytest.raises(B.E2egError) as e:
        B.e2eg_layer_transform_noalloc(B.E2EG_TRANSFORM_BWD, n, f, f, B.E2EG_BF16, 1, P, W, H, gH, gP, gW, stream)
    assert e.value.status == B.E2EG_ERR_CAPACITY and "static array" in str(e.value)
    torch.cuda.synchronize()
