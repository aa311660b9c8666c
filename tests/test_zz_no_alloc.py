"""subgen_exact_attend_noalloc (the entry point that allocates nothing; its split partials live in a buffer inside
the library) against subgen_exact_attend with a caller workspace: two calls in a row through the C ABI, the second
with a smaller input, so that the shared buffer still holds the first call's partials when the second one runs."""
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(S, n, d, g, dtype, seed):
    gen = torch.Generator(device="cpu").manual_seed(seed)
    K = torch.randn(S, n, d, generator=gen).to(dtype).to(DEV)
    V = torch.randn(S, n, d, generator=gen).to(dtype).to(DEV)
    Q = (torch.randn(S, g, d, generator=gen) / d ** 0.5 * 3).to(dtype).to(DEV)
    return K, V, Q


@pytest.mark.parametrize("dtype,d,g", [(torch.bfloat16, 128, 4), (torch.float32, 64, 1)])
def test_noalloc_entry_point_equals_the_workspace_one_twice_in_a_row(dtype, d, g):
    from paper_2402_06082_amd import binding as b
    L = b.load()
    assert L.subgen_exact_noalloc_max_bytes() == 32 << 20
    for S, n, seed in [(37, 9000, 1), (5, 700, 2)]:          # many splits per stream, then fewer streams and rows
        K, V, Q = make(S, n, d, g, dtype, seed)
        ref = b.exact_attend(K, V, Q)                         # existing entry point, caller workspace
        out = torch.full((S, g, d), float("nan"), dtype=torch.float32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(DEV)
        b.exact_attend_noalloc(K, V, Q, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(DEV) == before
        assert torch.isfinite(out).all()
        assert torch.equal(out, ref), (S, n, (out - ref).abs().max().item())   # same kernels, same split: same bits


def test_noalloc_entry_point_rejects_sizes_beyond_its_buffer():
    from paper_2402_06082_amd import binding as b
    L = b.load()
    S, d, g = 70000, 128, 4                                  # 70000 x 4 x 130 floats of partials: beyond 32 MiB
    assert L.subgen_exact_workspace_bytes(S, 8, d, g) > L.subgen_exact_noalloc_max_bytes()
    K, V, Q = make(S, 8, d, g, torch.bfloat16, 3)
    out = torch.zeros(S, g, d, dtype=torch.float32, device=DEV)
    with pytest.raises(b.SubgenError) as e:
        b.exact_attend_noalloc(K, V, Q, out)
    assert e.value.code == -5
    assert torch.equal(b.exact_attend(K, V, Q), b.exact_attend(K, V, Q))      # the workspace entry point still takes it
