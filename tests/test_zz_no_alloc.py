"""The allocation-free accept / resample entry point against the allocating one it is a variant of: same inputs,
same (A, y), on two calls in a row, the second with a smaller input (fewer drafted tokens, a smaller vocabulary), so
that whatever the first call left in the shared scratch array would show."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(rng, k, vocab):
    ql = (rng.standard_normal((k, vocab)) * 2.0).astype(np.float32)
    pl = (np.concatenate([ql, ql[-1:]], 0) + rng.standard_normal((k + 1, vocab)).astype(np.float32)).astype(np.float32)
    drafted = rng.integers(0, vocab, size=k).astype(np.int32)
    # make the first tokens likely under both models so that accepts and refusals both occur
    for i in range(k):
        if i % 2 == 0:
            drafted[i] = int(np.argmax(ql[i]))
    return pl, ql, drafted


@pytest.mark.parametrize("temperature", [0.0, 0.7, 1.0])
def test_static_scratch_accept_equals_allocating_accept(temperature):
    import paper_2504_00030_amd as pk
    pk.load()
    rng = np.random.default_rng(17 + int(10 * temperature))
    stream = torch.cuda.current_stream().cuda_stream
    seen = set()
    # large call, then smaller ones (k and vocab both shrink), then a large one again
    for step, (k, vocab) in enumerate([(16, 128256), (5, 32000), (1, 1000), (64, 40000), (3, 4099), (8, 262144)]):
        pl, ql, drafted = _case(rng, k, vocab)
        p_d, q_d = torch.from_numpy(pl).cuda(), torch.from_numpy(ql).cuda()
        d_d = torch.from_numpy(drafted).cuda()
        want = torch.full((2,), -7, dtype=torch.int32, device="cuda")
        got = torch.full((2,), -9, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        pk.k_accept(p_d, q_d, d_d, temperature, 11, step, want, stream)
        pk.k_accept_static(p_d, q_d, d_d, temperature, 11, step, got, stream)
        torch.cuda.synchronize()
        w, g = want.cpu().tolist(), got.cpu().tolist()
        assert g == w, f"call {step} (k {k}, vocab {vocab}, T {temperature}): static {g} != allocating {w}"
        assert 0 <= g[0] <= k and 0 <= g[1] < vocab
        seen.add(g[0] == k)
    assert temperature == 0.0 or len(seen) >= 1


def test_static_scratch_accept_rejects_sizes_beyond_its_array():
    import paper_2504_00030_amd as pk
    from paper_2504_00030_amd import binding
    pk.load()
    p = torch.zeros((3, 1024), device="cuda")
    q = torch.zeros((2, 1024), device="cuda")
    d = torch.zeros(2, dtype=torch.int32, device="cuda")
    out = torch.zeros(2, dtype=torch.int32, device="cuda")
    lib = pk.load()
    rc = lib.spec_k_accept_static(p.data_ptr(), q.data_ptr(), d.data_ptr(), 65, 1024, 1.0, 0, 0, out.data_ptr(), 0)
    assert rc == binding.SPEC_EINVAL
    rc = lib.spec_k_accept_static(p.data_ptr(), q.data_ptr(), d.data_ptr(), 2, 262145, 1.0, 0, 0, out.data_ptr(), 0)
    assert rc == binding.SPEC_EINVAL
    assert b"262144" in lib.spec_last_error(None)
    torch.cuda.synchronize()
