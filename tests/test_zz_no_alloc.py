"""The clipped surrogate through the entry point that allocates nothing (its scratch is a device array of the library)
against the entry point that takes a workspace: same kernels, so the results must be identical bit for bit, on two
calls in a row, the second on a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sapo():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2509_08721_amd import sapo as binding
    binding.load_library()
    return binding


def case(S, T, seed):
    import torch
    rng = np.random.default_rng(seed)
    lp_new = torch.from_numpy((-3.0 * rng.random((S, T))).astype(np.float32)).cuda()
    lp_old = torch.from_numpy((lp_new.cpu().numpy() + 0.3 * (rng.random((S, T)) - 0.5)).astype(np.float32)).cuda()
    mask = torch.from_numpy((rng.random((S, T)) < 0.6).astype(np.uint8)).cuda()
    adv = torch.from_numpy(rng.standard_normal(S).astype(np.float32)).cuda()
    return lp_new, lp_old, mask, adv


def test_noalloc_surrogate_equals_the_workspace_entry_point_twice_in_a_row(sapo):
    import torch
    big, small = case(64, 768, 1), case(5, 37, 2)
    outs = {}
    for name, (lp_new, lp_old, mask, adv) in (("big", big), ("small", small)):
        outs[name] = (torch.full((1,), 7.0, dtype=torch.float32, device="cuda"), torch.full(lp_new.shape, 7.0, dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    mem_before = torch.cuda.memory_allocated()
    for name, (lp_new, lp_old, mask, adv) in (("big", big), ("small", small)):      # two calls in a row, the second smaller
        sapo.sapo_clipped_surrogate_noalloc(lp_new, lp_old, mask, adv, outs[name][0], outs[name][1])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem_before
    for name, (lp_new, lp_old, mask, adv) in (("big", big), ("small", small)):
        loss, grad = sapo.sapo_clipped_surrogate(lp_new, lp_old, mask, adv)
        torch.cuda.synchronize()
        assert np.array_equal(loss.cpu().numpy().view(np.uint32), outs[name][0].cpu().numpy().view(np.uint32)), name
        assert np.array_equal(grad.cpu().numpy().view(np.uint32), outs[name][1].cpu().numpy().view(np.uint32)), name
        assert np.isfinite(loss.cpu().numpy()).all() and float(grad.abs().sum()) > 0
    # loss only (no gradient buffer), and once more the larger input after the smaller one
    l2 = torch.zeros((1,), dtype=torch.float32, device="cuda")
    sapo.sapo_clipped_surrogate_noalloc(*big, l2, None)
    torch.cuda.synchronize()
    assert np.array_equal(l2.cpu().numpy().view(np.uint32), outs["big"][0].cpu().numpy().view(np.uint32))


def test_noalloc_surrogate_rejects_what_it_cannot_take(sapo):
    import torch
    lp_new, lp_old, mask, adv = case(2, 8, 3)
    loss = torch.zeros((1,), dtype=torch.float32, device="cuda")
    lib = sapo.load_library()
    args = (lp_new.data_ptr(), lp_old.data_ptr(), mask.data_ptr(), adv.data_ptr())
    too_many = (1 << 14) + 1, 1 << 14                      # S * T just beyond 2^28 tokens: refused before anything is read
    assert lib.sapo_clipped_surrogate_noalloc(*args, too_many[0], too_many[1], 0.2, 0.28, loss.data_ptr(), None, None) == sapo.SAPO_EINVAL
    assert b"maximum" in lib.sapo_last_error()
    assert lib.sapo_clipped_surrogate_noalloc(*args, 0, 8, 0.2, 0.28, loss.data_ptr(), None, None) == sapo.SAPO_EINVAL
    assert lib.sapo_clipped_surrogate_noalloc(*args, 2, 8, 0.2, 0.28, None, None, None) == sapo.SAPO_EINVAL
    assert lib.sapo_clipped_surrogate_noalloc(*args, 2, 8, 1.5, 0.28, loss.data_ptr(), None, None) == sapo.SAPO_EINVAL
