"""The entry point for callers that cannot allocate (cdq_loss_static) against cdq_loss, through the C ABI: two
calls in a row on the library's static scratch array, the second on a smaller layer, each compared with what the
workspace-taking entry point returns for the same inputs.  Both run the same kernels in the same order, so the
results must be bit-equal; the test also checks that the call leaves the device allocator alone."""
import numpy as np
import pytest
import torch

from paper_2406_17542_amd import inputs

pytestmark = pytest.mark.gpu


def _layer(cdq, d_out, d_in, n, bits, group, seed):
    rng = np.random.default_rng(seed)
    X = torch.from_numpy(inputs.round_to_bf16(rng.standard_normal((n, d_in), dtype=np.float32))).cuda().to(torch.bfloat16)
    H = cdq.hessian(X)
    Wd = torch.from_numpy(inputs.make_wt(d_out, d_in, seed=seed)).cuda()
    scale, zero, Q = cdq.init_rtn(Wd, bits, group)
    return H, Wd, scale, zero, Q


def test_loss_static_matches_loss_on_two_calls_in_a_row():
    assert torch.cuda.is_available()
    from paper_2406_17542_amd import cdq
    cdq.lib()
    # the larger layer first (its partial sums fill more of the scratch array), then a smaller, ragged one
    cases = [(1000, 2048, 4096, 3, 2048, 1), (77, 384, 1024, 4, 128, 2)]
    layers = [_layer(cdq, *c) for c in cases]
    refs = [cdq.loss(H, Wd, s, z, Q, c[4]) for (H, Wd, s, z, Q), c in zip(layers, cases)]
    outs = [(torch.empty(c[0], dtype=torch.float64, device="cuda"), torch.empty(1, dtype=torch.float64, device="cuda")) for c in cases]
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    for (H, Wd, s, z, Q), c, (per, tot) in zip(layers, cases, outs):
        cdq.loss_static(H, Wd, s, z, Q, c[4], per, tot)
    torch.cuda.synchronize()
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before, "the binding allocated device memory"
    for (per_ref, tot_ref), (per, tot) in zip(refs, outs):
        assert torch.equal(per, per_ref)
        assert torch.equal(tot, tot_ref)
        assert float(tot) > 0.0
    # and once more on the first layer: the smaller call in between has left nothing behind that matters
    per, tot = outs[0]
    per.zero_(); tot.zero_()
    H, Wd, s, z, Q = layers[0]
    cdq.loss_static(H, Wd, s, z, Q, cases[0][4], per, tot)
    assert torch.equal(per, refs[0][0]) and torch.equal(tot, refs[0][1])


def test_loss_static_rejects_what_does_not_fit():
    from paper_2406_17542_amd import cdq
    L = cdq.lib()
    d_out, d_in = 65536, 16384                   # d_out * ceil(d_in/128) partial sums: 64 MiB, beyond the 24 MiB array
    assert cdq.workspace_bytes(cdq.OP_LOSS, 0, d_out, d_in) > (24 << 20)
    p = 0x1000                                   # never dereferenced: the size check comes first
    assert L.cdq_loss_static(p, p, p, p, p, d_out, d_in, d_in, p, p, None) == -4
