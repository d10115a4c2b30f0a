"""GPU parity of the fused in-place cross-entropy against the fp64 oracle on the same bf16 logits.

Tolerances: the loss is an fp32 reduction over up to 128K terms: |loss - oracle| <= 2e-4 (relative error of the
exponentials ~1e-6, of the logarithm likewise; the logits themselves are exact).  The gradient is rounded to bf16:
|g - oracle| <= 2^-8 |oracle| + 2^-8 |grad_scale| * 1e-3 (half an ulp would be 2^-9; the absolute term covers
probabilities whose exponentials carry the fp32 error of the row's log-sum-exp)."""
import numpy as np
import pytest
import torch

from oracle import fused_ce_oracle as orc

pytestmark = pytest.mark.gpu

CASES = [  # rows, vocab, row stride, spread of the logits
    (5, 8, 8, 2.0), (33, 4096, 4096, 3.0), (70, 128256, 128256, 2.0), (16, 131072, 131072, 6.0),
    (9, 32000, 32768, 4.0), (3, 151936, 151936, 2.0), (2, 262144, 262144, 1.0), (600, 1024, 1024, 8.0),
]


@pytest.mark.parametrize("rows,vocab,stride,spread", CASES)
def test_parity(rows, vocab, stride, spread):
    from paper_2509_21275_amd.fused_ce import fused_ce_inplace
    g = torch.Generator(device="cpu").manual_seed(1000 + rows + vocab)
    buf = (torch.randn((rows, stride), generator=g) * spread).to(torch.bfloat16)
    targets = torch.randint(0, vocab, (rows,), generator=g, dtype=torch.int32)
    if rows > 2:
        targets[1] = -100                           # an ignored row
        targets[2] = vocab - 1
    # make one row sharply peaked on its target and one peaked elsewhere
    buf[0, int(targets[0])] = 40.0
    if rows > 4:
        buf[4, (int(targets[4]) + 1) % vocab] = 30.0
    scale = 1.0 / rows
    want_loss, want_grad = orc.cross_entropy(buf[:, :vocab].double().numpy(), targets.numpy(), scale)
    dev_buf = buf.cuda()
    pad_before = dev_buf[:, vocab:].clone()
    loss = torch.full((rows,), float("nan"), device="cuda")
    fused_ce_inplace(dev_buf[:, :vocab], targets.cuda(), loss, scale)
    torch.cuda.synchronize()
    got_loss = loss.cpu().double().numpy()
    got_grad = dev_buf[:, :vocab].cpu().double().numpy()
    assert np.all(np.isfinite(got_loss)) and np.all(np.isfinite(got_grad))
    assert np.abs(got_loss - want_loss).max() <= 2e-4 * max(1.0, np.abs(want_loss).max())
    tol = 2.0 ** -8 * np.abs(want_grad) + 2.0 ** -8 * scale * 1e-3
    assert np.all(np.abs(got_grad - want_grad) <= tol), float((np.abs(got_grad - want_grad) - tol).max())
    assert torch.equal(dev_buf[:, vocab:], pad_before)        # the padding of a strided row is not touched
    if rows > 2:
        assert got_loss[1] == 0 and np.all(got_grad[1] == 0)  # ignored row


def test_empty_and_bad_arguments():
    import paper_2509_21275_amd as ca
    from paper_2509_21275_amd.fused_ce import fused_ce_inplace
    z = torch.zeros((0, 64), dtype=torch.bfloat16, device="cuda")
    fused_ce_inplace(z, torch.zeros((0,), dtype=torch.int32, device="cuda"), torch.zeros((0,), device="cuda"))
    z = torch.zeros((2, 12), dtype=torch.bfloat16, device="cuda")     # vocabulary not a multiple of 8
    with pytest.raises(ca.ChunkAttnError):
        fused_ce_inplace(z, torch.zeros((2,), dtype=torch.int32, device="cuda"), torch.zeros((2,), device="cuda"))
