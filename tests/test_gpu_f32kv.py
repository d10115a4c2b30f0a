"""GPU tests of chunk_attn_bwd_f32kv, the backward that keeps dK / dV in float32: parity with the fp64 oracle for
both head dimensions, accumulation over the slices of a split sequence (rounded once instead of once per slice),
uncovered rows, and agreement with chunk_attn_bwd on everything else."""
import numpy as np
import pytest
import torch

import synth
from gpu_util import TOL_GRAD, TOL_O, make_inputs, rel_err, run_gpu

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("d,Hq,Hkv", [(128, 8, 2), (64, 4, 4)])
def test_single_call_matches_oracle_and_bf16_path(oracle_mod, d, Hq, Hkv):
    # a hybrid chunk: tail slice behind a context, two short sequences; ragged sizes, several 128-key blocks
    case = synth.ChunkCase("hyb", synth.hybrid_chunk(300, 700, [150, 90]), 540, 1240, Hq, Hkv, d, 91)
    q, k, v, do = make_inputs(case)
    o, lse, dq, dk32, dv32 = run_gpu(case, q, k, v, do, f32kv=True)
    _, _, dq_b, dk_b, dv_b = run_gpu(case, q, k, v, do)
    assert dk32.dtype == torch.float32 and dv32.dtype == torch.float32
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    O, _ = orc.forward(); dQ, dK, dV = orc.backward()
    errs = dict(o=rel_err(o, O), dq=rel_err(dq, dQ), dk=rel_err(dk32, dK), dv=rel_err(dv32, dV))
    print(d, errs, flush=True)
    assert errs["o"] <= TOL_O and max(errs["dq"], errs["dk"], errs["dv"]) <= TOL_GRAD
    # same kernels, same sums: rounding the fp32 result gives the bf16 path's result bit for bit, dq is unchanged
    assert torch.equal(dq, dq_b)
    assert torch.equal(dk32.to(torch.bfloat16), dk_b) and torch.equal(dv32.to(torch.bfloat16), dv_b)


def test_accumulation_over_slices_is_rounded_once(oracle_mod):
    """8 slices of a 2048-token sequence, backward last to first, dK / dV accumulated over the calls in fp32: closer to
    the unsplit gradient than the bf16 buffers, which round after every slice."""
    n_slices, sl, Hq, Hkv, d = 8, 256, 8, 2, 128
    n = n_slices * sl
    q = synth.normal_bf16(777, 0, (n, Hq, d), "cuda"); k = synth.normal_bf16(777, 1, (n, Hkv, d), "cuda")
    v = synth.normal_bf16(777, 2, (n, Hkv, d), "cuda"); do = synth.normal_bf16(777, 3, (n, Hq, d), "cuda")
    dk32 = torch.zeros(k.shape, dtype=torch.float32, device="cuda"); dv32 = torch.zeros_like(dk32)
    dk16 = torch.zeros_like(k); dv16 = torch.zeros_like(v)
    for i in range(n_slices - 1, -1, -1):
        case = synth.ChunkCase(f"slice{i}", synth.split_slice(sl, sl * i), sl, n, Hq, Hkv, d, 0)
        qi = q[i * sl:(i + 1) * sl].contiguous(); doi = do[i * sl:(i + 1) * sl].contiguous()
        _, _, _, dk32, dv32 = run_gpu(case, qi, k, v, doi, accumulate=True, dk_init=dk32, dv_init=dv32, f32kv=True)
        _, _, _, dk16, dv16 = run_gpu(case, qi, k, v, doi, accumulate=True, dk_init=dk16, dv_init=dv16)
    whole = oracle_mod.Oracle([(0, n, 0, n)], q.cpu(), k.cpu(), v.cpu(), do.cpu())
    _, dK, dV = whole.backward()
    e32 = (rel_err(dk32, dK), rel_err(dv32, dV))
    e16 = (rel_err(dk16, dK), rel_err(dv16, dV))
    print("fp32 buffers", e32, "bf16 buffers", e16, flush=True)
    assert max(e32) <= TOL_GRAD and max(e16) <= TOL_GRAD
    # mean error over all elements: the fp32 buffers carry only the kernels' own bf16 operand rounding
    m32 = float(np.abs(dk32.double().cpu().numpy() - dK).mean()); m16 = float(np.abs(dk16.double().cpu().numpy() - dK).mean())
    assert m32 < m16


def test_uncovered_rows(oracle_mod):
    segs = [(0, 100, 10, 150), (100, 60, 200, 60)]
    case = synth.ChunkCase("gaps", [synth.Seg(*s) for s in segs], 160, 300, 4, 2, 128, 31)
    q, k, v, do = make_inputs(case)
    init_k = torch.full(k.shape, 3.0, dtype=torch.float32, device="cuda"); init_v = torch.full_like(init_k, -2.0)
    _, _, _, dk_acc, dv_acc = run_gpu(case, q, k, v, do, accumulate=True, dk_init=init_k, dv_init=init_v, f32kv=True)
    _, _, _, dk_ow, dv_ow = run_gpu(case, q, k, v, do, f32kv=True)
    cov = torch.zeros(300, dtype=torch.bool)
    for s in segs:
        cov[s[2]:s[2] + s[3]] = True
    assert torch.all(dk_acc.cpu()[~cov] == 3.0) and torch.all(dv_acc.cpu()[~cov] == -2.0)
    assert torch.all(dk_ow.cpu()[~cov] == 0) and torch.all(dv_ow.cpu()[~cov] == 0)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    _, dK, dV = orc.backward()
    c = cov.numpy()
    assert rel_err(dk_acc.cpu()[cov], dK[c] + 3.0) <= TOL_GRAD
    assert rel_err(dv_acc.cpu()[cov], dV[c] - 2.0) <= TOL_GRAD


def test_misaligned_pointer_is_rejected():
    import ctypes
    import paper_2509_21275_amd as ca
    desc = ca.make_desc([(0, 64, 0, 64)], 4, 2, 128, 64, 64, 0.1)
    ws = ca.alloc_workspace(desc)
    buf = torch.zeros(64 * 4 * 128 * 4, dtype=torch.bfloat16, device="cuda")
    f32 = torch.zeros(64 * 2 * 128 + 8, dtype=torch.float32, device="cuda")
    p = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    rc = ca._lib.chunk_attn_bwd_f32kv(ctypes.byref(desc), p(buf), p(buf), p(buf), p(buf), p(buf), p(f32), p(buf), p(f32, 4),
                                      p(f32), 0, p(ws), ws.numel(), None)
    assert rc == ca.INVALID_ARG
