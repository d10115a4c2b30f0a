"""Head dimensions other than the benchmark's 64 and 128: 256 (kernels of its own) and 96 (run as 128 on zero-padded
copies held in the workspace), through the C ABI against the fp64 oracle: scaled replicas of the five workloads, the
slice-by-slice accumulation of a split sequence in bf16 and float32 buffers, untouched / zeroed rows outside the key
ranges, workspace sizes, bit-reproducibility."""
import dataclasses

import numpy as np
import pytest
import torch

import synth
import paper_2509_21275_amd as ca
from gpu_util import TOL_GRAD, TOL_O, make_inputs, rel_err, run_gpu

pytestmark = pytest.mark.gpu

DIMS = [96, 256]


def _with_dim(case, d):
    return dataclasses.replace(case, name=f"{case.name}_d{d}", head_dim=d)


@pytest.mark.parametrize("d", DIMS)
@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_scaled_replicas(oracle_mod, idx, d):
    case = _with_dim(synth.scaled_case(idx, 16 if idx == 1 else 32), d)
    q, k, v, do = make_inputs(case)
    print(case.name, case.total_q, case.total_kv, flush=True)
    o, lse, dq, dk, dv = run_gpu(case, q, k, v, do)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    O, LSE = orc.forward(); dQ, dK, dV = orc.backward()
    errs = (rel_err(o, O), rel_err(dq, dQ), rel_err(dk, dK), rel_err(dv, dV), float(np.abs(lse.double().cpu().numpy() - LSE).max()))
    print(case.name, errs, flush=True)
    assert errs[0] <= TOL_O and max(errs[1:4]) <= TOL_GRAD and errs[4] <= 2e-2
    again = run_gpu(case, q, k, v, do)
    for x, y in zip((o, lse, dq, dk, dv), again):
        assert torch.equal(x, y)


@pytest.mark.parametrize("d", DIMS)
@pytest.mark.parametrize("f32kv", [False, True])
def test_split_sequence_accumulates_over_slices(oracle_mod, d, f32kv):
    """Four slices of one sequence, backward in reverse order, adding into shared dK/dV (bf16 or float32)."""
    n_slices, sl, Hq, Hkv = 4, 192, 4, 2
    n = n_slices * sl
    q = synth.normal_bf16(777, 0, (n, Hq, d), "cuda"); k = synth.normal_bf16(777, 1, (n, Hkv, d), "cuda")
    v = synth.normal_bf16(777, 2, (n, Hkv, d), "cuda"); do = synth.normal_bf16(777, 3, (n, Hq, d), "cuda")
    kv_dtype = torch.float32 if f32kv else torch.bfloat16
    dk = torch.zeros_like(k, dtype=kv_dtype); dv = torch.zeros_like(v, dtype=kv_dtype)
    o_all = torch.empty_like(q); dq_all = torch.empty_like(q)
    for i in range(n_slices - 1, -1, -1):
        case = synth.ChunkCase(f"slice{i}_d{d}", synth.split_slice(sl, sl * i), sl, n, Hq, Hkv, d, 0)
        print(case.name, "f32kv" if f32kv else "bf16", flush=True)
        qi = q[i * sl:(i + 1) * sl].contiguous(); doi = do[i * sl:(i + 1) * sl].contiguous()
        o, lse, dq, dk, dv = run_gpu(case, qi, k, v, doi, accumulate=True, dk_init=dk, dv_init=dv, f32kv=f32kv)
        o_all[i * sl:(i + 1) * sl] = o; dq_all[i * sl:(i + 1) * sl] = dq
    whole = oracle_mod.Oracle([(0, n, 0, n)], q.cpu(), k.cpu(), v.cpu(), do.cpu(), d ** -0.5)
    O, _ = whole.forward(); dQ, dK, dV = whole.backward()
    errs = (rel_err(o_all, O), rel_err(dq_all, dQ), rel_err(dk, dK), rel_err(dv, dV))
    print(errs, flush=True)
    assert errs[0] <= TOL_O and max(errs[1:]) <= TOL_GRAD


@pytest.mark.parametrize("d", DIMS)
def test_rows_outside_key_ranges(oracle_mod, d):
    segs = [(0, 100, 10, 150), (100, 60, 200, 60)]
    case = synth.ChunkCase(f"gaps_d{d}", [synth.Seg(*s) for s in segs], 160, 300, 4, 2, d, 31)
    q, k, v, do = make_inputs(case)
    init_k = torch.full_like(k, 3.0); init_v = torch.full_like(v, -2.0)
    _, _, _, dk_acc, dv_acc = run_gpu(case, q, k, v, do, accumulate=True, dk_init=init_k, dv_init=init_v)
    _, _, _, dk_ow, dv_ow = run_gpu(case, q, k, v, do)
    cov = torch.zeros(300, dtype=torch.bool)
    for s in segs:
        cov[s[2]:s[2] + s[3]] = True
    assert torch.all(dk_acc.cpu()[~cov] == 3.0) and torch.all(dv_acc.cpu()[~cov] == -2.0)
    assert torch.all(dk_ow.cpu()[~cov] == 0) and torch.all(dv_ow.cpu()[~cov] == 0)
    orc = oracle_mod.Oracle(case.segs, q.cpu(), k.cpu(), v.cpu(), do.cpu(), case.scale)
    _, dK, dV = orc.backward()
    c = cov.numpy()
    assert rel_err(dk_acc.cpu()[cov], dK[c] + 3.0) <= TOL_GRAD and rel_err(dv_acc.cpu()[cov], dV[c] - 2.0) <= TOL_GRAD


def test_padded_head_needs_a_larger_workspace_and_says_so():
    """head_dim 96 keeps zero-padded copies of its operands in the workspace: the sizes reported cover them, and a
    workspace sized for head_dim 128 alone is refused before anything is launched."""
    segs = synth.packed_chunk([300, 200])
    d96 = ca.make_desc(segs, 8, 2, 96, 500, 500, 96 ** -0.5)
    d128 = ca.make_desc(segs, 8, 2, 128, 500, 500, 128 ** -0.5)
    f96, b96 = ca.chunk_attn_workspace_bytes(d96)
    f128, b128 = ca.chunk_attn_workspace_bytes(d128)
    qb, kb = 500 * 8 * 128 * 2, 500 * 2 * 128 * 2
    assert f96 >= f128 + 2 * qb + 2 * kb and b96 >= b128 + 4 * qb + 2 * kb + 2 * 2 * kb
    q = torch.zeros((500, 8, 96), dtype=torch.bfloat16, device="cuda"); kv = torch.zeros((500, 2, 96), dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(q); lse = torch.empty((8, 500), dtype=torch.float32, device="cuda")
    ws = torch.empty(f128, dtype=torch.uint8, device="cuda")
    with pytest.raises(ca.ChunkAttnError) as e:
        ca.chunk_attn_fwd(d96, q, kv, kv, o, lse, ws)
    assert e.value.code == ca.WORKSPACE_TOO_SMALL
    torch.cuda.synchronize()
