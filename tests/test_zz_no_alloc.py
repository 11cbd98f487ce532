"""poly_lora_linear_static (the entry point that allocates nothing) against poly_lora_linear on the GPU."""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_14959_amd import binding, synth

pytestmark = pytest.mark.gpu


def _device_case(case):
    dev = "cuda"
    elt = torch.bfloat16 if case["dtype"] == synth.DT_BF16 else torch.float32
    up = lambda a, dt=elt: torch.from_numpy(np.ascontiguousarray(a)).to(device=dev, dtype=dt).contiguous()
    return dict(X=up(case["X"]), Wt=up(case["W"].T), At=up(np.swapaxes(case["A"], 1, 2)), Bt=up(np.swapaxes(case["B"], 1, 2)),
                bias=up(case["bias"], torch.float32) if case.get("bias") is not None else None,
                off=up(case["row_offsets"], torch.int32), ids=up(case["adapter_ids"], torch.int32),
                R=int(case["row_offsets"][-1]), elt=elt)


def _run_both(case, scale):
    """Same inputs through both entry points; all buffers exist before the static call, which itself gets no workspace."""
    d = _device_case(case)
    F, T, _ = d["X"].shape
    N = d["Wt"].shape[0]
    Y_ws = torch.full((d["R"], T, N), float("nan"), dtype=d["elt"], device="cuda")
    Y_st = torch.full((d["R"], T, N), float("nan"), dtype=d["elt"], device="cuda")
    st_ws = torch.full((1,), 99, dtype=torch.int32, device="cuda")
    st_st = torch.full((1,), 99, dtype=torch.int32, device="cuda")
    ws = torch.empty(binding.poly_lora_linear_workspace_bytes(F, T, case["r"], d["R"], case["dtype"]), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    binding.poly_lora_linear(d["X"], d["Wt"], d["bias"], d["At"], d["Bt"], scale, d["off"], d["ids"], d["R"], Y_ws, ws, dev_status=st_ws)
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    binding.poly_lora_linear_static(d["X"], d["Wt"], d["bias"], d["At"], d["Bt"], scale, d["off"], d["ids"], d["R"], Y_st, dev_status=st_st)
    assert torch.cuda.memory_stats()["allocation.all.allocated"] == before      # (torch's allocator at least was not asked)
    torch.cuda.synchronize()
    assert int(st_ws.item()) == 0 and int(st_st.item()) == 0
    return Y_ws.float().cpu().numpy(), Y_st.float().cpu().numpy()


def _check_against_checker(Y, want, dtype):
    err = float(np.abs(Y - want).max())
    assert err < (1e-4 if dtype == synth.DT_F32 else 2e-2), err


@pytest.mark.parametrize("dtype", [synth.DT_BF16, synth.DT_F32])
def test_two_calls_in_a_row_second_one_smaller(dtype):
    big = synth.make_lora_linear_case(dtype=dtype, seed=41, n_xblocks=7, T=197, Kdim=192, Ndim=576, n_adapters=6, r=8, per_block=2)
    small = synth.make_lora_linear_case(dtype=dtype, seed=42, n_xblocks=3, T=61, Kdim=64, Ndim=136, n_adapters=4, r=12, per_block=1)
    for case, scale in ((big, 1.5), (small, 0.75)):     # the second call finds the first one's leftovers in the scratch array
        Y_ws, Y_st = _run_both(case, scale)
        assert np.array_equal(Y_ws, Y_st)               # same kernels, same order of operations: bit for bit
        _check_against_checker(Y_st, oracle.lora_linear(case, s=scale), dtype)


def test_sizes_beyond_the_static_array_are_rejected_and_nothing_runs():
    case = synth.make_lora_linear_case(seed=43, n_xblocks=2, T=197, Kdim=64, Ndim=64, n_adapters=2, r=16, per_block=1)
    d = _device_case(case)
    R_big = 700                                          # 700 * 197 rows of 16 bf16 ranks = 4.4 MB of S alone
    assert binding.poly_lora_linear_workspace_bytes(2, 197, 16, R_big, synth.DT_BF16) > binding.STATIC_SCRATCH_BYTES
    Y = torch.full((2, 197, 64), float("nan"), dtype=torch.bfloat16, device="cuda")
    rc = binding.poly_lora_linear_static(d["X"], d["Wt"], d["bias"], d["At"], d["Bt"], 1.0, d["off"], d["ids"], R_big, Y, check=False)
    torch.cuda.synchronize()
    assert rc == binding.POLY_ECAP and torch.isnan(Y.float()).all()
