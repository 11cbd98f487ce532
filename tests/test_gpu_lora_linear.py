"""poly_lora_linear on the GPU against the CPU checker."""
import numpy as np
import pytest
import torch

import oracle
from paper_2507_14959_amd import binding, synth

pytestmark = pytest.mark.gpu


def gpu_lora_linear(case, scale=1.0, R_cap=None):
    dev = "cuda"
    elt = torch.bfloat16 if case["dtype"] == synth.DT_BF16 else torch.float32
    up = lambda a, dt=elt: torch.from_numpy(np.ascontiguousarray(a)).to(device=dev, dtype=dt).contiguous()
    X = up(case["X"]); Wt = up(case["W"].T); At = up(np.swapaxes(case["A"], 1, 2)); Bt = up(np.swapaxes(case["B"], 1, 2))
    bias = up(case["bias"], torch.float32) if case.get("bias") is not None else None
    off = up(case["row_offsets"], torch.int32); ids = up(case["adapter_ids"], torch.int32)
    R = int(case["row_offsets"][-1]) if R_cap is None else R_cap
    F, T, Kd = X.shape
    Y = torch.full((max(R, 1), T, Wt.shape[0]), float("nan"), dtype=elt, device=dev)
    st = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = torch.empty(max(binding.poly_lora_linear_workspace_bytes(F, T, case["r"], R, case["dtype"]), 256), dtype=torch.uint8, device=dev)
    binding.poly_lora_linear(X, Wt, bias, At, Bt, scale, off, ids, R, Y, ws, dev_status=st)
    torch.cuda.synchronize()
    return Y.float().cpu().numpy(), int(st.item())


def check(Y, want, dtype):
    err = np.abs(Y - want)
    if dtype == synth.DT_F32:
        assert err.max() < 1e-4, err.max()
    else:
        # bf16 output rounding (2^-9 relative) plus bf16 shrink output; fp32 accumulation
        assert err.max() < 2e-2, err.max()
        assert np.all(err <= 2.0 ** -8 * np.abs(want) + 2e-3), (err - 2.0 ** -8 * np.abs(want)).max()


@pytest.mark.parametrize("dtype", [synth.DT_F32, synth.DT_BF16])
@pytest.mark.parametrize("shape", [
    dict(n_xblocks=3, T=5, Kdim=24, Ndim=16, n_adapters=4, r=4, per_block=2),            # smaller than one tile
    dict(n_xblocks=5, T=197, Kdim=192, Ndim=576, n_adapters=6, r=8, per_block=2),        # DeiT-tiny qkv, ragged rows
    dict(n_xblocks=4, T=133, Kdim=72, Ndim=200, n_adapters=5, r=12, per_block=3),        # ragged rows, K, N and rank
    dict(n_xblocks=3, T=64, Kdim=256, Ndim=1100, n_adapters=3, r=40, per_block=1),       # wide tile path, rank > 32
])
def test_matches_checker(dtype, shape):
    case = synth.make_lora_linear_case(dtype=dtype, seed=31, **shape)
    Y, st = gpu_lora_linear(case, scale=1.5)
    assert st == 0
    check(Y, oracle.lora_linear(case, s=1.5), dtype)


def test_frames_without_adapters_and_row_bound_above_R():
    case = synth.make_lora_linear_case(n_xblocks=6, T=40, Kdim=64, Ndim=96, n_adapters=4, r=8, per_block=2, seed=5)
    off, ids = synth.sets_to_csr([[1], [], [0, 3], [], [], [2]])
    case["row_offsets"], case["adapter_ids"] = off, ids
    Y, st = gpu_lora_linear(case, R_cap=9)
    assert st == 0
    check(Y[:4], oracle.lora_linear(case), synth.DT_BF16)
    assert np.all(np.isnan(Y[4:]))                       # rows past row_offsets[F] stay untouched


def test_bad_adapter_id_sets_status_and_writes_nothing():
    case = synth.make_lora_linear_case(n_xblocks=2, T=8, Kdim=32, Ndim=32, n_adapters=4, r=8, per_block=1, seed=6)
    case["adapter_ids"] = np.array([1, 4], dtype=np.int32)
    Y, st = gpu_lora_linear(case)
    assert st == binding.POLY_ERANGE and np.all(np.isnan(Y))


def test_base_product_is_shared_by_row_blocks_of_one_input():
    # two row-blocks of the same X block with the same adapter must agree bit for bit
    case = synth.make_lora_linear_case(n_xblocks=2, T=50, Kdim=64, Ndim=128, n_adapters=3, r=16, per_block=1, seed=8)
    off, ids = synth.sets_to_csr([[2, 2, 1], [2]])
    case["row_offsets"], case["adapter_ids"] = off, ids
    Y, _ = gpu_lora_linear(case)
    assert np.array_equal(Y[0], Y[1]) and not np.array_equal(Y[0], Y[2])


def test_config5_full_size_every_row_block():
    """256 x 197 x 768 -> 2304, 64 adapters of rank 16, R = 512: the 256 x 256 tiles that run across block boundaries, the
    eight per-XCD runs and the fan-out of every X block into two row-blocks, all 512 row-blocks element by element."""
    case = synth.make_lora_linear_case()
    Y, st = gpu_lora_linear(case)
    assert st == 0 and Y.shape == (512, 197, 2304)
    worst = 0.0
    for b in range(0, 512, 32):                          # the checker in chunks of 32 row-blocks (116 MB of doubles each)
        want = oracle.lora_linear(case, b_begin=b, b_end=b + 32)
        check(Y[b:b + 32], want, synth.DT_BF16)
        worst = max(worst, float(np.abs(Y[b:b + 32] - want).max()))
    print(f"config 5: max-abs error over all 512 row-blocks {worst:.2e}")


def test_deep_layer_shape_no_shared_inputs_full_compare():
    """No two row-blocks share an input (one adapter per X block) and a block count that leaves the last 256-row tile ragged:
    600 blocks of 197 rows are 462 tiles (118 200 = 461 * 256 + 184), enough for the big tiles (>= 512 with three column tiles)."""
    case = synth.make_lora_linear_case(n_xblocks=600, T=197, Kdim=512, Ndim=768, n_adapters=9, r=16, per_block=1, seed=77)
    Y, st = gpu_lora_linear(case, scale=0.5)
    assert st == 0
    for b in range(0, 600, 100):
        check(Y[b:b + 100], oracle.lora_linear(case, s=0.5, b_begin=b, b_end=b + 100), synth.DT_BF16)
