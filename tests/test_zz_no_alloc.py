"""The entry point that allocates nothing (vp_output_fwd_noalloc: scratch in a static device array of
the library) against vp_output_fwd on the same inputs, called through the C ABI: two calls in a row,
the second with a smaller input, every output bit for bit (both run the same kernels)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _both(vp, N, h, Vs, dtype, save_logits, seed, offset):
    H, Ws, labels = si.small_output_case(N, h, Vs, 1, dtype, seed=seed, w_std=0.08)
    labels = labels + offset
    Hd, Wd, ld = to_dev(H), to_dev(Ws[0]), to_dev(labels)
    dt = vp.VP_F32 if dtype == "f32" else vp.VP_BF16
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    flags = vp.VP_SAVE_LOGITS if save_logits else 0
    f32 = dict(dtype=torch.float32, device="cuda")
    outs = []
    for which in ("workspace", "noalloc"):
        lm, ls, lt = torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32), torch.full((N,), 7.0, **f32)
        y = torch.zeros((N, Vs), dtype=tdt, device="cuda") if save_logits else None
        if which == "workspace":
            need = max(vp.vp_workspace_bytes(vp.binding.VP_CALL_OUTPUT_FWD, N, h, Vs, dt, flags), 256)
            ws = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda")
            vp.vp_output_fwd(Hd, Wd, ld, offset, lm, ls, lt, y, ws)
        else:
            vp.vp_output_fwd_noalloc(Hd, Wd, ld, offset, lm, ls, lt, y)
        torch.cuda.synchronize()
        outs.append((lm, ls, lt, y))
    for a, b in zip(*outs):
        if a is not None:
            assert torch.equal(a, b), "vp_output_fwd_noalloc differs from vp_output_fwd"
    assert bool(torch.isfinite(outs[1][1]).all()) and not bool((outs[1][0] == 7.0).any())


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_noalloc_forward_matches_forward_with_workspace_two_calls_in_a_row(dtype):
    import paper_2411_05288_amd as vp
    assert vp.vp_output_fwd_noalloc_max_scratch() == 4 << 20
    # first call: several column tiles and ragged edges; second call right after it: a smaller input,
    # which finds the first call's partials still in the scratch
    _both(vp, 700, 192, 1544, dtype, True, seed=811, offset=3000)
    _both(vp, 130, 64, 264, dtype, False, seed=812, offset=0)
    # (fp32 without kept logits holds the [N, Vs] logits in the scratch: 500 x 1544 x 4 bytes = 3.1 MB fits)
    _both(vp, 700 if dtype == "bf16" else 500, 192, 1544, dtype, False, seed=813, offset=0)


def test_noalloc_forward_refuses_sizes_beyond_its_scratch():
    import paper_2411_05288_amd as vp
    N, h, Vs = 8192, 64, 65536      # bf16: (2 * 256 + 1) * 8192 * 4 bytes = 16.8 MB of partials
    assert vp.vp_workspace_bytes(vp.binding.VP_CALL_OUTPUT_FWD, N, h, Vs, vp.VP_BF16, 0) > vp.vp_output_fwd_noalloc_max_scratch()
    H = torch.zeros((N, h), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((Vs, h), dtype=torch.bfloat16, device="cuda")
    lab = torch.zeros((N,), dtype=torch.int64, device="cuda")
    o = [torch.full((N,), 7.0, dtype=torch.float32, device="cuda") for _ in range(3)]
    with pytest.raises(vp.VPError, match="VP_ERR_UNSUPPORTED"):
        vp.vp_output_fwd_noalloc(H, W, lab, 0, o[0], o[1], o[2])
    torch.cuda.synchronize()
    assert all(bool((t == 7.0).all()) for t in o), "a refused call must launch nothing"


def test_noalloc_forward_at_the_size_of_the_largest_benchmark_shard():
    # cfg3's shard (N = 4096, Vs = 16032) needs 2.1 MB of partials: inside the static array
    import paper_2411_05288_amd as vp
    _both(vp, 4096, 256, 16032, "bf16", False, seed=814, offset=16032)
