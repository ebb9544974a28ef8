"""GPU parity of moe_dispatch_noalloc, the dispatch entry point that allocates nothing (its per-chunk
histograms live in a device array that is part of the library): every output must equal moe_dispatch's,
bit for bit, on two calls in a row, the second with a smaller input (the array keeps the first call's
contents).  Sizes above 16384 routes take the count / scan / rank kernels, which are the ones that use
the scratch; a small batch (one fused index kernel, no scratch) is covered too."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2502_06643_amd import binding as B
from paper_2502_06643_amd import synth
from paper_2502_06643_amd.layer import to_device, to_host

pytestmark = pytest.mark.gpu

INT_OUTPUTS = ("perm", "inv_perm", "expert_counts", "expert_start", "gpu_counts", "gpu_offsets")


def run(entry, x, idx, T, d, E, k, pl, G, dt):
    N = T * k
    i32 = dict(dtype=torch.int32, device="cuda")
    out = dict(send_buf=torch.zeros((N, d), dtype=x.dtype, device="cuda"), perm=torch.full((N,), -1, **i32),
               inv_perm=torch.full((N,), -1, **i32), expert_counts=torch.full((E,), -1, **i32),
               expert_start=torch.full((E,), -1, **i32), gpu_counts=torch.full((G,), -1, **i32),
               gpu_offsets=torch.full((G + 1,), -1, **i32))
    args = (x, dt, idx, T, d, E, k, pl, G, out["send_buf"], out["perm"], out["inv_perm"], out["expert_counts"],
            out["expert_start"], out["gpu_counts"], out["gpu_offsets"])
    if entry == "workspace":
        ws = torch.empty(max(256, B.moe_dispatch_workspace_bytes(T, E, k)), dtype=torch.uint8, device="cuda")
        B.moe_dispatch(*args, ws)
    else:
        B.moe_dispatch_noalloc(*args)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("dtype,d,E,k,G,sizes", [
    ("bf16", 256, 8, 2, 4, (20000, 9000)),          # 40000 then 18000 routes: both through count / scan / rank
    ("f32", 64, 64, 6, 8, (8192, 3000, 100)),       # 49152, 18000, then 600 routes (fused index kernel)
    ("bf16", 128, 256, 16, 256, (16000, 1100)),     # widest histograms: 250 chunks x 256 experts x 4 B = 250 KiB of the 256 KiB
])
def test_noalloc_dispatch_equals_dispatch_on_consecutive_calls(lib, dtype, d, E, k, G, sizes):
    dt = B.MOE_BF16 if dtype == "bf16" else B.MOE_F32
    pl_host = (np.arange(E) * 7 % G).astype(np.int32)
    pl = torch.from_numpy(pl_host).cuda()
    for call, T in enumerate(sizes):
        assert B.moe_dispatch_workspace_bytes(T, E, k) <= B.moe_dispatch_static_scratch_bytes()
        x_host = synth.normal(3 + call, 0, (T, d), 1.0, dtype)
        idx_host = synth.random_topk_idx(11 + call, T, E, k)
        x, idx = to_device(x_host), torch.from_numpy(idx_host).cuda()
        got = run("noalloc", x, idx, T, d, E, k, pl, G, dt)
        want = run("workspace", x, idx, T, d, E, k, pl, G, dt)
        ref = O.dispatch(x_host, idx_host, pl_host, G)
        for n in INT_OUTPUTS:
            np.testing.assert_array_equal(got[n].cpu().numpy(), want[n].cpu().numpy(), err_msg=f"call {call}: {n}")
            np.testing.assert_array_equal(got[n].cpu().numpy(), ref[n], err_msg=f"call {call}: {n} vs oracle")
        np.testing.assert_array_equal(to_host(got["send_buf"]), to_host(want["send_buf"]), err_msg=f"call {call}: send_buf")
        np.testing.assert_array_equal(to_host(got["send_buf"]), ref["send_buf"])


def test_noalloc_dispatch_refuses_what_its_buffer_cannot_hold(lib):
    T, E, k, G = 1 << 19, 256, 4, 4
    assert B.moe_dispatch_workspace_bytes(T, E, k) > B.moe_dispatch_static_scratch_bytes()
    one = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(RuntimeError, match="scratch"):
        B.moe_dispatch_noalloc(None, B.MOE_BF16, one, T, 8, E, k, one, G, None, one, one, one, one, one, one)
