"""Marshalling shared by the GPU tests: numpy workloads to device tensors, one library call, the tolerance check."""
import numpy as np

from helpers import error_report

# tolerance stated by the benchmark spec: max-abs <= 5e-3 and max-rel <= 1e-2, both required, max-rel being
# |g - o| / max(|o|, 1e-3)
MAX_ABS, MAX_REL = 5e-3, 1e-2


def arrays(w):
    return (w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens)


def to_dev(torch, arrs):
    dev = torch.device("cuda:0")
    q, kp, vp, bt, lens = arrs
    return (torch.from_numpy(q.view(np.int16)).to(dev).view(torch.bfloat16),
            torch.from_numpy(kp.view(np.int16)).to(dev).view(torch.bfloat16),
            torch.from_numpy(vp.view(np.int16)).to(dev).view(torch.bfloat16),
            torch.from_numpy(bt).to(dev), torch.from_numpy(lens).to(dev))


def run_gpu(torch, arrs, *, vector_kernels=False, scale=0.0, cu_budget=0, repeat=1):
    """One (or `repeat`) decode step(s) through the C ABI on a fresh handle; NaN-filled output buffers."""
    from paper_2604_23838_amd import binding as jb
    q, kp, vp, bt, lens = arrs
    B, Hq, D = q.shape
    tq, tk, tv, tbt, tl = to_dev(torch, arrs)
    op = jb.DecodeAttention(B, Hq, kp.shape[1], D, bt.shape[1], kp.shape[0], softmax_scale=scale, cu_budget=cu_budget)
    outs = []
    for _ in range(repeat):
        out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device="cuda:0")
        op(tq, tk, tv, tbt, tl, out, vector_kernels=vector_kernels)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    op.check_flags()
    op.close()
    return outs[0] if repeat == 1 else outs


def check(got, ref, what=""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    ma, mr = error_report(got, ref)
    print(f"{what}: max-abs {ma:.3e} max-rel(floor 1e-3) {mr:.3e}", flush=True)
    assert ma <= MAX_ABS and mr <= MAX_REL, f"{what}: max-abs {ma:.3e}, max-rel {mr:.3e}"
