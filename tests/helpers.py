"""Shared plumbing of the GPU parity tests: run the HIP path through the binding and compare
with the CPU oracle byte for byte."""
import numpy as np
import torch

from oracle import s3gd_oracle as O


def gpu_step(ctx, G, K, x0, lr, fused=False, dense_outputs=True, g_dev=None):
    """One step on the GPU.  Returns numpy outputs with the oracle's keys."""
    dev = torch.device("cuda:0")
    M, N = G.shape
    g = torch.from_numpy(G).to(dev) if g_dev is None else g_dev
    x = torch.from_numpy(np.ascontiguousarray(x0).copy()).to(dev)
    words = torch.full((M, K), 0x55555555, dtype=torch.int32, device=dev)
    counts = torch.full((M,), 0x55555555, dtype=torch.int32, device=dev)
    tally = votes = None
    if dense_outputs:
        tally = torch.full((N,), 0x55555555, dtype=torch.int32, device=dev)
        votes = torch.full((N,), 0x55, dtype=torch.int8, device=dev)
    if fused:
        ctx.step(g, K, x, float(lr), words, counts, tally, votes)
    else:
        ctx.topk_sign_encode(g, K, words, counts)
        ctx.majority_vote(words, counts, N, tally, votes)
        ctx.apply_update(x, votes, float(lr))
    torch.cuda.synchronize()
    assert ctx.last_async_status() == 0
    out = dict(words=words.cpu().numpy().view(np.uint32), counts=counts.cpu().numpy().view(np.uint32), x=x.cpu().numpy())
    if dense_outputs:
        out["tally"] = tally.cpu().numpy()
        out["votes"] = votes.cpu().numpy()
    return out


def assert_same(got, want, keys=("words", "counts", "tally", "votes", "x"), what=""):
    for k in keys:
        if k not in got:
            continue
        a, b = got[k], want[k]
        assert a.shape == b.shape and a.dtype == b.dtype, (what, k, a.shape, b.shape, a.dtype, b.dtype)
        if not np.array_equal(a.view(np.uint8), b.view(np.uint8)):
            bad = np.nonzero(a.reshape(-1).view(np.uint32 if a.dtype.itemsize == 4 else np.uint8)
                             != b.reshape(-1).view(np.uint32 if b.dtype.itemsize == 4 else np.uint8))[0]
            raise AssertionError(f"{what}: {k} differs at {bad.size} places, first {bad[:5]}: "
                                 f"got {a.reshape(-1)[bad[:5]]} want {b.reshape(-1)[bad[:5]]}")


def oracle_step(G, K, x0, lr):
    return O.step(G, K, x0, lr)
