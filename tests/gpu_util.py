"""Helpers of the GPU parity tests: run the HIP path through the binding, run the oracle, compare."""
import numpy as np
import torch

import paper_2507_05508_amd as P
from oracle import mlmc as O


def to_device(G: np.ndarray, ld=None, dev="cuda:0"):
    """Host rows -> CUDA tensor [M, d] (float32, or bfloat16 for uint16 bit patterns).  ld > d gives padded,
    possibly misaligned rows."""
    M, d = G.shape
    if G.dtype == np.uint16:
        t = torch.from_numpy(G.view(np.int16).copy()).view(torch.bfloat16)
    else:
        t = torch.from_numpy(G.copy())
    if ld is None or ld == d:
        return t.to(dev).contiguous()
    buf = torch.zeros((M, ld), dtype=t.dtype, device=dev)
    buf[:, :d] = t.to(dev)
    return buf[:, :d]


def u32(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def check_topk_against_oracle(plan, G, seed, step, msg, *, adaptive, norms_override=None, p=None):
    """Bit-exact comparison of one compress call with the oracle: levels, offsets, indices, values, tile table."""
    M, d = G.shape
    torch.cuda.synchronize()
    level = msg.level.cpu().numpy()
    row_off = msg.row_off.cpu().numpy()
    idx = u32(msg.idx)
    val = msg.val.cpu().numpy()
    tile_off = u32(msg.tile_off)
    if adaptive and norms_override is None and p is None:
        want = O.compress_topk(G, plan.ladder, None, seed, step)
    elif norms_override is not None:
        want = O.compress_topk(G, plan.ladder, None, seed, step, norms_override=norms_override)
    else:
        want = O.compress_topk(G, plan.ladder, p if p is not None else plan.p_fixed, seed, step)
    off = 0
    for i in range(M):
        w = want[i]
        assert level[i] == w["level"], (i, level[i], w["level"])
        assert row_off[i] == off
        n = len(w["idx"])
        assert np.array_equal(idx[off:off + n], w["idx"]), f"row {i}: indices differ"
        assert np.array_equal(val[off:off + n].view(np.uint32), w["val"].view(np.uint32)), f"row {i}: values differ"
        # tile table: entries with idx < t * TILE
        bounds = np.searchsorted(w["idx"], np.arange(plan.num_tiles + 1, dtype=np.int64) * P.MLMC_TILE, side="left")
        assert np.array_equal(tile_off[i], bounds.astype(np.uint32)), f"row {i}: tile offsets differ"
        off += n
    assert row_off[M] == off
    return want
