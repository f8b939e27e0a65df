"""pafu_step under HIP graph capture: the library enqueues kernels only (no memset, copy or allocation nodes), so a
step can be captured once and replayed.  Every replay is checked bit for bit against the eager call on the same
inputs, with eager work and synchronisations between the replays, and once against the oracle."""
import numpy as np
import pytest
import torch

from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import DEV, bits, step_workspace
from tests.test_gpu_step import _check_single, _single

pytestmark = pytest.mark.gpu


def _refill(cfg, args_pack, d0, seed):
    """New seeded features, Q, K, V written INTO the tensors the captured step reads; the weights stay."""
    args = args_pack[0]
    w, t, x_cache, x_chunk = args._keep
    d = wl.make_layer_inputs(cfg, seed=wl.BASE_SEED + seed)
    for key in ("W1", "b1", "W2", "b2"):
        d[key] = d0[key]
    rb = wl.round_to_bf16
    kv = {x: rb(d[x]) for x in ("K_cache", "V_cache", "Q", "K_chunk", "V_chunk")}

    def put(dst, a):
        dst.copy_(torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(dst.dtype).view(dst.shape))
    put(x_cache, d["X_cache"]); put(x_chunk, d["X_chunk"])
    put(t[0], kv["K_cache"]); put(t[1], kv["V_cache"]); put(t[2], kv["Q"]); put(t[3], kv["K_chunk"]); put(t[4], kv["V_chunk"])
    return d, kv


@pytest.mark.parametrize("shape", ["tiny", "split"])
def test_captured_step_replays_bit_identically(shape):
    if shape == "tiny":      # C0-sized, bf16: the launch-bound case a graph is for
        cfg = wl.scaled(wl.C0, dtype="bf16")
    else:                    # 32 work items on 256 CUs with a workspace: equal-run split + merge pass inside the graph
        cfg = wl.scaled(wl.C1, N=4, frame_tokens=600, chunk_frames=3, cache_frames=4, k=1200, M=256)
    k, L_B = cfg.k, cfg.Lc
    d = wl.make_layer_inputs(cfg)
    pack = _single(cfg, d, k, L_B, contiguous_features=False)
    args, kv, scores, ids, K_out, V_out, SL_out, O, n_kept = pack
    step_workspace(args)
    outs = (scores, ids, K_out, V_out, SL_out, O)

    B.pafu_step(args)                                   # eager once: one-time kernel attributes are set outside capture
    _check_single(cfg, d, k, L_B, pack)

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.pafu_step(args)                               # the binding launches on the capturing stream
    torch.cuda.synchronize()

    for rep in range(4):
        d2, kv2 = _refill(cfg, pack, d, 100 + rep)
        B.pafu_step(args)
        torch.cuda.synchronize()
        want = [bits(o).copy() for o in outs]
        for o in outs:
            o.fill_(-1 if o.dtype == torch.int32 else 0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, w_ in zip(outs, want):
            assert np.array_equal(bits(o), w_), (shape, rep)
        if rep == 3:                                    # and the replayed result is the oracle's
            pack2 = (args, kv2, scores, ids, K_out, V_out, SL_out, O, n_kept)
            _check_single(cfg, d2, k, L_B, pack2)
