"""Results are a pure function of the input bits: the same inputs at different addresses, after a copy that sweeps the
caches, through the single-list and the batched launches, give identical bits 20 times in a row, for scores, indices,
the compacted cache and the attention output (with and without the equal-run workspace, each against itself)."""
import numpy as np
import pytest
import torch

from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import DEV, attention_workspace

pytestmark = pytest.mark.gpu


def _run_all(inp, ws_bytes_shift=0):
    """score -> select -> compact -> attention (plain and with workspace) on the given device tensors."""
    n, Lc, N, D, k = inp["n"], inp["Lc"], inp["N"], inp["D"], inp["k"]
    scores = torch.empty(n + Lc, device=DEV)
    B.pafu_score(inp["X"], inp["W1"], None, inp["W2"], None, scores)
    sel_in = inp["S_ties"]                               # a list with heavy ties decides the selection
    ids = torch.empty(k, dtype=torch.int32, device=DEV)
    B.pafu_select_topk(sel_in, k, ids)
    K_out = torch.empty(k, N, D, device=DEV, dtype=torch.bfloat16)
    V_out = torch.empty_like(K_out)
    SL_out = torch.empty(k, device=DEV)
    B.pafu_compact_kv(inp["K"], inp["V"], sel_in, ids, k, K_out, V_out, SL_out)
    O = torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16)
    B.pafu_chunk_attention(inp["Q"], K_out, V_out, k, inp["Kn"], inp["Vn"], Lc, O)
    Lq1 = inp["Lq_short"]                                # a short chunk takes the equal-run split
    O2 = torch.empty(Lq1, N, D, device=DEV, dtype=torch.bfloat16)
    ws = attention_workspace(D)
    B.pafu_chunk_attention(inp["Q"][:Lq1], K_out, V_out, k, inp["Kn"][:Lq1], inp["Vn"][:Lq1], Lq1, O2, workspace=ws)
    return dict(scores=scores, ids=ids, K_out=K_out, V_out=V_out, SL_out=SL_out, O=O, O_split=O2)


def test_bits_do_not_depend_on_addresses_cache_state_or_batching():
    cfg = wl.C1
    n, Lc, N, D, k, H, M = cfg.n, cfg.Lc, cfg.N, cfg.D, cfg.k, cfg.H, cfg.M
    g = torch.Generator(device=DEV)
    g.manual_seed(20260121)
    r = lambda *shape: torch.randn(*shape, device=DEV, generator=g)
    base = dict(n=n, Lc=Lc, N=N, D=D, k=k, Lq_short=1560,
                X=r(n + Lc, H).to(torch.bfloat16), W1=(r(M, H) * 0.02).to(torch.bfloat16), W2=r(1, M) * 0.02,
                K=r(n, N, D).to(torch.bfloat16), V=r(n, N, D).to(torch.bfloat16), Q=r(Lc, N, D).to(torch.bfloat16),
                Kn=r(Lc, N, D).to(torch.bfloat16), Vn=r(Lc, N, D).to(torch.bfloat16),
                S_ties=torch.round(r(n) * 4.0) / 4.0)     # about 30 distinct values: the k-th is tied hundreds of times
    ref = _run_all(base)
    torch.cuda.synchronize()
    assert int(ref["ids"][-1]) > int(ref["ids"][0]) and torch.isfinite(ref["O"].float()).all()
    sweep_src = torch.empty(768 << 20, dtype=torch.uint8, device=DEV)       # larger than L2 + the memory-side cache
    sweep_dst = torch.empty_like(sweep_src)
    rng = np.random.default_rng(5)
    keep = []
    for it in range(20):
        keep.append(torch.empty(int(rng.integers(1, 64)) * 4096 + 256 * int(rng.integers(0, 16)), dtype=torch.uint8,
                                device=DEV))             # shifts the addresses of everything allocated after it
        inp = {key: (v.clone() if torch.is_tensor(v) else v) for key, v in base.items()}
        sweep_dst.copy_(sweep_src)                        # whatever the caches held is gone
        got = _run_all(inp)
        torch.cuda.synchronize()
        for key in ref:
            assert torch.equal(got[key], ref[key]), (it, key)
        assert all(got[key].data_ptr() != ref[key].data_ptr() for key in ref)
    # the batched launches (one workgroup per list / one launch for several layers) give the same bits as the single ones
    n_l = 3
    args = []
    outs = []
    for l in range(n_l):
        o = dict(scores=torch.empty(n + Lc, device=DEV), ids=torch.empty(k, dtype=torch.int32, device=DEV),
                 K_out=torch.empty(k, N, D, device=DEV, dtype=torch.bfloat16),
                 V_out=torch.empty(k, N, D, device=DEV, dtype=torch.bfloat16), SL_out=torch.empty(k, device=DEV),
                 O=torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16))
        outs.append(o)
        args.append(B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, Lc, base["X"][:n], base["X"][n:], base["W1"],
                                     None, base["W2"], None, base["K"], base["V"], None, base["Q"], base["Kn"],
                                     base["Vn"], o["scores"], o["ids"], o["K_out"], o["V_out"], o["SL_out"], o["O"]))
    B.pafu_step_layers(args)
    single = dict(scores=torch.empty(n + Lc, device=DEV), ids=torch.empty(k, dtype=torch.int32, device=DEV),
                  K_out=torch.empty(k, N, D, device=DEV, dtype=torch.bfloat16),
                  V_out=torch.empty(k, N, D, device=DEV, dtype=torch.bfloat16), SL_out=torch.empty(k, device=DEV),
                  O=torch.empty(Lc, N, D, device=DEV, dtype=torch.bfloat16))
    B.pafu_step(B.make_step_args(B.PAFU_MODE_SINGLE, N, D, n, Lc, k, Lc, base["X"][:n], base["X"][n:], base["W1"], None,
                                 base["W2"], None, base["K"], base["V"], None, base["Q"], base["Kn"], base["Vn"],
                                 single["scores"], single["ids"], single["K_out"], single["V_out"], single["SL_out"],
                                 single["O"]))
    torch.cuda.synchronize()
    for o in outs:
        for key in single:
            assert torch.equal(o[key], single[key]), key
    assert torch.equal(single["scores"], ref["scores"])
