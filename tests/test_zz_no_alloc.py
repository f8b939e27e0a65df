"""pafu_score_static (the entry point that allocates nothing: its scratch is a static device array inside the
library) against pafu_score on the same inputs, through the C ABI, on two calls in a row, the second with a smaller
input and a narrower hidden layer, so that stale scratch contents from the first call would show."""
import numpy as np
import pytest
import torch

from oracle import pafu_oracle as orc
from paper_2601_21896_amd import binding as B
from paper_2601_21896_amd import workloads as wl
from tests.gpu_util import DEV, SCORE_MAX_ABS, bits, dev, host

pytestmark = pytest.mark.gpu


def _case(T, F, M, n_out, seed, dtype="bf16"):
    rng = np.random.Generator(np.random.PCG64(seed))
    q = wl.round_to_bf16 if dtype == "bf16" else (lambda a: a)
    X = q(rng.standard_normal((T, F), dtype=np.float32))
    W1 = q(rng.standard_normal((M, F), dtype=np.float32) * np.float32(0.02))
    b1 = rng.standard_normal(M, dtype=np.float32) * np.float32(0.02)
    W2 = rng.standard_normal((n_out, M), dtype=np.float32) * np.float32(0.02)
    b2 = rng.standard_normal(n_out, dtype=np.float32) * np.float32(0.02)
    return X, W1, b1, W2, b2


def _both(X, W1, b1, W2, b2, dtype="bf16"):
    dt = dtype if dtype == "bf16" else None
    dX, dW1, db1, dW2, db2 = dev(X, dt), dev(W1, dt), dev(b1), dev(W2), dev(b2)
    T, M = X.shape[0], W1.shape[0]
    ws = torch.empty(B.pafu_score_workspace_bytes(M) // 4 + 1, device=DEV)
    want = torch.full((T + 4,), 9.0, device=DEV)
    got = torch.full((T + 4,), 9.0, device=DEV)
    B.pafu_score(dX, dW1, db1, dW2, db2, want[:T], workspace=ws)
    B.pafu_score_static(dX, dW1, db1, dW2, db2, got[:T])
    torch.cuda.synchronize()
    assert torch.all(got[T:] == 9.0)
    return got[:T], want[:T]


def test_score_static_matches_score_on_two_calls_in_a_row():
    first = _case(3000, 1536, 256, 12, seed=11)       # streaming MFMA kernel, 12 outputs averaged
    second = _case(777, 192, 64, 5, seed=12)          # smaller input, narrower hidden layer, another kernel
    third = _case(100, 40, 24, 3, seed=13, dtype="f32")   # plain-FMA kernel
    for case, dtype in ((first, "bf16"), (second, "bf16"), (third, "f32")):
        got, want = _both(*case, dtype=dtype)
        assert np.array_equal(bits(got), bits(want))                      # same kernels, same bits
        ref = orc.smlp_score(*case)
        assert np.abs(host(got) - ref).max() < SCORE_MAX_ABS
        assert np.abs(ref).max() > 1e-3


def test_score_static_rejects_a_hidden_layer_beyond_its_scratch():
    X = torch.zeros(4, 64, device=DEV, dtype=torch.bfloat16)
    W1 = torch.zeros(8193, 64, device=DEV, dtype=torch.bfloat16)
    W2 = torch.zeros(2, 8193, device=DEV)
    out = torch.full((4,), 3.0, device=DEV)
    with pytest.raises(B.PafuError) as e:
        B.pafu_score_static(X, W1, None, W2, None, out)
    assert e.value.status == -5
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)                      # nothing was enqueued
