"""The draft step on the library's own per-GPU scratch array (vt_draft_head_step_static).

For callers that cannot allocate.  Its results must be those of vt_draft_head_step bit for bit (same
kernels), and through it those of the oracle; two calls in a row share the array, the second with a
smaller input, so nothing the first call left behind may leak into the second.
"""

import numpy as np
import pytest
import torch

import oracle
import paper_2506_22694_amd as vt
from paper_2506_22694_amd import binding, synth

LOGP_TOL = 2e-3


def _dev():
    return torch.device("cuda:0")


def _to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:      # bf16 bit patterns
        return torch.from_numpy(a.view(np.int16)).to(_dev()).view(torch.bfloat16)
    return torch.from_numpy(a).to(_dev())


def _case(k, d, n, m, seed, dtype):
    W, map_ = synth.trimmed_head_direct(k, d, seed=seed, dtype=dtype)
    h = synth.hidden_rows(n, d, seed=seed, dtype=dtype)
    return W, map_, h


def _static_step(h, W, mp, n, k, m, want_lse=True, want_full=False):
    oi = torch.full((n, m), -7, dtype=torch.int32, device=_dev())
    ol = torch.full((n, m), 7.0, dtype=torch.float32, device=_dev())
    lse = torch.full((n,), 7.0, dtype=torch.float32, device=_dev()) if want_lse else None
    full = torch.full((n, k), 7.0, dtype=torch.float32, device=_dev()) if want_full else None
    vt.draft_head_step_static(h, W, mp, m, oi, ol, out_lse=lse, out_logp_full=full)
    torch.cuda.synchronize()
    return oi, ol, lse, full


@pytest.mark.gpu
def test_static_scratch_step_matches_workspace_step_two_calls_second_smaller():
    # first call: the headline shape (matrix-core kernel + merge kernel); second call, right behind it on the
    # same array: a smaller head with fewer rows (small-n kernel + merge kernel: other offsets inside the
    # array); then the first shape again
    cases = [(32768, 3072, 8, 8, 31, "bf16"), (1000, 512, 2, 3, 32, "bf16"), (32768, 3072, 8, 8, 31, "bf16"),
             (4096, 256, 4, 4, 33, "f32")]
    for (k, d, n, m, seed, dtype) in cases:
        W, map_, h = _case(k, d, n, m, seed, dtype)
        dW, dmap, dh = _to_dev(W), _to_dev(map_), _to_dev(h)
        oi, ol, lse, full = _static_step(dh, dW, dmap, n, k, m, want_full=(k <= 4096))
        wi, wl, wlse = vt.draft_head_step(dh, dW, dmap, m, return_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(oi, wi) and torch.equal(ol, wl) and torch.equal(lse, wlse), (k, d, n, m)
        ref = oracle.draft_head_step(h, W, map_, m)
        assert np.array_equal(oi.cpu().numpy(), ref["ids"]), (k, d, n, m)
        assert np.abs(ol.cpu().numpy().astype(np.float64) - ref["logp"]).max() <= LOGP_TOL
        assert np.abs(lse.cpu().numpy().astype(np.float64) - ref["lse"]).max() <= LOGP_TOL
        if full is not None:
            want = ref["z"] - ref["lse"][:, None]
            assert np.abs(full.cpu().numpy().astype(np.float64) - want).max() <= LOGP_TOL


@pytest.mark.gpu
def test_static_scratch_step_tree_shape_then_chain_shape():
    # 64 tree nodes x top-8 (1.2 MB of per-tile candidate lists in the array), then one row, top-1
    for (k, d, n, m, seed) in [(32768, 4096, 64, 8, 41), (32768, 2048, 1, 1, 42)]:
        W, map_, h = _case(k, d, n, m, seed, "bf16")
        dW, dmap, dh = _to_dev(W), _to_dev(map_), _to_dev(h)
        oi, ol, lse, _ = _static_step(dh, dW, dmap, n, k, m)
        wi, wl, wlse = vt.draft_head_step(dh, dW, dmap, m, return_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(oi, wi) and torch.equal(ol, wl) and torch.equal(lse, wlse), (k, d, n, m)


@pytest.mark.gpu
def test_static_scratch_step_rejects_shapes_beyond_its_array():
    L = vt.load_library()
    k, d, n, m = 32768, 8192, 256, 16          # the per-row tail would store 32 MiB of logits
    assert L.vt_draft_head_step_ws_bytes(n, k, d, m) > binding.VT_STATIC_WS_BYTES
    W, map_, h = _case(k, 128, n, m, 43, "bf16")     # the check depends on (n, k, m) here, not on real data
    dW, dmap, dh = _to_dev(W), _to_dev(map_), _to_dev(h)
    oi = torch.empty((n, m), dtype=torch.int32, device=_dev())
    ol = torch.empty((n, m), dtype=torch.float32, device=_dev())
    assert L.vt_draft_head_step_ws_bytes(n, k, 128, m) > binding.VT_STATIC_WS_BYTES
    with pytest.raises(vt.VocabTrimError) as e:
        vt.draft_head_step_static(dh, dW, dmap, m, oi, ol)
    assert e.value.status == 5
