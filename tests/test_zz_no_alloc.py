"""The allocation-free entry point against the handle-based one (needs an MI355X).  Collected last on purpose."""
import numpy as np
import pytest
import torch

from paper_2511_11062_amd import inputs
from paper_2511_11062_amd import lite_attn as la

pytestmark = pytest.mark.gpu


def _layer(name, heads, grid, seed, text=0):
    wl = inputs.Workload(name, 1, heads, grid, text_tokens=text, steps=2, seed=seed)
    seq = inputs.DriftSequence(wl, "cpu")
    return wl, [tuple(x.cuda().contiguous() for x in next(seq)) for _ in range(2)]


def test_static_entry_point_matches_the_handle_path():
    """lite_attn_fwd_static on two layers in a row, the second smaller than the first (so the static array still holds
    the first one's Skip-List, row schedule and V^T beyond what the second overwrites), two timesteps each with the
    caller-owned Skip-Mask carried from the first to the second: outputs and masks must equal what lite_attn_fwd
    gives with a handle -- the same kernels on the same inputs, so bit for bit, which is inside every tolerance."""
    stream = torch.cuda.current_stream().cuda_stream
    thr = [-3.0, -2.0]
    layers = [_layer("na_big", 3, (2, 24, 31), 51, text=40), _layer("na_small", 2, (1, 12, 25), 52)]   # N = 1528, 300
    assert layers[1][0].seqlen < layers[0][0].seqlen
    for wl, data in layers:
        H, N = wl.heads, wl.seqlen
        h = la.lite_attn_init_mask(1, H, N, protect=wl.protect, max_steps=2)
        la.lite_attn_set_stream(h, stream)
        ref = []
        try:
            for t, (q, k, v) in enumerate(data):
                o = torch.empty_like(q)
                la.lite_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), h, thr[t], t)
                torch.cuda.synchronize()
                ref.append((o, la.lite_attn_mask_export(h).copy()))
        finally:
            la.lite_attn_free_mask(h)
        desc = la.make_desc(1, H, N, protect=wl.protect, max_steps=1)
        mask = torch.zeros(la.static_mask_words(desc), dtype=torch.int64, device="cuda")     # the caller's Skip-Mask
        for t, (q, k, v) in enumerate(data):
            o = torch.full_like(q, float("nan"))
            la.lite_attn_fwd_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), desc, mask.data_ptr(),
                                    thr[t], stream)
            torch.cuda.synchronize()
            got_mask = mask.cpu().numpy().view(np.uint64)
            assert np.array_equal(got_mask, ref[t][1]), "%s step %d: Skip-Mask differs" % (wl.name, t)
            assert ref[t][1].any()
            d = (o.float() - ref[t][0].float()).abs()
            assert torch.isfinite(o).all()
            assert d.max().item() <= 1e-2 * ref[t][0].float().abs().max().item() and d.mean().item() <= 1e-3
            assert torch.equal(o, ref[t][0]), "%s step %d: output differs" % (wl.name, t)


def test_static_entry_point_refuses_what_does_not_fit():
    wl = inputs.WORKLOADS["wan14b"]
    desc = la.make_desc(1, wl.heads, wl.seqlen)
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    m = torch.zeros(8, dtype=torch.int64, device="cuda")
    with pytest.raises(la.LiteAttnError) as err:
        la.lite_attn_fwd_static(x.data_ptr(), x.data_ptr(), x.data_ptr(), x.data_ptr(), desc, m.data_ptr(), -1.0,
                                torch.cuda.current_stream().cuda_stream)
    assert err.value.code == -7
