"""The allocation-free decode entry point (scratch held by the library) against the ordinary one, through the
C ABI: same inputs, twin caches, two calls in a row on the shared scratch, the second with a smaller input."""
import pytest
import torch

from paper_2503_10714_amd import binding as zb
from paper_2503_10714_amd import synth
from tests import parity_util as pu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _twins(wl, parts):
    """Two caches with the same prefilled state (one device prefill each, from the same bytes)."""
    caches = []
    for _ in range(2):
        c = pu.make_cache(wl, DEV)
        c.set_decode_parts(parts)
        for l in range(wl.n_layers):
            Q, K, V, lens = synth.prompt(wl, l)
            c.prefill_compress(l, Q.to(DEV), K.to(DEV), V.to(DEV), lens)
        caches.append(c)
    return caches


def _step_both(wl, ref, sta, step):
    L, S, H, G, d = wl.n_layers, wl.n_seqs, wl.n_kv_heads, wl.q_per_kv, wl.head_dim
    qs, ks, vs = zip(*[synth.decode_inputs(wl, l, step) for l in range(L)])
    q, k, v = torch.stack(qs).to(DEV), torch.stack(ks).to(DEV), torch.stack(vs).to(DEV)
    out_r = torch.full((L, S, H, G, d), float("nan"), dtype=torch.float32, device=DEV)
    out_s = torch.full_like(out_r, float("nan"))
    info_r = tuple(torch.empty(L, S, H, dtype=torch.int32, device=DEV) for _ in range(3))
    info_s = tuple(torch.full((L, S, H), -7, dtype=torch.int32, device=DEV) for _ in range(3))
    zb.zsm_decode_step(ref.handle, 0, L, q, k, v, out_r, *info_r)
    zb.zsm_decode_step_static(sta.handle, 0, L, q, k, v, out_s, *info_s)
    torch.cuda.synchronize()
    assert torch.equal(out_s, out_r), (f"{wl.name} step {step}: outputs differ by {(out_s - out_r).abs().max().item():.3e}; not written: "
                                       f"static {torch.isnan(out_s).float().mean().item():.3f}, ordinary {torch.isnan(out_r).float().mean().item():.3f}")
    for a, b in zip(info_s, info_r):
        assert torch.equal(a, b), f"step {step}: decisions differ"


def _same_state(wl, ref, sta):
    for l in range(wl.n_layers):
        a, b = sta.export_layer(l), ref.export_layer(l)
        for key in a:
            assert torch.equal(a[key], b[key]), f"layer {l}: {key} differs"


def test_static_scratch_entry_point_matches_the_ordinary_one():
    big = synth.Workload(name="noalloc_big", n_layers=2, n_seqs=2, n_kv_heads=3, q_per_kv=3, head_dim=128, dtype="f16",
                         prompt_len=700, budget=301, decode_steps=6, window=16, outliers=True, n_residual=2)
    small = synth.Workload(name="noalloc_small", n_layers=1, n_seqs=1, n_kv_heads=2, q_per_kv=1, head_dim=64, dtype="f32",
                           prompt_len=150, budget=70, decode_steps=6, window=8, outliers=False)
    ref_b, sta_b = _twins(big, 3)
    ref_s, sta_s = _twins(small, 2)
    assert sta_b.decode_parts() == 3 and sta_s.decode_parts() == 2      # both launches are split: they use the scratch
    # two calls in a row on the library's scratch, the second with the smaller input; then on, alternating
    for step in range(big.decode_steps):
        _step_both(big, ref_b, sta_b, step)
        _step_both(small, ref_s, sta_s, step)
    _same_state(big, ref_b, sta_b)
    _same_state(small, ref_s, sta_s)
    # a launch that is not split needs no scratch and goes through as well
    sta_s.set_decode_parts(1); ref_s.set_decode_parts(1)
    _step_both(small, ref_s, sta_s, small.decode_steps)
    # so does a step over more than eight query heads per KV head (its pooled sums live in the cache buffer)
    mqa = synth.Workload(name="noalloc_mqa", n_layers=1, n_seqs=2, n_kv_heads=1, q_per_kv=12, head_dim=64, dtype="bf16",
                         prompt_len=200, budget=60, decode_steps=4, window=8, outliers=True, n_residual=1)
    ref_m, sta_m = _twins(mqa, 0)
    for step in range(mqa.decode_steps):
        _step_both(mqa, ref_m, sta_m, step)
    _same_state(mqa, ref_m, sta_m)
    for c in (ref_b, sta_b, ref_s, sta_s, ref_m, sta_m):
        c.close()


def test_static_scratch_limit_is_reported():
    """A split launch whose partial results exceed the library's array is refused before anything is enqueued."""
    c = zb.Cache(1, 8, 32, 4, 128, 2000, 2000, 1, "f16", device=DEV)     # 256 units x 4 heads x 4002 slots x 8 B = 33 MB
    c.set_decode_parts(2)
    assert c.decode_parts() == 2
    q = torch.zeros(1, 8, 32, 4, 128, dtype=torch.float16, device=DEV)
    k = torch.zeros(1, 8, 32, 128, dtype=torch.float16, device=DEV)
    out = torch.zeros(1, 8, 32, 4, 128, dtype=torch.float32, device=DEV)
    with pytest.raises(zb.ZsmError) as e:
        zb.zsm_decode_step_static(c.handle, 0, 1, q, k, k, out)
    assert e.value.status == -9 and "scratch" in str(e.value)
    st = c.export_layer(0)
    assert (st["n_seen"] == 0).all() and (st["w"] == 0).all()
    c.close()
