"""made_forward_logits_noalloc (the entry point that allocates nothing: its scratch memory is a static device
array) against made_forward_logits, through the C ABI: bit-identical logits on calls in a row that shrink, grow
and change model, so that the array's stale contents from one call are what the next one finds."""
import numpy as np
import pytest
import torch

from paper_2002_03629_amd import binding as B
from paper_2002_03629_amd import synth as S

pytestmark = pytest.mark.gpu


def _logits(h, fn, x, D, C):
    N = x.shape[0]
    out = torch.full((N, D, C), float("nan"), dtype=torch.float32, device="cuda")
    fn(h, torch.from_numpy(x).cuda(), N, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_noalloc_logits_equal_the_allocating_entry_point():
    rng = np.random.default_rng(5)
    models = {}
    try:
        for name in ("mid_bf16", "small_f32", "small_cat", "small_cat_onehot"):
            w = S.workload(name)
            net = S.make_network(w, with_bias=True)
            models[name] = (w, B.model_from_network(net))
        # two calls in a row on one model, the second smaller; then other models (other layouts of the array,
        # fp32 after bf16: stale bf16 pairs read as floats), then the first model again, larger than before
        plan = [("mid_bf16", 70), ("mid_bf16", 9), ("small_f32", 33), ("small_cat", 10), ("small_cat_onehot", 7),
                ("mid_bf16", 200), ("small_f32", 1)]
        for name, N in plan:
            w, h = models[name]
            hi = 2 if w.C == 1 else w.C
            x = rng.integers(0, hi, size=(N, w.D)).astype(np.uint8)
            ref = _logits(h, B.made_forward_logits, x, w.D, w.C)
            got = _logits(h, B.made_forward_logits_noalloc, x, w.D, w.C)
            assert np.isfinite(got).all(), (name, N)
            assert (got == ref).all(), (name, N, float(np.abs(got - ref).max()))
        # an empty batch does nothing; a batch beyond the static array is refused with the limit in the message
        w, h = models["mid_bf16"]
        B.made_forward_logits_noalloc(h, None, 0, None)
        per_row = (256 + 512 + 512) * 2                   # padded widths 196 -> 256, 500 -> 512 (twice), bf16
        too_many = (8 << 20) // per_row + 64
        x = torch.zeros((too_many, w.D), dtype=torch.uint8, device="cuda")
        out = torch.empty((too_many, w.D, 1), dtype=torch.float32, device="cuda")
        with pytest.raises(B.MadeError) as e:
            B.made_forward_logits_noalloc(h, x, too_many, out)
        assert e.value.code == B.MADE_ERR_ARG and "at most" in str(e.value)
        fits = (8 << 20) // per_row // 64 * 64
        xs = rng.integers(0, 2, size=(fits, w.D)).astype(np.uint8)
        assert (_logits(h, B.made_forward_logits_noalloc, xs, w.D, 1) == _logits(h, B.made_forward_logits, xs, w.D, 1)).all()
    finally:
        for _, h in models.values():
            B.made_free(h)


def test_noalloc_refuses_other_models_without_a_gpu_call():
    L = B.lib()
    assert L.made_forward_logits_noalloc(None, None, 4, None, None) == B.MADE_ERR_ARG
