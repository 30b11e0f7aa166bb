"""slide_predict_static (the entry point for callers that cannot allocate: all intermediates in a fixed
array inside the library) against slide_predict mode 1, which is itself checked against the oracle: same
ids, same scores, on two calls in a row, the second with a smaller input; in both input modes."""
import numpy as np
import pytest

from paper_2201_12667_amd import slide, synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

from helpers import FLOOR, REL, make_pair  # noqa: E402


def _sub_batch(b, n, dense):
    ye = int(b["y_indptr"][n])
    out = dict(batch=n, y_indptr=b["y_indptr"][:n + 1], y_indices=b["y_indices"][:ye])
    if dense:
        out["hidden"] = b["hidden"][:n]
    else:
        xe = int(b["x_indptr"][n])
        out.update(x_indptr=b["x_indptr"][:n + 1], x_indices=b["x_indices"][:xe], x_values=b["x_values"][:xe])
    return out


@pytest.mark.parametrize("name,wl", [
    ("sparse-input", synth.small(synth.HASH_DWTA, num_classes=150_001, batch=slide.STATIC_MAX_BATCH, K=4, L=5)),
    ("dense-hidden", synth.small(synth.HASH_SIMHASH, num_classes=40_009, batch=slide.STATIC_MAX_BATCH, input_dim=0,
                                 hidden_dim=200, K=6, L=4)),
])
def test_static_scratch_prediction_equals_workspace_prediction(name, wl):
    print("static scratch", name, flush=True)
    gen, model, orc = make_pair(wl)
    model.build_tables()
    dense = wl.input_dim == 0
    big = gen.batch(0)
    for step, (n, topk) in enumerate([(wl.batch, 7), (17, 64), (1, 3)]):    # second and third calls: smaller inputs
        hb = _sub_batch(gen.batch(step), n, dense) if n < wl.batch else big
        db = model.to_device(hb)
        out = (torch.full((n, topk), -7, dtype=torch.int32, device=model.dev),
               torch.full((n, topk), 123.0, dtype=torch.float32, device=model.dev))
        ids_s, sc_s = model.predict_static(db, topk, out)
        ids_w, sc_w = model.predict(db, topk, mode=1)
        torch.cuda.synchronize()
        assert model.status() == 0
        assert torch.equal(ids_s, ids_w), (name, step)
        assert torch.equal(sc_s, sc_w), (name, step)
        # and one sample against the oracle's double-precision scores
        i = n // 2
        h = orc.forward_hidden(hb).astype(np.float64)
        z = orc.p["W2"].astype(np.float64) @ h[i] + orc.p["b2"]
        order = np.lexsort((np.arange(z.size), -z))[:topk]
        got = sc_s[i].cpu().numpy()
        assert np.all(np.abs(got - z[order]) <= REL * np.abs(z[order]) + FLOOR * np.abs(z).max())
    # limits: a batch beyond the static maximum is refused on the host
    wl2 = synth.small(wl.hash_kind, num_classes=2000, batch=slide.STATIC_MAX_BATCH + 1, input_dim=wl.input_dim,
                      hidden_dim=wl.hidden_dim, K=wl.K, L=wl.L)
    gen2, big_model, _ = make_pair(wl2)
    big_model.build_tables()
    with pytest.raises(slide.SlideError) as e:
        big_model.predict_static(big_model.to_device(gen2.batch(0)), 5)
    assert e.value.code == slide.SLIDE_ENOMEM
    big_model.destroy()
    model.destroy()
