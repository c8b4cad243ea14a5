"""GPU parity of symi_expert_bwd_active + symi_adam_to_replicas_active: against the oracle
(whose gradient of a class without tokens is zero) and, bit for bit, against the plain pair."""
import numpy as np
import pytest
import torch

import paper_2504_19925_amd as symi
import workloads as wl
import harness as Hn
from tests.checks import check_iteration, small as _small

pytestmark = pytest.mark.gpu


def _starve(logits, classes):
    """No token picks these classes."""
    z = logits.clone()
    z[:, classes] = -1.0e4
    return z


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_active_pair_against_the_oracle(name):
    c = _small(name)
    print(f"[active] {name}: {c}", flush=True)
    st = Hn.State(c, shard=min(1, c.N - 1))
    st.active_grads = True
    for it in range(2):
        X, logits, dY = Hn.draw_inputs(c, it)
        logits = _starve(logits, [1, c.E - 1] if it == 0 else [0, 2, 3])
        check_iteration(st, X, logits, dY, hp_kw=dict(step=it + 1))
        assert int((st.hist == 0).sum()) >= 2
        st.hist_prev.copy_(st.hist)


@pytest.mark.parametrize("name", ["c1", "c2", "c4"])
def test_active_pair_equals_plain_pair_bit_for_bit(name):
    c = _small(name)
    print(f"[active==plain] {name}: {c}", flush=True)
    X, logits, dY = Hn.draw_inputs(c, 0)
    logits = _starve(logits, [0, 3, c.E - 2])
    weights = wl.make_class_weights(c, "cuda")
    adam, _ = Hn.make_adam(step=3)
    res = []
    for active in (False, True):
        st = Hn.State(c, shard=c.N - 1, weights=weights)
        st.active_grads = active
        st.m.uniform_(-1e-3, 1e-3, generator=torch.Generator("cuda").manual_seed(5))
        st.v.uniform_(0.0, 1e-6, generator=torch.Generator("cuda").manual_seed(6))
        st.place_current()
        st.forward(X, logits)
        st.dW1.fill_(float("nan") if active else 7.0)
        st.dW2.fill_(float("nan") if active else 7.0)
        st.backward(dY, logits)
        st.optimizer(adam)
        Hn.sync()
        res.append(st)
    a, b = res
    has = (a.hist > 0)
    assert 0 < int(has.sum()) < c.E
    for name_ in ("dXp", "dX", "dlogits", "master", "m", "v", "W1s", "W2s"):
        assert torch.equal(getattr(a, name_), getattr(b, name_)), name_
    assert torch.equal(a.dW1[has], b.dW1[has]) and torch.equal(a.dW2[has], b.dW2[has])
    assert not a.dW1[~has].any() and not a.dW2[~has].any()            # plain: zeros written
    assert torch.isnan(b.dW1[~has]).all() and torch.isnan(b.dW2[~has]).all()   # active: untouched


def test_active_adam_requires_the_current_placement():
    c = _small("c1")
    st = Hn.State(c)
    adam, _ = Hn.make_adam()
    lib = symi.binding.lib()
    import ctypes
    rc = lib.symi_adam_to_replicas_active(
        st.ctx.ptr, ctypes.byref(adam), st.dW1.data_ptr(), st.dW2.data_ptr(),
        st.master.data_ptr(), st.m.data_ptr(), st.v.data_ptr(), None, None,
        st.first_slot_next.data_ptr(), st.W1s.data_ptr(), st.W2s.data_ptr(), None)
    assert rc == -1 and "NULL" in symi.symi_last_error()
