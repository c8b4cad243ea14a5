"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on the five workload recipes at sizes the oracle finishes in seconds (several
tiles, ragged tails, empty groups), plus edge cases.  Integer outputs bit-exact; floats
within 1e-5 (fp32 path, routing data), 2e-2 (bf16 path), 1e-6 (Adam state)."""
import numpy as np
import pytest
import torch

import paper_2504_19925_amd as symi
import workloads as wl
from oracle import symi_oracle as O
import harness as Hn
from harness.metrics import TOL, check_close, relerr_elem
from tests.checks import OracleChain, check_iteration, small as _small

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4", "c5"])
def test_config_parity(name):
    """The whole schedule a config states (c2: 10 iterations, c4: 20, the others one) as ONE
    chain (Sec. 3.2 steps 1-8, Sec. 3.4): all N optimizer partitions step, the placement of
    iteration t+1 mimics the popularity of iteration t, and the forward of iteration t+1 runs
    on the slots that iteration t's symi_adam_to_replicas calls wrote.  Every iteration is
    checked stage by stage against the oracle (fed the GPU's own upstream state); the distance
    to an oracle that runs the whole chain on its own is reported at the end."""
    c = _small(name)
    print(f"[parity] {name}: {c}", flush=True)
    st = Hn.State(c, shard=min(1, c.N - 1), all_shards=True)
    chain = OracleChain(c, st.W1c, st.W2c)
    for it in range(c.iters):
        X, logits, dY = Hn.draw_inputs(c, it)
        check_iteration(st, X, logits, dY, hp_kw=dict(step=it + 1), chained=True)
        chain.step(X, logits, dY, Hn.make_adam(step=it + 1)[1])
        st.hist_prev.copy_(st.hist)     # the next iteration mimics this one's popularity ...
        st.advance()                    # ... with the placement the optimizer just filled
    drift = chain.drift(st)
    print(f"[parity] {name}: end-to-end drift after {c.iters} iteration(s) against the oracle's own chain "
          + " ".join(f"{k}={v:.2e}" for k, v in drift.items()), flush=True)
    # loose sanity bound only (the asserted tolerances are the stage-isolated ones above): the
    # weights move by at most lr per step, so two unrelated chains would end about
    # sqrt(2)*steps*lr/rms(w) apart in L2; chains that describe the same training run differ
    # only in the elements whose gradient is lost in the arithmetic's noise
    assert drift["master_l2"] < (1e-4 if c.dtype == "f32" else 0.2)


def test_placement_invariance_of_the_layer():
    """Replication changes where a row is processed, not the result: Y and the class
    gradients under a skewed placement equal those under the uniform one (bit for bit in
    the forward, because every row sees the same weights and reduction order)."""
    c = wl.scaled(wl.get_config("c2"), d=128, f=256, T=700, E=8, S_tot=24)
    X, logits, dY = Hn.draw_inputs(c, 0)
    outs = []
    for pop in ([0] * 8, [1000, 1, 1, 1, 1, 1, 1, 1], [0, 0, 0, 0, 0, 0, 0, 999]):
        st = Hn.State(c)
        st.hist_prev.copy_(torch.tensor(pop, dtype=torch.int32))
        st.place_current()
        st.forward(X, logits)
        st.backward(dY, logits)
        Hn.sync()
        outs.append((st.Y.clone(), st.dX.clone(), st.dW1.clone(), st.dW2.clone(),
                     st.counts.cpu().tolist()))
    assert outs[0][4] != outs[1][4] != outs[2][4]
    for o in outs[1:]:
        assert torch.equal(o[0], outs[0][0])
        assert torch.equal(o[1], outs[0][1])
        assert relerr_elem(Hn.npf(o[2]), Hn.npf(outs[0][2])) < 1e-5
        assert relerr_elem(Hn.npf(o[3]), Hn.npf(outs[0][3])) < 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_cases(dtype):
    base = wl.scaled(wl.get_config("c1"), dtype=dtype)
    cases = [
        wl.scaled(base, T=1, E=1, k=1, S_tot=1, N=1, d=8, f=8),            # smallest legal shape
        wl.scaled(base, T=5, E=4, k=4, S_tot=4, N=2, d=16, f=24),          # k = E, one slot per class
        wl.scaled(base, T=130, E=3, k=1, S_tot=64, N=3, d=40, f=72),       # many more slots than rows/classes
        wl.scaled(base, T=257, E=24, k=2, S_tot=24, N=1, d=72, f=200),     # E not a power of two
        wl.scaled(base, T=0, E=8, k=2, S_tot=16, N=4, d=128, f=256),       # empty batch
        wl.scaled(base, T=300, E=130, k=5, S_tot=257, N=2, d=64, f=64, router_matmul=False,
                  bias="zipf", zipf_s=1.2),                                # E > 128, S_tot > 256
    ]
    for c in cases:
        print(f"[edge] {c}", flush=True)
        st = Hn.State(c, shard=c.N - 1)
        X, logits, dY = Hn.draw_inputs(c, 0)
        check_iteration(st, X, logits, dY)


def test_tied_logits_and_renorm_off():
    c = wl.scaled(wl.get_config("c1"), T=512, E=64, k=6, S_tot=80, router_matmul=False)
    st = Hn.State(c, renorm=0)
    X, logits, dY = Hn.draw_inputs(c, 0)
    logits = (logits * 2).round() / 2          # many exact ties inside every row
    logits[::5] = 0.0                          # fully tied rows
    check_iteration(st, X, logits.contiguous(), dY)


def test_adam_weight_decay_grad_scale_and_later_steps():
    c = wl.scaled(wl.get_config("c2"), d=64, f=96, T=400, E=8, S_tot=12, N=4)
    st = Hn.State(c, shard=3)
    for it in range(3):
        X, logits, dY = Hn.draw_inputs(c, it)
        check_iteration(st, X, logits, dY, hp_kw=dict(step=it + 1, weight_decay=0.05,
                                                      grad_scale=0.125, lr=3e-3))
        st.hist_prev.copy_(st.hist)


def test_place_device_matches_oracle_on_random_popularities():
    """The device scheduler evaluates Algorithm 1's correction loops in closed form; it must
    reproduce the literal loops (the oracle) bit for bit, also on adversarial ties."""
    import random
    import paper_2504_19925_amd as symi
    rnd = random.Random(99)
    cases = [([5, 5, 4, 2], 16), ([1024, 1024, 0, 0, 0, 0, 0, 0], 16), ([0] * 64, 96), ([10, 3, 10, 5], 16),
             ([1000000] + [0] * 63, 64), ([7] * 16, 64), ([1] * 130, 257), ([3, 3, 3], 64)]
    for _ in range(400):
        E = rnd.choice([1, 2, 3, 8, 24, 64, 65, 128, 130, 300, 1024])
        S = rnd.randint(E, min(4096, 4 * E + 3))
        kind = rnd.random()
        if kind < 0.3:
            pop = [rnd.choice([0, 0, 1, 2, 2, 7]) for _ in range(E)]           # many ties
        elif kind < 0.6:
            pop = [int(100000 / (r + 1) ** 1.2) for r in range(E)]
            rnd.shuffle(pop)
        else:
            pop = [rnd.choice([0, 1, rnd.randint(0, 60000)]) for _ in range(E)]
        cases.append((pop, S))
    for pop, S in cases:
        E = len(pop)
        ctx = symi.symi_create(symi.SymiCfg.make(64, E, 1, 128, 256, S, 1, 0, "f32", 1))
        dev = dict(dtype=torch.int32, device="cuda")
        counts, placement, first = torch.zeros(E, **dev), torch.zeros(S, **dev), torch.zeros(E + 1, **dev)
        symi.symi_place(ctx, torch.tensor(pop, **dev), counts, placement, first)
        oc, op, of = O.place(pop, S)
        assert counts.cpu().tolist() == oc.tolist(), (pop[:16], S)
        assert placement.cpu().tolist() == op.tolist()
        assert first.cpu().tolist() == of.tolist()


def test_backward_on_two_streams_equals_backward_on_one():
    """symi_expert_bwd may run its two chains of products on two streams (small batches); the
    results are the same bits as with every kernel on the caller's stream (a context created
    with SYMI_CTX_NO_OVERLAP), also when the caller's stream is not the default one."""
    c = _small("c2")
    weights = wl.make_class_weights(c, "cuda")
    X, logits, dY = Hn.draw_inputs(c, 0)
    outs = []
    for flags, own_stream in ((0, False), (symi.CTX_NO_OVERLAP, False), (0, True)):
        st = Hn.State(c, weights=weights, flags=flags)
        st.place_current()
        st.forward(X, logits)
        for t in (st.dX, st.dW1, st.dW2, st.dXp):
            t.fill_(float("nan"))
        if own_stream:
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                st.backward(dY, logits)
            torch.cuda.current_stream().wait_stream(s)
        else:
            st.backward(dY, logits)
        Hn.sync()
        outs.append([t.clone() for t in (st.dX, st.dW1, st.dW2, st.dgate, st.dlogits)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b)


def test_shape_limits_of_the_interface():
    """The largest class, choice and slot counts the interface accepts (E = 1024, k = 16,
    S_tot = 4096), two iterations so that the second placement is a replicated one."""
    base = wl.scaled(wl.get_config("c1"), dtype="bf16")
    c = wl.scaled(base, T=700, E=1024, k=16, S_tot=4096, N=4, d=64, f=64, router_matmul=False,
                  bias="zipf", zipf_s=0.5)
    st = Hn.State(c, shard=1)
    for it in range(2):
        X, logits, dY = Hn.draw_inputs(c, it)
        check_iteration(st, X, logits, dY)
        st.hist_prev.copy_(st.hist)


def test_forward_backward_under_graph_capture():
    """The calls can be captured into a HIP graph (including the helper-stream fork/join of the
    backward): every replay, with eager work and synchronisations in between, reproduces the
    eager results bit for bit."""
    c = _small("c2")
    st = Hn.State(c)
    X, logits, dY = Hn.draw_inputs(c, 0)
    st.place_current()
    st.forward(X, logits)
    st.backward(dY, logits)          # eager reference
    Hn.sync()
    outs = (st.Y, st.dX, st.dW1, st.dW2, st.dgate, st.dlogits, st.hist, st.row_of_assign, st.slot_offsets)
    want = [t.clone() for t in outs]
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        st.forward(X, logits)
        st.backward(dY, logits)
        torch.cuda.current_stream().synchronize()
        g.capture_begin()
        st.forward(X, logits)
        st.backward(dY, logits)
        g.capture_end()
    torch.cuda.current_stream().wait_stream(s)
    Hn.sync()
    scratch = torch.empty(1 << 20, device="cuda")
    for rep in range(4):
        for t in outs:
            t.zero_() if t.dtype == torch.int32 else t.fill_(float("nan"))
        scratch.normal_()            # eager work between the replays
        Hn.sync()
        g.replay()
        Hn.sync()
        for t, w in zip(outs, want):
            assert torch.equal(t, w), f"replay {rep}"


def test_whole_steps_replayed_from_graphs_equal_eager_steps():
    """Layer, backward, placement and optimizer of consecutive iterations captured as one HIP
    graph per distinct step (inputs of period 2, placement buffers of period 2) and replayed:
    the optimizer state and the slots end up bit for bit where eager launches put them."""
    c = _small("c2")
    weights = wl.make_class_weights(c, "cuda")
    inputs = [Hn.draw_inputs(c, it) for it in range(2)]
    adam, _ = Hn.make_adam(step=2)

    def make():
        st = Hn.State(c, shard=1, weights=weights)
        st.active_grads = True
        st.place_current()
        return st

    def step(st, i):
        X, logits, dY = inputs[i % 2]
        st.forward(X, logits)
        st.backward(dY, logits)
        st.optimizer(adam)
        st.advance()

    a, b = make(), make()
    for st in (a, b):
        step(st, 0)
    Hn.sync()
    for i in range(1, 6):
        step(a, i)
    Hn.sync()
    graphs = []
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    scratch = torch.empty(1 << 20, device="cuda")
    with torch.cuda.stream(side):
        for i in (1, 2):
            g = torch.cuda.CUDAGraph()
            g.capture_begin()
            step(b, i)
            g.capture_end()
            graphs.append(g)
        Hn.sync()
        for i in range(1, 6):
            graphs[(i - 1) % 2].replay()
            scratch.normal_()         # eager work and a synchronisation between the replays
            Hn.sync()
    torch.cuda.current_stream().wait_stream(side)
    b.advance()                       # five replays: an odd number of role swaps on the device side
    Hn.sync()
    for name in ("master", "m", "v", "W1s", "W2s", "Y", "dX", "dlogits", "hist", "placement",
                 "first_slot", "slot_offsets"):
        assert torch.equal(getattr(a, name), getattr(b, name)), name


def test_sliced_reductions_with_ragged_lengths():
    """A few m-tiles and long reductions: the two narrow products (Yp over f, dXp over 2f) have
    their tiles' reductions cut into slices (2 and 4 here on a 256-CU part), the last slice
    ending in a partial 64-deep step; checked element by element against the oracle, and
    equal, up to the order of the fp32 sums, to the uncut products."""
    c = wl.scaled(wl.get_config("c2"), E=8, S_tot=16, N=4, d=512, f=2056, T=1100, iters=1)
    print(f"[sliced] {c}", flush=True)
    st = Hn.State(c, shard=2)
    X, logits, dY = Hn.draw_inputs(c, 0)
    check_iteration(st, X, logits, dY)
    st.forward(X, logits)            # again: the optimizer has rewritten the slots meanwhile
    st.backward(dY, logits)
    Hn.sync()
    Yp, dXp = st.Yp.clone(), st.dXp.clone()
    whole = symi.symi_create(st.cfg, symi.CTX_NO_SLICING)      # same buffers, reductions left whole
    st.ctx, sliced = whole, st.ctx
    st.forward(X, logits)
    st.backward(dY, logits)
    Hn.sync()
    st.ctx = sliced
    for a, b in ((st.Yp, Yp), (st.dXp, dXp)):
        a, b = a.float(), b.float()
        assert ((a - b).abs() <= 2.0 ** -7 * b.abs() + 2.0 ** -12 * b.abs().max()).all()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n_tiles = int(((st.slot_offsets[1:] - st.slot_offsets[:-1] + 255) // 256).sum()) * (c.d // 256)
    if 0 < n_tiles % min(cus, 256) <= min(cus, 256) // 2:
        assert not torch.equal(st.Yp, Yp) and not torch.equal(st.dXp, dXp)   # slices were used


@pytest.mark.timeout(600)
@pytest.mark.parametrize("shape", ["4_column_tiles", "8_column_tiles", "3_and_5_column_tiles"])
def test_tiles_dealt_out_in_xcd_blocks(shape):
    """Products of more than 256 tiles: the grouped GEMM deals each whole round of 256 tiles out
    to the XCDs in blocks (a permutation of the launch order inside the round) and leaves the
    rest, here a ragged and partly sliced last round, in launch order; with 8 column tiles the
    W1 gradient's 64 tiles per class are dealt out too.  With 3 and 5 column tiles the rounds are
    8 m-tiles, one per XCD.  Every output element by element against the oracle."""
    kw = {"4_column_tiles": dict(d=1024, f=512, T=8192), "8_column_tiles": dict(d=2048, f=1024, T=4700),
          "3_and_5_column_tiles": dict(d=768, f=640, T=2100)}[shape]
    c = wl.scaled(wl.get_config("c2"), E=8, S_tot=16, N=4, iters=1, **kw)
    print(f"[xcd blocks] {c}", flush=True)
    st = Hn.State(c, shard=1)
    X, logits, dY = Hn.draw_inputs(c, 0)
    check_iteration(st, X, logits, dY)
    rows = (st.slot_offsets[1:] - st.slot_offsets[:-1]).cpu().numpy()
    n_tiles = int(((rows + 255) // 256).sum()) * (c.d // 256)
    assert n_tiles > (256 if shape != "3_and_5_column_tiles" else 16 * (c.d // 256)), n_tiles
