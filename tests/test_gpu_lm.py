"""GPU parity: embedding lookup, log-softmax, output layer and the whole language-model step
(Eq. 6 from token to distribution) against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_vec_close, host, planes_host, to_dev
from paper_1802_00150_amd import inputs

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def amq():
    import paper_1802_00150_amd as m
    m.binding.lib()
    return m


@pytest.fixture(autouse=True)
def threads():
    oracle.set_threads(oracle.host_threads())
    yield
    oracle.set_threads(1)


@pytest.mark.parametrize("vocab,n,k,B", [(50, 70, 2, 5), (1000, 300, 2, 1), (333, 1024, 3, 64), (17, 129, 4, 3),
                                         (64, 5000, 1, 2)])
def test_embedding_lookup(amq, vocab, n, k, B):
    import torch
    g = np.random.default_rng(vocab + n + k)
    emb = (g.standard_normal((vocab, n)) * 0.1).astype(np.float32)
    Ep, ae = oracle.quantize_rows(emb, k, 2)
    ids = g.integers(0, vocab, size=B).astype(np.int64)
    ids[-1] = ids[0]                      # a repeated id
    say("embedding vocab=%d n=%d k=%d B=%d" % (vocab, n, k, B))
    Xr, br = oracle.embedding_lookup(Ep, ae, n, ids)
    Xg, bg = amq.embedding_lookup(to_dev(Ep), to_dev(ae), n, torch.from_numpy(ids).to("cuda:0"))
    assert np.array_equal(planes_host(Xg), Xr)
    assert np.array_equal(host(bg), br)


def test_embedding_lookup_out_of_range_id_gives_zero_vector(amq):
    import torch
    g = np.random.default_rng(5)
    emb = (g.standard_normal((20, 200)) * 0.1).astype(np.float32)
    Ep, ae = oracle.quantize_rows(emb, 2, 2)
    ids = np.array([3, 20, -1, 19, 1 << 40], np.int64)
    Xg, bg = amq.embedding_lookup(to_dev(Ep), to_dev(ae), 200, torch.from_numpy(ids).to("cuda:0"))
    Xg, bg = planes_host(Xg), host(bg)
    Xr, br = oracle.embedding_lookup(Ep, ae, 200, np.array([3, 19], np.int64))
    assert np.array_equal(Xg[:, [0, 3]], Xr) and np.array_equal(bg[[0, 3]], br)
    assert not Xg[:, [1, 2, 4]].any() and not bg[[1, 2, 4]].any()


@pytest.mark.parametrize("B,V", [(1, 1), (3, 7), (2, 1000), (5, 4097), (4, 10000), (1, 42000), (64, 42000),
                                 (2, 65536), (3, 70001)])
def test_log_softmax(amq, B, V):
    g = np.random.default_rng(B * 100003 + V)
    Y = (g.standard_normal((B, V)) * 3.0 + g.standard_normal((B, 1)) * 20.0).astype(np.float32)
    say("log_softmax B=%d V=%d" % (B, V))
    ref = oracle.log_softmax(Y)
    d = to_dev(Y)
    out = amq.log_softmax(d)
    assert_vec_close(host(out), ref, "logprob")
    assert np.array_equal(host(d), Y)            # input untouched
    amq.log_softmax(d, out=d)                    # in place
    assert np.array_equal(host(d), host(out))
    assert np.allclose(np.exp(host(out).astype(np.float64)).sum(axis=1), 1.0, atol=1e-4)


@pytest.mark.parametrize("V,H,B,k_w,k_a", [(130, 72, 3, 2, 2), (1000, 300, 1, 2, 3), (777, 256, 20, 3, 3),
                                           (10000, 1024, 37, 2, 3), (4100, 1500, 18, 2, 2), (300, 2100, 5, 4, 4),
                                           # vocabularies above 32768 with 32 or more rows: the product with several
                                           # batch tiles per wave and one (max, sum) pair per workgroup; V ragged
                                           # against 16 and against 4, last batch group partly empty
                                           (33001, 64, 40, 2, 2), (40003, 200, 100, 2, 2), (35002, 130, 33, 3, 3)])
def test_softmax_layer(amq, V, H, B, k_w, k_a):
    g = np.random.default_rng(V + H + B)
    Ws = (g.standard_normal((V, H)) * 0.05).astype(np.float32)
    bs = (g.standard_normal(V) * 0.3).astype(np.float32)
    h = np.tanh(g.standard_normal((B, H))).astype(np.float32)
    Wsp, als = oracle.quantize_rows(Ws, k_w, 2)
    dW, dA = to_dev(Wsp), to_dev(als)
    for bias in (None, bs):
        say("softmax layer V=%d H=%d B=%d W%d/A%d bias=%s" % (V, H, B, k_w, k_a, bias is not None))
        logits, ref = oracle.softmax_layer(Wsp, als, H, bias, h, k_a, 2)
        got = amq.softmax_layer(dW, dA, H, None if bias is None else to_dev(bias), to_dev(h), k_a, 2)
        assert_vec_close(host(got), ref, "logprob")


def lm_oracle_step(q, ids, h, c, k_as):
    Xp, bx = oracle.embedding_lookup(q["Ep"], q["ae"], q["E"], ids)
    h1, c1 = oracle.lstm_step_xq(q["Wxp"], q["ax"], q["Whp"], q["ah"], q["E"], q["H"], q["bias"], Xp, bx, h, c, 2)
    _, lp = oracle.softmax_layer(q["Wsp"], q["as"], q["H"], q["bs"], h1, k_as, 2)
    return h1, c1, lp


def lm_setup(cfg, k_ws):
    k = cfg["k_w"]
    q = dict(E=cfg["E"], H=cfg["H"], bs=cfg["bs"])
    q["Ep"], q["ae"] = oracle.quantize_rows(cfg["emb"], k, 2)
    q["Wxp"], q["ax"] = oracle.quantize_rows(cfg["Wx"], k, 2)
    q["Whp"], q["ah"] = oracle.quantize_rows(cfg["Wh"], k, 2)
    q["Wsp"], q["as"] = oracle.quantize_rows(cfg["Ws"], k_ws, 2)
    g = np.random.default_rng(cfg["H"])
    q["bias"] = (g.standard_normal(4 * cfg["H"]) * 0.1).astype(np.float32)
    return q


def lm_gpu_step(amq, q, dq, ids, dh, dc, k_a, k_as):
    import torch
    return amq.lm_step(dq["Ep"], dq["ae"], q["E"], dq["Wxp"], dq["ax"], dq["Whp"], dq["ah"], q["H"], dq["bias"],
                       dq["Wsp"], dq["as"], dq["bs"], torch.from_numpy(np.ascontiguousarray(ids)).to("cuda:0"),
                       dh, dc, k_a, k_as, 2)


# small and ragged shapes: batch 3 and 1 take the register-resident kernel, 20 the matrix cores
@pytest.mark.parametrize("E,H,V,B,k,k_ws,k_as", [(40, 24, 130, 3, 2, 2, 2), (300, 300, 10000, 1, 2, 2, 3),
                                                 (128, 256, 1000, 20, 3, 3, 3), (200, 136, 555, 33, 2, 3, 2)])
def test_lm_step_teacher_forced_and_free_running(amq, E, H, V, B, k, k_ws, k_as):
    steps = 4
    cfg = inputs.language_model(trial=E + B, steps=steps, B=B, H=H, E=E, vocab=V, k=k)
    q = lm_setup(cfg, k_ws)
    dq = {n: to_dev(q[n]) for n in ("Ep", "ae", "Wxp", "ax", "Whp", "ah", "Wsp", "as", "bias", "bs")}
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    fh, fc = to_dev(h), to_dev(c)                 # free-running GPU state
    for t in range(steps):
        say("lm step E=%d H=%d V=%d B=%d t=%d" % (E, H, V, B, t))
        ids = cfg["ids"][t]
        h1, c1, lp = lm_oracle_step(q, ids, h, c, k_as)
        dh, dc = to_dev(h), to_dev(c)             # teacher-forced: the oracle's previous state
        got = lm_gpu_step(amq, q, dq, ids, dh, dc, k, k_as)
        assert_vec_close(host(dc), c1, "c")
        assert_vec_close(host(dh), h1, "h")
        assert_vec_close(host(got), lp, "logprob")
        got_free = lm_gpu_step(amq, q, dq, ids, fh, fc, k, k_as)
        assert_vec_close(host(fh), h1, "h free-running")
        assert_vec_close(host(got_free), lp, "logprob free-running")
        h, c = h1, c1


@pytest.mark.parametrize("B", [1, 64])
def test_lm_step_full_size(amq, B):
    """Hidden 1024, vocabulary 42000 (the output layer is 42000 x 1024), W2/A2."""
    cfg = inputs.language_model(trial=0, steps=2, B=B)
    q = lm_setup(cfg, 2)
    dq = {n: to_dev(q[n]) for n in ("Ep", "ae", "Wxp", "ax", "Whp", "ah", "Wsp", "as", "bias", "bs")}
    g = np.random.default_rng(B)
    h = np.tanh(g.standard_normal((B, 1024))).astype(np.float32) * np.float32(0.5)
    c = g.standard_normal((B, 1024)).astype(np.float32)
    for t in range(2):
        say("lm full size B=%d t=%d" % (B, t))
        ids = cfg["ids"][t]
        h1, c1, lp = lm_oracle_step(q, ids, h, c, 2)
        dh, dc = to_dev(h), to_dev(c)
        got = lm_gpu_step(amq, q, dq, ids, dh, dc, 2, 2)
        assert_vec_close(host(dc), c1, "c")
        assert_vec_close(host(dh), h1, "h")
        assert_vec_close(host(got), lp, "logprob")
        h, c = h1, c1


@pytest.mark.parametrize("E,H,V,B,k,k_ws,k_as,steps", [(300, 300, 10000, 1, 2, 2, 3, 5), (128, 256, 1000, 1, 3, 3, 3, 70),
                                                       (40, 24, 130, 3, 2, 2, 2, 4), (200, 136, 555, 20, 2, 3, 2, 3),
                                                       (1024, 1024, 42000, 1, 2, 2, 2, 3),
                                                       # batch above 1: 4096 // 1500 = 2 steps per pass of the
                                                       # output layer, so 5 steps take three passes
                                                       (40, 24, 130, 1500, 2, 2, 2, 5),
                                                       # full size at batch 64: one 192-row pass of the output layer
                                                       (1024, 1024, 42000, 64, 2, 2, 2, 3)])
def test_lm_sequence(amq, E, H, V, B, k, k_ws, k_as, steps):
    """Whole sequences through one call (batch 1: the recurrence in one launch over the chip, the
    output layer on all steps of a piece together) against the oracle's step-by-step loop."""
    import torch
    cfg = inputs.language_model(trial=E + B + steps, steps=steps, B=B, H=H, E=E, vocab=V, k=k)
    q = lm_setup(cfg, k_ws)
    dq = {n: to_dev(q[n]) for n in ("Ep", "ae", "Wxp", "ax", "Whp", "ah", "Wsp", "as", "bias", "bs")}
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    ref = []
    for t in range(steps):
        h, c, lp = lm_oracle_step(q, cfg["ids"][t], h, c, k_as)
        ref.append(lp)
    say("lm sequence E=%d H=%d V=%d B=%d steps=%d" % (E, H, V, B, steps))
    dh = torch.zeros((B, H), device="cuda:0")
    dc = torch.zeros((B, H), device="cuda:0")
    out = torch.full((steps, B, V), float("nan"), device="cuda:0")
    amq.lm_sequence(dq["Ep"], dq["ae"], E, dq["Wxp"], dq["ax"], dq["Whp"], dq["ah"], H, dq["bias"], dq["Wsp"],
                    dq["as"], dq["bs"], torch.from_numpy(np.ascontiguousarray(cfg["ids"])).to("cuda:0"), dh, dc, k,
                    k_as, 2, logprob=out)
    got = host(out)
    for t in range(steps):
        assert_vec_close(got[t], ref[t], "logprob step %d" % t)
    assert_vec_close(host(dh), h, "h final")
    assert_vec_close(host(dc), c, "c final")
    if B > 1:
        # the sequence call regroups the recurrent work (inputs looked up a step ahead, W_x x_t off the chain,
        # h-side sums + cell in a second launch) without changing a bit of it: the state it leaves is the
        # state that step-by-step calls leave
        sh, sc = torch.zeros((B, H), device="cuda:0"), torch.zeros((B, H), device="cuda:0")
        for t in range(steps):
            lm_gpu_step(amq, q, dq, cfg["ids"][t], sh, sc, k, k_as)
        assert np.array_equal(host(dh), host(sh)), "h differs from step-by-step calls"
        assert np.array_equal(host(dc), host(sc)), "c differs from step-by-step calls"


def test_lm_sequence_give_up_turns_log_probabilities_into_nan(amq):
    # Same failure path as in the plain LSTM sequence (waits that give up at their second poll, through the
    # test hook): the output layer must not present log-probabilities computed from an incomplete recurrence.
    import torch
    E, H, V, B, k, k_ws, k_as, steps, piece = 128, 256, 1000, 1, 3, 3, 3, 70, 64
    cfg = inputs.language_model(trial=777, steps=steps, B=B, H=H, E=E, vocab=V, k=k)
    q = lm_setup(cfg, k_ws)
    dq = {n: to_dev(q[n]) for n in ("Ep", "ae", "Wxp", "ax", "Whp", "ah", "Wsp", "as", "bias", "bs")}
    ids = torch.from_numpy(np.ascontiguousarray(cfg["ids"])).to("cuda:0")
    dh = torch.zeros((B, H), device="cuda:0")
    dc = torch.zeros((B, H), device="cuda:0")
    out = torch.zeros((steps, B, V), device="cuda:0")
    ws = torch.empty(int(amq.binding.lib().amq_lm_sequence_workspace_bytes(E, H, V, B, k, k_as)), dtype=torch.uint8,
                     device="cuda:0")
    say("lm sequence with waits that give up at once")
    amq.binding.debug_set_sequence_spin_limit(1)
    try:
        amq.lm_sequence(dq["Ep"], dq["ae"], E, dq["Wxp"], dq["ax"], dq["Whp"], dq["ah"], H, dq["bias"], dq["Wsp"],
                        dq["as"], dq["bs"], ids, dh, dc, k, k_as, 2, ws=ws, logprob=out)
        torch.cuda.synchronize()
    finally:
        amq.binding.debug_set_sequence_spin_limit(0)
    assert amq.lstm_sequence_abandoned(ws, E, H, 1, k)
    bad = np.isnan(host(out)).all(axis=(1, 2))
    first = int(np.argmax(bad))
    assert bad.any() and first % piece == 0 and bad[first:].all() and not np.isnan(host(out)[:first]).any()
    # and the same call without the hook completes, with the flag cleared
    dh.zero_()
    dc.zero_()
    amq.lm_sequence(dq["Ep"], dq["ae"], E, dq["Wxp"], dq["ax"], dq["Whp"], dq["ah"], H, dq["bias"], dq["Wsp"],
                    dq["as"], dq["bs"], ids, dh, dc, k, k_as, 2, ws=ws, logprob=out)
    assert not amq.lstm_sequence_abandoned(ws, E, H, 1, k)
    assert not np.isnan(host(out)).any()
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    for t in range(steps):
        h, c, lp = lm_oracle_step(q, cfg["ids"][t], h, c, k_as)
    assert_vec_close(host(out)[steps - 1], lp, "logprob of the last step")


@pytest.mark.parametrize("E,H,V,B,k,k_ws,k_as,steps", [
    (300, 300, 10000, 1, 2, 2, 3, 5),         # batch 1, few rows: 64 rows at a time through the ordinary layer
    (128, 256, 1000, 1, 3, 3, 3, 70),         # two pieces of the batch-1 recurrence
    (200, 136, 555, 20, 2, 3, 2, 3),
    (40, 24, 130, 1500, 2, 2, 2, 5),          # three passes of 3000, 3000 and 1500 rows, 64 rows at a time
    (1024, 1024, 42000, 1, 2, 2, 2, 35),      # the 35 rows of a batch-1 sequence: logits never written
    (1024, 1024, 42000, 64, 2, 2, 2, 3),      # 192 rows, logits never written
    (64, 40, 33001, 40, 2, 2, 2, 2),          # ragged vocabulary above 32768, 80 rows
])
def test_lm_sequence_score(amq, E, H, V, B, k, k_ws, k_as, steps):
    """Log-probability of given next words only, against the oracle's full log-probabilities."""
    import torch
    cfg = inputs.language_model(trial=E + B + steps + 1, steps=steps, B=B, H=H, E=E, vocab=V, k=k)
    q = lm_setup(cfg, k_ws)
    dq = {n: to_dev(q[n]) for n in ("Ep", "ae", "Wxp", "ax", "Whp", "ah", "Wsp", "as", "bias", "bs")}
    g = np.random.default_rng(steps + B)
    targets = g.integers(0, V, size=(steps, B)).astype(np.int64)
    targets[0, 0] = 0
    targets[-1, -1] = V - 1
    h = np.zeros((B, H), np.float32)
    c = np.zeros((B, H), np.float32)
    ref = np.zeros((steps, B), np.float64)
    for t in range(steps):
        h, c, lp = lm_oracle_step(q, cfg["ids"][t], h, c, k_as)
        ref[t] = lp[np.arange(B), targets[t]]
    say("lm score E=%d H=%d V=%d B=%d steps=%d" % (E, H, V, B, steps))
    dh = torch.zeros((B, H), device="cuda:0")
    dc = torch.zeros((B, H), device="cuda:0")
    out = torch.full((steps, B), float("nan"), device="cuda:0")
    amq.lm_sequence_score(dq["Ep"], dq["ae"], E, dq["Wxp"], dq["ax"], dq["Whp"], dq["ah"], H, dq["bias"], dq["Wsp"],
                          dq["as"], dq["bs"], torch.from_numpy(np.ascontiguousarray(cfg["ids"])).to("cuda:0"),
                          torch.from_numpy(targets).to("cuda:0"), dh, dc, k, k_as, 2, out=out)
    got = host(out).astype(np.float64)
    # the bar of the full log-probabilities: 1e-4 relative plus 1e-4 of the row's r.m.s. (about log V)
    tol = 1e-4 * np.abs(ref) + 1e-4 * np.log(V)
    bad = ~(np.abs(got - ref) <= tol)
    assert not bad.any(), "%d mismatches, worst %g" % (bad.sum(), np.abs(got - ref).max())
    assert_vec_close(host(dh), h, "h final")
    assert_vec_close(host(dc), c, "c final")


def test_lm_sequence_score_index_outside_vocabulary(amq):
    import torch
    E, H, V, B, steps = 64, 40, 33001, 40, 1
    cfg = inputs.language_model(trial=5, steps=steps, B=B, H=H, E=E, vocab=V, k=2)
    q = lm_setup(cfg, 2)
    dq = {n: to_dev(q[n]) for n in ("Ep", "ae", "Wxp", "ax", "Whp", "ah", "Wsp", "as", "bias", "bs")}
    targets = np.full((steps, B), 7, np.int64)
    targets[0, 3] = V
    targets[0, 5] = -1
    for Bsel in (B, 2):   # both forms of the output pass
        dh = torch.zeros((Bsel, H), device="cuda:0")
        dc = torch.zeros((Bsel, H), device="cuda:0")
        ids = torch.from_numpy(np.ascontiguousarray(cfg["ids"][:, :Bsel])).to("cuda:0")
        tg = targets[:, :Bsel].copy()
        tg[0, 1] = V + 5
        out = host(amq.lm_sequence_score(dq["Ep"], dq["ae"], E, dq["Wxp"], dq["ax"], dq["Whp"], dq["ah"], H, dq["bias"],
                                         dq["Wsp"], dq["as"], dq["bs"], ids, torch.from_numpy(tg).to("cuda:0"), dh, dc, 2,
                                         2, 2))
        bad = (tg < 0) | (tg >= V)
        assert np.isnan(out[bad]).all() and np.isfinite(out[~bad]).all()
