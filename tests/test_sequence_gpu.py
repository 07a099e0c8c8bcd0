"""GPU parity of the whole-step persistent launch (quasar_sequence_*): a chain of dependent
linears plus the fused vocabulary/acceptance phase in ONE launch, against the oracle's own
chain (each oracle output rounded once to bf16 feeds the next oracle linear), and bit-for-bit
against the single-call entry points."""
import numpy as np
import pytest
import torch

from oracle import quasar_ref as ref
from paper_2603_01399_amd import synth
from gpu_util import bf16_to_dev, bf16_to_host, f32_to_dev, i32_to_dev

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def qb():
    assert torch.cuda.is_available()
    from paper_2603_01399_amd import binding
    return binding


def layer_shapes(hidden, kv, inter):
    return (("q", hidden, hidden), ("k", hidden, kv), ("v", hidden, kv), ("o", hidden, hidden),
            ("gate", hidden, inter), ("up", hidden, inter), ("down", inter, hidden))


def build_model(qb, n_layers, hidden, kv, inter, seed, bf16=False):
    """Seeded weights with unit gain (std 1/sqrt(K)) so that a chain of linears stays O(1)."""
    layers = []
    for li in range(n_layers):
        lin = {}
        for i, (name, K, N) in enumerate(layer_shapes(hidden, kv, inter)):
            w = synth.normal_weights(N, K, seed=seed + 100 * li + i, std=1.0 / np.sqrt(K))
            if bf16:
                lin[name] = dict(K=K, N=N, wb=synth.to_bf16_bits(w), wp=qb.pack_bf16_weights(f32_to_dev(w)), sc=None)
            else:
                q, s = ref.quantize_weights(w)
                wq, sc = qb.quantize_weights(f32_to_dev(w))
                lin[name] = dict(K=K, N=N, q=q, s=s, wp=wq, sc=sc)
        layers.append(lin)
    return layers


def oracle_linear(l, xb):
    y = ref.bf16_linear(xb, l["wb"]) if "wb" in l else ref.w8_linear(xb, l["q"], l["s"])
    return y, ref.f64_to_bf16_bits(y)


def oracle_chain(layers, x0):
    outs = []
    h = x0
    for lin in layers:
        o = {}
        o["q"] = oracle_linear(lin["q"], h)
        o["k"] = oracle_linear(lin["k"], h)
        o["v"] = oracle_linear(lin["v"], h)
        o["o"] = oracle_linear(lin["o"], o["q"][1])
        o["gate"] = oracle_linear(lin["gate"], o["o"][1])
        o["up"] = oracle_linear(lin["up"], o["o"][1])
        o["down"] = oracle_linear(lin["down"], o["gate"][1])
        h = o["down"][1]
        outs.append(o)
    return outs, h


def gpu_buffers(layers, M, x0):
    dev = "cuda"
    bufs = []
    h = bf16_to_dev(x0)
    for lin in layers:
        b = {n: torch.zeros((M, lin[n]["N"]), dtype=torch.bfloat16, device=dev) for n in lin}
        b["in"] = h
        h = b["down"]
        bufs.append(b)
    return bufs, h


def linear_list(layers, bufs):
    lst = []
    for lin, b in zip(layers, bufs):
        src = {"q": b["in"], "k": b["in"], "v": b["in"], "o": b["q"], "gate": b["o"], "up": b["o"], "down": b["gate"]}
        for name in ("q", "k", "v", "o", "gate", "up", "down"):
            l = lin[name]
            lst.append((src[name], l["wp"], l["sc"], l["N"], b[name]))
    return lst


@pytest.mark.parametrize("M,hidden,kv,inter,bf16", [
    (8, 256, 64, 768, False),
    (8, 512, 128, 8320, False),     # down projection K = 8320: activations staged in two chunks
    (3, 256, 64, 768, False),
    (16, 256, 64, 768, False),
    (32, 256, 64, 1536, False),
    (8, 256, 64, 768, True),
    (8, 5120, 512, 2560, False),    # 80 steps: five per wave (units padded to eight slots); 320 tiles: one or two per workgroup
    (4, 1280, 256, 6400, False),    # 20 and 100 steps: uneven shares of one or two and six or seven steps per wave
])
def test_sequence_chain_vs_oracle_and_single_calls(qb, M, hidden, kv, inter, bf16):
    print("sequence", M, hidden, kv, inter, bf16, flush=True)
    n_layers, V = 3, 2048
    layers = build_model(qb, n_layers, hidden, kv, inter, seed=9000 + M, bf16=bf16)
    x0 = synth.activations_bf16(M, hidden, seed=9100 + M)
    wv = synth.normal_weights(V, hidden, seed=9200 + M, std=1.0 / np.sqrt(hidden))
    if bf16:
        head = dict(wb=synth.to_bf16_bits(wv), wp=qb.pack_bf16_weights(f32_to_dev(wv)), sc=None)
    else:
        qh, sh = ref.quantize_weights(wv)
        wq, sc = qb.quantize_weights(f32_to_dev(wv))
        head = dict(q=qh, s=sh, wp=wq, sc=sc)

    want, h_last = oracle_chain(layers, x0)
    draft = np.arange(1, M, dtype=np.int32) if M > 1 else np.zeros(0, np.int32)
    if bf16:
        vout = ref.lmhead_verify(h_last, head["wb"], None, draft, weights_are_bf16=True)
    else:
        vout = ref.lmhead_verify(h_last, head["q"], head["s"], draft)

    # ---- one persistent launch
    bufs, h_dev = gpu_buffers(layers, M, x0)
    out_argmax = torch.full((M,), -1, dtype=torch.int32, device="cuda")
    out_accept = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    seq = qb.Sequence(linear_list(layers, bufs),
                      verify=(h_dev, head["wp"], head["sc"], V, i32_to_dev(draft) if len(draft) else None,
                              out_argmax, out_accept))
    assert seq.nphases == 4 * n_layers + 1          # q|k|v, o, gate|up, down per layer + the head
    # every buffer is written once: all dependent phases wait for their data, none at a barrier
    assert seq.n_barriers == 0 and seq.n_flag_waits == 4 * n_layers
    seq.run()
    torch.cuda.synchronize()
    assert not seq.timed_out()
    for li in range(n_layers):
        for name in ("q", "k", "v", "o", "gate", "up", "down"):
            got = ref.bf16_bits_to_f64(bf16_to_host(bufs[li][name]))
            err = ref.rel_maxabs_err(got, want[li][name][0])
            assert err <= TOL, (li, name, err)
    clear = (vout["top1"] - vout["top2"]) > TOL * vout["maxabs"]
    assert clear.any()
    am = out_argmax.cpu().numpy()
    assert np.array_equal(am[clear], vout["argmax"][clear])
    if np.all(clear[: min(vout["n_acc"], M - 1) + 1]):
        assert int(out_accept.cpu()[0]) == vout["n_acc"]

    # ---- the same step through the single-call entry points: identical bits
    bufs2, h2 = gpu_buffers(layers, M, x0)
    for (x, wp, sc, N, y) in linear_list(layers, bufs2):
        if bf16:
            qb.bf16_linear(x, wp, N, y)
        else:
            qb.w8_linear(x, wp, sc, N, y)
    ws = qb.make_workspace(M, V, hidden)
    dd = i32_to_dev(draft) if len(draft) else None
    if bf16:
        am2, acc2 = qb.bf16_lmhead_verify(h2, head["wp"], V, dd, ws)
    else:
        am2, acc2 = qb.lmhead_verify(h2, head["wp"], head["sc"], V, dd, ws)
    torch.cuda.synchronize()
    for li in range(n_layers):
        for name in ("q", "k", "v", "o", "gate", "up", "down"):
            assert torch.equal(bufs[li][name].view(torch.int16), bufs2[li][name].view(torch.int16)), (li, name)
    assert torch.equal(am2, out_argmax) and torch.equal(acc2, out_accept)

    # ---- repeatable
    first = [bufs[li]["down"].clone() for li in range(n_layers)]
    for _ in range(5):
        seq.run()
    torch.cuda.synchronize()
    assert not seq.timed_out()
    for li in range(n_layers):
        assert torch.equal(first[li].view(torch.int16), bufs[li]["down"].view(torch.int16))


def test_sequence_rows_off_cache_line_boundaries(qb):
    """Activation rows that do not start on 128-byte lines (row stride 264 elements), chained through the
    whole-step launch: results equal the single calls bit for bit."""
    print("sequence odd strides", flush=True)
    M, H, L = 8, 256, 4
    ws = []
    for i in range(L):
        w = synth.normal_weights(H, H, seed=9600 + i, std=1.0 / np.sqrt(H))
        ws.append(qb.quantize_weights(f32_to_dev(w)))
    x0 = bf16_to_dev(synth.activations_bf16(M, H, seed=9650))
    def run(fn):
        big = [torch.zeros((M, H + 8), dtype=torch.bfloat16, device="cuda") for _ in range(L + 1)]
        act = [b[:, :H] for b in big]                                 # row stride H + 8
        act[0].copy_(x0)
        fn(act)
        torch.cuda.synchronize()
        return act
    def as_sequence(act):
        seq = qb.Sequence([(act[i], ws[i][0], ws[i][1], H, act[i + 1]) for i in range(L)])
        assert seq.n_barriers == 0
        seq.run()
        torch.cuda.synchronize()
        assert not seq.timed_out()
    def as_calls(act):
        for i in range(L):
            qb.w8_linear(act[i], ws[i][0], ws[i][1], H, act[i + 1])
    a, b = run(as_sequence), run(as_calls)
    for i in range(L + 1):
        assert torch.equal(a[i].contiguous().view(torch.int16), b[i].contiguous().view(torch.int16)), i


def test_sequence_input_rewritten_after_it_was_read_is_read_fresh(qb):
    """x -> a, a -> x, x -> c: the last phase reads x after an earlier phase of the same launch has both
    read (cached) and then rewritten it; it must see the new contents.  Also a three-layer ping-pong that
    starts in one of the two buffers."""
    print("sequence rewritten input", flush=True)
    M, H = 8, 512
    ws, refq = [], []
    for i in range(3):
        w = synth.normal_weights(H, H, seed=9900 + i, std=1.0 / np.sqrt(H))
        ws.append(qb.quantize_weights(f32_to_dev(w)))
    x0 = bf16_to_dev(synth.activations_bf16(M, H, seed=9950))
    def bufs3():
        return [torch.zeros((M, H), dtype=torch.bfloat16, device="cuda") for _ in range(3)]
    for order in ((0, 1, 0, 2), (0, 1, 0, 1)):          # buffer index read by / written by consecutive linears
        xs = bufs3()
        xs[0].copy_(x0)
        lin = [(xs[order[i]], ws[i][0], ws[i][1], H, xs[order[i + 1]]) for i in range(3)]
        seq = qb.Sequence(lin)
        assert seq.n_barriers >= 2
        seq.run()
        torch.cuda.synchronize()
        assert not seq.timed_out()
        ys = bufs3()
        ys[0].copy_(x0)
        for i in range(3):
            qb.w8_linear(ys[order[i]], ws[i][0], ws[i][1], H, ys[order[i + 1]])
        torch.cuda.synchronize()
        for j in range(3):
            assert torch.equal(xs[j].view(torch.int16), ys[j].view(torch.int16)), (order, j)


def test_sequence_rerun_with_new_input_sees_fresh_activations(qb):
    """The same prepared sequence is run again after its input (same address) was overwritten:
    every intermediate buffer is produced again and must be read fresh, not from a cache line
    that still holds the previous step's value."""
    print("sequence rerun", flush=True)
    M, hidden, kv, inter, n_layers = 8, 256, 64, 768, 3
    layers = build_model(qb, n_layers, hidden, kv, inter, seed=9800)
    x_a = synth.activations_bf16(M, hidden, seed=9801)
    x_b = synth.activations_bf16(M, hidden, seed=9802)
    bufs, h_dev = gpu_buffers(layers, M, x_a)
    seq = qb.Sequence(linear_list(layers, bufs))
    for xb in (x_a, x_b, x_a, x_b):
        bufs[0]["in"].copy_(bf16_to_dev(xb))
        seq.run()
        torch.cuda.synchronize()
        assert not seq.timed_out()
        want, _ = oracle_chain(layers, xb)
        for li in range(n_layers):
            for name in ("q", "o", "up", "down"):
                got = ref.bf16_bits_to_f64(bf16_to_host(bufs[li][name]))
                assert ref.rel_maxabs_err(got, want[li][name][0]) <= TOL, (li, name)


def test_sequence_replayed_from_a_captured_graph(qb):
    """The whole-step launch captured into a HIP graph (its two kernels, no memset node) and
    replayed several times, with eager work and new inputs between the replays: every replay must
    give the bits of the eager run on the same input."""
    print("sequence graph replay", flush=True)
    M, hidden, kv, inter, n_layers = 8, 256, 64, 768, 2
    layers = build_model(qb, n_layers, hidden, kv, inter, seed=9850)
    inputs = [synth.activations_bf16(M, hidden, seed=9851 + i) for i in range(3)]
    bufs, h_dev = gpu_buffers(layers, M, inputs[0])
    seq = qb.Sequence(linear_list(layers, bufs))
    eager = []
    for xb in inputs:
        bufs[0]["in"].copy_(bf16_to_dev(xb))
        seq.run()
        torch.cuda.synchronize()
        eager.append([bf16_to_host(bufs[li]["down"]) for li in range(n_layers)])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        seq.run()                                            # warm-up on the capture stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            seq.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for rep in range(6):
        i = rep % 3
        bufs[0]["in"].copy_(bf16_to_dev(inputs[i]))
        scratch.add_(1.0)                                    # unrelated eager work between the replays
        for li in range(n_layers):
            bufs[li]["down"].zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert not seq.timed_out()
        for li in range(n_layers):
            assert np.array_equal(bf16_to_host(bufs[li]["down"]), eager[i][li]), (rep, li)


def test_sequence_reused_buffers_fall_back_to_barriers(qb):
    """Ping-pong activation buffers (written more than once per step) must be ordered by
    device-wide barriers; results stay identical to the single-call path."""
    print("sequence ping-pong", flush=True)
    M, H, L = 8, 512, 6
    ws = []
    for i in range(L):
        w = synth.normal_weights(H, H, seed=9700 + i, std=1.0 / np.sqrt(H))
        ws.append((ref.quantize_weights(w), qb.quantize_weights(f32_to_dev(w))))
    x0 = synth.activations_bf16(M, H, seed=9750)
    xd = bf16_to_dev(x0)
    pp = [torch.zeros((M, H), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    lin = []
    for i in range(L):
        src = xd if i == 0 else pp[i % 2]
        lin.append((src, ws[i][1][0], ws[i][1][1], H, pp[(i + 1) % 2]))
    seq = qb.Sequence(lin)
    assert seq.n_barriers >= L - 2 and seq.nphases == L
    for _ in range(3):
        seq.run()
    torch.cuda.synchronize()
    assert not seq.timed_out()
    h = x0
    for i in range(L):
        y = ref.w8_linear(h, ws[i][0][0], ws[i][0][1])
        h = ref.f64_to_bf16_bits(y)
    got = ref.bf16_bits_to_f64(bf16_to_host(pp[L % 2]))
    assert ref.rel_maxabs_err(got, y) <= TOL
    ref_out = [torch.zeros((M, H), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    for i in range(L):
        src = xd if i == 0 else ref_out[i % 2]
        qb.w8_linear(src, ws[i][1][0], ws[i][1][1], H, ref_out[(i + 1) % 2])
    torch.cuda.synchronize()
    assert torch.equal(ref_out[L % 2].view(torch.int16), pp[L % 2].view(torch.int16))


def test_sequence_planted_head_exact(qb):
    print("sequence planted head", flush=True)
    M, K, V = 8, 512, 8192
    h = synth.activations_bf16(M, K, seed=9500)
    w = synth.normal_weights(V, K, seed=9501)
    t = synth.distinct_targets(M, V, seed=9502)
    synth.plant_targets(w, h, t)
    wq, sc = qb.quantize_weights(f32_to_dev(w))
    hd = bf16_to_dev(h)
    for j in (0, 3, 7):
        d = synth.draft_with_matches(t, j, V, M - 1)
        out_argmax = torch.full((M,), -1, dtype=torch.int32, device="cuda")
        out_accept = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        seq = qb.Sequence([], verify=(hd, wq, sc, V, i32_to_dev(d), out_argmax, out_accept))
        seq.run()
        torch.cuda.synchronize()
        assert not seq.timed_out()
        assert np.array_equal(out_argmax.cpu().numpy(), t) and int(out_accept.cpu()[0]) == j


def test_sequence_argument_errors(qb):
    print("sequence arg errors", flush=True)
    x = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    y = torch.zeros((8, 256), dtype=torch.bfloat16, device="cuda")
    wq = torch.zeros(256 * 256, dtype=torch.int8, device="cuda")
    sc = torch.zeros(256, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError) as e:
        qb.Sequence([(x, wq, sc, 256, x)])               # in place
    assert e.value.status == 2
    wb = torch.zeros(256 * 256, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(qb.QuasarError) as e:
        qb.Sequence([(x, wq, sc, 256, y), (y, wb, None, 256, torch.zeros_like(y))])   # mixed weight types
    assert e.value.status == 5


@pytest.mark.parametrize("M,hidden,kv,inter,bf16", [
    (8, 512, 128, 8320, False),     # K = 8320 in two chunks of 65 KB
    (5, 1280, 256, 4096, False),    # uneven step shares, ragged M
    (8, 256, 64, 768, True),        # bf16 weights
    (1, 4096, 1024, 1024, False),   # full-size K: 64 KB of activations beside the second workgroup
])
def test_sequence_two_workgroups_per_compute_unit_same_bits(qb, M, hidden, kv, inter, bf16):
    """The form with two alternating workgroups of 8 waves per compute unit (asked for explicitly: a
    chain of dependent phases would not choose it) against the single calls and against the form
    with one workgroup of 16 waves: identical bits, including ping-pong buffers (barriers) and the
    vocabulary phase; the time stamps of a stamped run are ordered."""
    print("sequence two workgroups per unit", M, hidden, kv, inter, bf16, flush=True)
    n_layers, V = 2, 2048
    layers = build_model(qb, n_layers, hidden, kv, inter, seed=9300 + M, bf16=bf16)
    x0 = synth.activations_bf16(M, hidden, seed=9310 + M)
    wv = synth.normal_weights(V, hidden, seed=9320 + M, std=1.0 / np.sqrt(hidden))
    head = (qb.pack_bf16_weights(f32_to_dev(wv)), None) if bf16 else qb.quantize_weights(f32_to_dev(wv))
    draft = i32_to_dev(np.arange(1, M, dtype=np.int32)) if M > 1 else None
    results = {}
    try:
        for form in (2, 1):
            qb.set_sequence_form(form)
            bufs, h_dev = gpu_buffers(layers, M, x0)
            am = torch.full((M,), -1, dtype=torch.int32, device="cuda")
            acc = torch.full((1,), -1, dtype=torch.int32, device="cuda")
            seq = qb.Sequence(linear_list(layers, bufs), verify=(h_dev, head[0], head[1], V, draft, am, acc))
            assert seq.workgroups_per_cu == form
            for _ in range(3):
                seq.run()
            stamps = seq.run_stamped().cpu().numpy()
            torch.cuda.synchronize()
            assert not seq.timed_out()
            results[form] = (bufs, am, acc)
            assert stamps.shape == (seq.nphases, seq.workgroups_per_cu * torch.cuda.get_device_properties(0).multi_processor_count, 8)
            took = stamps[:, :, 2] > 0                      # workgroups with a share in the phase
            assert took.any(axis=1).all()
            for a, b in ((0, 1), (1, 2), (2, 3), (3, 4)):
                assert (stamps[:, :, a][took] <= stamps[:, :, b][took]).all(), (a, b)
            # gate|up reads all of o's output: its input was seen complete only after every workgroup with a
            # share in o had summed its last tile.  (o and down read one member matrix of their producer phase
            # - q of q|k|v, gate of gate|up - and wait for the workgroups that wrote that matrix only.)
            for p in range(2, seq.nphases, 4):
                if took[p].any() and took[p - 1].any():
                    assert stamps[p, :, 1][took[p]].min() >= stamps[p - 1, :, 3][took[p - 1]].max()
            # nobody saw an input complete before the first of its producers had raised its flag
            for p in range(1, seq.nphases):
                if took[p].any() and took[p - 1].any() and p % 4 != 0:
                    assert stamps[p, :, 1][took[p]].min() >= stamps[p - 1, :, 4][took[p - 1]].min()
    finally:
        qb.set_sequence_form(0)
    bufs2, h2 = gpu_buffers(layers, M, x0)
    for (x, wp, sc, N, y) in linear_list(layers, bufs2):
        qb.bf16_linear(x, wp, N, y) if bf16 else qb.w8_linear(x, wp, sc, N, y)
    ws = qb.make_workspace(M, V, hidden)
    am2, acc2 = (qb.bf16_lmhead_verify(h2, head[0], V, draft, ws) if bf16
                 else qb.lmhead_verify(h2, head[0], head[1], V, draft, ws))
    torch.cuda.synchronize()
    for form in (2, 1):
        bufs, am, acc = results[form]
        for li in range(n_layers):
            for name in ("q", "k", "v", "o", "gate", "up", "down"):
                assert torch.equal(bufs[li][name].view(torch.int16), bufs2[li][name].view(torch.int16)), (form, li, name)
        assert torch.equal(am, am2) and torch.equal(acc, acc2), form


def test_sequence_of_independent_linears_takes_the_alternating_form(qb):
    """Phases that do not wait for each other (every linear reads a resident input): prepare picks two
    workgroups per compute unit by itself; bits equal the single calls; W8A8 form too."""
    print("sequence independent phases", flush=True)
    from oracle import quasar_w8a8_ref as a8
    M, K = 8, 1024
    xs = [bf16_to_dev(synth.activations_bf16(M, K, seed=9400 + i)) for i in range(4)]
    ws = []
    for i in range(4):
        w = synth.normal_weights(512, K, seed=9410 + i, std=1.0 / np.sqrt(K))
        ws.append((ref.quantize_weights(w), qb.quantize_weights(f32_to_dev(w))))
    for w8a8 in (False, True):
        ys = [torch.zeros((M, 512), dtype=torch.bfloat16, device="cuda") for _ in range(4)]
        seq = qb.Sequence([(xs[i], ws[i][1][0], ws[i][1][1], 512, ys[i]) for i in range(4)], w8a8=w8a8)
        assert seq.nphases == 4 and seq.n_flag_waits == 0 and seq.n_barriers == 0
        assert seq.workgroups_per_cu == 2
        for _ in range(2):
            seq.run()
        torch.cuda.synchronize()
        assert not seq.timed_out()
        for i in range(4):
            one = qb.w8a8_linear(xs[i], ws[i][1][0], ws[i][1][1], 512) if w8a8 else qb.w8_linear(xs[i], ws[i][1][0], ws[i][1][1], 512)
            assert torch.equal(one.view(torch.int16), ys[i].view(torch.int16)), (w8a8, i)
            if w8a8:
                assert np.array_equal(bf16_to_host(ys[i]), a8.w8a8_linear(bf16_to_host(xs[i]), ws[i][0][0], ws[i][0][1])), i
