"""GPU parity of sq_decode_layer (rotate + quantize and the W4A4 GEMM in one launch, at most 32
tokens) against the two calls it replaces -- the results must be the same bits -- and against the
CPU oracle of the whole layer.

The weights here are random codes and random steps (the GEMM is exact on any codes); the
activations, lists and rotation factors are the seeded layers of the other tests."""

import numpy as np
import pytest

from paper_2511_22316_amd import synth
from parity_util import dev, host

pytestmark = pytest.mark.gpu


def _weights(N, K, seed):
    g = np.random.default_rng(seed)
    return synth.random_codes(N, K, seed), g.uniform(1e-4, 5e-3, N).astype(np.float32)


class Layer:
    """Device-side constants of one layer plus a zeroed workspace for the single-launch call."""

    def __init__(self, L, N, T_max, seed=5):
        import torch
        import paper_2511_22316_amd as sq
        self.L, self.N = L, N
        self.n1, self.n2 = L.R1.shape[0], L.R2.shape[0]
        self.K = self.n1 * self.n2
        self.Qw_h, self.sw_h = _weights(N, self.K, seed)
        self.Qw, self.sw = dev(self.Qw_h), dev(self.sw_h)
        self.prepared = torch.empty((sq.sq_prepared_rotation_bytes(self.n1, self.n2),), dtype=torch.uint8, device="cuda")
        sq.sq_prepare_rotation(dev(L.R1), dev(L.R2), self.prepared)
        self.ws = torch.zeros((sq.sq_decode_layer_workspace_bytes(T_max, self.K),), dtype=torch.uint8, device="cuda")

    def two_calls(self, X):
        import torch
        import paper_2511_22316_amd as sq
        L, T = self.L, X.shape[0]
        Q = torch.empty((T, self.K // 2), dtype=torch.uint8, device="cuda")
        s = torch.empty((T,), dtype=torch.float32, device="cuda")
        Y = torch.full((T, self.N), -3.0, dtype=torch.float16, device="cuda")
        sq.sq_rotate_quantize_prepared(dev(X), L.giv_i, L.giv_j, L.giv_theta, self.prepared, self.n1, self.n2, Q, s)
        sq.sq_w4a4_gemm(Q, s, self.Qw, self.sw, Y)
        torch.cuda.synchronize()
        return Y

    def one_launch(self, X, Y=None):
        import torch
        import paper_2511_22316_amd as sq
        L, T = self.L, X.shape[0]
        if Y is None:
            Y = torch.full((T, self.N), -5.0, dtype=torch.float16, device="cuda")
        sq.sq_decode_layer(dev(X), L.giv_i, L.giv_j, L.giv_theta, self.prepared, self.n1, self.n2, self.Qw, self.sw,
                           Y, self.ws)
        torch.cuda.synchronize()
        return Y

    def counters(self):
        return host(self.ws[:16]).view(np.int32)


def _layer_of(name):
    return synth.layer(synth.CONFIGS[name])


@pytest.mark.parametrize("name,T,N", [("decode", 8, 28672), ("decode", 1, 1000), ("decode", 32, 16400),
                                      ("decode", 7, 4096), ("tiny", 16, 512), ("tiny", 3, 96),
                                      ("attn_proj", 5, 4096), ("attn_proj", 31, 20000)])
def test_decode_layer_equals_the_two_calls(name, T, N):
    print(f"case decode layer {name} T={T} N={N}", flush=True)
    import torch
    L = _layer_of(name)
    X = L.X[:T] if L.X.shape[0] >= T else synth.activations(synth.CONFIGS[name], T)
    lay = Layer(L, N, T)
    want = lay.two_calls(X)
    got = lay.one_launch(X)
    assert torch.equal(got, want)
    assert list(lay.counters()) == [0, 0, 0, 0]


@pytest.mark.parametrize("n1,n2,T,N", [(32, 32, 3, 700), (32, 64, 9, 2048), (16, 32, 32, 1024)])
def test_decode_layer_other_shapes(n1, n2, T, N):
    print(f"case decode layer shape {n1}x{n2} T={T} N={N}", flush=True)
    import torch
    cfg = synth.LayerConfig(f"d_{n1}x{n2}", T, n1, n2, N, 6, "normal", 2, 300.0, 0.01, 20.0, 0.02, 900 + n1 + n2)
    L = synth.layer(cfg)
    lay = Layer(L, N, T)
    assert torch.equal(lay.one_launch(L.X), lay.two_calls(L.X))


def test_decode_layer_wide_list_and_repeated_calls():
    """A list that touches all 128 columns (the instantiation with eight repair steps), and call
    after call on the same workspace without clearing it in between."""
    print("case decode layer wide list, repeated calls", flush=True)
    import torch
    cfg = synth.CONFIGS["decode"]
    L0 = synth.layer(cfg)
    gi = np.arange(64, dtype=np.int32)
    gj = gi + 64 + 128 * 3                       # other rows, the other 64 columns
    gt = np.linspace(-1.0, 1.2, 64).astype(np.float32)
    L = synth.Layer(cfg, L0.X, gi, gj, gt, L0.R1, L0.R2, L0.R1_f64, L0.R2_f64)
    lay = Layer(L, 28672, 8)
    X3 = synth.activations(cfg, 24)
    for k in range(3):
        X = X3[8 * k: 8 * k + 8 - k]             # 8, 7, 6 tokens
        assert torch.equal(lay.one_launch(X), lay.two_calls(X)), f"call {k}"
        assert list(lay.counters()) == [0, 0, 0, 0]


def test_decode_layer_against_the_oracle(oracle):
    print("case decode layer against the oracle", flush=True)
    cfg = synth.CONFIGS["decode"]
    L = synth.layer(cfg)
    N = 2048
    lay = Layer(L, N, 8)
    Y = host(lay.one_launch(L.X)).astype(np.float64)
    Qo, so = oracle.quantize_rows(oracle.rotate(L.X, L.giv_i, L.giv_j, L.giv_theta, L.R1, L.R2))
    Yo, _ = oracle.gemm(Qo, so, lay.Qw_h, lay.sw_h)
    Yo = Yo.astype(np.float64)
    rel = np.linalg.norm(Y - Yo, axis=1) / np.linalg.norm(Yo, axis=1)
    assert rel.max() <= 1e-2, f"worst row error {rel.max():.3e}"


def test_decode_layer_strided_and_empty():
    print("case decode layer strides / empty", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    L = _layer_of("tiny")
    T, N = 6, 200
    lay = Layer(L, N, T)
    X = L.X[:T]
    want = lay.two_calls(X)
    Xw = torch.full((T, lay.K + 16), 777.0, dtype=torch.float16, device="cuda")
    Xw[:, : lay.K] = dev(X)
    Yw = torch.full((T, N + 9), -1.0, dtype=torch.float16, device="cuda")
    sq.sq_decode_layer(Xw[:, : lay.K], L.giv_i, L.giv_j, L.giv_theta, lay.prepared, lay.n1, lay.n2, lay.Qw, lay.sw,
                       Yw[:, :N], lay.ws)
    torch.cuda.synchronize()
    assert torch.equal(Yw[:, :N], want)
    assert torch.all(Yw[:, N:] == -1.0)
    # no tokens: nothing is enqueued, the workspace is not touched
    sq.sq_decode_layer(Xw[:0, : lay.K], L.giv_i, L.giv_j, L.giv_theta, lay.prepared, lay.n1, lay.n2, lay.Qw, lay.sw,
                       Yw[:0, :N], lay.ws)
    torch.cuda.synchronize()
    assert list(lay.counters()) == [0, 0, 0, 0]


def test_decode_layer_gives_up_instead_of_waiting_forever():
    """The wait for the rotated tokens is bounded.  With a 'done' counter that starts below zero it
    can never be satisfied: every block must give up after the (here tiny) bound, leave Y alone,
    raise the error word and exit; the counters come out cleared, and the next call works."""
    print("case decode layer bounded wait", flush=True)
    import torch
    L = _layer_of("tiny")
    T, N = 16, 512
    lay = Layer(L, N, T)
    X = L.X[:T]
    want = lay.two_calls(X)
    import paper_2511_22316_amd as sq
    sq.sq_debug_set_option(sq.binding.SQ_DEBUG_DECODE_SPIN_LIMIT, 40)
    try:
        lay.ws[:16] = torch.from_numpy(np.array([-5, 0, 0, 0], np.int32).view(np.uint8)).cuda()
        Y = lay.one_launch(X)
        assert torch.all(Y == -5.0)
        assert list(lay.counters()) == [0, 0, 0, 1]
        # the status call reports it once and clears the word
        with pytest.raises(sq.SQError) as e:
            sq.sq_decode_layer_status(lay.ws)
        assert e.value.code == 6
        sq.sq_decode_layer_status(lay.ws)
        assert list(lay.counters()) == [0, 0, 0, 0]
    finally:
        sq.sq_debug_set_option(sq.binding.SQ_DEBUG_DECODE_SPIN_LIMIT, 0)
    lay.ws[:16] = 0
    assert torch.equal(lay.one_launch(X), want)
    assert list(lay.counters()) == [0, 0, 0, 0]
    sq.sq_decode_layer_status(lay.ws)


def test_decode_layer_captured_in_a_graph_replays_correctly():
    """The call records into a HIP graph (it allocates nothing, clears nothing from the host and
    leaves its counters ready for the next launch): three replays in a row on fresh contents of
    the static input buffer, with eager work and a synchronization in between, equal the two eager
    calls bit for bit."""
    print("case decode layer graph capture", flush=True)
    import torch
    import paper_2511_22316_amd as sq
    L = _layer_of("decode")
    T, N = 8, 4096
    lay = Layer(L, N, T)
    X3 = synth.activations(synth.CONFIGS["decode"], 24)
    Xin = torch.empty((T, lay.K), dtype=torch.float16, device="cuda")
    Y = torch.full((T, N), -5.0, dtype=torch.float16, device="cuda")

    def call(stream):
        sq.sq_decode_layer(Xin, L.giv_i, L.giv_j, L.giv_theta, lay.prepared, lay.n1, lay.n2, lay.Qw, lay.sw, Y, lay.ws,
                           stream=stream)

    side = torch.cuda.Stream()
    Xin.copy_(dev(X3[:T]))
    torch.cuda.synchronize()
    with torch.cuda.stream(side):                   # warm-up outside capture (one-time kernel attributes)
        call(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        call(side)
    for k in range(3):
        X = X3[8 * k: 8 * k + 8]
        Xin.copy_(dev(X))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = Y.clone()
        want = lay.two_calls(X)                     # eager work between the replays
        assert torch.equal(got, want), f"replay {k}"
        assert list(lay.counters()) == [0, 0, 0, 0]


@pytest.mark.parametrize("name,T,N", [("attn_proj", 32, 4096), ("decode", 9, 1024)])
def test_decode_layer_without_a_givens_list(name, T, N):
    """P = 0: the rotation is the Kronecker factors alone; and an odd number of tokens with two
    tokens per group (the last group is half empty)."""
    print(f"case decode layer no list {name} T={T}", flush=True)
    import torch
    cfg = synth.CONFIGS[name]
    L0 = synth.layer(cfg)
    e = np.zeros(0, np.int32)
    L = synth.Layer(cfg, L0.X, e, e, np.zeros(0, np.float32), L0.R1, L0.R2, L0.R1_f64, L0.R2_f64)
    X = synth.activations(cfg, T)
    lay = Layer(L, N, T)
    assert torch.equal(lay.one_launch(X), lay.two_calls(X))
    if name == "attn_proj":                       # 31 tokens: sixteen groups, the last one half empty
        assert torch.equal(lay.one_launch(X[:31]), lay.two_calls(X[:31]))
    assert list(lay.counters()) == [0, 0, 0, 0]
