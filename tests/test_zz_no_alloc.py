"""sq_decode_layer_static (the single-launch layer with its workspace inside the library, for
callers that cannot allocate device memory) against sq_decode_layer with a caller's workspace:
the same bits, call after call on the one array every call on a GPU shares -- the second call
with fewer tokens and a smaller layer, so that leftovers of the first would show."""
import numpy as np
import pytest

from paper_2511_22316_amd import synth
from parity_util import dev

pytestmark = pytest.mark.gpu


def _weights(N, K, seed):
    g = np.random.default_rng(seed)
    return synth.random_codes(N, K, seed), g.uniform(1e-4, 5e-3, N).astype(np.float32)


def _case(name, T, N, seed):
    import torch
    import paper_2511_22316_amd as sq
    cfg = synth.CONFIGS[name]
    L = synth.layer(cfg, max(T, 1))
    n1, n2, K = cfg.n1, cfg.n2, cfg.K
    Qw_h, sw_h = _weights(N, K, seed)
    Qw, sw, X = dev(Qw_h), dev(sw_h), dev(L.X[:T])
    prepared = torch.empty((sq.sq_prepared_rotation_bytes(n1, n2),), dtype=torch.uint8, device="cuda")
    sq.sq_prepare_rotation(dev(L.R1), dev(L.R2), prepared)
    ws = torch.zeros((sq.sq_decode_layer_workspace_bytes(T, K),), dtype=torch.uint8, device="cuda")
    want = torch.full((T, N), -3.0, dtype=torch.float16, device="cuda")
    got = torch.full((T, N), -5.0, dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    return dict(L=L, n1=n1, n2=n2, X=X, Qw=Qw, sw=sw, prepared=prepared, ws=ws, want=want, got=got)


def test_static_workspace_entry_matches_the_workspace_entry():
    import torch
    import paper_2511_22316_amd as sq
    # every buffer of both calls exists before the first call of the entry point under test
    cases = [_case("decode", 8, 28672, 11), _case("attn_proj", 3, 4096, 12), _case("decode", 32, 16400, 13),
             _case("tiny", 1, 96, 14)]
    for c in cases:
        L = c["L"]
        sq.sq_decode_layer(c["X"], L.giv_i, L.giv_j, L.giv_theta, c["prepared"], c["n1"], c["n2"], c["Qw"], c["sw"],
                           c["want"], c["ws"])
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for k, c in enumerate(cases):
        print(f"case static workspace call {k}: T={c['X'].shape[0]} K={c['X'].shape[1]} N={c['Qw'].shape[0]}", flush=True)
        L = c["L"]
        sq.sq_decode_layer_static(c["X"], L.giv_i, L.giv_j, L.giv_theta, c["prepared"], c["n1"], c["n2"], c["Qw"],
                                  c["sw"], c["got"])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for k, c in enumerate(cases):
        assert torch.equal(c["got"], c["want"]), f"call {k} differs from sq_decode_layer"
    # the same calls again, in reverse order, on the array the first round left behind
    for c in reversed(cases):
        c["got"].fill_(-7.0)
    for c in reversed(cases):
        L = c["L"]
        sq.sq_decode_layer_static(c["X"], L.giv_i, L.giv_j, L.giv_theta, c["prepared"], c["n1"], c["n2"], c["Qw"],
                                  c["sw"], c["got"])
    torch.cuda.synchronize()
    for k, c in enumerate(cases):
        assert torch.equal(c["got"], c["want"]), f"second round, call {k} differs from sq_decode_layer"
    sq.sq_decode_layer_status(None)          # no workgroup of any of these calls gave up its wait


def test_static_workspace_entry_rejects_what_does_not_fit():
    import torch
    import paper_2511_22316_amd as sq
    c = _case("decode", 8, 512, 15)
    L = c["L"]
    X33 = torch.zeros((33, c["X"].shape[1]), dtype=torch.float16, device="cuda")
    Y33 = torch.zeros((33, 512), dtype=torch.float16, device="cuda")
    with pytest.raises(sq.SQError) as e:
        sq.sq_decode_layer_static(X33, L.giv_i, L.giv_j, L.giv_theta, c["prepared"], c["n1"], c["n2"], c["Qw"],
                                  c["sw"], Y33)
    assert e.value.code == 2                 # SQ_ERR_SHAPE: more tokens than the array holds
    # no tokens: nothing is enqueued, no error
    sq.sq_decode_layer_static(X33[:0], L.giv_i, L.giv_j, L.giv_theta, c["prepared"], c["n1"], c["n2"], c["Qw"],
                              c["sw"], Y33[:0])
