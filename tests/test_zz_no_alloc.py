"""rnnt_beam_decode_static (the entry point for callers that cannot allocate device memory) against
rnnt_beam_decode + rnnt_beam_results: the same kernels on the same inputs, so every output must be identical,
bit for bit, on two calls in a row, the second with a smaller input (the static workspace keeps the first
call's contents).  Through the C ABI, on an MI355X."""
import numpy as np
import pytest

import synth_inputs as S
from gpu_common import to_gpu

pytestmark = pytest.mark.gpu


def _both_ways(A, dec, c, enc, L, beam, lm=None, lm_weight=0.0):
    import torch
    B, T = enc.shape[0], enc.shape[1]
    d_enc, d_len = to_gpu(enc, torch.float32), to_gpu(L, torch.int32)
    cap = T * c["s"] + 1
    tokens = torch.full((B, beam, cap), -1, dtype=torch.int32, device="cuda")
    lens = torch.full((B, beam), -7, dtype=torch.int32, device="cuda")
    scores = torch.full((B, beam), 7.0, dtype=torch.float64, device="cuda")
    steps = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    flags = torch.full((2,), -7, dtype=torch.int32, device="cuda")
    dec.decode_static(d_enc, d_len, tokens, lens, scores, steps, flags, beam=beam, lm=lm, lm_weight=lm_weight)
    torch.cuda.synchronize()
    got = dict(tokens=tokens.cpu().numpy(), lens=lens.cpu().numpy(), scores=scores.cpu().numpy(),
               n_steps=steps.cpu().numpy(), flags=flags.cpu().numpy())
    dec.decode(d_enc, d_len, beam=beam, lm=lm, lm_weight=lm_weight)
    want = dec.results(cap=cap)
    return got, want


def _same(got, want):
    np.testing.assert_array_equal(got["flags"], [0, 0])
    np.testing.assert_array_equal(got["n_steps"], want["n_steps"])
    np.testing.assert_array_equal(got["lens"], want["lens"])
    np.testing.assert_array_equal(got["scores"], want["scores"])  # bit-identical float64
    B, K = want["lens"].shape
    for b in range(B):
        for j in range(K):
            n = max(int(want["lens"][b, j]), 0)
            np.testing.assert_array_equal(got["tokens"][b, j, :n], want["tokens"][b, j, :n])
            assert np.all(got["tokens"][b, j, n:] == -1)  # nothing written beyond the length


@pytest.mark.parametrize("kind", ["lstm_rnnt", "tdt_aes", "stateless", "lm"])
def test_static_workspace_decode_equals_the_allocating_one_twice(kind):
    import paper_2506_00185_amd as A
    over = dict(lstm_rnnt=dict(), tdt_aes=dict(model="tdt", durations=[0, 1, 2], algo="aes", gamma=2.3),
                stateless=dict(pred="stateless", ctx=2, algo="aes"), lm=dict(beam=8))[kind]
    c = S.custom_config(B=9, T=33, T_min=12, D=96, H=64, P=64, E=32, V=70, beam=over.pop("beam", 4), s=3, **over)
    w = S.perturb_biases(S.make_weights(c, 910), 911)
    L = S.make_lengths(c, 912)
    enc = S.make_enc(c, L, 913)
    lm, lam = None, 0.0
    if kind == "lm":
        lm, lam = A.NGramLM(S.make_lm(V=c["V"], order=3, n_target=3000, zipf_s=1.1, seed=914)), 0.3
    dec = A.BeamDecoder(c, w)
    # first call: the whole batch; second call: fewer and shorter utterances at a narrower beam
    got, want = _both_ways(A, dec, c, enc, L, c["beam"], lm, lam)
    _same(got, want)
    assert np.all(want["n_steps"] > 0)
    B2, T2 = 4, 20
    L2 = np.minimum(L[:B2], T2).astype(np.int32)
    got2, want2 = _both_ways(A, dec, c, np.ascontiguousarray(enc[:B2, :T2]), L2, max(c["beam"] // 2, 1), lm, lam)
    _same(got2, want2)


def test_static_workspace_rejects_what_does_not_fit():
    import torch
    import paper_2506_00185_amd as A
    # 64 MiB cannot hold the encoder projection of 200 x 400 frames at H = 256 (82 MB)
    c = S.custom_config(B=200, T=400, T_min=400, D=32, H=256, P=32, E=32, V=20, beam=2, s=1)
    dec = A.BeamDecoder(c, S.make_weights(c, 920))
    B, T, K = c["B"], c["T"], c["beam"]
    enc = torch.zeros((B, T, c["D"]), dtype=torch.float32, device="cuda")
    lengths = torch.full((B,), T, dtype=torch.int32, device="cuda")
    tokens = torch.zeros((B, K, 8), dtype=torch.int32, device="cuda")
    lens = torch.zeros((B, K), dtype=torch.int32, device="cuda")
    scores = torch.zeros((B, K), dtype=torch.float64, device="cuda")
    steps = torch.zeros((B,), dtype=torch.int32, device="cuda")
    with pytest.raises(A.RnntBeamError, match="static workspace"):
        dec.decode_static(enc, lengths, tokens, lens, scores, steps)
