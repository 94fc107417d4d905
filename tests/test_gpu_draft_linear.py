"""GPU-vs-oracle parity of s4c_draft_linear (Eq. 3, h = Linear(concat[e, f])) through the C ABI.
bf16 in/out with fp32 accumulation: |g - o| <= 2^-8 |o| + 2e-3 element by element (half an ulp of
the bf16 result is 2^-9 |o|; the fp32 sum of <= 32768 products of O(1/sqrt(K)) terms adds ~1e-5)."""
import numpy as np
import pytest
import torch

from oracle import s4c_oracle as O
from paper_2506_14158_amd import binding as B, synth
from paper_2506_14158_amd.device import np_to_torch

pytestmark = pytest.mark.gpu


def make(T, H, Hout, seed, bias=True):
    rng = np.random.default_rng(seed)
    bf = lambda x: synth.f32_to_bf16_bits(x.astype(np.float32))
    e, f = bf(rng.standard_normal((T, H))), bf(rng.standard_normal((T, H)))
    W = bf(rng.standard_normal((Hout, 2 * H)) / np.sqrt(2 * H))
    b = bf(rng.standard_normal(Hout)) if bias else None
    return e, f, W, b


def run(e, f, W, b):
    out = torch.full((e.shape[0], W.shape[0]), float("nan"), dtype=torch.bfloat16, device="cuda")
    ws = B.alloc_workspace(B.s4c_draft_linear_workspace_size(e.shape[0], e.shape[1], W.shape[0]))
    if ws is not None:
        ws.view(torch.float32).fill_(float("nan"))       # partial sums are written before they are read
    B.s4c_draft_linear(np_to_torch(e), np_to_torch(f), np_to_torch(W), out, None if b is None else np_to_torch(b), ws)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


def close(g, o):
    assert np.isfinite(g).all()
    err = np.abs(g - o)
    assert (err <= 2.0 ** -8 * np.abs(o) + 2e-3).all(), float((err - 2.0 ** -8 * np.abs(o)).max())


@pytest.mark.parametrize("T,H,Hout,bias", [(300, 64, 256, True), (1, 32, 256, False), (256, 32, 512, True),
                                           (777, 1024, 768, True), (2048, 512, 1024, False)])
def test_element_by_element(T, H, Hout, bias):
    e, f, W, b = make(T, H, Hout, T + H, bias)
    close(run(e, f, W, b), O.draft_linear(e, f, W, b))


@pytest.mark.parametrize("T,H,Hout,bias", [(1, 4096, 4096, True), (15, 4096, 4096, False), (60, 4096, 4096, True),
                                           (128, 4096, 4096, True), (60, 5120, 5120, True), (33, 96, 256, True),
                                           (128, 32, 512, False), (17, 1056, 768, True), (100, 8192, 1024, True)])
def test_few_tokens_element_by_element(T, H, Hout, bias):
    """Up to 128 tokens (a draft tree at batch 1; 4096 / 5120 are the hidden sizes of Vicuna 7B / 13B): the
    weight-streaming kernel with split-K, every output element against the oracle."""
    e, f, W, b = make(T, H, Hout, 1000 + T + H, bias)
    close(run(e, f, W, b), O.draft_linear(e, f, W, b))


@pytest.mark.parametrize("T,H,Hout", [(256, 5120, 5120), (200, 4096, 4096), (512, 1024, 512), (513, 1024, 512), (129, 96, 256)])
def test_a_few_hundred_tokens_run_in_passes(T, H, Hout):
    """129 .. 512 tokens (config 3's four trees are 256): the weight-streaming kernel in equal passes of at most
    128 tokens, the last one possibly shorter; 513 tokens is the first size of the tiled kernel."""
    e, f, W, b = make(T, H, Hout, 2000 + T + H, True)
    close(run(e, f, W, b), O.draft_linear(e, f, W, b))


def test_few_tokens_selector_weights_are_exact_and_deterministic():
    T, H = 60, 512
    e, f, _, _ = make(T, H, H, 5)
    one = synth.f32_to_bf16_bits(np.eye(H, dtype=np.float32))
    zero = np.zeros((H, H), dtype=np.uint16)
    assert np.array_equal(run(e, f, np.ascontiguousarray(np.hstack([one, zero])), None), synth.bf16_bits_to_f32(e).astype(np.float64))
    assert np.array_equal(run(e, f, np.ascontiguousarray(np.hstack([zero, one])), None), synth.bf16_bits_to_f32(f).astype(np.float64))
    e, f, W, b = make(60, 4096, 4096, 8)
    first = run(e, f, W, b)
    for _ in range(3):
        assert np.array_equal(run(e, f, W, b), first)


def test_selector_weights_are_exact():
    """W = [I | 0] returns e, W = [0 | I] returns f, bit for bit (every product is x * 1 or x * 0)."""
    T, H = 300, 256
    e, f, _, _ = make(T, H, H, 3)
    one = synth.f32_to_bf16_bits(np.eye(H, dtype=np.float32))
    zero = np.zeros((H, H), dtype=np.uint16)
    ge = run(e, f, np.ascontiguousarray(np.hstack([one, zero])), None)
    gf = run(e, f, np.ascontiguousarray(np.hstack([zero, one])), None)
    assert np.array_equal(ge, synth.bf16_bits_to_f32(e).astype(np.float64))
    assert np.array_equal(gf, synth.bf16_bits_to_f32(f).astype(np.float64))


def test_full_size_sampled():
    """A 70B-sized head (hidden 8192) on the 2048 tokens of config 5's trees: sampled tokens x sampled features."""
    T, H, Hout = 2048, 8192, 8192
    e, f, W, b = make(T, H, Hout, 11)
    g = run(e, f, W, b)
    rng = np.random.default_rng(1)
    ts, os_ = np.sort(rng.choice(T, 24, replace=False)), np.sort(rng.choice(Hout, 96, replace=False))
    ts[0], ts[-1], os_[0], os_[-1] = 0, T - 1, 0, Hout - 1
    ref = O.draft_linear(np.ascontiguousarray(e[ts]), np.ascontiguousarray(f[ts]), np.ascontiguousarray(W[os_]),
                         np.ascontiguousarray(b[os_]))
    close(g[np.ix_(ts, os_)], ref)


def test_rejects_unsupported_shapes():
    t = lambda *s: torch.zeros(*s, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.S4CError):       # Hout must be a multiple of 256
        B.s4c_draft_linear(t(4, 64), t(4, 64), t(100, 128), t(4, 100))
    with pytest.raises(B.S4CError):       # H must be a multiple of 32
        B.s4c_draft_linear(t(4, 40), t(4, 40), t(256, 80), t(4, 256))
    with pytest.raises(B.S4CError):       # few tokens: the workspace is required
        B.s4c_draft_linear(t(4, 64), t(4, 64), t(256, 128), t(4, 256))
    with pytest.raises(TypeError):
        B.s4c_draft_linear(t(4, 64).float(), t(4, 64).float(), t(256, 128).float(), t(4, 256).float())
