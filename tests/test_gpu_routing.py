"""GPU parity of the routing-score update (spec_routing_scores, through the C ABI) against the CPU
oracle.  The kernel sums products in fp32 per lane and fp64 across lanes; scores lie in [0, 1] and
must agree to 1e-5 absolute (the confidences stay away from the singular corners c = 1, d = 0)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2503_10325_amd import workloads as W

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def sv():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2503_10325_amd import binding
    binding.lib()
    return binding


def run_gpu(sv, ri: W.RoutingInputs, emb_f32=False):
    from paper_2503_10325_amd.runner import bf16_to_device
    dev = "cuda"
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    emb = t(W.bf16_bits_to_f32(ri.embedding)) if emb_f32 else bf16_to_device(ri.embedding, dev)
    B, _, N = ri.conf.shape
    scores = torch.full((B, N), -1.0, dtype=torch.float32, device=dev)
    sv.spec_routing_scores(t(ri.k_len), t(ri.conf), t(ri.draft_tokens), t(ri.accept_len), t(ri.out_tokens), emb, scores)
    torch.cuda.synchronize()
    return scores.cpu().numpy()


def ref(ri: W.RoutingInputs, emb_f32=False):
    emb = W.bf16_bits_to_f32(ri.embedding) if emb_f32 else ri.embedding
    return oracle.routing_scores(ri.k_len, ri.conf, ri.draft_tokens, ri.accept_len, ri.out_tokens, emb)


@pytest.mark.parametrize("shape", [(5, 6, 4, 1000, 128), (9, 7, 3, 517, 100), (3, 64, 16, 300, 72), (32, 6, 4, 32000, 4096)])
@pytest.mark.parametrize("emb_f32", [False, True])
def test_routing_scores_match_oracle(sv, shape, emb_f32):
    B, K, N, V, E = shape
    if emb_f32 and V * E > 4_000_000:
        pytest.skip("bf16 table only at full size")
    ri = W.make_routing_inputs(B, K, N, V, E, seed=3)
    got, want = run_gpu(sv, ri, emb_f32), ref(ri, emb_f32)
    assert np.isfinite(got).all() and got.min() >= 0.0 and got.max() <= 1.0 + 1e-6
    assert np.abs(got - want).max() <= TOL
    assert want.max() > 0.2                                # the case has accepted positions that count


def test_routing_scores_corners(sv):
    """Zero-length drafts, nothing accepted, everything accepted, c at 0 and 1, a zero embedding row."""
    ri = W.make_routing_inputs(6, 5, 2, 50, 64, seed=1)
    ri.k_len[:] = [0, 5, 5, 3, 5, 5]
    ri.accept_len[:] = [0, 0, 5, 3, 2, 5]
    ri.conf[4] = 0.0
    ri.conf[5] = 1.0
    ri.embedding[7] = 0                                     # bf16 bits of +0
    ri.out_tokens[2, 1] = 7
    ri.draft_tokens[2, 3, 0] = 7
    got, want = run_gpu(sv, ri), ref(ri)
    assert np.abs(got - want).max() <= TOL
    assert got[0].max() == 0.0 and got[1].max() == 0.0 and got[4].max() == 0.0
