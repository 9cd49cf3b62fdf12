"""Random static builds (Sec. 4.1 setup: a window of R tokens, `keep_residual` = k newest tokens stay in fp16, all
older ones are quantized at once, the last group possibly partial): records, window, states and the decoded output
against the oracle at both code widths, and the refusal of a further append.

The seeds listed include the cases that exposed a defect: a partial last group whose token count modulo 32 lies in
1..16 (the state update reads tokens in blocks of 32; the half of the last block that no valid token reaches must hold
zeros), long prompts that go through the chunked build, sequences that fit the window whole."""
import numpy as np
import pytest

import kvlinc_synth as synth  # noqa: F401  (path set up by conftest)
from tests import kvlinc_testlib as tl
from tests.test_gpu_parity import _all_pairs, _build

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    import paper_2510_05373_amd as kvmod
    return kvmod


@pytest.mark.parametrize("seed", [0, 3, 4, 6, 7, 8, 9, 21, 32, 37])
def test_random_static_builds(kv, seed):
    import torch
    rng = np.random.default_rng(7000 + seed)
    B = int(rng.integers(1, 6)); H_kv = int(rng.choice([1, 2, 3, 8])); gq = int(rng.integers(1, 9)); H_q = gq * H_kv
    R = 4 * int(rng.integers(1, 33)); keep = int(rng.integers(1, R + 1))
    hi = int(rng.choice([40, 300, 1500, 9000]))
    lengths = [int(rng.integers(1, hi + 1)) for _ in range(B)]
    if rng.random() < 0.3: lengths[0] = keep  # everything stays in the window
    if rng.random() < 0.3: lengths[-1] = keep + 128 * int(rng.integers(1, 4))  # whole groups only
    if rng.random() < 0.2: lengths[B // 2] = max(1, keep - 1)
    bits = int(rng.choice([2, 4])); corr = bool(rng.random() < 0.8)
    print("[static] seed %d B=%d heads %d/%d R=%d keep=%d lengths %s bits %d correction %d"
          % (seed, B, H_q, H_kv, R, keep, lengths, bits, corr), flush=True)
    cache, K, V, Wq, Wk = _build(kv, 700 + seed, B, H_q, H_kv, lengths, R=R, keep=keep, correction=corr,
                                 capacity=max(lengths) + 300, bits=bits)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    if sum(lengths) * H_kv < 6000:
        pairs = _all_pairs(B, H_kv)
    else:
        pairs = list({(int(rng.integers(0, B)), int(rng.integers(0, H_kv))) for _ in range(3)})
    tl.check_cache_against_oracle(cache, K, V, lengths, pairs, Wk=Wk, keep=keep)
    q = tl.gen_q(700 + seed, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    assert np.isfinite(out.astype(np.float32)).all()
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), pairs, H_q, H_kv, Wq, Wk, bits=bits)
    tl.check_outputs(out, want)
    # a sequence with a partial last group accepts no further token and stays as it is
    nq0, nr0 = cache.n_quant.cpu().tolist(), cache.n_res.cpu().tolist()
    z = torch.zeros(B, H_kv, 1, 128, dtype=torch.float16, device="cuda")
    cache.append(z, z, keep_residual=keep)
    torch.cuda.synchronize()
    st = int(cache.status.item())
    nq1, nr1 = cache.n_quant.cpu().tolist(), cache.n_res.cpu().tolist()
    partial = [nq % 128 != 0 for nq in nq0]
    for b in range(B):
        if partial[b]:
            assert (nq1[b], nr1[b]) == (nq0[b], nr0[b]), (b, nq0, nr0, nq1, nr1)
    assert (not any(partial)) or (st & kv.KVLINC_ST_STATIC), (st, partial)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("valid", [1, 9, 16, 17, 33, 48, 66, 105, 127])
def test_partial_last_group_of_every_kind_of_size(kv, valid, bits):
    """One full group and a last group of `valid` tokens: states and output for sizes on both sides of the 16- and
    32-token steps of the state update."""
    import torch
    keep, R = 20, 32
    lengths = [128 + valid + keep, valid + keep]
    cache, K, V, Wq, Wk = _build(kv, 740 + valid, 2, 4, 2, lengths, R=R, keep=keep, capacity=512, bits=bits)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    assert cache.n_quant.cpu().tolist() == [128 + valid, valid] and cache.n_res.cpu().tolist() == [keep, keep]
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(2, 2), Wk=Wk, keep=keep)
    q = tl.gen_q(740 + valid, 2, 4)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, [128 + valid, valid], _all_pairs(2, 2), 4, 2, Wq, Wk, bits=bits)
    tl.check_outputs(out, want)
