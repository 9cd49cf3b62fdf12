"""Bulk appends of long prompts -- the build that shares the groups of a (sequence, KV head) out in chunks over the
chip (Sec. 3.2: the states are sums over tokens, Eq. 5) -- onto caches that already hold tokens, with ragged `n_new`
in the same call (a sequence that takes the whole prompt next to one that takes one token, or none), followed by
one-token appends; random variants (code width, Alg. 1-literal merge, sliding value window, 16-bit state storage,
which is not chunked).  Records, window, states and decoded output against the oracle."""
import numpy as np
import pytest

import kvlinc_synth as synth
from tests import kvlinc_testlib as tl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    import paper_2510_05373_amd as kvmod
    return kvmod


@pytest.mark.parametrize("seed", [0, 2, 3, 7, 11, 18])
def test_long_prompts_onto_caches_that_hold_tokens(kv, seed):
    import torch
    rng = np.random.default_rng(11000 + seed)
    B = int(rng.integers(1, 5)); H_kv = int(rng.choice([1, 2, 4, 8])); gq = int(rng.integers(1, 9)); H_q = gq * H_kv
    bits = int(rng.choice([2, 4])); literal, sliding, state16 = (bool(rng.random() < 0.3) for _ in range(3))
    flags = (kv.KVLINC_FLAG_ALG1_LITERAL if literal else 0) | (kv.KVLINC_FLAG_SLIDING_VALUES if sliding else 0)
    cfg = 1100 + seed
    first = [int(rng.integers(0, 700)) for _ in range(B)]
    T = int(rng.integers(8192, 14000))
    second = [int(rng.choice([0, 1, int(rng.integers(2, 300)), T, int(rng.integers(8192, T + 1)), int(rng.integers(300, T + 1))]))
              for _ in range(B)]
    third = [int(rng.integers(0, 3)) for _ in range(B)]
    lengths = [a + b + c for a, b, c in zip(first, second, third)]
    print("[chunked] seed %d B=%d heads %d/%d first %s second %s (T=%d) third %s bits %d literal %d sliding %d state16 %d"
          % (seed, B, H_q, H_kv, first, second, T, third, bits, literal, sliding, state16), flush=True)
    Wq, Wk = synth.adapters_q(cfg, H_q), synth.adapters_k(cfg, H_kv)
    Kh, Vh = tl.gen_kv(cfg, B, H_kv, [max(n, 1) for n in lengths])
    cache = kv.KVLincCache(B, H_q, H_kv, max(lengths) + 300, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), bits=bits, flags=flags,
                           state_storage="fp16" if state16 else "fp32")
    pos = [0] * B
    after_call = []
    for part in (first, second, third):
        Tc = T if part is second else max(max(part), 1)
        k = np.zeros((B, H_kv, Tc, 128), dtype=np.float16)
        v = np.zeros_like(k)
        for b in range(B):
            k[b, :, :part[b]] = Kh[b, :, pos[b]:pos[b] + part[b]]
            v[b, :, :part[b]] = Vh[b, :, pos[b]:pos[b] + part[b]]
            pos[b] += part[b]
        cache.append(tl.to_dev(k), tl.to_dev(v), n_new=tl.to_dev(np.asarray(part, dtype=np.int32)))
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        after_call.append(list(pos))
    n_quant, n_res = cache.n_quant.cpu().numpy(), cache.n_res.cpu().numpy()
    for b in range(B):
        if lengths[b] > 0:
            assert (int(n_quant[b]), int(n_res[b])) == tl.o_cache.window_split(lengths[b])
        else:
            assert (int(n_quant[b]), int(n_res[b])) == (0, 0)
    q = tl.gen_q(cfg, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    live = [b for b in range(B) if lengths[b] > 0]
    pairs = list({(int(rng.choice(live)), int(rng.integers(0, H_kv))) for _ in range(2)}) if live else []
    want = {}
    for (b, g) in pairs:
        n = lengths[b]
        k, v = Kh[b, g, :n], Vh[b, g, :n]
        # 16-bit storage rounds the state at the end of every call that flushed
        points = sorted({tl.o_cache.window_split(c[b])[0] for c in after_call if c[b] > 0}) if state16 else None
        tl.check_pair_against_oracle(cache, b, g, k, v, int(n_quant[b]), int(n_res[b]), None if state16 else Wk[g])
        ref = tl.o_cache.build_cache(k, v, int(n_quant[b]), Wk=Wk[g], bits=bits, state_rounding=points)
        for h in range(g * gq, (g + 1) * gq):
            want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h], literal_alg1=literal,
                                            value_window="sliding" if sliding else "block")
    if want:
        tl.check_outputs(out, want)
    assert int(cache.split_done.abs().sum().item()) == 0
