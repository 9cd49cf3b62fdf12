"""Random batches of many sequences with long, unequal contexts (the shape of Sec. 4.4's throughput runs: tens of
sequences per step) and random variants: bulk build, up to two one-token appends, decode.  Two (sequence, KV head)
pairs carry the synthetic data of the parity tests and are compared with the oracle (records, window, states, output);
the others hold device-generated N(0, 1) rows and must come out finite."""
import numpy as np
import pytest

import kvlinc_synth as synth
from tests import kvlinc_testlib as tl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    import paper_2510_05373_amd as kvmod
    return kvmod


@pytest.mark.parametrize("seed", [3, 5, 19, 20, 37])
def test_random_batches(kv, seed):
    import torch
    rng = np.random.default_rng(9000 + seed)
    B = int(rng.choice([1, 2, 5, 17, 40])); H_kv = int(rng.choice([1, 2, 4, 8])); gq = int(rng.integers(1, 9)); H_q = gq * H_kv
    hi = int(rng.choice([2000, 9000, 20000])) if B * H_kv <= 64 else int(rng.choice([1500, 4000]))
    lengths = [int(rng.integers(1, hi + 1)) for _ in range(B)]
    bits = int(rng.choice([2, 4])); literal, sliding, state16 = (bool(rng.random() < 0.3) for _ in range(3))
    flags = (kv.KVLINC_FLAG_ALG1_LITERAL if literal else 0) | (kv.KVLINC_FLAG_SLIDING_VALUES if sliding else 0)
    cfg = 900 + seed
    print("[batches] seed %d B=%d heads %d/%d longest %d bits %d literal %d sliding %d state16 %d"
          % (seed, B, H_q, H_kv, max(lengths), bits, literal, sliding, state16), flush=True)
    Wq, Wk = synth.adapters_q(cfg, H_q), synth.adapters_k(cfg, H_kv)
    pairs = list({(int(rng.integers(0, B)), int(rng.integers(0, H_kv))) for _ in range(2)})
    T = max(lengths)
    gen = torch.Generator(device="cuda"); gen.manual_seed(seed)
    Kd = torch.randn(B, H_kv, T, 128, device="cuda", generator=gen).half()
    Vd = torch.randn(B, H_kv, T, 128, device="cuda", generator=gen).half()
    hist = {}
    for (b, g) in pairs:
        n = lengths[b]
        k, v = synth.keys(cfg, b, g, n), synth.values(cfg, b, g, n)
        Kd[b, g, :n] = torch.from_numpy(k).cuda()
        Vd[b, g, :n] = torch.from_numpy(v).cuda()
        hist[(b, g)] = (k, v)
    cache = kv.KVLincCache(B, H_q, H_kv, T + 300, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), bits=bits, flags=flags,
                           state_storage="fp16" if state16 else "fp32")
    tail = int(rng.integers(0, 3))
    pre = [max(0, n - tail) for n in lengths]
    cache.append(Kd[:, :, :max(max(pre), 1)].contiguous(), Vd[:, :, :max(max(pre), 1)].contiguous(),
                 n_new=tl.to_dev(np.asarray(pre, dtype=np.int32)))
    for s in range(tail):
        n_new = np.asarray([1 if pre[b] + s < lengths[b] else 0 for b in range(B)], dtype=np.int32)
        idx = [min(pre[b] + s, T - 1) for b in range(B)]
        kn = torch.stack([Kd[b, :, idx[b]] for b in range(B)]).unsqueeze(2).contiguous()
        vn = torch.stack([Vd[b, :, idx[b]] for b in range(B)]).unsqueeze(2).contiguous()
        cache.append(kn, vn, n_new=tl.to_dev(n_new))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    n_quant, n_res = tl.check_counters(cache, lengths)
    q = tl.gen_q(cfg, B, H_q)
    out = cache.decode(tl.to_dev(q), max_context=[0, T][int(rng.integers(0, 2))]).cpu().numpy()
    assert np.isfinite(out.astype(np.float32)).all()
    want = {}
    for (b, g) in pairs:
        k, v = hist[(b, g)]
        # 16-bit storage rounds the state at the end of every call that flushed
        first = tl.o_cache.window_split(pre[b])[0]
        points = list(range(first, int(n_quant[b]) + 1, 128)) if state16 else None
        tl.check_pair_against_oracle(cache, b, g, k, v, int(n_quant[b]), int(n_res[b]), None if state16 else Wk[g])
        ref = tl.o_cache.build_cache(k, v, int(n_quant[b]), Wk=Wk[g], bits=bits, state_rounding=points)
        for h in range(g * gq, (g + 1) * gq):
            want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h], literal_alg1=literal,
                                            value_window="sliding" if sliding else "block")
    tl.check_outputs(out, want)
    assert int(cache.split_done.abs().sum().item()) == 0
