"""GPU parity on seeded random shapes: batch, head counts, lengths (with the window boundaries mixed in), a bulk
prefix followed by a few one-token appends, correction on or off, 2-bit and 4-bit codes, the variants of the path (literal Alg. 1, sliding value window, 16-bit state) drawn at random, and the three kinds of launch bound.  Records, window,
states and outputs of two random (sequence, KV head) pairs per case are compared with the oracle."""
import numpy as np
import pytest

import kvlinc_synth as synth
from tests import kvlinc_testlib as tl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kv():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2510_05373_amd as kvmod
    return kvmod


@pytest.mark.parametrize("seed,bits", [(0, 2), (1, 2), (2, 2), (3, 4), (4, 4), (5, 2), (6, 4), (7, 2), (8, 4), (9, 2)])
def test_random_shapes(kv, seed, bits):
    import torch
    rng = np.random.default_rng(1000 + seed)
    vrng = np.random.default_rng(5000 + seed)  # the variants of the path, drawn apart from the shapes
    for it in range(12):
        B = int(rng.integers(1, 7))
        H_kv = int(rng.choice([1, 2, 3]))
        gq = int(rng.integers(1, 9))
        H_q = gq * H_kv
        hi = int(rng.choice([400, 3000, 6000]))
        lengths = [int(rng.integers(0, hi + 1)) for _ in range(B)]
        if rng.random() < 0.3:
            lengths[int(rng.integers(0, B))] = int(rng.choice([0, 1, 127, 128, 129, 255, 256, 257]))
        if max(lengths) == 0:
            lengths[0] = 1
        cfg = 100 * (seed + 1) + it
        literal, sliding, state16 = (bool(vrng.random() < 0.3) for _ in range(3))
        flags = (kv.KVLINC_FLAG_ALG1_LITERAL if literal else 0) | (kv.KVLINC_FLAG_SLIDING_VALUES if sliding else 0)
        print("  [case] seed %d #%d B=%d heads %d/%d lengths %s literal %d sliding %d state16 %d"
              % (seed, it, B, H_q, H_kv, lengths, literal, sliding, state16), flush=True)
        K, V = tl.gen_kv(cfg, B, H_kv, lengths)
        corr = rng.random() < 0.8
        Wq = synth.adapters_q(cfg, H_q) if corr else None
        Wk = synth.adapters_k(cfg, H_kv) if corr else None
        cache = kv.KVLincCache(B, H_q, H_kv, max(lengths) + int(rng.integers(1, 600)),
                               Wq=None if Wq is None else tl.to_dev(Wq), Wk=None if Wk is None else tl.to_dev(Wk), bits=bits,
                               flags=flags, state_storage="fp16" if state16 else "fp32")
        tail = int(rng.integers(0, 4))  # the last `tail` tokens arrive one at a time
        pre = [max(0, n - tail) for n in lengths]
        Kd, Vd = tl.to_dev(K), tl.to_dev(V)
        T = max(max(pre), 1)
        cache.append(Kd[:, :, :T].contiguous(), Vd[:, :, :T].contiguous(),
                     n_new=tl.to_dev(np.asarray(pre, dtype=np.int32)))
        for s in range(tail):
            n_new = np.asarray([1 if pre[b] + s < lengths[b] else 0 for b in range(B)], dtype=np.int32)
            idx = [min(pre[b] + s, K.shape[2] - 1) for b in range(B)]
            kn = torch.stack([Kd[b, :, idx[b]] for b in range(B)]).unsqueeze(2).contiguous()
            vn = torch.stack([Vd[b, :, idx[b]] for b in range(B)]).unsqueeze(2).contiguous()
            cache.append(kn, vn, n_new=tl.to_dev(n_new))
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        n_quant, n_res = tl.check_counters(cache, lengths)
        q = tl.gen_q(cfg, B, H_q)
        bound = [0, max(lengths), max(lengths) + 1000][int(rng.integers(0, 3))]
        out = cache.decode(tl.to_dev(q), max_context=bound).cpu().numpy()
        assert np.isfinite(out.astype(np.float32)).all()
        for b in range(B):
            if lengths[b] == 0:
                assert not out[b].any()
        pairs = {(int(rng.integers(0, B)), int(rng.integers(0, H_kv))) for _ in range(2)}
        pairs = [p for p in pairs if lengths[p[0]] > 0]
        want = {}
        for (b, g) in pairs:
            # (with the state stored in 16 bits only there is no fp32 S to compare: the output comparison covers it)
            tl.check_pair_against_oracle(cache, b, g, K[b, g, :lengths[b]], V[b, g, :lengths[b]], int(n_quant[b]),
                                         int(n_res[b]), None if (Wk is None or state16) else Wk[g])
            # the 16-bit state was rounded at the end of every call that flushed: after the bulk build and after each flush since
            first = tl.o_cache.window_split(pre[b])[0]
            points = list(range(first, int(n_quant[b]) + 1, 128)) if (state16 and corr) else None
            ref = tl.o_cache.build_cache(K[b, g, :lengths[b]], V[b, g, :lengths[b]], int(n_quant[b]), Wk=None if Wk is None else Wk[g],
                                         bits=bits, state_rounding=points)
            for h in range(g * gq, (g + 1) * gq):
                want[(b, h)] = tl.o_attn.decode(q[b, h], ref, None if Wq is None else Wq[h], literal_alg1=literal,
                                                value_window="sliding" if sliding else "block")
        if pairs:
            tl.check_outputs(out, want)
        assert int(cache.split_done.abs().sum().item()) == 0
