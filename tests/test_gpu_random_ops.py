"""GPU parity on seeded random SEQUENCES OF CALLS: bulk appends with per-sequence row limits, one-token appends (some
sequences sitting out), appends with a non-finite row in one KV head of one sequence (that sequence must stay as it
was, the others take their rows), appends that exhaust the capacity of one sequence, and decode calls in between.  A
host model keeps every sequence's token history; the cache is a pure function of it (Sec. 3.3, last sentence: quantized
in blocks after attention has used the tokens), so counters, records, window, states and outputs are compared with the
oracle built from the history alone, at random points and for every (sequence, KV head) at the end."""
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


@pytest.mark.parametrize("seed,bits,sliding", [(0, 2, False), (1, 2, True), (2, 4, False), (3, 2, False), (4, 4, True), (5, 2, False),
                                                 (35, 2, True), (36, 4, True), (38, 2, True)])
def test_random_call_sequences(kv, seed, bits, sliding):
    import torch
    rng = np.random.default_rng(7000 + seed)
    B = int(rng.integers(1, 5))
    H_kv = int(rng.choice([1, 2, 3]))
    gq = int(rng.choice([1, 2, 4, 7]))
    H_q = gq * H_kv
    capacity = int(rng.choice([1024, 1536]))  # tokens the group records hold per sequence (+ the window)
    cfg = 700 + seed
    Wq, Wk = synth.adapters_q(cfg, H_q), synth.adapters_k(cfg, H_kv)
    literal, state16 = seed % 3 == 1, seed % 4 == 2  # the other variants of the path, by the seed
    cache = kv.KVLincCache(B, H_q, H_kv, capacity, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), bits=bits,
                           flags=(kv.KVLINC_FLAG_SLIDING_VALUES if sliding else 0) | (kv.KVLINC_FLAG_ALG1_LITERAL if literal else 0),
                           state_storage="fp16" if state16 else "fp32")
    rounded_at = [[] for _ in range(B)]  # 16-bit state: the quantized-token counts at which a call ended that had flushed
    hist_k = [np.zeros((H_kv, 0, 128), dtype=np.float16) for _ in range(B)]
    hist_v = [np.zeros((H_kv, 0, 128), dtype=np.float16) for _ in range(B)]

    def rows(T):
        k = (rng.standard_normal((B, H_kv, T, 128)) * rng.choice([0.5, 1.0, 3.0])).astype(np.float16)
        v = (rng.standard_normal((B, H_kv, T, 128)) * rng.choice([0.5, 1.0, 3.0])).astype(np.float16)
        return k, v

    def fits(b, n):  # does sequence b hold n more tokens?  (its quantized part may take max_groups groups)
        total = hist_k[b].shape[1] + n
        return tl.o_cache.window_split(total)[0] <= cache.max_groups * 128

    def check(pairs, decode):
        lengths = [h.shape[1] for h in hist_k]
        n_quant, n_res = tl.check_counters(cache, lengths)
        q = tl.gen_q(cfg, B, H_q, step=int(rng.integers(0, 1000)))
        out = None
        if decode:  # through one of the entry points, with one of the kinds of launch bound
            qd = tl.to_dev(q)
            bound = [0, max(lengths), max(lengths) + 700][int(rng.integers(0, 3))]
            if rng.random() < 0.3:
                od = torch.empty_like(qd)
                assert kv.kvlinc_decode_attention_noalloc(cache, qd, od, max_context=bound) == kv.KVLINC_OK
            else:
                od = cache.decode(qd, max_context=bound)
            out = od.cpu().numpy()
        want = {}
        for (b, g) in pairs:
            if lengths[b] == 0:
                if decode:
                    assert not out[b].any()
                continue
            ref = tl.check_pair_against_oracle(cache, b, g, hist_k[b][g], hist_v[b][g], int(n_quant[b]), int(n_res[b]),
                                               None if state16 else Wk[g])
            if state16:  # (no fp32 S to compare; the states enter through the output)
                ref = tl.o_cache.build_cache(hist_k[b][g], hist_v[b][g], int(n_quant[b]), Wk=Wk[g], bits=bits, state_rounding=rounded_at[b])
            if decode:
                for h in range(g * gq, (g + 1) * gq):
                    want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h], literal_alg1=literal, value_window="sliding" if sliding else "block")
        if want:
            tl.check_outputs(out, want)
        assert int(cache.split_done.abs().sum().item()) == 0

    n_ops = 40
    seen = {"poison": 0, "capacity": 0, "appends": 0}
    for op_i in range(n_ops):
        kind = rng.choice(["bulk", "one", "one", "one", "poison", "burst"])
        T = {"bulk": int(rng.integers(2, 400)), "one": 1, "poison": int(rng.choice([1, 1, 40])), "burst": 1}[kind]
        reps = int(rng.integers(20, 140)) if kind == "burst" else 1  # a burst: many one-token appends in a row
        for _ in range(reps):
            k, v = rows(T)
            n_new = np.asarray([int(rng.integers(0, T + 1)) if rng.random() < 0.4 else T for _ in range(B)], dtype=np.int32)
            expect = 0
            bad_b = -1
            if kind == "poison":
                bad_b = int(rng.integers(0, B))
                if n_new[bad_b] == 0:
                    n_new[bad_b] = T
                row, g = int(rng.integers(0, n_new[bad_b])), int(rng.integers(0, H_kv))
                which = rng.choice(["k_nan", "v_inf", "v_overflow"])
                if which == "k_nan":
                    k[bad_b, g, row, int(rng.integers(0, 128))] = np.float16("nan")
                elif which == "v_inf":
                    v[bad_b, g, row, int(rng.integers(0, 128))] = np.float16("-inf")
                else:
                    v[bad_b, g, row] = np.float16(6e4)  # finite, but its rotation leaves binary16
                expect |= kv.KVLINC_ST_NONFINITE
            taken = []
            for b in range(B):
                n = int(n_new[b])
                if b == bad_b or n == 0:
                    continue
                if not fits(b, n):
                    expect |= kv.KVLINC_ST_CAPACITY  # refused as a whole, the sequence stays as it is
                    continue
                taken.append(b)
            cache.status.zero_()
            cache.append(tl.to_dev(k), tl.to_dev(v), n_new=tl.to_dev(n_new))
            torch.cuda.synchronize()
            got = int(cache.status.item())
            seen["appends"] += 1
            seen["poison"] += int(bool(got & kv.KVLINC_ST_NONFINITE))
            seen["capacity"] += int(bool(got & kv.KVLINC_ST_CAPACITY))
            if bad_b >= 0 and not fits(bad_b, int(n_new[bad_b])):
                # the poisoned sequence is also out of room: it is refused for that before its rows are looked at
                assert got & kv.KVLINC_ST_CAPACITY and got & ~(kv.KVLINC_ST_CAPACITY | kv.KVLINC_ST_NONFINITE) == 0, (kind, got)
            else:
                assert got == expect, (kind, got, expect)
            for b in taken:
                n = int(n_new[b])
                nq_before = tl.o_cache.window_split(hist_k[b].shape[1])[0]
                hist_k[b] = np.concatenate([hist_k[b], k[b, :, :n]], axis=1)
                hist_v[b] = np.concatenate([hist_v[b], v[b, :, :n]], axis=1)
                nq_after = tl.o_cache.window_split(hist_k[b].shape[1])[0]
                if nq_after != nq_before:
                    rounded_at[b].append(nq_after)
        if rng.random() < 0.35 or kind == "poison":
            pairs = [(int(rng.integers(0, B)), int(rng.integers(0, H_kv))) for _ in range(2)]
            if bad_b >= 0:
                pairs.append((bad_b, int(rng.integers(0, H_kv))))
            print("  [ops] seed %d op %d (%s): lengths %s, checking %s" % (seed, op_i, kind, [h.shape[1] for h in hist_k], pairs), flush=True)
            check(pairs, decode=True)
    check([(b, g) for b in range(B) for g in range(H_kv)], decode=True)
    print("  [ops] seed %d: %d appends, %d with a refused non-finite row, %d with a sequence at its capacity; final lengths %s"
          % (seed, seen["appends"], seen["poison"], seen["capacity"], [h.shape[1] for h in hist_k]), flush=True)
    assert seen["poison"] > 0 or seen["capacity"] > 0  # (a sequence that is out of room is refused for that first)
