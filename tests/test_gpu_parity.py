"""GPU parity: the HIP path through the C ABI against the oracle, element by element (needs an MI355X)."""
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


def _build(kv, cfg, B, H_q, H_kv, lengths, R=128, keep=None, correction=True, capacity=None, bits=2, flags=0):
    K, V = tl.gen_kv(cfg, B, H_kv, lengths)
    Wq = synth.adapters_q(cfg, H_q) if correction else None
    Wk = synth.adapters_k(cfg, H_kv) if correction else None
    cache = kv.KVLincCache(B, H_q, H_kv, capacity or int(max(lengths)) + 512, R=R,
                           Wq=None if Wq is None else tl.to_dev(Wq), Wk=None if Wk is None else tl.to_dev(Wk),
                           bits=bits, flags=flags)
    n_new = tl.to_dev(np.asarray(lengths, dtype=np.int32))
    cache.append(tl.to_dev(K), tl.to_dev(V), n_new=n_new, keep_residual=0 if keep is None else keep)
    return cache, K, V, Wq, Wk


def _all_pairs(B, H_kv):
    return [(b, g) for b in range(B) for g in range(H_kv)]


@pytest.mark.parametrize("correction", [True, False])
def test_bulk_append_and_decode_small_ragged(kv, correction):
    """Several tiles, ragged lengths (one below a group, one an exact multiple, one with a long tail)."""
    import torch
    B, H_q, H_kv = 4, 8, 2
    lengths = [700, 128, 57, 1025]
    cache, K, V, Wq, Wk = _build(kv, 11, B, H_q, H_kv, lengths, correction=correction)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(B, H_kv), Wk=Wk)
    q = tl.gen_q(11, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)


def test_one_token_appends_cross_flushes(kv):
    """Bulk prefix, then one-token appends through two window flushes; state after every flush boundary and at the
    end must equal the oracle's pure function of the token history."""
    import torch
    B, H_q, H_kv = 2, 8, 2
    start, steps = [250, 127], 300
    total = [s + steps for s in start]
    K, V = tl.gen_kv(12, B, H_kv, total)
    Wq, Wk = synth.adapters_q(12, H_q), synth.adapters_k(12, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    T0 = max(start)
    k0 = torch.zeros(B, H_kv, T0, 128, dtype=torch.float16, device="cuda")
    v0 = torch.zeros_like(k0)
    for b in range(B):
        k0[b, :, :start[b]] = Kd[b, :, :start[b]]
        v0[b, :, :start[b]] = Vd[b, :, :start[b]]
    cache.append(k0, v0, n_new=tl.to_dev(np.asarray(start, dtype=np.int32)))
    lengths = list(start)
    for step in range(steps):
        kn = torch.stack([Kd[b, :, lengths[b]:lengths[b] + 1] for b in range(B)]).contiguous()
        vn = torch.stack([Vd[b, :, lengths[b]:lengths[b] + 1] for b in range(B)]).contiguous()
        cache.append(kn, vn)
        lengths = [n + 1 for n in lengths]
        if step in (0, 5, 6, 7, 133, 134, 135, steps - 1):
            tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(B, H_kv), Wk=Wk)
            q = tl.gen_q(12, B, H_q, step)
            out = cache.decode(tl.to_dev(q)).cpu().numpy()
            want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv,
                                    Wq, Wk)
            tl.check_outputs(out, want)
    assert int(cache.status.item()) == 0


def test_config1_partial_tail_group(kv):
    """Workload 1: batch 1, 32/8 heads, context 1024, 32-token window -> 7 full groups + a 96-token tail group."""
    c = synth.CONFIGS[1]
    lengths = [c["n"]]
    cache, K, V, Wq, Wk = _build(kv, 1, c["B"], c["H_q"], c["H_kv"], lengths, R=c["R"], keep=c["keep"], capacity=1024)
    assert cache.n_quant.cpu().tolist() == [992] and cache.n_res.cpu().tolist() == [32]
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(1, 8), Wk=Wk, keep=32)
    q = tl.gen_q(1, 1, 32)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, [992], _all_pairs(1, 8), 32, 8, Wq, Wk)
    tl.check_outputs(out, want)
    # a sequence with a partial last group accepts no further token
    import torch
    z = torch.zeros(1, 8, 1, 128, dtype=torch.float16, device="cuda")
    cache.append(z, z, keep_residual=32)
    torch.cuda.synchronize()
    assert int(cache.status.item()) & kv.KVLINC_ST_STATIC
    assert cache.n_quant.cpu().tolist() == [992] and cache.n_res.cpu().tolist() == [32]


@pytest.mark.parametrize("gq,H_kv", [(1, 2), (7, 2), (2, 1), (8, 1), (3, 2), (5, 1), (6, 3), (4, 5)])
def test_other_head_ratios(kv, gq, H_kv):
    B, H_q = 2, gq * H_kv
    lengths = [400, 300]
    cache, K, V, Wq, Wk = _build(kv, 13, B, H_q, H_kv, lengths)
    q = tl.gen_q(13, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)


def test_many_short_sequences(kv):
    """More sequences than compute units, each a few hundred tokens: every sequence one split, several generations of
    workgroups, correction workgroups far outnumbering the places."""
    B, H_q, H_kv = 300, 2, 1
    lengths = [129 + (37 * b) % 400 for b in range(B)]
    cache, K, V, Wq, Wk = _build(kv, 20, B, H_q, H_kv, lengths)
    q = tl.gen_q(20, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    pairs = [(b, 0) for b in (0, 1, 63, 64, 127, 128, 255, 256, 298, 299)]
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), pairs, H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)
    assert np.isfinite(out.astype(np.float32)).all() and int(cache.split_done.abs().sum().item()) == 0


def test_cache_filled_to_its_last_group(kv):
    """Capacity 4 groups: a bulk build of 512 tokens, then one-token appends.  Token 513 flushes into the last group;
    at 640 tokens every group and the window are full and decode must still be exact (a wave's first request is
    clamped to the last record); token 641 would need a fifth group: the status bit is set and the sequence stays."""
    import torch
    B, H_q, H_kv = 2, 4, 1
    total = 641
    K, V = tl.gen_kv(21, B, H_kv, [total, total])
    Wq, Wk = synth.adapters_q(21, H_q), synth.adapters_k(21, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 512, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    assert cache.max_groups == 4
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :512].contiguous(), Vd[:, :, :512].contiguous())
    for t in range(512, 640):
        cache.append(Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous())
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    assert cache.n_quant.cpu().tolist() == [512, 512] and cache.n_res.cpu().tolist() == [128, 128]
    lengths = [640, 640]
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(B, H_kv), Wk=Wk)
    q = tl.gen_q(21, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, [512, 512], _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)
    cache.append(Kd[:, :, 640:641].contiguous(), Vd[:, :, 640:641].contiguous())
    torch.cuda.synchronize()
    assert int(cache.status.item()) & kv.KVLINC_ST_CAPACITY
    assert cache.n_quant.cpu().tolist() == [512, 512] and cache.n_res.cpu().tolist() == [128, 128]
    out2 = cache.decode(tl.to_dev(q)).cpu().numpy()
    assert np.array_equal(out.view(np.uint16), out2.view(np.uint16))


@pytest.mark.parametrize("key_gain,query_gain", [(32, 4), (256, 16)])
def test_large_magnitudes_stay_finite(kv, key_gain, query_gain):
    """Keys and queries far larger than any activation of the paper's models (|k| up to 7e3): the binary16 operands
    of the matrix products must not overflow, and the (then one-hot) softmax must still match the oracle."""
    B, H_q, H_kv = 1, 4, 1
    lengths = [700]
    K, V = tl.gen_kv(22, B, H_kv, lengths)
    K = (K.astype(np.float32) * key_gain).astype(np.float16)
    q = (tl.gen_q(22, B, H_q).astype(np.float32) * query_gain).astype(np.float16)
    assert np.isfinite(K.astype(np.float32)).all()
    Wq, Wk = synth.adapters_q(22, H_q), synth.adapters_k(22, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache.append(tl.to_dev(K), tl.to_dev(V))
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    assert int(cache.status.item()) == 0 and np.isfinite(out.astype(np.float32)).all()
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), [(0, 0)], H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)


def test_degenerate_inputs(kv):
    import torch
    B, H_q, H_kv = 3, 4, 1
    # sequence 0 empty, sequence 1 a single token, sequence 2 constant keys/values (scale 0 everywhere)
    lengths = [0, 1, 300]
    K, V = tl.gen_kv(14, B, H_kv, lengths)
    K[2, :, :300] = np.float16(0.75)
    V[2, :, :300] = np.float16(-1.5)
    Wq, Wk = synth.adapters_q(14, H_q), synth.adapters_k(14, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
    tl.check_cache_against_oracle(cache, K, V, lengths, [(1, 0), (2, 0)], Wk=Wk)
    # constant keys: every key code is 0 (stored as the bit pair 1,1: all-ones words) and every key scale is 0
    assert (cache.groups[2, 0, :2, :1024] == -1).all() and not cache.groups[2, 0, :2, 2048:2112].any()
    q = tl.gen_q(14, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    assert not out[0].any()  # no tokens -> zeros
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), [(1, 0), (2, 0)], H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)
    assert int(cache.status.item()) == 0


def test_signed_zeros_give_a_positive_zero_point(kv):
    """A group minimum that is a negative zero is stored as +0 (the quantizer contract), on the GPU as in the oracle:
    a key channel of negative zeros only, one whose only zero is a -0 below positive values, and zeros of both signs."""
    B, H_q, H_kv = 1, 4, 1
    lengths = [256]
    K, V = tl.gen_kv(19, B, H_kv, lengths)
    K[0, 0, :, 3] = np.float16(-0.0)
    K[0, 0, :, 5] = np.abs(K[0, 0, :, 5]) + np.float16(0.25)
    K[0, 0, 17, 5] = np.float16(-0.0)
    K[0, 0, ::2, 9] = np.float16(-0.0)
    K[0, 0, 1::2, 9] = np.float16(0.0)
    Wq, Wk = synth.adapters_q(19, H_q), synth.adapters_k(19, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache.append(tl.to_dev(K), tl.to_dev(V))
    tl.check_cache_against_oracle(cache, K, V, lengths, [(0, 0)], Wk=Wk)
    rec = cache.groups[0, 0, 0].cpu().numpy().view(np.uint32)
    kz = rec[2112:2176]  # key zero-points, channel 2i in the low half of word i
    assert (kz[1] >> 16) == 0 and (kz[4] >> 16) == 0, "channels 3 and 9: zero-point +0"
    assert (kz[2] >> 16) == 0, "channel 5: minimum -0 stored as +0"


def test_status_bits_and_rejections(kv):
    import torch
    B, H_q, H_kv = 1, 4, 1
    cache = kv.KVLincCache(B, H_q, H_kv, 256)  # capacity: 2 groups
    k = torch.randn(B, H_kv, 600, 128, device="cuda").half()
    cache.append(k, k)  # would need 4 groups
    torch.cuda.synchronize()
    assert int(cache.status.item()) == kv.KVLINC_ST_CAPACITY
    assert cache.n_quant.item() == 0 and cache.n_res.item() == 0 and not cache.groups.any()
    cache.status.zero_()
    k[0, 0, 5, 7] = float("inf")
    cache.append(k[:, :, :300].contiguous(), k[:, :, :300].contiguous())
    torch.cuda.synchronize()
    assert int(cache.status.item()) == kv.KVLINC_ST_NONFINITE
    assert cache.n_quant.item() == 0 and cache.n_res.item() == 0 and not cache.split_done.any()
    # host-side rejections: nothing is launched
    q = torch.zeros(B, H_q, 128, dtype=torch.float16, device="cuda")
    ws = torch.empty(4, device="cuda")
    assert kv.kvlinc_decode_attention(cache, q, q.clone(), ws) == kv.KVLINC_EWORKSPACE
    assert kv.kvlinc_append_quantize(cache, k, k, None, 0, 0) == kv.KVLINC_EINVAL
    assert kv.kvlinc_append_quantize(cache, k, k, None, 600, 200) == kv.KVLINC_EINVAL


def test_row_limits_outside_0_T_are_clamped(kv):
    """n_new below 0 reads as 0, above T as T (the kernels never read beyond the T rows that were passed), in a
    one-token append, a bulk append that stays in the window and one that flushes."""
    import torch
    B, H_q, H_kv = 3, 4, 2
    for T in (1, 40, 300):
        lengths = [0, T, T]
        K, V = tl.gen_kv(21, B, H_kv, [T, T, T])
        cache = kv.KVLincCache(B, H_q, H_kv, 1024)
        cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray([-7, T + 1000, T], dtype=np.int32)))
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        tl.check_cache_against_oracle(cache, K, V, lengths, [(1, 0), (1, 1), (2, 0)], check_states=False)
        assert cache.n_quant.cpu().tolist()[0] == 0 and cache.n_res.cpu().tolist()[0] == 0


def test_two_caches_stepped_on_two_streams_give_the_same_bits(kv):
    """Calls on different caches may overlap in time: two caches (2-bit and 4-bit codes) stepped through appends, a
    window flush and decodes on two streams at once end with the bits of the same steps taken one after the other."""
    import torch
    dev = torch.device("cuda:0")

    def run(concurrent):
        g = torch.Generator(device=dev)
        g.manual_seed(77)
        B, H_q, H_kv, n0, steps = 3, 8, 2, 600, 150
        Wq = (torch.randn(H_q, 2, 128, 128, device=dev, generator=g) / 128 ** 0.5).half()
        Wk = (torch.randn(H_kv, 2, 128, 128, device=dev, generator=g) / 128 ** 0.5).half()
        caches, data, outs = [], [], []
        for j in range(2):
            c = kv.KVLincCache(B, H_q, H_kv, n0 + steps + 200, Wq=Wq, Wk=Wk, bits=2 + 2 * j)
            K = torch.randn(B, H_kv, n0, 128, device=dev, generator=g).half()
            V = torch.randn(B, H_kv, n0, 128, device=dev, generator=g).half()
            c.append(K, V)
            data.append(tuple(torch.randn(steps, B, h, n, 128, device=dev, generator=g).half().squeeze(3)
                              for h, n in ((H_kv, 1), (H_kv, 1), (H_q, 1))))
            caches.append(c)
            outs.append(torch.empty(steps, B, H_q, 128, dtype=torch.float16, device=dev))
            c.workspace(n0 + steps + 1)
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream(), torch.cuda.Stream()] if concurrent else [torch.cuda.current_stream()] * 2
        for s in range(steps):
            for j in range(2):
                kn, vn, qq = data[j]
                caches[j].append(kn[s].unsqueeze(2), vn[s].unsqueeze(2), stream=streams[j])
                caches[j].decode(qq[s], out=outs[j][s], max_context=n0 + steps + 1, stream=streams[j])
        torch.cuda.synchronize()
        for c in caches:
            assert int(c.status.item()) == 0 and not c.split_done.any()
        return ([o.cpu().numpy().view(np.uint16) for o in outs] + [c.groups.cpu().numpy() for c in caches]
                + [c.S16.cpu().numpy().view(np.uint16) for c in caches] + [c.n_quant.cpu().numpy() for c in caches])

    for x, y in zip(run(False), run(True)):
        assert np.array_equal(x, y)


def _live_state(cache):
    """Everything a sequence's state consists of, as host arrays: counters, live group records and window rows, states."""
    nq, nr = cache.n_quant.cpu().numpy().copy(), cache.n_res.cpu().numpy().copy()
    out = {"n_quant": nq, "n_res": nr, "split_done": cache.split_done.cpu().numpy().copy()}
    for b in range(cache.B):
        ng = -(-int(nq[b]) // 128)
        out["groups%d" % b] = cache.groups[b, :, :ng].cpu().numpy().copy()
        out["k_res%d" % b] = cache.k_res[b, :, :int(nr[b])].cpu().numpy().view(np.uint16).copy()
        out["v_res%d" % b] = np.stack([tl.o_layout.unpack_value_window(cache.v_res[b, g].cpu().numpy(), int(nr[b]))
                                       for g in range(cache.H_kv)]).view(np.uint16).copy()
    if cache.S is not None:
        out["S"] = cache.S.cpu().numpy().view(np.uint32).copy()
        out["P"] = cache.P.cpu().numpy().view(np.uint32).copy()
        out["S16"] = cache.S16.cpu().numpy().view(np.uint16).copy()
    return out


def _assert_same_state(a, b):
    assert a.keys() == b.keys()
    for k in a:
        assert np.array_equal(a[k], b[k]), k


@pytest.mark.parametrize("H_kv,bad_head", [(2, 1), (2, 0), (1, 0), (3, 2)])
def test_rejected_append_leaves_the_sequence_unchanged(kv, H_kv, bad_head):
    """A non-finite new token -- in any KV head, arriving alone or inside a bulk append, in a key, a value, or as a
    value whose rotation overflows fp16 -- sets KVLINC_ST_NONFINITE and leaves counters, live records, window and states
    of that sequence bit for bit as they were; the other sequence of the batch takes its tokens; a clean retry works."""
    import torch
    B, gq = 2, 2
    H_q = gq * H_kv
    lengths = [383, 250]  # sequence 0: one token short of a full window (the next append is plain, the one after flushes)
    cache, K, V, Wq, Wk = _build(kv, 31, B, H_q, H_kv, lengths)
    rng = np.random.default_rng(5)
    fresh = lambda T: (rng.standard_normal((B, H_kv, T, 128)).astype(np.float16),
                       rng.standard_normal((B, H_kv, T, 128)).astype(np.float16))
    total = [list(lengths)]

    def attempt(kn, vn, poison, n_new=None):
        """Append with `poison` applied to sequence 0 only: sequence 0 must be refused, sequence 1 must take its rows."""
        before = _live_state(cache)
        kp, vp = kn.copy(), vn.copy()
        poison(kp, vp)
        cache.status.zero_()
        cache.append(tl.to_dev(kp), tl.to_dev(vp), n_new=None if n_new is None else tl.to_dev(np.asarray(n_new, dtype=np.int32)))
        torch.cuda.synchronize()
        assert int(cache.status.item()) == kv.KVLINC_ST_NONFINITE
        after = _live_state(cache)
        T = kn.shape[2] if n_new is None else n_new[1]
        assert after["n_quant"][0] == before["n_quant"][0] and after["n_res"][0] == before["n_res"][0]
        assert after["n_quant"][1] + after["n_res"][1] == before["n_quant"][1] + before["n_res"][1] + T
        for k in before:  # everything of sequence 0
            if k.endswith("0"):
                assert np.array_equal(before[k], after[k]), k
        if "S" in before:
            for k in ("S", "P", "S16"):
                assert np.array_equal(before[k][0], after[k][0]), k
        assert not after["split_done"].any()
        total[0][1] += T
        return kn[1], vn[1]

    hist_k, hist_v = [K[1, :, :lengths[1]]], [V[1, :, :lengths[1]]]
    # 1. one token, NaN in a key of `bad_head`
    kn, vn = fresh(1)
    k1, v1 = attempt(kn, vn, lambda k, v: k.__setitem__((0, bad_head, 0, 17), np.float16("nan")))
    hist_k.append(k1); hist_v.append(v1)
    # a clean token fills sequence 0's window: the next one-token append has to flush it
    kn, vn = fresh(1)
    cache.append(tl.to_dev(kn), tl.to_dev(vn))
    K = np.concatenate([K[:, :, :lengths[0]], kn], axis=2)  # (sequence 0's rows; sequence 1 is tracked in hist_*)
    V = np.concatenate([V[:, :, :lengths[0]], vn], axis=2)
    lengths = [lengths[0] + 1, lengths[1]]
    hist_k.append(kn[1]); hist_v.append(vn[1])
    assert cache.n_res.cpu().tolist()[0] == 128
    # 2. one token that would flush, a finite value row whose rotation overflows fp16 (all channels 6e4 -> 6.8e5)
    kn, vn = fresh(1)
    k1, v1 = attempt(kn, vn, lambda k, v: v.__setitem__((0, bad_head, 0), np.float16(6e4)))
    hist_k.append(k1); hist_v.append(v1)
    # 3. a bulk append of 300 rows (it would flush sequence 0's window twice), Inf in a value of `bad_head` at row 200
    kn, vn = fresh(300)
    k1, v1 = attempt(kn, vn, lambda k, v: v.__setitem__((0, bad_head, 200, 3), np.float16("inf")))
    hist_k.append(k1); hist_v.append(v1)
    # 4. the same with a row limit: the fault lies in a row that is appended (row 4 of 5)
    kn, vn = fresh(300)
    k1, v1 = attempt(kn, vn, lambda k, v: k.__setitem__((0, bad_head, 4, 100), np.float16("-inf")), n_new=[5, 7])
    hist_k.append(k1[:, :7]); hist_v.append(v1[:, :7])
    # a fault in a row beyond the limit is not looked at
    kn, vn = fresh(8)
    kp = kn.copy()
    kp[0, bad_head, 6, 0] = np.float16("nan")
    cache.status.zero_()
    cache.append(tl.to_dev(kp), tl.to_dev(vn), n_new=tl.to_dev(np.asarray([3, 8], dtype=np.int32)))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0
    K0 = np.concatenate([K[0, :, :lengths[0]], kn[0, :, :3]], axis=1)
    V0 = np.concatenate([V[0, :, :lengths[0]], vn[0, :, :3]], axis=1)
    hist_k.append(kn[1]); hist_v.append(vn[1])
    K1, V1 = np.concatenate(hist_k, axis=1), np.concatenate(hist_v, axis=1)
    n0, n1 = K0.shape[1], K1.shape[1]
    tl.check_counters(cache, [n0, n1])
    n_quant, n_res = cache.n_quant.cpu().numpy(), cache.n_res.cpu().numpy()
    q = tl.gen_q(31, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = {}
    for b, (Kb, Vb) in enumerate(((K0, V0), (K1, V1))):
        for g in range(H_kv):
            ref = tl.check_pair_against_oracle(cache, b, g, Kb[g], Vb[g], int(n_quant[b]), int(n_res[b]), Wk[g])
            for h in range(g * gq, (g + 1) * gq):
                want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h])
    tl.check_outputs(out, want)


@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("log2_gain", [-8, -4, 4, 8])
@pytest.mark.parametrize("which", ["values", "keys"])
def test_magnitudes_far_from_one_keep_the_tolerance(kv, which, log2_gain, bits):
    """Values (resp. keys) scaled by 2^-8 .. 2^8: the operands of the matrix products carry block exponents, so the
    output stays inside the tolerance whatever the magnitude (relative to the output's own size)."""
    B, H_q, H_kv = 2, 8, 2
    lengths = [900, 517]
    K, V = tl.gen_kv(33, B, H_kv, lengths)
    gain = np.float32(2.0 ** log2_gain)
    if which == "values":
        V = (V.astype(np.float32) * gain).astype(np.float16)
    else:
        K = (K.astype(np.float32) * gain).astype(np.float16)
    Wq, Wk = synth.adapters_q(33, H_q), synth.adapters_k(33, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), bits=bits)
    cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
    q = tl.gen_q(33, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy().astype(np.float64)
    assert int(cache.status.item()) == 0
    n_quant, n_res = tl.check_counters(cache, lengths)
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(B, H_kv), Wk=Wk)  # (records, window, states at that magnitude)
    want = tl.oracle_decode(K, V, q, lengths, n_quant, _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk, bits=bits)
    # the tolerance is stated for outputs of order one: compare at the values' own scale
    unit = float(gain) if which == "values" else 1.0
    scaled = {k: v / unit for k, v in want.items()}
    tl.check_outputs(out / unit, scaled)


def test_state_beyond_the_binary16_range_is_flagged_and_saturated(kv):
    """Values with a common sign make S grow with the context: rotated values of 442 in every channel and 20480 quantized
    tokens put entries of S near 442 * 20480 / 128 = 7e4 > 65504.  The append reports KVLINC_ST_STATE_RANGE, the 16-bit
    copy holds +-65504 there, and nothing is Inf or NaN."""
    import torch
    B, H_q, H_kv = 1, 4, 1
    n = 20480 + 128
    K, _ = tl.gen_kv(34, B, H_kv, [n])
    V = np.zeros_like(K)
    V[..., 0] = np.float16(5000.0)  # rotation: 5000 / sqrt(128) = 442 in all 128 channels
    Wq, Wk = synth.adapters_q(34, H_q), synth.adapters_k(34, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, n, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache.append(tl.to_dev(K[:, :, :4096]), tl.to_dev(V[:, :, :4096]))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0  # still in range at 4096 tokens
    cache.append(tl.to_dev(K[:, :, 4096:]), tl.to_dev(V[:, :, 4096:]))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == kv.KVLINC_ST_STATE_RANGE
    S = cache.S.cpu().numpy()
    S16 = cache.S16.cpu().numpy().astype(np.float32)
    assert np.isfinite(S).all() and np.abs(S).max() > 65504.0
    assert np.isfinite(S16).all() and np.abs(S16).max() == 65504.0
    out = cache.decode(tl.to_dev(tl.gen_q(34, B, H_q))).cpu().numpy()
    assert np.isfinite(out.astype(np.float32)).all()


def test_state_stored_in_16_bits_only(kv):
    """S == NULL: the state lives in its binary16 tiles.  A bulk build (one rounding), then one-token appends across
    three window flushes (one rounding each), against the oracle with the same rounding points: the tiles are equal
    almost everywhere and within one rounding flip per rounding point elsewhere (the GPU sums a group in binary32), P
    and the records as always, outputs inside the tolerance.  The same history with the fp32 master copy gives tiles that differ (it rounds the exact sum)."""
    import torch
    B, H_q, H_kv = 2, 8, 2
    pre, extra = [700, 333], 300
    lengths = [p + extra for p in pre]
    K, V = tl.gen_kv(35, B, H_kv, lengths)
    Wq, Wk = synth.adapters_q(35, H_q), synth.adapters_k(35, H_kv)
    caches = {}
    for storage in ("fp16", "fp32"):
        cache = kv.KVLincCache(B, H_q, H_kv, 2048, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), state_storage=storage)
        Kd, Vd = tl.to_dev(K), tl.to_dev(V)
        cache.append(Kd[:, :, :max(pre)].contiguous(), Vd[:, :, :max(pre)].contiguous(),
                     n_new=tl.to_dev(np.asarray(pre, dtype=np.int32)))
        for s in range(extra):
            kn = torch.stack([Kd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            vn = torch.stack([Vd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            cache.append(kn, vn)
        torch.cuda.synchronize()
        assert int(cache.status.item()) == 0
        caches[storage] = cache
    cache = caches["fp16"]
    assert cache.S is None
    n_quant, n_res = tl.check_counters(cache, lengths)
    q = tl.gen_q(35, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = {}
    gq = H_q // H_kv
    for b in range(B):
        first = tl.o_cache.window_split(pre[b])[0]          # quantized tokens after the bulk build
        points = list(range(first, int(n_quant[b]) + 1, 128))  # ... and after every flush since
        for g in range(H_kv):
            n = lengths[b]
            ref = tl.o_cache.build_cache(K[b, g, :n], V[b, g, :n], int(n_quant[b]), Wk=Wk[g], state_rounding=points)
            tl.check_pair_against_oracle(cache, b, g, K[b, g, :n], V[b, g, :n], int(n_quant[b]), int(n_res[b]), None)
            S16 = tl.o_layout.unpack_state_tiles(cache.S16[b, g].cpu().numpy())
            # A group's sum differs in its last binary32 bits, which now and then flips a rounding: one unit in the
            # last place of that entry AS IT WAS THEN -- an entry that has since cancelled to a small value keeps the
            # absolute difference -- and at most one flip per rounding point.  So: equal bits almost everywhere, and
            # everywhere within (rounding points) x (unit in the last place of the largest entry).
            ulps = np.abs(tl._ordered16(S16) - tl._ordered16(ref["S"].astype(np.float16)))
            s_max = np.abs(ref["S"]).max()
            ulp_max = 2.0 ** (np.floor(np.log2(s_max)) - 10)
            assert np.abs(S16.astype(np.float64) - ref["S"]).max() <= len(points) * ulp_max, (b, g, int(ulps.max()))
            assert (ulps == 0).mean() > 0.9
            P = cache.P[b, g].cpu().numpy().astype(np.float64)
            assert np.abs(P - ref["P"]).max() <= tl.STATE_P_ELEMENT * np.abs(ref["P"]).max()
            for h in range(g * gq, (g + 1) * gq):
                want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h])
    tl.check_outputs(out, want)
    assert not torch.equal(caches["fp16"].S16, caches["fp32"].S16)  # several roundings against one
    assert torch.equal(caches["fp16"].groups, caches["fp32"].groups) and torch.equal(caches["fp16"].P, caches["fp32"].P)


def test_alg1_literal_correction_mode(kv):
    """KVLINC_FLAG_ALG1_LITERAL: the correction terms are added to the max-shifted sums without the factor e^-M, as the
    last lines of Alg. 1 print them; against the oracle's switch of the same name, and different from the Eq. 5 mode."""
    B, H_q, H_kv = 2, 8, 2
    lengths = [1500, 777]
    K, V = tl.gen_kv(36, B, H_kv, lengths)
    Wq, Wk = synth.adapters_q(36, H_q), synth.adapters_k(36, H_kv)
    outs = {}
    for flags in (0, kv.KVLINC_FLAG_ALG1_LITERAL):
        cache = kv.KVLincCache(B, H_q, H_kv, 2048, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), flags=flags)
        cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
        q = tl.gen_q(36, B, H_q)
        outs[flags] = cache.decode(tl.to_dev(q)).cpu().numpy()
        assert int(cache.status.item()) == 0
        n_quant = cache.n_quant.cpu().numpy()
    gq = H_q // H_kv
    want = {}
    for b in range(B):
        for g in range(H_kv):
            n = lengths[b]
            ref = tl.o_cache.build_cache(K[b, g, :n], V[b, g, :n], int(n_quant[b]), Wk=Wk[g])
            for h in range(g * gq, (g + 1) * gq):
                want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h], literal_alg1=True)
    tl.check_outputs(outs[kv.KVLINC_FLAG_ALG1_LITERAL], want)
    diff = np.abs(outs[0].astype(np.float64) - outs[kv.KVLINC_FLAG_ALG1_LITERAL].astype(np.float64)).max()
    assert diff > 1e-3  # the two modes are different functions of the same cache


def test_run_to_run_determinism(kv):
    import torch
    B, H_q, H_kv = 2, 8, 2
    lengths = [1500, 900]
    cache, K, V, Wq, Wk = _build(kv, 15, B, H_q, H_kv, lengths)
    q = tl.to_dev(tl.gen_q(15, B, H_q))
    first = cache.decode(q).clone()
    for _ in range(5):
        assert torch.equal(cache.decode(q), first)
    cache2, *_ = _build(kv, 15, B, H_q, H_kv, lengths)
    for name in ("groups", "k_res", "v_res", "S", "P"):
        assert torch.equal(getattr(cache, name), getattr(cache2, name)), name


@pytest.mark.parametrize("n_quant,n_res", [(0, 1), (0, 64), (0, 65), (0, 128), (128, 1), (128, 63), (256, 64),
                                           (256, 65), (384, 127), (1024, 128)])
def test_window_boundaries(kv, n_quant, n_res):
    """Every way the fp16 window can meet its two 64-token halves, with and without quantized groups before it."""
    B, H_q, H_kv = 2, 8, 2
    n = n_quant + n_res
    lengths = [n, n]
    cache, K, V, Wq, Wk = _build(kv, 16, B, H_q, H_kv, lengths)
    assert cache.n_quant.cpu().tolist() == [n_quant] * B and cache.n_res.cpu().tolist() == [n_res] * B
    q = tl.gen_q(16, B, H_q)
    out = cache.decode(tl.to_dev(q), max_context=n).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, [n_quant] * B, _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)


@pytest.mark.parametrize("B", [1, 2, 3, 5, 7, 32, 33, 47])
def test_batch_sizes_around_the_correction_width(kv, B):
    """The correction workgroups serve 4 sequences each: batches that do not fill the last one, small and large."""
    H_q, H_kv = 4, 1
    lengths = [300 + (131 * b) % 917 for b in range(B)]
    cache, K, V, Wq, Wk = _build(kv, 17, B, H_q, H_kv, lengths)
    q = tl.gen_q(17, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    tl.check_outputs(out, want)


@pytest.mark.parametrize("gq", [4, 7])
def test_unequal_lengths_take_unequal_splits(kv, gq):
    """A batch whose sequences differ 80-fold in length: the launch gives each a number of splits in proportion to its
    groups (here 1 to 10), down to a sequence without any quantized token; every row must still match."""
    import torch
    B, H_kv = 5, 2
    H_q = gq * H_kv
    lengths = [300, 2500, 5000, 57, 1290]
    cache, K, V, Wq, Wk = _build(kv, 18, B, H_q, H_kv, lengths)
    q = tl.gen_q(18, B, H_q)
    out = cache.decode(tl.to_dev(q))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0 and int(cache.split_done.abs().sum().item()) == 0
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    tl.check_outputs(out.cpu().numpy(), want)
    assert torch.equal(cache.decode(tl.to_dev(q)), out)  # same bits on a second call


def test_result_does_not_depend_on_the_launch_bound(kv):
    """max_context only sizes the launch: any upper bound gives the same result up to the summation order."""
    import torch
    B, H_q, H_kv = 1, 4, 1
    lengths = [2000]
    cache, K, V, Wq, Wk = _build(kv, 18, B, H_q, H_kv, lengths, capacity=16384)
    q = tl.gen_q(18, B, H_q)
    want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
    outs = []
    for bound in (2000, 2048, 5000, 0):  # 0 = the cache's capacity
        out = cache.decode(tl.to_dev(q), max_context=bound).cpu().numpy()
        tl.check_outputs(out, want)
        outs.append(out.astype(np.float64))
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() <= 2e-3
    assert int(cache.split_done.abs().sum().item()) == 0


def test_timed_entry_point_gives_the_same_bits(kv):
    """kvlinc_decode_attention_timed is kvlinc_decode_attention plus two events on the dispatch."""
    import ctypes
    import torch
    B, H_q, H_kv = 2, 8, 2
    lengths = [900, 1300]
    cache, K, V, Wq, Wk = _build(kv, 19, B, H_q, H_kv, lengths)
    q = tl.to_dev(tl.gen_q(19, B, H_q))
    plain = cache.decode(q).clone()
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    e0, e1 = ctypes.c_void_p(), ctypes.c_void_p()
    assert hip.hipEventCreate(ctypes.byref(e0)) == 0 and hip.hipEventCreate(ctypes.byref(e1)) == 0
    out = torch.empty_like(q)
    ws = cache.workspace(0)
    rc = kv.kvlinc_decode_attention_timed(cache, q, out, ws, e0.value, e1.value)
    assert rc == kv.KVLINC_OK
    torch.cuda.synchronize()
    ms = ctypes.c_float()
    assert hip.hipEventElapsedTime(ctypes.byref(ms), e0, e1) == 0
    assert 0.0 < ms.value < 50.0
    assert torch.equal(out, plain)
    hip.hipEventDestroy(e0)
    hip.hipEventDestroy(e1)


def _sliding_reference(K, V, q, lengths, n_quant, H_q, H_kv, Wq, Wk):
    want = {}
    gq = H_q // H_kv
    for b in range(len(lengths)):
        for g in range(H_kv):
            n = int(lengths[b])
            ref = tl.o_cache.build_cache(K[b, g, :n], V[b, g, :n], int(n_quant[b]), Wk=None if Wk is None else Wk[g])
            for h in range(g * gq, (g + 1) * gq):
                want[(b, h)] = tl.o_attn.decode(q[b, h], ref, None if Wq is None else Wq[h], value_window="sliding")
    return want


@pytest.mark.parametrize("gq", [4, 7])
@pytest.mark.parametrize("correction", [True, False])
def test_sliding_value_window(kv, gq, correction):
    """KVLINC_FLAG_SLIDING_VALUES (Sec. 4.1, setup): the values of the newest 128 tokens are the fp16 ones whatever the
    key window holds.  A bulk build (which has to store the newest group's values into the window) and one-token appends
    across a flush (which leave them there), decoded after every few appends, against the oracle's sliding mode; the
    records, states and window rows are those of the block mode."""
    import torch
    B, H_kv = 3, 2
    H_q = gq * H_kv
    pre = [517, 128 + 77, 60]      # key windows of 5, 77 and 60 tokens; the last sequence has nothing quantized
    extra = 140                    # every sequence crosses a flush
    lengths = [p + extra for p in pre]
    K, V = tl.gen_kv(36, B, H_kv, lengths)
    Wq, Wk = (synth.adapters_q(36, H_q), synth.adapters_k(36, H_kv)) if correction else (None, None)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=None if Wq is None else tl.to_dev(Wq), Wk=None if Wk is None else tl.to_dev(Wk),
                           flags=kv.KVLINC_FLAG_SLIDING_VALUES)
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :max(pre)].contiguous(), Vd[:, :, :max(pre)].contiguous(), n_new=tl.to_dev(np.asarray(pre, dtype=np.int32)))
    worst_gap = 0.0
    for s in range(extra + 1):
        cur = [p + s for p in pre]
        if s in (0, 1, 50, 67, 68, 69, 123, 124, 139, 140):
            q = tl.gen_q(36, B, H_q, step=s)
            out = cache.decode(tl.to_dev(q)).cpu().numpy().astype(np.float64)
            assert int(cache.status.item()) == 0
            n_quant, n_res = tl.check_counters(cache, cur)
            want = _sliding_reference(K, V, q, cur, n_quant, H_q, H_kv, Wq, Wk)
            tl.check_outputs(out, want)
            # the block mode's answer differs (so the comparison above tells the two apart)
            blockw = tl.oracle_decode(K, V, q, cur, n_quant, _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk)
            worst_gap = max(worst_gap, max(np.abs(want[k] - blockw[k]).max() for k in want))
        if s < extra:
            kn = torch.stack([Kd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            vn = torch.stack([Vd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            cache.append(kn, vn)
    assert worst_gap > 1e-3
    # records, states and window rows are what the block mode stores
    n_quant, n_res = tl.check_counters(cache, lengths)
    for b in range(B):
        for g in range(H_kv):
            tl.check_pair_against_oracle(cache, b, g, K[b, g, :lengths[b]], V[b, g, :lengths[b]], int(n_quant[b]), int(n_res[b]),
                                         None if Wk is None else Wk[g], check_states=correction)


def test_sliding_value_window_keeps_a_refused_append_out_of_the_live_value_slots(kv):
    """With the sliding window the value slots behind the key window are live.  A one-token append with a non-finite
    key in ONE kv head must leave them alone in ALL kv heads: the decode result after the refused append equals the one
    before it, bit for bit."""
    import torch
    B, H_q, H_kv = 2, 8, 4
    n0 = 128 + 40
    K, V = tl.gen_kv(37, B, H_kv, [n0 + 1] * B)
    cache = kv.KVLincCache(B, H_q, H_kv, 512, flags=kv.KVLINC_FLAG_SLIDING_VALUES)
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :n0].contiguous(), Vd[:, :, :n0].contiguous())
    q = tl.to_dev(tl.gen_q(37, B, H_q))
    before = cache.decode(q).clone()
    v_before = cache.v_res.clone()
    kn = Kd[:, :, n0:n0 + 1].clone()
    kn[1, 2, 0, 5] = float("inf")
    cache.append(kn, Vd[:, :, n0:n0 + 1].contiguous())
    torch.cuda.synchronize()
    assert int(cache.status.item()) & kv.KVLINC_ST_NONFINITE
    nr = cache.n_res.cpu().numpy()
    assert list(nr) == [41, 40]
    assert torch.equal(cache.v_res[1], v_before[1])
    cache.status.zero_()
    after = cache.decode(q)
    assert torch.equal(after[1], before[1])


@pytest.mark.parametrize("H_kv", [1, 2])
def test_long_prompt_build_in_chunks(kv, H_kv):
    """A bulk append of few sequences and many groups is shared out in chunks of groups over the chip (their shares of
    S and P meet by atomic additions): records and window bit-exact, states within the element-wise bounds, for a long
    sequence, and for a short one in the same call (whose single chunk keeps the state in registers); then the decode."""
    B, H_q = 2, 4 * H_kv
    lengths = [8192 + 77, 300]
    K, V = tl.gen_kv(38, B, H_kv, lengths)
    Wq, Wk = synth.adapters_q(38, H_q), synth.adapters_k(38, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 8192 + 512, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
    assert int(cache.status.item()) == 0
    n_quant, n_res = tl.check_counters(cache, lengths)
    for b in range(B):
        for g in range(H_kv):
            tl.check_pair_against_oracle(cache, b, g, K[b, g, :lengths[b]], V[b, g, :lengths[b]], int(n_quant[b]), int(n_res[b]), Wk[g])
    q = tl.gen_q(38, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy().astype(np.float64)
    tl.check_outputs(out, tl.oracle_decode(K, V, q, lengths, n_quant, _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk))
    # a second call on top (the chunks add to a state that is not zero): 8192 more tokens for sequence 0 only
    more = [8192, 0]
    K2, V2 = tl.gen_kv(39, B, H_kv, [8192, 8192])
    cache2 = kv.KVLincCache(B, H_q, H_kv, 2 * 8192 + 512, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache2.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
    cache2.append(tl.to_dev(K2), tl.to_dev(V2), n_new=tl.to_dev(np.asarray(more, dtype=np.int32)))
    assert int(cache2.status.item()) == 0
    total = [lengths[0] + 8192, lengths[1]]
    n_quant, n_res = tl.check_counters(cache2, total)
    for g in range(H_kv):
        Kall = np.concatenate([K[0, g, :lengths[0]], K2[0, g]]); Vall = np.concatenate([V[0, g, :lengths[0]], V2[0, g]])
        tl.check_pair_against_oracle(cache2, 0, g, Kall, Vall, int(n_quant[0]), int(n_res[0]), Wk[g])
        tl.check_pair_against_oracle(cache2, 1, g, K[1, g, :lengths[1]], V[1, g, :lengths[1]], int(n_quant[1]), int(n_res[1]), Wk[g])


@pytest.mark.parametrize("H_kv", [1, 2])
def test_long_prompt_build_in_chunks_refuses_as_a_whole(kv, H_kv):
    """A non-finite value in a late group of one kv head: no chunk of any head may have touched the states."""
    import torch
    B, H_q = 1, 4 * H_kv
    n0, n1 = 300, 8192
    K, V = tl.gen_kv(40, B, H_kv, [n0 + n1])
    Wq, Wk = synth.adapters_q(40, H_q), synth.adapters_k(40, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, n0 + n1 + 512, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :n0].contiguous(), Vd[:, :, :n0].contiguous())
    before = {nm: getattr(cache, nm).clone() for nm in ("S", "P", "S16", "n_quant", "n_res", "k_res", "v_res")}
    ng = int(cache.n_quant[0].item()) // 128
    rec_before = cache.groups[:, :, :ng].clone()
    vbad = Vd[:, :, n0:].clone()
    vbad[0, H_kv - 1, 7000, 3] = float("nan")
    cache.append(Kd[:, :, n0:].contiguous(), vbad)
    torch.cuda.synchronize()
    assert int(cache.status.item()) & kv.KVLINC_ST_NONFINITE
    for nm, t in before.items():
        assert torch.equal(getattr(cache, nm), t), nm
    assert torch.equal(cache.groups[:, :, :ng], rec_before)
    assert not cache.split_done.any()
    # and the same append without the fault goes through
    cache.status.zero_()
    cache.append(Kd[:, :, n0:].contiguous(), Vd[:, :, n0:].contiguous())
    assert int(cache.status.item()) == 0
    n_quant, n_res = tl.check_counters(cache, [n0 + n1])
    for g in range(H_kv):
        tl.check_pair_against_oracle(cache, 0, g, K[0, g], V[0, g], int(n_quant[0]), int(n_res[0]), Wk[g])


# ---- 4-bit codes (Eq. 1 at N = 4) ---------------------------------------------------------------------------------

@pytest.mark.parametrize("gq,H_kv,correction", [(4, 2, True), (4, 2, False), (8, 1, True), (1, 3, True), (7, 2, True)])
def test_four_bit_codes_bulk_and_decode(kv, gq, H_kv, correction):
    """A cache with 4-bit codes: records (two 2-bit planes per tile), window, states and counters bit for bit / within
    the state bounds against the oracle at bits = 4, and the decode output within the output tolerance; ragged lengths
    with a sequence below one group, an exact multiple and several groups per wave."""
    import torch
    B, H_q = 4, gq * H_kv
    lengths = [700, 128, 57, 2300]
    cache, K, V, Wq, Wk = _build(kv, 41, B, H_q, H_kv, lengths, correction=correction, bits=4)
    torch.cuda.synchronize()
    assert int(cache.status.item()) == 0 and cache.groups.shape[-1] == 4352
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(B, H_kv), Wk=Wk)
    q = tl.gen_q(41, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    n_quant = cache.n_quant.cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, n_quant, _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk, bits=4)
    tl.check_outputs(out, want)
    # the 2-bit answer on the same inputs differs by more than the tolerance, so the comparison tells the widths apart
    two = tl.oracle_decode(K, V, q, lengths, n_quant, [(0, 0)], H_q, H_kv, Wq, Wk, bits=2)
    assert max(np.abs(two[k] - want[k]).max() for k in two) > 2 * tl.OUT_MAX_ABS


def test_four_bit_codes_one_token_appends_cross_a_flush(kv):
    """One-token appends through a window flush with 4-bit codes, a partial tail group from a static window, and a
    refused append that leaves the sequence as it was."""
    import torch
    B, H_q, H_kv = 2, 8, 2
    start, steps = [250, 127], 140
    total = [s + steps for s in start]
    K, V = tl.gen_kv(42, B, H_kv, total)
    Wq, Wk = synth.adapters_q(42, H_q), synth.adapters_k(42, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), bits=4)
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :max(start)].contiguous(), Vd[:, :, :max(start)].contiguous(),
                 n_new=tl.to_dev(np.asarray(start, dtype=np.int32)))
    lengths = list(start)
    for step in range(steps):
        kn = torch.stack([Kd[b, :, lengths[b]:lengths[b] + 1] for b in range(B)]).contiguous()
        vn = torch.stack([Vd[b, :, lengths[b]:lengths[b] + 1] for b in range(B)]).contiguous()
        cache.append(kn, vn)
        lengths = [n + 1 for n in lengths]
        if step in (0, 5, 6, 7, 133, 134, steps - 1):
            tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(B, H_kv), Wk=Wk)
            q = tl.gen_q(42, B, H_q, step)
            out = cache.decode(tl.to_dev(q)).cpu().numpy()
            want = tl.oracle_decode(K, V, q, lengths, cache.n_quant.cpu().numpy(), _all_pairs(B, H_kv), H_q, H_kv, Wq, Wk, bits=4)
            tl.check_outputs(out, want)
    assert int(cache.status.item()) == 0
    # a non-finite key in one head: refused, nothing of the sequence changes
    before = [t.clone() for t in (cache.groups, cache.k_res, cache.v_res, cache.S, cache.P, cache.S16, cache.n_quant, cache.n_res)]
    kn = torch.zeros(B, H_kv, 1, 128, dtype=torch.float16, device="cuda")
    kn[1, 1, 0, 5] = float("inf")
    cache.append(kn, torch.zeros_like(kn), n_new=tl.to_dev(np.asarray([0, 1], dtype=np.int32)))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == kv.KVLINC_ST_NONFINITE
    nq, nr = cache.n_quant.cpu().tolist(), cache.n_res.cpu().tolist()
    for old, new in zip(before[4:], (cache.P, cache.S16, cache.n_quant, cache.n_res)):
        assert torch.equal(old, new)
    assert torch.equal(before[3], cache.S)
    for b in range(B):
        assert torch.equal(before[0][b, :, :nq[b] // 128], cache.groups[b, :, :nq[b] // 128])
        assert torch.equal(before[1][b, :, :nr[b]], cache.k_res[b, :, :nr[b]])


def test_four_bit_codes_static_window_and_sliding_values(kv):
    """4-bit codes with the static 32-token window of workload 1 (a partial tail group) and with the sliding value
    window."""
    c = synth.CONFIGS[1]
    lengths = [c["n"]]
    cache, K, V, Wq, Wk = _build(kv, 1, c["B"], c["H_q"], c["H_kv"], lengths, R=c["R"], keep=c["keep"], capacity=1024, bits=4)
    assert cache.n_quant.cpu().tolist() == [992] and cache.n_res.cpu().tolist() == [32]
    tl.check_cache_against_oracle(cache, K, V, lengths, _all_pairs(1, 8), Wk=Wk, keep=32)
    q = tl.gen_q(1, 1, 32)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = tl.oracle_decode(K, V, q, lengths, [992], _all_pairs(1, 8), 32, 8, Wq, Wk, bits=4)
    tl.check_outputs(out, want)
    # sliding value window: bulk build, then appends; the newest group's last tokens take their values from the window
    import torch
    B, H_q, H_kv = 2, 8, 2
    pre, extra = [517, 205], 30
    lengths = [p + extra for p in pre]
    K, V = tl.gen_kv(43, B, H_kv, lengths)
    Wq, Wk = synth.adapters_q(43, H_q), synth.adapters_k(43, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), flags=kv.KVLINC_FLAG_SLIDING_VALUES, bits=4)
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :max(pre)].contiguous(), Vd[:, :, :max(pre)].contiguous(), n_new=tl.to_dev(np.asarray(pre, dtype=np.int32)))
    for s in range(extra + 1):
        cur = [p + s for p in pre]
        if s in (0, 1, 29, 30):
            q = tl.gen_q(43, B, H_q, step=s)
            out = cache.decode(tl.to_dev(q)).cpu().numpy().astype(np.float64)
            n_quant, n_res = tl.check_counters(cache, cur)
            want = {}
            for b in range(B):
                for g in range(H_kv):
                    ref = tl.o_cache.build_cache(K[b, g, :cur[b]], V[b, g, :cur[b]], int(n_quant[b]), Wk=Wk[g], bits=4)
                    for h in range(4 * g, 4 * g + 4):
                        want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h], value_window="sliding")
            tl.check_outputs(out, want)
        if s < extra:
            kn = torch.stack([Kd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            vn = torch.stack([Vd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            cache.append(kn, vn)
    assert int(cache.status.item()) == 0


def test_a_step_replayed_from_a_hip_graph(kv):
    """One step -- kvlinc_append_quantize (one token) + kvlinc_decode_attention_noalloc -- captured into a HIP graph and
    replayed 140 times across a window flush, with the program's own eager copies and synchronisations between the
    replays; every replay gives the bits of an eager twin cache that takes the same tokens through the workspace entry
    point.  (The library records kernels only: no memset nodes, no allocation.)"""
    import torch
    B, H_q, H_kv = 3, 8, 2
    pre = [300, 127, 64]
    steps = 140
    total = [p + steps for p in pre]
    K, V = tl.gen_kv(51, B, H_kv, total)
    Wq, Wk = tl.to_dev(synth.adapters_q(51, H_q)), tl.to_dev(synth.adapters_k(51, H_kv))
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    n0 = tl.to_dev(np.asarray(pre, dtype=np.int32))
    caches = [kv.KVLincCache(B, H_q, H_kv, 1024, Wq=Wq, Wk=Wk) for _ in range(2)]
    for c in caches:
        c.append(Kd[:, :, :max(pre)].contiguous(), Vd[:, :, :max(pre)].contiguous(), n_new=n0)
    graphed, eager = caches
    k_in = torch.zeros(B, H_kv, 1, 128, dtype=torch.float16, device="cuda")
    v_in = torch.zeros_like(k_in)
    q_in = torch.zeros(B, H_q, 128, dtype=torch.float16, device="cuda")
    out_g = torch.zeros_like(q_in)
    # the static buffer's address is looked up on the first call on a device: not inside a capture
    assert kv.kvlinc_decode_attention_noalloc(graphed, q_in, out_g, max_context=1024) == kv.KVLINC_OK
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            assert kv.kvlinc_append_quantize(graphed, k_in, v_in, stream=side) == kv.KVLINC_OK
            assert kv.kvlinc_decode_attention_noalloc(graphed, q_in, out_g, max_context=1024, stream=side) == kv.KVLINC_OK
    torch.cuda.synchronize()
    # the capture itself ran nothing: the caches still agree
    assert torch.equal(graphed.n_res, eager.n_res) and torch.equal(graphed.n_quant, eager.n_quant)
    q_all = tl.to_dev(np.stack([tl.gen_q(51, B, H_q, step=s) for s in range(steps)]))
    for s in range(steps):
        kn = torch.stack([Kd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
        vn = torch.stack([Vd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
        k_in.copy_(kn); v_in.copy_(vn); q_in.copy_(q_all[s])
        torch.cuda.synchronize()
        g.replay()
        eager.append(kn, vn)
        want = eager.decode(q_all[s], max_context=1024)
        torch.cuda.synchronize()
        assert torch.equal(out_g, want), s
    assert int(graphed.status.item()) == 0 and int(graphed.split_done.abs().sum().item()) == 0
    for name in ("groups", "k_res", "n_quant", "n_res", "S", "P", "S16"):
        assert torch.equal(getattr(graphed, name), getattr(eager, name)), name
    lengths = [p + steps for p in pre]
    want = tl.oracle_decode(K, V, q_all[steps - 1].cpu().numpy(), lengths, graphed.n_quant.cpu().numpy(), [(0, 1), (2, 0)], H_q, H_kv,
                            synth.adapters_q(51, H_q), synth.adapters_k(51, H_kv))
    tl.check_outputs(out_g.cpu().numpy(), want)


@pytest.mark.parametrize("bits", [2, 4])
def test_all_variants_together(kv, bits):
    """State stored in 16 bits only, the literal last lines of Alg. 1 and the sliding value window in one cache, at both
    code widths: a bulk build, then one-token appends across a flush, decoded against the oracle with all three switches
    (the variants are separate descriptor fields and kernel instantiations; this is the case where they all meet)."""
    import torch
    B, H_q, H_kv = 2, 8, 2
    pre, extra = [390, 140], 140
    lengths = [p + extra for p in pre]
    K, V = tl.gen_kv(61, B, H_kv, lengths)
    Wq, Wk = synth.adapters_q(61, H_q), synth.adapters_k(61, H_kv)
    flags = kv.KVLINC_FLAG_ALG1_LITERAL | kv.KVLINC_FLAG_SLIDING_VALUES
    cache = kv.KVLincCache(B, H_q, H_kv, 1024, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk), state_storage="fp16", flags=flags, bits=bits)
    Kd, Vd = tl.to_dev(K), tl.to_dev(V)
    cache.append(Kd[:, :, :max(pre)].contiguous(), Vd[:, :, :max(pre)].contiguous(), n_new=tl.to_dev(np.asarray(pre, dtype=np.int32)))
    gq = H_q // H_kv
    for s in range(extra + 1):
        cur = [p + s for p in pre]
        if s in (0, 3, 119, 120, 140):
            q = tl.gen_q(61, B, H_q, step=s)
            out = cache.decode(tl.to_dev(q)).cpu().numpy()
            assert int(cache.status.item()) == 0
            n_quant, n_res = tl.check_counters(cache, cur)
            want = {}
            for b in range(B):
                first = tl.o_cache.window_split(pre[b])[0]
                points = list(range(first, int(n_quant[b]) + 1, 128))  # the state was rounded after the build and every flush
                for g in range(H_kv):
                    ref = tl.o_cache.build_cache(K[b, g, :cur[b]], V[b, g, :cur[b]], int(n_quant[b]), Wk=Wk[g], bits=bits,
                                                 state_rounding=points)
                    for h in range(g * gq, (g + 1) * gq):
                        want[(b, h)] = tl.o_attn.decode(q[b, h], ref, Wq[h], literal_alg1=True, value_window="sliding")
            tl.check_outputs(out, want)
        if s < extra:
            kn = torch.stack([Kd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            vn = torch.stack([Vd[b, :, pre[b] + s] for b in range(B)]).unsqueeze(2).contiguous()
            cache.append(kn, vn)
    n_quant, n_res = tl.check_counters(cache, lengths)
    for b in range(B):
        for g in range(H_kv):
            tl.check_pair_against_oracle(cache, b, g, K[b, g, :lengths[b]], V[b, g, :lengths[b]], int(n_quant[b]), int(n_res[b]), None)


@pytest.mark.parametrize("bits,sliding,correction", [(4, True, True), (2, True, False), (4, False, False)])
def test_long_prompt_build_in_chunks_variants(kv, bits, sliding, correction):
    """The chunked build of a long prompt (groups shared out over the chip) at 4-bit codes, with the sliding value window
    (the last arrival stores the newest group's fp16 values) and for a cache without correction states."""
    B, H_q, H_kv = 2, 8, 2
    lengths = [8192 + 513, 8192 - 31]
    K, V = tl.gen_kv(62, B, H_kv, lengths)
    Wq, Wk = (synth.adapters_q(62, H_q), synth.adapters_k(62, H_kv)) if correction else (None, None)
    cache = kv.KVLincCache(B, H_q, H_kv, 8192 + 1024, Wq=None if Wq is None else tl.to_dev(Wq), Wk=None if Wk is None else tl.to_dev(Wk),
                           bits=bits, flags=kv.KVLINC_FLAG_SLIDING_VALUES if sliding else 0)
    cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
    assert int(cache.status.item()) == 0
    n_quant, n_res = tl.check_counters(cache, lengths)
    q = tl.gen_q(62, B, H_q)
    out = cache.decode(tl.to_dev(q)).cpu().numpy()
    want = {}
    for b in range(B):
        for g in range(H_kv):
            ref = tl.check_pair_against_oracle(cache, b, g, K[b, g, :lengths[b]], V[b, g, :lengths[b]], int(n_quant[b]), int(n_res[b]),
                                               None if Wk is None else Wk[g])
            for h in range(4 * g, 4 * g + 4):
                want[(b, h)] = tl.o_attn.decode(q[b, h], ref, None if Wq is None else Wq[h], value_window="sliding" if sliding else "block")
    tl.check_outputs(out, want)
    assert int(cache.split_done.abs().sum().item()) == 0


@pytest.mark.parametrize("H_kv", [1, 2])
def test_sliding_value_window_refuses_a_bulk_append_before_any_row_is_stored(kv, H_kv):
    """Sliding value window, a bulk append that flushes nothing, a non-finite value in its 6th row: not even the five
    rows ahead of it may be stored, because the value slots behind the key window hold the newest group's fp16 values
    (with one kv head no other head's workgroup could have warned: every bulk append to such a cache is scanned first)."""
    import torch
    B, H_q = 2, 4 * H_kv
    lengths = [512 + 92, 300]
    cache, K, V, Wq, Wk = _build(kv, 63, B, H_q, H_kv, lengths, flags=kv.KVLINC_FLAG_SLIDING_VALUES)
    q = tl.to_dev(tl.gen_q(63, B, H_q))
    before_out = cache.decode(q).clone()
    before = {nm: getattr(cache, nm).clone() for nm in ("v_res", "n_quant", "n_res", "S", "P", "S16")}
    rng = np.random.default_rng(9)
    kn = rng.standard_normal((B, H_kv, 18, 128)).astype(np.float16)
    vn = rng.standard_normal((B, H_kv, 18, 128)).astype(np.float16)
    vn[0, H_kv - 1, 5, 77] = np.float16("nan")
    cache.append(tl.to_dev(kn), tl.to_dev(vn), n_new=tl.to_dev(np.asarray([18, 0], dtype=np.int32)))
    torch.cuda.synchronize()
    assert int(cache.status.item()) == kv.KVLINC_ST_NONFINITE
    for nm, t in before.items():
        assert torch.equal(getattr(cache, nm), t), nm  # (all of v_res: live slots and window rows alike)
    assert torch.equal(cache.decode(q), before_out)
    assert not cache.split_done.any()
