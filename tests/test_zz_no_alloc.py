"""The allocation-free decode entry point (kvlinc_decode_attention_noalloc) gives the bits of kvlinc_decode_attention: two
calls in a row through the C ABI, the second on a smaller input, each compared with the workspace entry point on the
same cache; and a launch that needs more than the static buffer is refused before anything is enqueued."""
import ctypes

import numpy as np
import pytest

import kvlinc_synth as synth
from tests import kvlinc_testlib as tl

pytestmark = pytest.mark.gpu


def _case(kv, cfg, B, H_q, H_kv, lengths):
    import torch
    K, V = tl.gen_kv(cfg, B, H_kv, lengths)
    Wq, Wk = synth.adapters_q(cfg, H_q), synth.adapters_k(cfg, H_kv)
    cache = kv.KVLincCache(B, H_q, H_kv, max(lengths) + 256, Wq=tl.to_dev(Wq), Wk=tl.to_dev(Wk))
    cache.append(tl.to_dev(K), tl.to_dev(V), n_new=tl.to_dev(np.asarray(lengths, dtype=np.int32)))
    q = tl.to_dev(tl.gen_q(cfg, B, H_q))
    want = cache.decode(q, max_context=max(lengths)).clone()
    torch.cuda.synchronize()
    return cache, q, want, (K, V, Wq, Wk)


def test_noalloc_entry_point_matches_the_workspace_entry_point():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2510_05373_amd as kv
    big = _case(kv, 41, 6, 16, 4, [5000, 3000, 4097, 129, 2500, 4800])
    small = _case(kv, 42, 2, 8, 2, [700, 300])
    for cache, q, want, _ in (big, small):  # the second call reuses the buffer the first one left dirty
        need = kv.kvlinc_decode_workspace_bytes(cache, int((cache.n_quant + cache.n_res).max().item()))
        assert 0 < need <= kv.KVLINC_STATIC_SCRATCH_BYTES
        out = torch.full_like(q, float("nan"))
        rc = kv.kvlinc_decode_attention_noalloc(cache, q, out, max_context=int((cache.n_quant + cache.n_res).max().item()))
        assert rc == kv.KVLINC_OK, kv.kvlinc_strerror(rc)
        torch.cuda.synchronize()
        assert torch.equal(out, want)
        assert int(cache.split_done.abs().sum().item()) == 0 and int(cache.status.item()) == 0
    # and against the oracle, so that "equal" is not "equally wrong"
    cache, q, want, (K, V, Wq, Wk) = small
    ref = tl.oracle_decode(K, V, q.cpu().numpy(), [700, 300], cache.n_quant.cpu().numpy(), [(0, 0), (1, 1)], 8, 2, Wq, Wk)
    out = torch.empty_like(q)
    assert kv.kvlinc_decode_attention_noalloc(cache, q, out, max_context=700) == kv.KVLINC_OK
    tl.check_outputs(out.cpu().numpy(), ref)
    # a launch beyond the static buffer is refused on the host: nothing is enqueued, `out` keeps its contents
    wide = kv.KVLincCache(256, 32, 8, 4096)
    qw = torch.zeros(256, 32, 128, dtype=torch.float16, device="cuda")
    ow = torch.full_like(qw, 7.0)
    assert kv.kvlinc_decode_workspace_bytes(wide, 4096) > kv.KVLINC_STATIC_SCRATCH_BYTES
    assert kv.kvlinc_decode_attention_noalloc(wide, qw, ow, max_context=4096) == kv.KVLINC_ESCRATCH
    torch.cuda.synchronize()
    assert bool((ow == 7.0).all())
    assert "scratch" in kv.kvlinc_strerror(kv.KVLINC_ESCRATCH)
