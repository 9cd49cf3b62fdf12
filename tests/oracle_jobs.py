"""Oracle references for many (sequence, KV head) pairs at the full workload sizes, computed by a few worker processes.

A job names a seeded pair -- (config, sequence, KV head, tokens, quantized tokens, query step) -- and the worker
regenerates its inputs from kvlinc_synth, builds the oracle's cache and decodes the pair's query heads.  Nothing here
imports torch or touches the GPU: the workers are fresh interpreters started as child processes by the test process.

What comes back per job: SHA-1 digests of the packed group records and of the window rows (the bit-exact fields; on a
mismatch the test recomputes that one pair in-process for a field-by-field report), the correction states S, P (fp64)
and the outputs y [G_q, 128] (fp64).
"""
import hashlib
import json
import os
import subprocess
import sys
import tempfile

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sha(a):
    return hashlib.sha1(np.ascontiguousarray(a).tobytes()).hexdigest()


def run_job(job):
    """job: dict(cfg, b, g, n, nq, H_q, H_kv, step, R[, bits]) -> dict of references (see the module docstring)."""
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    import kvlinc_synth as synth
    from oracle import attention as o_attn
    from oracle import kvcache as o_cache
    from oracle import layout as o_layout
    cfg, b, g, n, nq = job["cfg"], job["b"], job["g"], job["n"], job["nq"]
    H_q, H_kv = job["H_q"], job["H_kv"]
    gq = H_q // H_kv
    K, V = synth.keys(cfg, b, g, n), synth.values(cfg, b, g, n)
    Wk, Wq = synth.adapters_k(cfg, H_kv)[g], synth.adapters_q(cfg, H_q)
    q = synth.queries(cfg, b, H_q, job["step"])
    bits = job.get("bits", 2)
    ref = o_cache.build_cache(K, V, nq, Wk=Wk, bits=bits)
    rec = (o_layout.pack_records if bits == 2 else o_layout.pack_records4)(ref["k_codes"], ref["v_codes"], ref["k_scale"], ref["k_zero"], ref["v_scale"], ref["v_zero"])
    y = np.stack([o_attn.decode(q[h], ref, Wq[h]) for h in range(g * gq, (g + 1) * gq)])
    return dict(rec_sha=sha(rec), kres_sha=sha(ref["k_res"].view(np.uint16)),
                vres_sha=sha(ref["v_res"].view(np.uint16)),  # the live window rows [n_res, 128], oldest first
                S=ref["S"], P=ref["P"], y=y)


def _worker_main(argv):
    jobs = json.load(open(argv[1]))
    out = {}
    for i, job in enumerate(jobs):
        r = run_job(job)
        for k, v in r.items():
            out["%d/%s" % (job["id"], k)] = np.asarray(v)
        print("[oracle worker %s] job %d/%d done (config %d, sequence %d, head %d, %d tokens)"
              % (argv[3], i + 1, len(jobs), job["cfg"], job["b"], job["g"], job["n"]), flush=True)
    np.savez(argv[2], **out)


def run_jobs_parallel(jobs, workers=None):
    """Runs the jobs on `workers` child processes (plain interpreters, no GPU); returns [result dict] in job order.
    Progress lines of the workers go to this process's stdout."""
    if workers is None:
        workers = max(1, min(8, (os.cpu_count() or 2) - 1, len(jobs)))
    jobs = [dict(j, id=i) for i, j in enumerate(jobs)]
    # longest jobs first, dealt round-robin, so that the workers end together
    order = sorted(jobs, key=lambda j: -j["n"])
    shares = [order[w::workers] for w in range(workers)]
    tmp = tempfile.mkdtemp(prefix="kvlinc_oracle_")
    procs = []
    env = dict(os.environ, OMP_NUM_THREADS="2", OPENBLAS_NUM_THREADS="2", MKL_NUM_THREADS="2")
    for w, share in enumerate(shares):
        if not share:
            continue
        jf, of = os.path.join(tmp, "jobs%d.json" % w), os.path.join(tmp, "out%d.npz" % w)
        json.dump(share, open(jf, "w"))
        procs.append((subprocess.Popen([sys.executable, "-u", os.path.abspath(__file__), jf, of, str(w)], env=env), of))
    results = [None] * len(jobs)
    for p, of in procs:
        rc = p.wait()
        assert rc == 0, "oracle worker failed with exit code %d" % rc
        data = np.load(of)
        for key in data.files:
            i, name = key.split("/")
            i = int(i)
            if results[i] is None:
                results[i] = {}
            v = data[key]
            results[i][name] = str(v) if v.dtype.kind == "U" else v
        os.remove(of)
    assert all(r is not None for r in results)
    return results


if __name__ == "__main__":
    _worker_main(sys.argv)
