"""Reference ("oracle") implementation of the KVLinC 2-bit decode path, NumPy on the CPU.

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is slow, plain and written to be checked against the
paper by eye.  Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
it; the product (the HIP library and its Python binding) never does, and the two share no code.

What each module follows:

* ``hadamard``   -- the orthogonal Hadamard rotation applied to values (Sec. 3.1, Obs. 3).
* ``quantizer``  -- asymmetric N-bit min/max quantization, group-wise, Q_C / Q_T (Sec. 2, Eq. 1).
* ``kvcache``    -- K_q = Q_C(K), V_q = Q_T(V H), the fp16 window of recent tokens (Sec. 4.1 setup),
                    and the correction states S_n, P_n (Sec. 3.2, Eq. 5).
* ``attention``  -- corrected single-query attention (Eq. 3, Eq. 4, Eq. 5, Eq. 6) and the
                    block-parallel decode with its merge (Sec. 3.3, Alg. 1).
* ``layout``     -- the physical order of the packed cache: 9216-byte group records (two 4 KB tiles of
                    2-bit codes plus scales and zero-points) and the window's value order (an encoding
                    of ours; the paper only fixes "16 codes per 32-bit word", Sec. 3.3).
* ``accounting`` -- average bits per cached element (Table 1, "KV Cache" column).

Arithmetic is fp64 except where a floating-point value decides an integer or a stored 16-bit
pattern (quantization codes, stored scale / zero-point, the rotated fp16 value); there the
``spec32`` routines take the decision in binary32 with a fixed operation order, which is the
contract the GPU kernels are held to bit for bit.  Every such routine has an ``exact`` (fp64)
twin so the distance between the two can be measured.

Parity pins (tests/test_oracle_*.py): Eq. 1 round-trip bound and level range, Eq. 2 error law,
H H^T = d I and FWHT == dense product, bits -> 16 convergence to textbook softmax attention,
rotation invariance, split/merge invariance (Alg. 1), zero-state and zero-weight closed forms,
Eq. 4 == Eq. 5, the printed 2.46 / 2.71 average-bit figures, a hand-computed tiny case in exact
rational arithmetic.  Unpinned: anything that needs trained adapters, model weights or the
paper's datasets (accuracy tables, the end-to-end speed-up) -- "parity unpinned".
"""
