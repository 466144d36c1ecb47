"""CPU oracle for the bidirectional KV-cache production path.

THIS PACKAGE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 NumPy
statement of what the hot path computes, written from the paper, and shares no
code with the HIP library.  Only ``tests/``, ``__graft_entry__.smoke()`` and
the ``cpu_baseline`` leg of ``bench.py`` may import it.  The product path never
routes through it.

Modules
-------
transformer   the KV cache of a decoder prompt (Sec. 3 "Attention and KV cache",
              "Chunk Prefill"): monolithic, chunked and token-by-token prefill.
meet_point    TTFT of a split, brute-force optimal meet point, the greedy race
              of Alg. 1, and a discrete-event replay of the claim protocol.
store         packing of a KV cache into the page images the storage tier holds.

Parity status: the arithmetic of every function here is pinned by
``tests/test_oracle_*.py`` (hand-worked values, closed forms, invariants,
brute force).  The absolute KV values of a *random* model have no printed
reference in the paper; they are pinned through three structurally different
prefill routines agreeing, plus hand-worked one- and two-token models.
"""
