"""CPU oracle for the retrieve -> verify -> accept -> commit step.  TEST INFRASTRUCTURE ONLY.

Plain, slow, written from the paper's definitions (Sec. 2.1 Eq. 1-4, Sec. 3.2-3.4 Eq. 5-8) in
float64 numpy.  It shares no code with the HIP library and must never be imported by the
product package: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.

Pin status (checked by `pytest -m "not gpu"`):
    retrieval.retrieve      pinned: explicit-trie brute force, hand-worked pools, special cases
    decoder.verify_forward  pinned: torch CPU reference ops, cache/no-cache/sequential
                            consistency, closed forms (zero weights, RoPE properties)
    acceptance.*            pinned: full-sort brute force, closed forms, strict == greedy
No value printed in the paper can pin absolute outputs (it prints none for this path).
"""
