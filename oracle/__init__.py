"""CPU oracle for the mixed action+decode attention step over a shared prefix KV.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
directory; only the tests, the smoke check and the benchmark's CPU-baseline leg
do.  The oracle shares no code with the HIP path: it holds every stream's keys
and values as plain un-paged lists and recomputes attention from the textbook
definition in float64.

Modules
-------
attention   float64 attention over the visible set of each query (numpy).
brute       the same definition in pure-Python loops, for tiny cases.
pool_model  the indexing oracle: free stack, refcounts, block tables, slots.
replay      runs an operation trace through pool_model + attention.
schedule    the per-frame execution flow (Alg. 1) under arbitrary arrivals, and the
            ablation variants, as a plain simulation.

Parity status: every function here is pinned by the non-GPU tests (brute force,
closed forms, a library attention routine, the paper's shared == isolated
invariant, and its worked scheduling example).  Token buffers, EOS and sampling
of the language expert are out of scope and therefore "parity unpinned".
"""
