"""CPU oracle for the ExpertWeave MoE-layer hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct statement of what the path computes, written from
the paper (arxiv 2508.17624): Sec. 2.1 (router top-k, dispatch, grouped expert
computation, combine), Sec. 4.1 (ESFT expert map and the rerouted top-k set),
Sec. 4.2 (virtual weight tensor, page pool, sub-page sharing) and Sec. 3.1
(adapter sparsity and memory fragmentation factors).

It shares no code with the HIP path and imports nothing from it.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import it; the product path
never does.

    oracle.moe    numpy, fp64: every stage and every intermediate of one MoE layer
    oracle.brute  pure-Python loops over tokens/experts, fp64: pins oracle.moe on tiny inputs
    oracle.pool   page accounting of the virtual weight tensor, S_i and F_mem

Parity status: every function is pinned by tests marked "not gpu" (brute force,
closed forms, invariants, library special cases, figures and tables quoted in the
paper's text); none is "parity unpinned".
"""
