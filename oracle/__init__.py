"""Float64 CPU oracle for Einsum Networks (arxiv 2004.06231).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, obviously-correct
NumPy implementation of what the HIP library computes.  It exists so that the
GPU results can be checked against something written directly from the paper.
Only the test-suite, the smoke check and the CPU-baseline leg of the benchmark
may import it; the product package never does, and this package never imports
the product package or loads its shared library.

Modules
-------
structure : region graphs (random binary trees, Poon-Domingos), replica
            assignment, topological layers (Algorithm 1), parameter layout.
einet     : forward pass (Sec. 3.2-3.4, Eq. 3, App. B), EM statistics (Eq. 6)
            and M-step (Eq. 7-9), all in float64.
train     : the stochastic-EM loop over mini-batches (Eq. 8-9, Sec. 4.2) and the
            mixture of several EiNets (Sec. 4.2).
init      : the counter-based random initialisation of the parameters.
sampling  : top-down sampling, unconditional and given evidence, with leaf samples
            or leaf means (Sec. 2, Sec. 4.2, App. D).
"""
