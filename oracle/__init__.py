"""CPU oracle of the fused GEMM + ring reduce-scatter path.  Test infrastructure only."""
