"""CPU oracle of the tile-centric mixed-precision GEMM.  Test infrastructure only."""
