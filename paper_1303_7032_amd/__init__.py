"""MI355X (gfx950) library for batched retrieval in the Gripon-Berrou clustered associative
memory: clique storage into a bit-packed adjacency, sum-of-sum, sum-of-max and the hybrid
rule, iterated to a fixed point.  `binding` wraps the C ABI of include/gbnn.h; `inputs`
draws the seeded synthetic workloads; `build` compiles the HIP library in-tree."""
