"""CPU oracle for the speculative-decoding step (test infrastructure, NOT a product code path).

Plain, slow, float64 numpy (plus one small C file for the acceptance rules) written from the
paper's statement of the step: a single-layer drafter expands a token tree, the target model
verifies all tree tokens in one forward pass, the longest drafted prefix that the target agrees
with is accepted together with one token of the target's own, and the accepted path's keys and
values are kept in the cache (Section 2.2 "Mechanism of Speculative Decoding", Section 4.1
"Model Architecture", Section 5.1 "Tree-based Drafting").

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.  It
shares no code with the HIP library and never receives values computed by it.

Parity status of each function is stated in its module header; anything marked
"parity unpinned" has no check other than itself.
"""
