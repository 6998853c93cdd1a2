"""CPU oracle for the Ulysses-shard hot path.  TEST INFRASTRUCTURE ONLY.

Plain fp64 definitions of the sequence<->head re-layout and of causal
grouped-query softmax attention (forward and backward), written from the
paper's statement of the problem (Section 2, Figure 1; Section 3.1
challenges 1-3) and the textbook operator its attention nodes denote.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package.  It shares no code with the HIP path and never calls it.
"""
