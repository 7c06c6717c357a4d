"""CPU oracle for the TSM hot path: TEST INFRASTRUCTURE ONLY.

Plain float64 numpy plus one C file of direct-summation convolutions, written
from the paper's description of the operator and network.  Only the tests, the
smoke check and the benchmark's CPU-baseline leg may import it; it shares no
code with the HIP library and the product path never calls it."""
