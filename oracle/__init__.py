"""CPU oracle of the spatial-temporal serving step (arXiv 2504.19516).

TEST INFRASTRUCTURE ONLY. Plain, slow, obviously-correct implementations of what the
HIP path computes: the transformer step over a paged KV cache (`transformer`), the
SM-scaling roofline latency model (`latency`) and the SLO-aware scheduler replay
(`scheduler`). Only tests, the smoke check and the benchmark's CPU-baseline leg may
import this package; the product path never does and shares no code with it.
"""
