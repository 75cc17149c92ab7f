"""CPU oracle of the DAS batched verification step -- TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this.  Only tests, the smoke check and
the bench's cpu_baseline leg may.
"""
from .model import (build, OracleModel, OracleSeq, greedy_accept, stochastic_accept,
                    softmax_weights, inverse_cdf, num_threads)
from .pagetable import PageTableMirror
