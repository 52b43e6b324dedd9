"""CPU oracle for the BiLD decoding path: test infrastructure, not product.

Plain float64 numpy written from the paper's definitions.  Only the tests, the
smoke check and the benchmark's CPU-baseline leg import it; the HIP library
and its Python binding never do, and the two share no code.

Parity status: the policies, the softmax statistics, the cached/T-row
equivalence, every layer primitive and the limiting cases of Algorithm 1 are
pinned by tests that run without a GPU.  The token values produced on the
benchmark configurations themselves are PARITY UNPINNED beyond those checks:
the paper prints no worked trace, so the oracle is the sole authority there.
"""
from . import bild, model, policy, sampling
from .bild import Request, Result, Stats, bild_generate, greedy
from .model import DecoderCache, Model
from .sampling import Sampler
