"""zkmi: the tlookup / sumcheck prover hot path of zkLLM on one AMD MI355X.

The work is done by ``libzkmi.so`` (hand-written HIP for gfx950, built in-tree by
``paper_2404_16109_amd.build``); this package is argument marshalling only.
PyTorch is used to own device memory and to name the stream.  There is no CPU
fallback: if the library is missing, importing the binding raises.
"""
from .binding import *  # noqa: F401,F403
