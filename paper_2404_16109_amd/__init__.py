"""zkmi: the tlookup / sumcheck prover hot path of zkLLM on one AMD MI355X.

The work is done by ``libzkmi.so`` (hand-written HIP for gfx950, built in-tree by
``paper_2404_16109_amd.build``); this package is argument marshalling only.
PyTorch is used to own device memory and to name the stream.  There is no CPU
fallback: the first use of any entry point loads the library and raises if it
has not been built.  (``paper_2404_16109_amd.build`` and ``.synth`` can be
imported without it.)
"""
import importlib


def __getattr__(name):
    if name.startswith("__"):
        raise AttributeError(name)
    if name in ("build", "synth", "binding"):
        return importlib.import_module("." + name, __name__)
    binding = importlib.import_module(".binding", __name__)
    return getattr(binding, name)
