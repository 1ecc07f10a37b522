"""MI355X-native Float8 linear layer (forward + backward).

`f8` is the thin ctypes binding over the C-ABI library built from csrc/;
`workloads` names the Llama-3.1-shaped synthetic inputs.  The binding loads
the library on first use and raises if it has not been built.
"""
from . import workloads  # noqa: F401
