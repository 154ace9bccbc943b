"""Persistent sparse recurrent step for AMD MI355X: Python binding of libsprnn.so.

``binding`` marshals arguments into the C ABI declared in ``include/sprnn.h``; ``workloads`` draws the
seeded synthetic inputs; ``build`` compiles the HIP library in-tree.  Nothing here computes the
recurrent step on the CPU.
"""
from .binding import SparseRNN, SprnnError, pack_host, load_library, status_string  # noqa: F401
