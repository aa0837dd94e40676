"""DropMatch MC-dropout LM-head verification for MI355X (gfx950).

`paper_2603_03333_amd.binding` is the ctypes binding of the C-ABI library
(libdropmatch.so, built from csrc/ by `paper_2603_03333_amd.build`);
`paper_2603_03333_amd.workloads` holds seeded synthetic inputs.  Nothing is loaded at
import time; the library loads on the first call into the binding.
"""
__all__ = ["binding", "build", "workloads"]
