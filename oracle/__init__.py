"""CPU oracle for the garbled-circuit hot path -- TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares no code with the GPU library and never imports it.

  oracle.dash_oracle.c : the garbler / evaluator (plain C, one gate at a time)
  oracle.capi          : ctypes wrapper around it (marshalling only)
  oracle.plain         : plain integer definitions of what the circuits compute
"""
from .capi import Oracle, build, lib  # noqa: F401
