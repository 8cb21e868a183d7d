"""CPU oracle for ActorQ int8 policy inference.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It never imports the HIP library or its Python binding.
"""
from .policy import OraclePolicy, lib, c_qparams_asym, c_quantize_asym, c_quantize_sym_rows  # noqa: F401
