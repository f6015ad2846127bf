"""CPU oracle for the HISA / RNS-CKKS hot path.  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the cpu_baseline leg of bench.py may import
this package.  It shares no code with paper_1810_00845_amd.
"""
from .ckks import Ct, Oracle, OracleError, Pt, build, lib, round_half_away  # noqa: F401
