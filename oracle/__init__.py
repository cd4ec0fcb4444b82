"""CPU oracle for the AdaHOP per-GEMM path -- TEST INFRASTRUCTURE ONLY.

Importable from tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg; the product
package never imports it and shares no code with it.
"""
