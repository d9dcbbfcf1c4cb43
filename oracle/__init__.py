"""CPU oracle for the TEAM MoE-layer hot path.  TEST INFRASTRUCTURE ONLY.

Imported by tests/, by ``__graft_entry__.smoke()`` and by the CPU-baseline leg of ``bench.py``; the product
package never imports it.  ``c_oracle`` wraps the plain-C definition (double accumulators), ``moe_numpy`` is a
second, independently written NumPy fp64 implementation used to cross-check the first.
"""
