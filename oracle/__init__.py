"""CPU oracle of the DynSplit-KV hot path: test infrastructure, never a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package; the HIP library and its Python binding never do.
"""
