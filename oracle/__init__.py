"""CPU oracle of the W4A16 skinny GEMM: test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares no code with paper_2402_00025_amd and never imports it.
"""
