"""Float64 CPU oracle for the SwitchHead attention layer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library, its Python
binding) imports or calls this package; only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may.  The oracle shares no code with the HIP path.
"""
