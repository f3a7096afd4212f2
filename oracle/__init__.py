"""fp64 CPU oracle for the sketched linear layer (SKLinear).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this
package: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg
do.  It shares no code with the HIP library and never calls it.
"""
