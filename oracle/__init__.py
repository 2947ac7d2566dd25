"""CPU oracle for the STree tree-masked SSD pass: TEST INFRASTRUCTURE ONLY.

Plain fp64 implementations written from the paper's definitions; they share no
code with the HIP library and nothing in the product path may import this
package.  Only ``tests/``, the smoke check and the benchmark's ``cpu_baseline``
leg use it.

``ref``          ctypes wrapper of ``stree_oracle.c`` (path-unrolled sequential
                 recurrence = primary oracle, per-node-state recurrence, linear
                 scan, tree conv, commit, tree index, unroll counts)
``matrix_form``  numpy statement of the paper's matrix form (tree mask L,
                 A_tree = L A_log, M_x, M_u) for tiny trees
"""
