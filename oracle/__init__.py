"""CPU oracle for the split-precision optimizer step: test infrastructure only.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package.  See oracle/mpo_ref.h for what each routine follows in the paper.
"""
