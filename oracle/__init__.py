"""CPU oracle for the EOQ full-int8 training step -- TEST INFRASTRUCTURE ONLY.

A plain, slow implementation of what the paper defines (Sections 3.1-3.2),
written independently of the HIP library.  It may be imported by tests, by the
smoke check and by the CPU-baseline leg of the benchmark, and by nothing else;
the product package never imports it and it never imports the product package.
"""
