"""Plain CPU oracle for the Parle training step: TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the bench's CPU-baseline leg may import this
package.  It shares no code with the HIP path and never imports it.
Pin status: every function here is pinned by tests/test_oracle_*.py against
closed forms, finite differences, brute force or library routines, except the
exact training trajectory of the full-size networks, for which the paper prints
no intermediate values ("parity unpinned" for the architecture details that the
paper leaves to its citations; see the module headers).
"""
