"""CPU oracle for the batched token-sampling stage: test infrastructure, not product code.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It shares no code with the HIP path."""
