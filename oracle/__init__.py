"""CPU oracle for the schedule-executed training step (test infrastructure).

Plain fp64 NumPy, NCHW, written from the paper's definitions; slow on purpose.
Only the tests, the smoke check and the benchmark's CPU-baseline leg may
import it.  It shares no code with the HIP library and never calls it.
"""
