"""Seeded, synthetic inputs for the schedule-executed training step.

This package only *describes* work: it writes graph and schedule text, and
draws seeded random tensors.  It holds none of the method's arithmetic and
no executor; both the CPU oracle and the HIP library read what it writes,
each with a parser of its own.
"""
