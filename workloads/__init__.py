"""Seeded synthetic inputs for the batched peak-memory estimator.

This package only *describes* inputs: decoder tensor/event tables, configuration
grids and explicit allocator event lists.  It holds none of the estimator's
arithmetic (no rounding, no chunking, no peak computation); the CPU oracle and
the HIP path each consume what it produces and share nothing else.
"""
