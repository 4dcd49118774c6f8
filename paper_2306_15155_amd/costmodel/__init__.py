"""Learned per-primitive cost models (Section 3.5 of the paper: graph features + embedding sizes -> primitive time,
gradient-boosted trees, one additive prediction per composition).

``collect`` times the primitives of every composition on a grid of synthetic graphs on the GPU at hand,
``train`` fits small gradient-boosted regression trees to those timings and writes the tables the library embeds
(``csrc/learned_model.inc``).  Both are tools around the library, not part of its hot path.
"""
