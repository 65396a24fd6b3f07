"""Test and benchmark harness: a graph builder, exhaustive ground truth and graph diagnostics.

Nothing here is part of the library (``paper_2604_16402_amd``) or of the oracle (``oracle``);
the library imports none of it.
"""
