"""Seeded synthetic workloads shared by the CPU oracle and the HIP path.

This package holds only *data*: layer-graph descriptions of the member models
(`zoo`), and the seeded generators for their weights, the input batches and the
request stream (`gen`).  It contains none of the method's arithmetic: no
convolution, no pooling, no DAG compilation.  Both executors consume the bytes
produced here; neither imports the other.
"""
from . import zoo, gen  # noqa: F401
