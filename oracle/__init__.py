"""CPU oracle for the HA-RAG mixed-precision KV-chunk load.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py.  Nothing in the product package imports it, and it
imports nothing from the product package.

`codec`      ctypes view of ha_rag_oracle.c (quantise, pack, dequantise, scatter)
`placement`  Algorithm 1 (rank -> precision class) and Algorithm 2 (tier lookup,
             promotion, LRU) as plain Python
"""
from . import codec, placement  # noqa: F401
