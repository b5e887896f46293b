"""CPU oracle for the KV-cache chunk path.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product (paper_2510_09665_amd) never does.  See lmc_oracle.c for what
is computed and which passages of the paper it follows.
"""
from .oracle import (  # noqa: F401
    ORC_OK, ORC_INVAL, ORC_NOMEM, ORC_MISS, ORC_BADSLOT, ORC_BUSY,
    build, chunk_bytes, fnv1a64, gather, gather_chunk, hash_chunks, scatter, scatter_chunk,
    OracleStore, time_pass,
)
