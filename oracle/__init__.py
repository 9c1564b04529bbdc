"""CPU oracle (test infrastructure only): see oracle.c and oracle.py."""
from .oracle import (  # noqa: F401
    METRIC_L2,
    METRIC_IP,
    OracleIVFPQ,
    assign,
    build,
    canon_ip,
    canon_l2,
    coarse_probe,
    flat_search,
    kmeans,
    train_ivfpq,
    refine,
    num_threads,
    pq_decode,
    pq_encode,
    recall,
)
