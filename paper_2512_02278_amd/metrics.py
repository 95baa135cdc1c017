"""Traffic accounting for the search path.

``paper_model_*`` restate the paper's own bandwidth model (Sec. 2, equation for
bt_q; Sec. 3.2 Stage 3: V = I * w * d_g vectors per query, QPS = BW / bytes).
``algorithmic_bytes_per_query`` is the refinement used for the roofline: it counts
what the method must move given how many rows were actually scored (the visited
filter removes most of the I*w*d_g references) and adds the graph rows, the query
and the result, which the paper's model leaves out.
"""
from __future__ import annotations


def paper_model_vectors(iterations: int, width: int, degree: int) -> int:
    """V = I * w * d_g (Sec. 3.2, Stage 3)."""
    return iterations * width * degree


def paper_model_bytes(n_vectors: int, dim: int, bytes_per_elem: int) -> int:
    """Bytes/query = V * d * b: each candidate vector fetched once (Sec. 2, bt_q)."""
    return n_vectors * dim * bytes_per_elem


def paper_model_qps(hbm_bytes_per_s: float, bytes_per_query: float) -> float:
    """QPS = BW_HBM / (bytes per query) (Sec. 3.2, Stage 3)."""
    return hbm_bytes_per_s / bytes_per_query


def algorithmic_bytes_per_query(n_dist: float, n_parents: float, row_bytes: int, degree: int, query_bytes: int,
                                k: int) -> float:
    """Vector rows scored + graph rows read + the query + the k (id, distance) results."""
    return n_dist * row_bytes + n_parents * degree * 4 + query_bytes + k * 8
