"""The C-ABI library without a GPU: it loads, exports what include/ann.h declares, and
turns every bad argument into an error code (no launch is attempted on these paths)."""
import ctypes
import os
import re

import pytest

from paper_2512_02278_amd import ann

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000  # a non-null, 16-byte aligned address that is never dereferenced on these paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ann.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ann_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = ann.lib()
    names = declared_functions()
    assert set(names) == set(ann.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None


def test_public_header_is_plain_c(tmp_path):
    """include/ann.h is the boundary: it must compile as C99 and as C++ on its own, with no HIP or torch types."""
    import subprocess

    src = tmp_path / "use_header.c"
    src.write_text('#include "ann.h"\nint main(void) { return ANN_OK; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, "ann.h")).read(), flags=re.S)
    assert not re.search(r"\bhip\w+|\btorch|\bat::", text) and "#include <stdint.h>" in text


def desc(**kw):
    d = ann.ann_index_desc_t()
    d.vectors, d.n, d.dim, d.dtype, d.row_stride_bytes = FAKE, 1000, 128, ann.ANN_U8, 128
    d.graph, d.degree, d.metric, d.n_entry, d.entry_mode, d.seed = FAKE, 32, ann.ANN_L2, 32, 0, 1
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def load(d):
    h = ctypes.c_void_p()
    rc = ann.lib().ann_index_load(ctypes.byref(d), ctypes.byref(h))
    return rc, h


def test_load_and_free_roundtrip():
    rc, h = load(desc())
    assert rc == ann.ANN_OK and h.value
    assert ann.lib().ann_lds_bytes(h, 128, 4) > 0
    assert ann.lib().ann_free(h) == ann.ANN_OK
    assert ann.lib().ann_free(None) == ann.ANN_OK


def test_set_option_checks_its_arguments():
    L = ann.lib()
    rc, h = load(desc(entry_mode=1, centroids=FAKE, cluster_offsets=FAKE, n_clusters=40, route_c=2, dim=100, dtype=ann.ANN_F32,
                      row_stride_bytes=400))  # 400-byte rows: no matrix-core routing, so nothing touches a device
    assert rc == ann.ANN_OK
    base = L.ann_lds_bytes(h, 128, 4)
    assert L.ann_index_set_option(h, ann.ANN_OPT_VISITED_WINDOW_BITS, 0) == ann.ANN_OK
    assert L.ann_lds_bytes(h, 128, 4) == base - 8192 // 8 + 4 * (1 << 9)      # no bitmap; the hash gets one more bit
    assert L.ann_index_set_option(h, ann.ANN_OPT_VISITED_WINDOW_BITS, 100) == ann.ANN_OK   # rounded up to 128 bits
    assert L.ann_lds_bytes(h, 128, 4) == base - 8192 // 8 + 128 // 8
    assert L.ann_index_set_option(h, ann.ANN_OPT_VISITED_WINDOW_BITS, (1 << 17) + 1) == ann.ANN_EINVAL
    assert L.ann_index_set_option(h, ann.ANN_OPT_VISITED_WINDOW_BITS, -1) == ann.ANN_EINVAL
    assert L.ann_index_set_option(h, ann.ANN_OPT_VISITED_HASH_BITS_BIAS, 5) == ann.ANN_EINVAL
    assert L.ann_index_set_option(h, ann.ANN_OPT_VISITED_HASH_BITS_BIAS, -1) == ann.ANN_OK
    assert L.ann_index_set_option(h, ann.ANN_OPT_CLUSTER_ORDER_MIN_QUERIES, -1) == ann.ANN_OK
    assert L.ann_index_set_option(h, ann.ANN_OPT_MATRIX_CORE_ROUTING, 0) == ann.ANN_OK
    assert L.ann_index_set_option(h, ann.ANN_OPT_LANES_PER_ROW, 32) == ann.ANN_OK
    assert L.ann_index_set_option(h, ann.ANN_OPT_LANES_PER_ROW, 8) == ann.ANN_EUNSUPPORTED   # 8 lanes x 3 pieces hold 384 bytes
    assert L.ann_index_set_option(h, ann.ANN_OPT_LANES_PER_ROW, 5) == ann.ANN_EUNSUPPORTED
    assert L.ann_index_set_option(h, ann.ANN_OPT_LANES_PER_ROW, 0) == ann.ANN_OK
    assert L.ann_index_set_option(h, 99, 0) == ann.ANN_EINVAL
    assert "unknown option" in ann.ann_last_error()
    assert L.ann_index_set_option(None, ann.ANN_OPT_MATRIX_CORE_ROUTING, 0) == ann.ANN_EINVAL
    assert L.ann_free(h) == ann.ANN_OK


def test_static_scratch_size_in_header_and_binding_agree():
    text = open(os.path.join(ROOT, "include", "ann.h")).read()
    m = re.search(r"#define\s+ANN_STATIC_SCRATCH_BYTES\s+\(([^)]*)\)", text)
    assert m and eval(m.group(1)) == ann.ANN_STATIC_SCRATCH_BYTES
    L = ann.lib()
    rc, h = load(desc())
    # argument errors come before any device work; an empty batch launches nothing
    assert L.ann_search_static(h, FAKE, 0, 10, 64, 1, 5, FAKE, FAKE, None) == ann.ANN_OK
    assert L.ann_search_static(h, FAKE, 5, 0, 64, 1, 5, FAKE, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_search_static(None, FAKE, 5, 10, 64, 1, 5, FAKE, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_free(h) == ann.ANN_OK


def test_product_sources_read_no_environment_variables():
    """Nothing outside the C ABI steers the library: its sources never call getenv."""
    import glob

    for path in glob.glob(os.path.join(ROOT, "paper_2512_02278_amd", "csrc", "*")):
        assert "getenv" not in open(path).read(), path


@pytest.mark.parametrize("kw,code", [
    (dict(vectors=None), ann.ANN_EINVAL),
    (dict(graph=None), ann.ANN_EINVAL),
    (dict(n=0), ann.ANN_EINVAL),
    (dict(n=2**31), ann.ANN_EINVAL),
    (dict(dtype=7), ann.ANN_EINVAL),
    (dict(metric=5), ann.ANN_EINVAL),
    (dict(dim=100, row_stride_bytes=112), ann.ANN_EINVAL),      # 100 bytes: not a multiple of 16
    (dict(row_stride_bytes=64), ann.ANN_EINVAL),                # stride below the row length
    (dict(row_stride_bytes=136), ann.ANN_EINVAL),               # stride not a multiple of 16
    (dict(row_stride_bytes=1 << 31), ann.ANN_EINVAL),           # stride of 2^31 bytes or more
    (dict(vectors=FAKE + 8), ann.ANN_EINVAL),                   # misaligned
    (dict(degree=0), ann.ANN_EINVAL),
    (dict(n_entry=0), ann.ANN_EINVAL),
    (dict(n_entry=513), ann.ANN_EINVAL),
    (dict(entry_mode=3), ann.ANN_EINVAL),
    (dict(entry_mode=1), ann.ANN_EINVAL),                       # routed without centroids
    (dict(entry_mode=1, centroids=FAKE, cluster_offsets=FAKE, n_clusters=4, route_c=5), ann.ANN_EINVAL),
    (dict(entry_mode=1, centroids=FAKE, cluster_offsets=FAKE, n_clusters=40, route_c=9), ann.ANN_EINVAL),
    (dict(dim=1552, row_stride_bytes=1552), ann.ANN_EUNSUPPORTED),  # rows above 1536 elements: no variant built
])
def test_load_rejects(kw, code):
    rc, h = load(desc(**kw))
    assert rc == code and not h.value
    assert ann.ann_last_error()


def test_search_argument_errors_and_empty_batch():
    L = ann.lib()
    rc, h = load(desc())
    assert rc == ann.ANN_OK

    def search(nq=10, k=10, itopk=64, width=1, max_iters=5, q=FAKE, ids=FAKE, dists=FAKE):
        return L.ann_search(h, q, nq, k, itopk, width, max_iters, ids, dists, None)

    assert search(nq=0) == ann.ANN_OK                   # nothing to do, nothing launched
    assert search(nq=0, q=None, ids=None, dists=None) == ann.ANN_OK
    assert search(nq=-1) == ann.ANN_EINVAL
    assert search(k=0) == ann.ANN_EINVAL
    assert search(k=65) == ann.ANN_EINVAL               # k above itopk
    assert search(max_iters=-1) == ann.ANN_EINVAL
    assert search(itopk=513, k=10) == ann.ANN_EUNSUPPORTED
    assert search(width=17) == ann.ANN_EUNSUPPORTED     # 17 * 32 neighbours per round: above 512
    assert search(width=0) == ann.ANN_EUNSUPPORTED
    assert search(q=None) == ann.ANN_EINVAL
    assert search(ids=None) == ann.ANN_EINVAL
    assert search(dists=None) == ann.ANN_EINVAL
    assert search(q=FAKE + 4) == ann.ANN_EINVAL
    assert "aligned" in ann.ann_last_error()
    assert L.ann_route(h, FAKE, 4, FAKE, None) == ann.ANN_EINVAL  # not a routed index
    assert L.ann_free(h) == ann.ANN_OK
    assert L.ann_search(None, FAKE, 1, 1, 1, 1, 1, FAKE, FAKE, None) == ann.ANN_EINVAL


def test_binding_refuses_host_tensors():
    import torch

    x = torch.zeros((100, 128), dtype=torch.uint8)
    g = torch.zeros((100, 32), dtype=torch.int32)
    with pytest.raises(ValueError):
        ann.ann_index_load(x, g)


def test_combine_entry_points_reject_bad_arguments():
    L = ann.lib()
    rc, h = load(desc())
    assert rc == ann.ANN_OK
    assert L.ann_gather_vectors(h, FAKE, 0, FAKE, None) == ann.ANN_OK          # nothing to do
    assert L.ann_gather_vectors(h, FAKE, -1, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_gather_vectors(h, None, 4, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_gather_vectors(h, FAKE, 4, FAKE + 4, None) == ann.ANN_EINVAL  # misaligned output
    assert L.ann_gather_vectors(None, FAKE, 4, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_free(h) == ann.ANN_OK

    def merge(key_dtype=ann.ANN_U8, nq=4, per_query=30, k=10, ids=FAKE, keys=FAKE, oi=FAKE, ok=FAKE):
        return L.ann_merge_topk(key_dtype, ids, keys, nq, per_query, k, oi, ok, None)

    assert merge(nq=0) == ann.ANN_OK
    assert merge(key_dtype=9) == ann.ANN_EINVAL
    assert merge(nq=-2) == ann.ANN_EINVAL
    assert merge(per_query=0) == ann.ANN_EUNSUPPORTED
    assert merge(per_query=513) == ann.ANN_EUNSUPPORTED
    assert merge(k=31) == ann.ANN_EINVAL                 # k above per_query
    assert merge(k=0) == ann.ANN_EINVAL
    assert merge(ids=None) == ann.ANN_EINVAL
    assert merge(ok=None) == ann.ANN_EINVAL
    rc, h2 = load(desc())
    assert L.ann_calibration_gather(h2, FAKE, 0, FAKE, None) == ann.ANN_OK
    assert L.ann_calibration_gather(h2, None, 8, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_calibration_gather(h2, FAKE, 8, None, None) == ann.ANN_EINVAL
    assert L.ann_calibration_gather(h2, FAKE, -3, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_calibration_gather(None, FAKE, 8, FAKE, None) == ann.ANN_EINVAL
    assert L.ann_free(h2) == ann.ANN_OK
    assert L.ann_calibration_copy(FAKE, FAKE, 0, None) == ann.ANN_OK
    assert L.ann_calibration_copy(FAKE, FAKE, 24, None) == ann.ANN_EINVAL      # not a multiple of 16
    assert L.ann_calibration_copy(None, FAKE, 32, None) == ann.ANN_EINVAL


def test_graph_construction_rejects_bad_arguments():
    L = ann.lib()

    def prune(knn=FAKE, n=1000, d_in=64, d_out=32, out=FAKE):
        return L.ann_graph_prune(knn, n, d_in, d_out, out, None)

    assert prune(knn=None) == ann.ANN_EINVAL
    assert prune(out=None) == ann.ANN_EINVAL
    assert prune(n=0) == ann.ANN_EINVAL
    assert prune(n=2**31) == ann.ANN_EINVAL
    assert prune(d_out=0) == ann.ANN_EINVAL
    assert prune(d_in=16, d_out=17) == ann.ANN_EINVAL           # d_out above d_in
    assert prune(d_in=129, d_out=32) == ann.ANN_EUNSUPPORTED
    assert prune(d_in=128, d_out=65) == ann.ANN_EUNSUPPORTED
    need = L.ann_graph_optimize_workspace_bytes(1000, 64, 32)
    assert need >= 1000 * 32 * 12 + 1000 * 12 and need % 256 == 0
    assert L.ann_graph_optimize_workspace_bytes(0, 64, 32) == ann.ANN_EINVAL
    assert L.ann_graph_optimize_workspace_bytes(1000, 200, 32) == ann.ANN_EUNSUPPORTED
    big = L.ann_graph_optimize_workspace_bytes(100_000_000, 64, 32)
    assert 38e9 < big < 42e9                                     # pruned rows + (position, source) words + offsets

    def optimize(knn=FAKE, n=1000, d_in=64, d_out=32, out=FAKE, ws=FAKE, ws_bytes=need):
        return L.ann_graph_optimize(knn, n, d_in, d_out, out, ws, ws_bytes, None)

    assert optimize(knn=None) == ann.ANN_EINVAL
    assert optimize(ws=None) == ann.ANN_EINVAL
    assert optimize(ws=FAKE + 16) == ann.ANN_EINVAL             # workspace not 256-byte aligned
    assert optimize(ws_bytes=need - 1) == ann.ANN_EINVAL
    assert "needed" in ann.ann_last_error()
    assert optimize(d_out=65, d_in=128) == ann.ANN_EUNSUPPORTED


def test_reciprocal_division_used_for_graph_slots_is_exact():
    """The kernel turns s / degree (s < 1024, degree <= 512) into (s * ceil(2^20 / degree)) >> 20."""
    for d in range(1, 513):
        inv = ((1 << 20) + d - 1) // d
        assert all(((s * inv) >> 20) == s // d for s in range(1024)), d
