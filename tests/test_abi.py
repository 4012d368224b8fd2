"""The C-ABI library loads, exports every symbol include/retexo.h declares, and
rejects bad arguments before touching the device (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2302_13053_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "retexo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(retexo_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    names = declared_symbols()
    assert len(names) >= 15
    for n in names:
        assert getattr(lib, n) is not None, n
    assert sorted(B.EXPORTS) == names
    # and the Python binding offers a function of the same name for each
    for n in names:
        assert callable(getattr(B, n)), n


def test_status_strings():
    for code in range(0, -12, -1):
        assert B.status_string(code) != "unknown status"
    assert B.status_string(-99) == "unknown status"


FAKE = 0x1000   # non-NULL address that is never dereferenced: all checks below fail before any launch


def test_transform_argument_errors():
    assert B.retexo_transform(-1, 4, 4, FAKE, 4, FAKE, 0, 0, FAKE * 2, 4) == B.E_SIZE
    assert B.retexo_transform(8, 4, 4, FAKE, 3, FAKE, 0, 0, FAKE * 64, 4) == B.E_LD
    assert B.retexo_transform(8, 4, 4, FAKE, 4, FAKE, 0, 0, FAKE * 64, 3) == B.E_LD
    assert B.retexo_transform(8, 4, 4, 0, 4, FAKE, 0, 0, FAKE * 64, 4) == B.E_NULL
    assert B.retexo_transform(8, 4, 4, FAKE, 4, 0, 0, 0, FAKE * 64, 4) == B.E_NULL
    assert B.retexo_transform(8, 4, 4, FAKE, 4, FAKE, 0, 0, 0, 4) == B.E_NULL
    assert B.retexo_transform(8, 4, 4, FAKE, 4, FAKE, 0, B.F_SELF_CONCAT, FAKE * 64, 4) == B.E_FLAGS
    assert B.retexo_transform(8, 4, 4, FAKE, 4, FAKE, 0, 0, FAKE + 16, 4) == B.E_ALIAS
    assert B.retexo_transform(0, 4, 4, 0, 4, 0, 0, 0, 0, 4) == B.OK        # empty: no-op


def test_plan_and_aggregate_argument_errors():
    st, plan = B.retexo_plan_create(-1, FAKE, FAKE)
    assert st == B.E_SIZE and plan is None
    st, plan = B.retexo_plan_create(4, 0, FAKE)
    assert st == B.E_NULL and plan is None
    st, plan = B.retexo_plan_create(4, FAKE, FAKE, flags=B.F_RELU)
    assert st == B.E_FLAGS and plan is None
    assert B.retexo_aggregate(0, B.MEAN, 4, 1, FAKE, 4, 0, 0, 0.2, 0, FAKE * 64, 4, 0, 0) == B.E_NULL
    assert B.retexo_round(0, B.MEAN, 4, 4, 1, FAKE, 4, 0, 0, 0, 0, 0.2, 0, FAKE * 64, 4, 0, 0) == B.E_NULL
    assert B.retexo_workspace_bytes(0, 4, B.MEAN) == B.E_NULL
    assert B.retexo_plan_destroy(0) == B.OK
    assert B.retexo_plan_nnz(0) == B.E_NULL


def test_csr_argument_errors():
    assert B.retexo_csr_workspace_bytes(-1, 4, False) == B.E_SIZE
    assert B.retexo_csr_workspace_bytes(1 << 30, 4, False) == B.E_SIZE
    st, _ = B.retexo_csr_from_coo(-1, FAKE, FAKE, 4, False, FAKE, FAKE, 8, FAKE, 1 << 20)
    assert st == B.E_SIZE
    st, _ = B.retexo_csr_from_coo(4, FAKE, FAKE, 4, False, 0, FAKE, 8, FAKE, 1 << 20)
    assert st == B.E_NULL
    st, _ = B.retexo_csr_from_coo(4, 0, FAKE, 4, False, FAKE, FAKE, 8, FAKE, 1 << 20)
    assert st == B.E_NULL
    st, _ = B.retexo_csr_from_coo(4, FAKE, FAKE, 4, False, FAKE, FAKE, 8, 0, 1 << 20)
    assert st == B.E_WORKSPACE
    st, _ = B.retexo_csr_from_coo(4, FAKE, FAKE, 4, False, FAKE, FAKE, 8, FAKE + 8, 1 << 20)
    assert st == B.E_WORKSPACE     # misaligned


def test_options():
    assert B.retexo_set_option("agg_slab_cols", 0) == B.OK
    assert B.retexo_set_option("agg_slab_major", -1) == B.OK
    assert B.retexo_set_option("agg_heavy_degree", 2048) == B.OK
    for name, default in (("agg_parts", -1), ("agg_max_vec", 4), ("agg_gat_fast", 1), ("agg_gat_flash", 1),
                          ("agg_gat_in_rows", 1), ("agg_wide_offsets", 0)):
        assert B.retexo_set_option(name, default) == B.OK
    assert B.retexo_set_option("no_such_option", 1) == B.E_FLAGS
