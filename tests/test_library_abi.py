"""CPU-only checks of the boundary: the built C-ABI library loads and exports every symbol the
header declares; struct layouts in the binding match the header's field order."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "persia_emb.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(emb_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary_calls():
    names = declared_functions()
    for required in ("emb_create", "emb_destroy", "emb_lookup_pool", "emb_backward_update", "emb_hash_rows",
                     "emb_read_dedup", "emb_read_rows", "emb_last_error"):
        assert required in names


def test_library_loads_and_exports_every_declared_symbol():
    from paper_2111_05897_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libpersia_emb.so is not built: run `python paper_2111_05897_amd/build.py`")
    lib = binding.load_library()
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in persia_emb.h but not exported"
    assert lib.emb_stage_count() >= 1
    names = [lib.emb_stage_name(i).decode() for i in range(lib.emb_stage_count())]
    assert "gather_pool" in names and "reduce_update" in names
    # error path that needs no GPU: null arguments are rejected, with a message
    assert lib.emb_create(None, None) == binding.EMB_EINVAL
    assert b"null" in lib.emb_last_error(None)


def test_binding_struct_layouts():
    from paper_2111_05897_amd import binding as b
    assert C.sizeof(b.emb_table_desc) == 16
    assert C.sizeof(b.emb_slot_desc) == 16
    assert C.sizeof(b.emb_batch) == 32
    assert C.sizeof(b.emb_config) == 80
    assert b.emb_config.init_seed.offset == 56 and b.emb_config.max_batch.offset == 72
    assert b.emb_batch.ids.offset == 16


def test_workload_shapes_match_the_configurations():
    from paper_2111_05897_amd import workload as W
    w = W.make_workload(2)
    assert (w.batch, w.cfg.num_slots, w.cfg.tables[0].rows, w.cfg.tables[0].dim) == (16384, 100, 1 << 26, 64)
    w3 = W.make_workload(3)
    assert sum(t.rows for t in w3.cfg.tables) == 1 << 27 and w3.cfg.pooled_width == 9920
    w1 = W.make_workload(1, scale=1 / 16)
    b = W.make_batch(w1)
    lens = b.offsets[1:] - b.offsets[:-1]
    assert lens.min() >= 1 and lens.max() <= 20 and abs(lens.mean() - 10.5) < 0.3
    assert b.num_ids == len(b.ids)
    b2 = W.make_batch(w1)
    assert (b2.ids == b.ids).all() and (W.make_batch(w1, 1).ids[:100] != b.ids[:100]).any()
    w2 = W.make_workload(2, scale=1 / 64)
    l2 = W.bag_lengths(w2, 0)
    assert l2.min() >= 1 and l2.max() <= 64 and abs(l2.mean() - 8.0) < 0.2
