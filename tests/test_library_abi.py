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
    return sorted(set(re.findall(r"\b((?:emb|mlp|hyb)_[a-z_]+)\s*\(", text)))


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


def _config(b, tables, slots, **kw):
    t = (b.emb_table_desc * len(tables))(*[b.emb_table_desc(*x) for x in tables])
    s = (b.emb_slot_desc * len(slots))(*[b.emb_slot_desc(x[0], x[2] if len(x) > 2 else 0, x[1]) for x in slots])
    f = dict(hash=1, opt=1, lr=0.05, eps=1e-8, acc_init=0.1, init_lo=-0.01, init_hi=0.01, device=0, init_seed=1,
             max_ids=64, max_batch=8, reserved=0)
    f.update(kw)
    cfg = b.emb_config(len(tables), len(slots), t, s, f["hash"], f["opt"], f["lr"], f["eps"], f["acc_init"], f["init_lo"],
                       f["init_hi"], f["device"], f["init_seed"], f["max_ids"], f["max_batch"], f["reserved"])
    cfg._keep = (t, s)
    return cfg


def test_argument_validation_happens_on_the_host_before_any_device_call():
    """Every malformed configuration is turned away with EMB_EINVAL and a message by checks that run before the
    library touches a device (so they can be exercised here, without a GPU); null contexts likewise."""
    from paper_2111_05897_amd import binding as b
    lib = b.load_library()
    h = C.c_void_p()
    bad = {
        "dim 12": _config(b, [(100, 12, 0)], [(0, 1)]),
        "unknown dtype": _config(b, [(100, 8, 7)], [(0, 1)]),
        "table with 0 rows": _config(b, [(0, 8, 0)], [(0, 1)]),
        "too many rows": _config(b, [(1 << 30, 8, 0), (1 << 30, 8, 0)], [(0, 1), (1, 2)]),
        "slot names a missing table": _config(b, [(100, 8, 0)], [(3, 1)]),
        "slot.reserved": _config(b, [(100, 8, 0)], [(0, 1, 9)]),
        "config.reserved": _config(b, [(100, 8, 0)], [(0, 1)], reserved=1),
        "unknown hash": _config(b, [(100, 8, 0)], [(0, 1)], hash=5),
        "unknown optimizer": _config(b, [(100, 8, 0)], [(0, 1)], opt=2),
        "negative eps": _config(b, [(100, 8, 0)], [(0, 1)], eps=-1.0),
        "lr not finite": _config(b, [(100, 8, 0)], [(0, 1)], lr=float("nan")),
        "init range reversed": _config(b, [(100, 8, 0)], [(0, 1)], init_lo=1.0, init_hi=-1.0),
        "max_batch 0": _config(b, [(100, 8, 0)], [(0, 1)], max_batch=0),
        "max_ids too large": _config(b, [(100, 8, 0)], [(0, 1)], max_ids=1 << 31),
        "bags overflow": _config(b, [(100, 8, 0)], [(0, 1)] * 4096, max_batch=1 << 20),
        "gradient positions overflow": _config(b, [(100, 128, 0), (100, 128, 0)], [(0, 1), (1, 2)] * 500, max_batch=1 << 20),
    }
    for name, cfg in bad.items():
        assert lib.emb_create(C.byref(cfg), C.byref(h)) == b.EMB_EINVAL, name
        assert lib.emb_last_error(None), name
        assert not h.value, name
    small_cache = (C.c_uint64 * 1)(10)            # fewer slots than one batch may need
    cfg = _config(b, [(1000, 8, 0)], [(0, 1)])
    assert lib.emb_create_cached(C.byref(cfg), small_cache, C.byref(h)) == b.EMB_EINVAL
    assert b"cache_rows" in lib.emb_last_error(None)
    # null contexts
    batch = b.emb_batch(1, 0, 0, None, None)
    assert lib.emb_lookup_pool(None, C.byref(batch), None, None) == b.EMB_EINVAL
    assert lib.emb_backward_update(None, C.byref(batch), None, None) == b.EMB_EINVAL
    assert lib.emb_backward_update_static(None, C.byref(batch), None, None) == b.EMB_EINVAL
    assert lib.emb_hash_rows(None, C.byref(batch), None, None) == b.EMB_EINVAL
    assert lib.emb_dedup_sizes(None, None, None) == b.EMB_EINVAL
    assert lib.emb_read_rows(None, 0, None, 0, None, None) == b.EMB_EINVAL
    assert lib.emb_destroy(None) == b.EMB_OK
    assert lib.emb_static_max_ids() == 1 << 18
    # the value codec's arguments (pointers are only looked at, never followed, before the checks)
    fake = C.c_void_p(0x1000)
    assert lib.emb_codec_compress(fake, 4, 6, 1024.0, fake, fake, None) == b.EMB_EINVAL          # block_len % 4
    assert lib.emb_codec_compress(fake, 4, 8, 1.0e6, fake, fake, None) == b.EMB_EINVAL           # kappa beyond fp16
    assert lib.emb_codec_decompress(None, fake, 4, 8, 1024.0, fake, None) == b.EMB_EINVAL        # null buffer
    assert lib.emb_codec_compress(None, 0, 8, 1024.0, None, None, None) == b.EMB_OK              # nothing to do


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
