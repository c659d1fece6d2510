"""The C boundary without a GPU: the library loads, exports every declared
symbol, and rejects bad arguments before touching the device."""
import os
import re

import pytest

from paper_2208_14228_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    inc = os.path.join(ROOT, "include")
    txt = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    txt = re.sub(r"/\*.*?\*/", "", txt, flags=re.S)
    return sorted(set(re.findall(r"\b(es_[a-z_]+)\s*\(", txt)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 20
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names
    assert "gfx950" in B.es_version()


def test_strerror():
    assert B.es_strerror(0) == "ok"
    for s in (B.ES_EINVAL, B.ES_ESTATE, B.ES_ENOMEM, B.ES_EHIP):
        assert B.es_strerror(s) not in ("ok", "unknown status")
    assert B.es_strerror(-99) == "unknown status"


def test_init_rejects_bad_layouts_before_any_device_work():
    bad = [
        (0, 8, [(0, 8)], 1, ()),                 # no logical workers
        (70000, 8, [(0, 8)], 1, ()),             # too many
        (2, 8, [(0, 8)], 0, ()),                 # chunk alignment 0
        (2, 8, [(0, 4)], 1, ()),                 # does not cover [0, P)
        (2, 8, [(0, 4), (5, 3)], 1, ()),         # gap
        (2, 8, [(0, 5), (4, 4)], 1, ()),         # overlap
        (2, 8, [(4, 4), (0, 4)], 1, ()),         # not ascending
        (2, 8, [(0, 8)], 1, (16, 0)),            # empty state segment
    ]
    for n, P, buckets, A, segs in bad:
        st, h = B.es_init(n, P, buckets, A, segs)
        assert st == B.ES_EINVAL and h == 0, (n, P, buckets, A, segs)


def test_null_handle_is_rejected_everywhere():
    assert B.es_destroy(0) == B.ES_EINVAL
    assert B.es_sync(0) == B.ES_EINVAL
    assert B.es_ctx_save(0, 0) == B.ES_EINVAL
    assert B.es_ctx_restore(0, 0) == B.ES_EINVAL
    assert B.es_ctx_switch(0, 0, 1) == B.ES_EINVAL
    assert B.es_accumulate(0, 0, 0, 0) == B.ES_EINVAL
    assert B.es_accumulate_batch(0, 0, [0], [0]) == B.ES_EINVAL
    assert B.es_accumulate_in_place(0, 0, 0) == B.ES_EINVAL
    assert B.es_accumulate_many(0, [0], [0]) == B.ES_EINVAL
    assert B.es_est_boundary(0, 0, None, [0], [0]) == B.ES_EINVAL
    assert B.es_grad_slot(0, 0, 0) == 0
    assert B.es_ring_order_reduce(0, 0) == B.ES_EINVAL
    assert B.es_sgd_step(0, 0, 0, 0, 0.1, 0.9) == B.ES_EINVAL
    assert B.es_reduce_sgd_step(0, 0, 0, 0, 0.1, 0.9) == B.ES_EINVAL
    assert B.es_set_option(0, "nontemporal", 1) == B.ES_EINVAL
    assert B.es_stage_fence(0) == B.ES_EINVAL
    assert B.es_grad_sq_norm(0, 0, 0) == B.ES_EINVAL
    assert B.es_clip_sgd_step(0, 0, 0, 0, 0, 1.0, 0.0, 0.1, 0.9) == B.ES_EINVAL
    assert B.es_bn_batch_stats(0, 2, 2, 8, 0, 0, 0, 0) == B.ES_EINVAL
    assert B.es_checkpoint_bytes(0) == 0
    assert B.es_checkpoint_export(0, 0, 0, 0, 0, 0) == B.ES_EINVAL
    assert B.es_checkpoint_import(0, 0, 0, 0, 0)[0] == B.ES_EINVAL
    assert B.es_dropout_mask(0, 0, 0, 0, 0, 0.1) == B.ES_EINVAL
    assert B.es_set_streams(0, 0, 0, 0) == B.ES_EINVAL
    assert B.es_last_hip_error(0) == 0


def test_allocation_free_norm_rejects_bad_arguments_before_any_device_work():
    assert B.es_grad_sq_norm_static(16, 4, 0, 0) == B.ES_EINVAL                 # no output
    assert B.es_grad_sq_norm_static(0, 4, 16, 0) == B.ES_EINVAL                 # no input
    assert B.es_grad_sq_norm_static(20, 4, 16, 0) == B.ES_EINVAL                # input not 16-byte aligned
    assert B.es_grad_sq_norm_static(16, (1 << 30) + 1, 16, 0) == B.ES_EINVAL    # beyond the fixed array


def test_product_does_not_import_the_oracle():
    """The HIP path and its binding never touch oracle/ (and the oracle never imports them)."""
    pkg = os.path.join(ROOT, "paper_2208_14228_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", src, flags=re.M), f
                assert "es_oracle" not in src, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2208_14228_amd" not in src and "libes.so" not in src, f
