"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every function include/quest.h declares, and rejects bad arguments with the
documented status codes before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2406_10774_amd import binding


def declared_functions(repo_root):
    text = open(os.path.join(repo_root, "include", "quest.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(quest_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    lib = binding.load()
    names = declared_functions(repo_root)
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def make_cache(**kw):
    base = dict(batch=1, num_heads=32, head_dim=128, page_size=16, max_pages_per_seq=2048,
                flags=0, num_phys_pages=2048, k_pool=0x1000, v_pool=0x1000, meta=0x1000,
                page_table=0x1000, seq_lens=0x1000)
    base.update(kw)
    return binding.quest_cache(**base)


def test_workspace_bytes_is_pure_and_consistent():
    lib = binding.load()
    out = ctypes.c_size_t(0)
    c = make_cache()
    assert lib.quest_workspace_bytes(ctypes.byref(c), 128, ctypes.byref(out)) == 0
    sparse = out.value
    assert lib.quest_workspace_bytes(ctypes.byref(c), 0, ctypes.byref(out)) == 0
    dense = out.value
    # one 256-byte counter slot per head + (D + 2) floats per (head, split);
    # the dense path uses at least as many splits
    assert (sparse - 32 * 256) % (32 * 130 * 4) == 0 and (dense - 32 * 256) % (32 * 130 * 4) == 0
    assert dense >= sparse > 0
    assert lib.quest_workspace_bytes(ctypes.byref(c), 128, None) == -1


def test_topk_workspace_bytes_follows_the_two_stage_rule():
    """quest.h: rows of 16384 pages or more are selected in two stages, a 4096-page chunk
    keeping its best k_pages as (score, page) candidates, while a row has at most 8192
    of them and they are fewer than half of the row; everything else needs no workspace."""
    lib = binding.load()
    out = ctypes.c_size_t(7)

    def need(max_pages, k_pages, **kw):
        c = make_cache(max_pages_per_seq=max_pages, **kw)
        assert lib.quest_topk_workspace_bytes(ctypes.byref(c), k_pages, ctypes.byref(out)) == 0
        return out.value

    heads = make_cache().num_heads
    assert need(16383, 64) == 0                                   # short rows: one work-group per row
    assert need(16384, 64) == heads * 4 * 64 * 8                  # 4 chunks
    assert need(32769, 256) == heads * 9 * 256 * 8                # the ninth chunk holds one page
    assert need(32769, 256, batch=3) == 3 * heads * 9 * 256 * 8
    assert need(32769, 1024) == 0                                 # 9216 candidates: too many
    assert need(65535, 512) == heads * 16 * 512 * 8
    assert need(65535, 4097) == 0                                 # more than a chunk holds
    assert need(16384, 4096) == 0                                 # candidates would be the whole row
    c = make_cache(max_pages_per_seq=32769)
    assert lib.quest_topk_workspace_bytes(ctypes.byref(c), 256, None) == -1
    assert lib.quest_topk_workspace_bytes(ctypes.byref(c), 0, ctypes.byref(out)) == 0 and out.value == 0


@pytest.mark.parametrize("kw,status", [
    (dict(head_dim=64), -3), (dict(page_size=24), -3), (dict(page_size=128), -3), (dict(batch=0), -2),
    (dict(num_heads=70000), -2), (dict(page_table=None), -1), (dict(seq_lens=None), -1),
    (dict(max_pages_per_seq=0), -2), (dict(num_kv_heads=5), -2), (dict(num_kv_heads=-1), -2),
])
def test_bad_cache_is_rejected_on_the_host(kw, status):
    lib = binding.load()
    c = make_cache(**kw)
    assert lib.quest_build_meta(ctypes.byref(c), None) == status
    assert lib.quest_estimate(ctypes.byref(c), 0x1000, 0x1000, None) == status
    assert lib.quest_last_error()          # a message is available


def test_null_and_range_arguments():
    lib = binding.load()
    c = make_cache()
    r = ctypes.byref(c)
    assert lib.quest_build_meta(None, None) == -1
    assert lib.quest_estimate(r, None, 0x1000, None) == -1
    assert lib.quest_estimate(r, 0x1000, None, None) == -1
    assert lib.quest_append_meta(r, None, None, 0, None) == -1
    assert lib.quest_append_meta(r, 0x1000, None, 1, None) == -1     # pool write needs v_new
    assert lib.quest_topk(r, 0x1000, 0, 0x1000, None, None, 0, None) == -2    # k_pages < 1
    assert lib.quest_topk(r, None, 4, 0x1000, None, None, 0, None) == -1
    assert lib.quest_sparse_decode(r, 0x1000, 0x1000, 0, 1.0, 0x1000, 0, None, 0x1000, 1 << 30,
                                   None) == -2
    # workspace too small / missing
    assert lib.quest_sparse_decode(r, 0x1000, 0x1000, 128, 1.0, 0x1000, 0, None, 0x1000, 16,
                                   None) == -4
    assert lib.quest_sparse_decode(r, 0x1000, 0x1000, 128, 1.0, 0x1000, 0, None, None, 0,
                                   None) == -4
    assert b"workspace" in lib.quest_last_error()
    # selection + attention from given scores: same rules
    assert lib.quest_select_decode(r, 0x1000, None, 128, 1.0, 0x1000, None, 0x1000, 0, None, 0x1000,
                                   1 << 30, None) == -1              # scores
    assert lib.quest_select_decode(r, 0x1000, 0x1000, 0, 1.0, 0x1000, None, 0x1000, 0, None, 0x1000,
                                   1 << 30, None) == -2              # k_pages < 1
    assert lib.quest_select_decode(r, 0x1000, 0x1000, 128, 1.0, 0x1000, None, 0x1000, 0, None, None,
                                   0, None) == -4


def test_product_package_does_not_import_the_oracle(repo_root):
    pkg = os.path.join(repo_root, "paper_2406_10774_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("the CPU oracle's tests", ""), f
