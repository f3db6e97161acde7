"""GPU parity for grouped-query attention (fewer KV heads than query heads): the chain and
the one-call step against the oracle's reading (a page's score for a KV head is the largest
of its query heads' scores; one page list per KV head), for groups of 2, 4 and 8 and two
page sizes."""
import numpy as np
import pytest

from paper_2406_10774_amd import synth
from test_gpu_chain import run_chain, run_decode_steps

pytestmark = pytest.mark.gpu


def ragged(cid, kv_heads, S=16):
    lens = (1, S * 5 + 3, S * 70 + S - 1, S * 33)
    return synth.Workload(cid, f"gqa-S{S}", len(lens), kv_heads, lens, token_budget=S * 12,
                          planted_per_head=4, page_size=S, decode_steps=24)


@pytest.mark.parametrize("kv_heads,group", [(3, 2), (2, 3), (2, 4), (1, 8)])
def test_chain(kv_heads, group):
    run_chain(ragged(500 + group, kv_heads), steps=5, permute=True, group=group)


@pytest.mark.parametrize("S", [8, 32])
def test_chain_other_page_sizes(S):
    run_chain(ragged(510 + S, 2, S=S), steps=4, permute=True, group=4)


@pytest.mark.parametrize("flags", [0, 1, 8])
def test_decode_step(flags):
    # two launches, three launches, two launches with the newest page kept
    run_decode_steps(ragged(520, 2), steps=8, permute=True, flags=flags, group=4)


def test_long_context_group_of_4():
    w = synth.Workload(530, "gqa-long", 1, 8, (16384 + 5,), token_budget=2048, planted_per_head=16,
                       decode_steps=4)
    run_chain(w, steps=3, permute=True, group=4)
