"""GPU parity for page sizes other than the paper's default of 16 (Figure 8 of arXiv
2406.10774 sweeps the page size): the whole chain, the single-call step and the dense path
against the oracle, on ragged batches whose last pages are partial, with pages of 8, 32 and
64 tokens (16 again as the control of the shared code)."""
import numpy as np
import pytest

from paper_2406_10774_amd import synth
from test_gpu_chain import run_chain, run_decode_steps

pytestmark = pytest.mark.gpu


def ragged(S, cid):
    # a one-token sequence, a few pages plus a partial one, many pages ending one token short
    # of a full page, an exact multiple, and one that crosses several page boundaries while
    # the test appends
    lens = (1, S * 5 + 3, S * 70 + S - 1, S * 33, S * 41 + S - 2)
    return synth.Workload(cid, f"ragged-S{S}", len(lens), 3, lens, token_budget=S * 12,
                          planted_per_head=4, page_size=S, decode_steps=24)


@pytest.mark.parametrize("S", [8, 16, 32, 64])
def test_chain_ragged(S):
    run_chain(ragged(S, 200 + S), steps=6, permute=True)


@pytest.mark.parametrize("S", [8, 32, 64])
@pytest.mark.parametrize("flags", [0, 1])
def test_decode_step_ragged(S, flags):
    # two launches (the attention launch selects its pages) and three launches
    run_decode_steps(ragged(S, 300 + S), steps=8, permute=True, flags=flags)


@pytest.mark.parametrize("S", [8, 32, 64])
def test_long_context_many_splits(S):
    """One long sequence: several splits per head, page list much shorter than the context."""
    w = synth.Workload(400 + S, f"long-S{S}", 1, 8, (16384 + 5,), token_budget=2048,
                       planted_per_head=16, page_size=S, decode_steps=4)
    run_chain(w, steps=3, permute=True)
