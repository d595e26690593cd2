"""Teams of workgroups per channel (cbd_config.workgroups_per_channel): the same results as one workgroup per
channel, against the checker."""
import numpy as np
import pytest

from paper_2306_15685_amd import synth
from paper_2306_15685_amd import binding as B

import gpu_harness as GH
from oracle import OracleGraph
from test_gpu_parity import run_batch, mid_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    return torch


@pytest.mark.parametrize("k", [2, 4, 8])
def test_team_random_graph(torch_cuda, k):
    """HCLG-style random graph with epsilon closures up to a few levels deep, ragged chunks, a partial result per
    chunk, contexts per channel."""
    print(f"team of {k}: random graph", flush=True)
    g, L, ctxs, offs = mid_inputs(torch_cuda)
    s = run_batch(torch_cuda, g, L, ctxs, offs, beam=13.0, max_active=0, chunks=[1, 7, 16, 24], hash_log2=16,
                  workgroups_per_channel=k)
    assert s["eps_arcs"] > 0 and s["frames"] == L.shape[0] * L.shape[1]


def test_team_histogram_pruning(torch_cuda):
    print("team of 4: max-active engaged", flush=True)
    g, L, ctxs, offs = mid_inputs(torch_cuda, seed=12)
    s = run_batch(torch_cuda, g, L, ctxs, offs, beam=14.0, max_active=150, chunks=[12, 12, 24], hash_log2=16,
                  workgroups_per_channel=4, use_final=False)
    assert s["max_tokens"] > 150


def test_team_lexicon_loop_long_hub_row(torch_cuda):
    """A hub row of 1,500 arcs (shared out over the team once it has been announced, by one member's waves in the
    frame after the reset), word-end epsilon arcs that all lead back to the hub, max-active engaged."""
    print("team of 4: lexicon loop", flush=True)
    torch = torch_cuda
    g = synth.make_lexicon_graph(24, 1500, seed_stream=(91,))
    C, T = 5, 40
    L = synth.make_loglikes(C, T, g.num_pdfs, 2.0, seed_stream=(91,), device="cuda")
    w = synth.scaled(synth.WORKLOADS["e2e"], channels=C, ctx_min=20, ctx_max=60, config_id=91)
    ctxs, offs = synth.make_contexts(w, g)
    s = run_batch(torch, g, L, ctxs, offs, beam=8.0, max_active=400, chunks=[3, 10, 27], hash_log2=16, lookup_mode=1,
                  workgroups_per_channel=4)
    assert s["max_tokens"] > 400
