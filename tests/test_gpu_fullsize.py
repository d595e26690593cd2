"""Full-size parity: the five benchmark workloads in the launch configuration bench.py times
(runner.Session.step), checked against the CPU checker on sampled channels (every partial and
final result, counters) and, on many more channels, by properties that need no checker:
the returned arc path is connected from the start state, consumes exactly the decoded frames,
re-accumulating its cost in fp32 in path order gives the returned cost bit for bit, and the
words are the path's output labels."""
import numpy as np
import pytest

from paper_2306_15685_amd import synth, runner
from paper_2306_15685_amd import binding as B

import gpu_harness as GH
import helpers as H
from oracle import OracleGraph, OracleChannel

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    return torch


@pytest.fixture(scope="module")
def big_graph():
    """The 10M-state graph shared by the large, dynamic and stress workloads (same seed stream)."""
    w = synth.WORKLOADS["large"]
    g = synth.make_graph(w.num_states, w.num_pdfs, w.num_words, w.eps_prob, seed_stream=(w.config_id,),
                         mean_degree=w.mean_degree, word_frac=w.word_frac)
    return g, OracleGraph.from_graph(g)


def check_workload(torch, w, g, og, sample, prop_channels, graph_handle=None):
    inp = runner.make_inputs(w, g)
    sess = runner.Session(inp, graph_handle=graph_handle)
    try:
        finals = sess.step(keep_results=True, collect_stats=False)
        partials = sess.partials
        n_seg = w.segments
        assert len(finals) == n_seg
        # --- sampled channels against the checker: every chunk's partial result, the final one, counters
        for c in sample:
            ch = OracleChannel(og, w.beam, w.max_active)
            for s in range(n_seg):
                lists, offs = inp.contexts[s]
                ch.set_context(lists[c], offs[c])
                ch.reset()
                Lh = inp.loglikes[s][c].cpu().numpy()
                t = 0
                while t < w.frames:
                    n = min(w.chunk, w.frames - t)
                    ch.advance(Lh[t:t + n])
                    t += n
                    if w.partial_every_chunk and t < w.frames:
                        st, wl, al, cost, na, nw = next(r for (ss, tt, r) in partials if ss == s and tt == t)
                        GH.assert_best_equal((int(st[c]), wl[c], al[c], float(cost[c])), ch.best_path(False),
                                             f"{w.name} seg {s} ch {c} partial t={t}")
                st, wl, al, cost, na, nw = finals[s]
                GH.assert_best_equal((int(st[c]), wl[c], al[c], float(cost[c])), ch.best_path(True),
                                     f"{w.name} seg {s} ch {c} final")
            stc = sess.stats(c)   # counters of the last segment
            assert stc["emit_arcs"] == ch.emit_arcs and stc["tokens"] == ch.stat(1), f"{w.name} ch {c} counters"
            assert stc["active_tokens"] == ch.stat(2) and stc["max_tokens"] == ch.stat(3)
        # --- properties on many channels
        for s in range(n_seg if n_seg <= 2 else 2):
            lists, offs = inp.contexts[s]
            st, wl, al, cost, na, nw = finals[s]
            assert (st == 0).all(), f"{w.name}: channel in error state {st[st != 0][:4]}"
            for c in prop_channels:
                Lh = inp.loglikes[s][c].cpu().numpy()
                ctx = set(lists[c].tolist())
                c2, frames, words2, end = H.rescore_path(g, al[c], Lh, lambda t: ctx, lambda t: float(offs[c]))
                assert frames == w.frames, f"{w.name} ch {c}: path consumes {frames} frames"
                assert np.float32(cost[c]) == c2, f"{w.name} ch {c}: cost {cost[c]} vs re-scored {c2}"
                assert wl[c].tolist() == words2, f"{w.name} ch {c}: words are not the path's labels"
        total = sess.stats(-1)
        return total
    finally:
        sess.close()


def test_medium_all_channels(torch_cuda):
    w = synth.WORKLOADS["medium"]
    g = synth.graph_for(w)
    og = OracleGraph.from_graph(g)
    check_workload(torch_cuda, w, g, og, sample=range(w.channels), prop_channels=range(w.channels))


def test_e2e_units_lexicon_loop(torch_cuda):
    """Second workload: 64 channels over a 20,000-word lexicon loop of end-to-end units."""
    w = synth.WORKLOADS["e2e"]
    g = synth.graph_for(w)
    og = OracleGraph.from_graph(g)
    total = check_workload(torch_cuda, w, g, og, sample=[0, 31, 63], prop_channels=range(0, w.channels, 8))
    assert total["max_tokens"] > 2500   # far denser token activity than the HCLG-style workloads


@pytest.mark.timeout(900)
def test_large_online(torch_cuda, big_graph):
    g, og = big_graph
    w = synth.WORKLOADS["large"]
    rng = np.random.default_rng(1)
    sample = [0, w.channels - 1] + rng.choice(w.channels, 6, replace=False).tolist()
    total = check_workload(torch_cuda, w, g, og, sample=sample, prop_channels=range(0, w.channels, 4))
    assert total["slow_frames"] < total["frames"] // 100   # LDS tables carry the workload, the fallback is rare


@pytest.mark.timeout(900)
def test_dynamic_context_switching(torch_cuda, big_graph):
    """512 channels, 20 utterances each with a fresh context per channel (fewer channels are
    sampled for the checker because each costs 20 utterances)."""
    g, og = big_graph
    w = synth.WORKLOADS["dynamic"]
    check_workload(torch_cuda, w, g, og, sample=[0, 257, w.channels - 1], prop_channels=range(0, w.channels, 16))


@pytest.mark.timeout(900)
def test_throughput_stress(torch_cuda, big_graph):
    g, og = big_graph
    w = synth.WORKLOADS["stress"]
    rng = np.random.default_rng(2)
    sample = [0, w.channels - 1] + rng.choice(w.channels, 4, replace=False).tolist()
    check_workload(torch_cuda, w, g, og, sample=sample, prop_channels=range(0, w.channels, 64))


@pytest.mark.timeout(600)
def test_three_minute_utterance(torch_cuda):
    """Sec. 5.3 decodes 3-minute recordings: 6000 frames of 30 ms in one utterance, in 50-frame chunks, with a
    partial result now and then.  All back-pointer records of the utterance stay in device memory (no
    garbage collection is needed at these sizes), so this checks record indices and the long traceback."""
    torch = torch_cuda
    w = synth.scaled(synth.WORKLOADS["medium"], channels=4, frames=6000, chunk=50, config_id=62)
    g = synth.graph_for(synth.WORKLOADS["medium"])
    og = OracleGraph.from_graph(g)
    L = synth.make_loglikes(w.channels, w.frames, w.num_pdfs, w.sigma, seed_stream=(62,), device="cuda")
    ctxs, offs = synth.make_contexts(w, g)
    dec = GH.GpuDecoder(g, w.channels, w.beam, w.max_active, max_frames=w.frames, records_per_frame=1024,
                        max_context_arcs=max(len(x) for x in ctxs))
    try:
        orcs = GH.oracle_channels(g, 2, w.beam, w.max_active, og=og)
        Lh = L[:2].cpu().numpy()
        dec.set_contexts(ctxs, offs)
        dec.reset()
        for c in range(2):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        for t in range(0, w.frames, w.chunk):
            dec.advance(L, t, t + w.chunk)
            for c in range(2):
                orcs[c].advance(Lh[c, t:t + w.chunk])
            if (t // w.chunk) % 40 == 39:
                for c in range(2):
                    GH.assert_best_equal(dec.best(c), orcs[c].best_path(False), f"partial at frame {t + w.chunk} ch {c}")
        for c in range(2):
            rc, words, arcs, cost = dec.best(c, True)
            GH.assert_best_equal((rc, words, arcs, cost), orcs[c].best_path(True), f"final ch {c}")
            assert len(arcs) >= w.frames
        st = dec.stats(-1)
        assert st["status"] == 0 and st["frames"] == w.channels * w.frames
    finally:
        dec.close()
