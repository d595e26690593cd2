"""Full-size parity: the benchmark workloads in the launch configuration bench.py times
(runner.Session.step), on the graphs bench.py builds, with EVERY channel of every segment checked
against the CPU checker (each partial result, the final result, the counters).  On some channels the
results are also checked by properties that need no checker: the returned arc path is connected from
the start state, consumes exactly the decoded frames, re-accumulating its cost in fp32 in path order
gives the returned cost bit for bit, and the words are the path's output labels."""
import os
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2306_15685_amd import synth, runner
from paper_2306_15685_amd import binding as B

import gpu_harness as GH
import helpers as H
from oracle import OracleGraph, OracleChannel
from oracle import word_arcs as oracle_word_arcs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    return torch


@pytest.fixture(scope="module")
def big_graph():
    """The 10M-state graph that the large, dynamic and stress workloads share (bench.py builds the same one)."""
    w = synth.WORKLOADS["large"]
    g = synth.graph_for(w)
    for other in ("dynamic", "stress"):
        assert synth.WORKLOADS[other].graph_id == w.config_id
    return g, OracleGraph.from_graph(g)


def oracle_workers():
    return max(1, min(16, len(os.sched_getaffinity(0))))


def check_workload(torch, w, g, og, prop_channels, graph_handle=None, **session_kw):
    """Every channel of every segment against the checker: each chunk's partial result, the final result and (for
    the last segment) the counters.  The checker's channels run on a pool of host threads, one checker object per
    thread, reused from channel to channel (ctypes releases the interpreter lock during the calls)."""
    inp = runner.make_inputs(w, g)
    sess = runner.Session(inp, graph_handle=graph_handle, **session_kw)
    try:
        n_seg = w.segments
        if inp.sequences is not None:
            # the lists were made by the library from word sequences (Algorithm 1): the checker's own Algorithm 1
            # must select the same arcs for every channel, and its lists are the ones its decoding then uses
            checked = []
            with ThreadPoolExecutor(max_workers=oracle_workers()) as ex:
                for s in range(n_seg):
                    per_channel, offs = inp.sequences[s]
                    want = list(ex.map(lambda seqs: oracle_word_arcs.arcs_for_sequences(g, seqs), per_channel))
                    got, offs2 = inp.contexts[s]
                    assert np.array_equal(offs, offs2)
                    for c in range(w.channels):
                        assert np.array_equal(np.sort(got[c]), want[c]), f"{w.name} seg {s} ch {c}: Algorithm 1 arcs"
                    checked.append((want, offs))
            sizes = [x.size for want, _ in checked for x in want]
            print(f"{w.name}: {len(sizes)} arc lists from word sequences equal to the checker's "
                  f"({min(sizes)}-{max(sizes)} arcs)", flush=True)
            assert min(sizes) > 0 and any(len(q) > 1 for seqs in inp.sequences[0][0] for q in seqs)
            oracle_contexts = checked
        else:
            oracle_contexts = inp.contexts
        finals = sess.step(keep_results=True, collect_stats=False)
        partials = {(ss, tt): r for (ss, tt, r) in sess.partials}
        assert len(finals) == n_seg
        tls = threading.local()
        last_counters = {}

        def one_channel(s, c, Lh, lists, offs):
            ch = getattr(tls, "ch", None)
            if ch is None:
                ch = tls.ch = OracleChannel(og, w.beam, w.max_active)
            ch.set_context(lists[c], offs[c])
            ch.reset()
            t = 0
            while t < w.frames:
                n = min(w.chunk, w.frames - t)
                ch.advance(Lh[c, t:t + n])
                t += n
                if w.partial_every_chunk and t < w.frames:
                    st, wl, al, cost, na, nw = partials[(s, t)]
                    GH.assert_best_equal((int(st[c]), wl[c], al[c], float(cost[c])), ch.best_path(False),
                                         f"{w.name} seg {s} ch {c} partial t={t}")
            st, wl, al, cost, na, nw = finals[s]
            GH.assert_best_equal((int(st[c]), wl[c], al[c], float(cost[c])), ch.best_path(True),
                                 f"{w.name} seg {s} ch {c} final")
            if s == n_seg - 1:
                last_counters[c] = (ch.emit_arcs, ch.stat(1), ch.stat(2), ch.stat(3))
            return c

        with ThreadPoolExecutor(max_workers=oracle_workers()) as ex:
            for s in range(n_seg):
                lists, offs = oracle_contexts[s]
                Lh = inp.loglikes[s].cpu().numpy()
                done = list(ex.map(lambda c: one_channel(s, c, Lh, lists, offs), range(w.channels)))
                assert len(done) == w.channels
                del Lh
                print(f"{w.name}: segment {s + 1}/{n_seg}: {w.channels} channels equal to the checker", flush=True)
        for c in range(w.channels):   # counters of the last segment
            stc = sess.stats(c)
            emit, toks, act, mx = last_counters[c]
            assert stc["emit_arcs"] == emit and stc["tokens"] == toks, f"{w.name} ch {c} counters"
            assert stc["active_tokens"] == act and stc["max_tokens"] == mx, f"{w.name} ch {c} counters"
        # --- extra, on some channels: properties that need no checker
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
    check_workload(torch_cuda, w, g, og, prop_channels=range(w.channels))


@pytest.mark.parametrize("team", [1, 4])
def test_e2e_units_lexicon_loop(torch_cuda, team):
    """Second workload: 64 channels over a 20,000-word lexicon loop of end-to-end units, decoded by one workgroup
    per channel (tables in device memory) and by teams of four (tables in the members' LDS)."""
    w = synth.WORKLOADS["e2e"]
    g = synth.graph_for(w)
    og = OracleGraph.from_graph(g)
    total = check_workload(torch_cuda, w, g, og, prop_channels=range(0, w.channels, 8), workgroups_per_channel=team)
    assert total["max_tokens"] > 2500   # far denser token activity than the HCLG-style workloads


@pytest.mark.timeout(600)
def test_word_sequence_contexts(torch_cuda):
    """Sec. 4.1 end to end: every channel's biasing list is given as word sequences, the library's Algorithm 1
    turns them into arc lists (checked against the checker's Algorithm 1, list by list), and the decoding with
    them is checked on every channel.  The graph keeps word labels four arcs apart (see synth.make_graph)."""
    w = synth.WORKLOADS["words"]
    g = synth.graph_for(w)
    og = OracleGraph.from_graph(g)
    total = check_workload(torch_cuda, w, g, og, prop_channels=range(0, w.channels, 16))
    assert total["frames"] == w.channels * w.frames


@pytest.mark.timeout(900)
def test_large_online(torch_cuda, big_graph):
    g, og = big_graph
    w = synth.WORKLOADS["large"]
    total = check_workload(torch_cuda, w, g, og, prop_channels=range(0, w.channels, 16))
    assert total["slow_frames"] < total["frames"] // 100   # LDS tables carry the workload, the fallback is rare


@pytest.mark.timeout(900)
def test_dynamic_context_switching(torch_cuda, big_graph):
    """512 channels, 20 utterances each with a fresh context per channel."""
    g, og = big_graph
    w = synth.WORKLOADS["dynamic"]
    check_workload(torch_cuda, w, g, og, prop_channels=range(0, w.channels, 64))


@pytest.mark.timeout(900)
def test_throughput_stress(torch_cuda, big_graph):
    g, og = big_graph
    w = synth.WORKLOADS["stress"]
    check_workload(torch_cuda, w, g, og, prop_channels=range(0, w.channels, 256))


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
