"""Compaction of the back-pointer records on the GPU.  Partial and final results are read off the best current
token's sequence (Sec. 1, Sec. 3.2), so records that no current token has on its path can be dropped; this is
what lets utterances as long as the 3-minute recordings of Sec. 5.3 run in a small record buffer.  Checked two
ways: the records after a compaction equal a mark-and-renumber written out here in numpy on the records
downloaded before it (bit-exact), and decoding with compactions gives the CPU checker's partial and final
results throughout."""
import numpy as np
import pytest

from paper_2306_15685_amd import synth
from paper_2306_15685_amd import binding as B

import gpu_harness as GH
from oracle import OracleGraph

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    torch.cuda.set_device(0)
    return torch


def inputs(C, T, S=60_000, P=500, seed=31, finals=False, eps=0.10):
    g = synth.make_graph(S, P, 2000, eps, seed_stream=(seed,), with_finals=finals)
    L = synth.make_loglikes(C, T, P, 4.0, seed_stream=(seed,), device="cuda")
    w = synth.scaled(synth.WORKLOADS["large"], channels=C, ctx_min=30, ctx_max=60, config_id=80 + seed)
    ctxs, offs = synth.make_contexts(w, g)
    return g, L, ctxs, offs


def mark_and_renumber(arcs, prev, fb, kept_base, live):
    """What a compaction must leave.  Records below kept_base (the beginning all paths share, as found before) and
    the current frame's (from fb on) stay; of the others, those on a predecessor chain from a live current token.
    Kept records keep their order.  kept_base then moves up past the marked records below the highest place, a
    multiple of 32 records above the old kept_base, that exactly one marked link crosses.
    -> (arcs, prev, frame_base, n_records, kept_base) after the compaction, and which records were kept."""
    n = arcs.size
    young = fb - kept_base
    keep = np.zeros(n, bool)
    keep[:kept_base] = True
    keep[fb:] = True
    links = []     # (lower end, upper end) of every marked link, relative to kept_base; -1 = below it
    for i in np.nonzero(live)[0]:
        q = prev[fb + i]
        if q < fb:
            links.append((max(q - kept_base, -1), young))
        while kept_base <= q < fb and not keep[q]:
            keep[q] = True
            links.append(tuple(sorted((max(prev[q] - kept_base, -1), q - kept_base))))
            q = prev[q]
    new = np.cumsum(keep) - 1
    p = prev[keep]
    safe = np.maximum(p, 0)
    new_prev = np.where((p >= 0) & keep[safe], new[safe], -1).astype(np.int32)
    new_kept = kept_base
    for b in range(young // 32, -1, -1):
        if sum(1 for lo, hi in links if lo < 32 * b <= hi) == 1:
            new_kept = kept_base + int(keep[kept_base:kept_base + 32 * b].sum())
            break
    return arcs[keep], new_prev, int(new[fb]), int(keep.sum()), new_kept, keep


def top_of_chain(prev, kb):
    """The record below kb that no other record below kb points at."""
    pointed = set(int(x) for x in prev[:kb] if x >= 0)
    tops = [i for i in range(kb) if i not in pointed]
    assert len(tops) == 1
    return tops[0]


def is_one_chain(prev, kb):
    """Records [0, kb) form a single predecessor chain ending at the start record."""
    q, seen = top_of_chain(prev, kb), 0
    while q >= 0:
        assert q < kb
        seen += 1
        q = int(prev[q])
    return seen == kb


def live_mask(dec, c, arcs, fb):
    """Which of the current frame's records belong to tokens the frame cutoff has not dropped (within a frame an
    arc names its token: it leads to one state, and a state has one token)."""
    rc, st, co, ar = dec.tokens(c)
    assert rc == 0
    return np.isin(arcs[fb:], ar)


@pytest.mark.parametrize("table_location", [1, 2])
def test_records_after_compaction_equal_mark_and_renumber(torch_cuda, table_location):
    """Exact contents of the record buffer after the first compaction (nothing kept from before), after later ones
    (an older generation in place), and after one that finds nothing to drop."""
    C, T = 3, 60
    g, L, ctxs, offs = inputs(C, T)
    dec = GH.GpuDecoder(g, C, 12.0, 300, max_frames=T, table_location=table_location)
    try:
        dec.set_contexts(ctxs, offs)
        dec.reset()
        dropped = 0
        for k, (t0, t1) in enumerate([(0, 1), (1, 13), (13, 14), (14, 40), (40, 60)]):
            dec.advance(L, t0, t1)
            for c in range(C):
                arcs, prev, fb, kb = dec.records(c)
                want = mark_and_renumber(arcs, prev, fb, kb, live_mask(dec, c, arcs, fb))
                dec.compact(np.array([c], np.int32))
                arcs2, prev2, fb2, kb2 = dec.records(c)
                assert np.array_equal(arcs2, want[0]) and np.array_equal(prev2, want[1]), f"chunk {k} ch {c}"
                assert fb2 == want[2] and arcs2.size == want[3] and kb2 == want[4], f"chunk {k} ch {c}"
                # what lies below the new base is one chain, and every live token's path runs into it
                if kb2 > 0:
                    assert np.all(prev2[1:kb2] == np.arange(kb2 - 1)) or is_one_chain(prev2, kb2)
                    for i in np.nonzero(live_mask(dec, c, arcs2, fb2))[0]:
                        q = fb2 + i
                        while q >= kb2:
                            q = prev2[q]
                        assert q == top_of_chain(prev2, kb2), f"chunk {k} ch {c} token {i}"
                dropped += arcs.size - arcs2.size
                # a second call right away has nothing younger than what the first one kept
                dec.compact(np.array([c], np.int32))
                arcs3, prev3, fb3, kb3 = dec.records(c)
                assert np.array_equal(arcs3, arcs2) and np.array_equal(prev3, prev2) and fb3 == fb2 and kb3 >= kb2
        st = dec.stats(-1)
        assert st["records_dropped"] == dropped > 0 and st["status"] == 0
    finally:
        dec.close()


def test_results_with_compaction_every_chunk(torch_cuda):
    """Channels 0 and 2 are compacted after every chunk, 1 and 3 never: every partial result, the final result
    (with final costs) and the final token tables agree with the checker on all four."""
    torch = torch_cuda
    C, T, chunk = 4, 240, 8
    g, L, ctxs, offs = inputs(C, T, seed=32, finals=True)
    Lh = L.cpu().numpy()
    dec = GH.GpuDecoder(g, C, 12.0, 250, max_frames=T)
    some = np.array([0, 2], np.int32)
    try:
        og = OracleGraph.from_graph(g)
        orcs = GH.oracle_channels(g, C, 12.0, 250, og=og)
        dec.set_contexts(ctxs, offs)
        dec.reset()
        dec.compact()     # right after the start of the utterance: only the start token's closure exists
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        for t in range(0, T, chunk):
            dec.advance(L, t, t + chunk)
            dec.compact(some)
            for c in range(C):
                orcs[c].advance(Lh[c, t:t + chunk])
            st, wl, al, cost, na, nw = B.cbd_best_paths(dec.dh, dec.all, False, capacity=4 * T + 16)
            for c in range(C):
                GH.assert_best_equal((int(st[c]), wl[c], al[c], float(cost[c])), orcs[c].best_path(False),
                                     f"partial t={t + chunk} ch={c}")
        for c in range(C):
            GH.assert_tables_equal(dec.tokens(c), orcs[c].tokens(), f"final table ch={c}")
            GH.assert_best_equal(dec.best(c, True), orcs[c].best_path(True), f"final ch={c}")
        s0, s1 = dec.stats(0), dec.stats(1)
        assert s0["compactions"] >= T // chunk - 1 and s1["compactions"] == 0
        assert s0["records"] < s1["records"] // 10      # most records are on no current token's path
    finally:
        dec.close()


def test_long_utterance_in_a_small_record_buffer(torch_cuda):
    """Sec. 5.3's recordings are 3 minutes long: 6000 frames of 30 ms.  The record buffer here has room for about
    330 frames; with automatic compaction the utterance decodes to the checker's result, without it the channel
    stops with a capacity error."""
    torch = torch_cuda
    T, chunk, C = 6000, 50, 2
    w = synth.scaled(synth.WORKLOADS["medium"], channels=C, frames=T, chunk=chunk, config_id=63)
    g = synth.graph_for(synth.WORKLOADS["medium"])
    og = OracleGraph.from_graph(g)
    L = synth.make_loglikes(C, T, w.num_pdfs, w.sigma, seed_stream=(63,), device="cuda")
    Lh = L.cpu().numpy()
    ctxs, offs = synth.make_contexts(w, g)
    kw = dict(max_frames=100, records_per_frame=512, max_context_arcs=max(len(x) for x in ctxs))
    capacity = 512 * 101 + 2048      # records per channel (the decoder's sizing rule with hash_log2 = 12)
    dec = GH.GpuDecoder(g, C, w.beam, w.max_active, compact_records_above=20_000, **kw)
    plain = GH.GpuDecoder(g, C, w.beam, w.max_active, graph_handle=dec.gh, **kw)
    try:
        orcs = GH.oracle_channels(g, C, w.beam, w.max_active, og=og)
        for d in (dec, plain):
            d.set_contexts(ctxs, offs)
            d.reset()
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        for t in range(0, T, chunk):
            dec.advance(L, t, t + chunk)
            plain.advance(L, t, t + chunk)
            for c in range(C):
                orcs[c].advance(Lh[c, t:t + chunk])
            if (t // chunk) % 30 == 29:
                for c in range(C):
                    GH.assert_best_equal(dec.best(c), orcs[c].best_path(False), f"partial at frame {t + chunk} ch {c}")
        for c in range(C):
            rc, words, arcs, cost = dec.best(c, True)
            GH.assert_best_equal((rc, words, arcs, cost), orcs[c].best_path(True), f"final ch {c}")
            assert len(arcs) >= T
            s = dec.stats(c)
            assert s["status"] == 0 and s["frames"] == T and s["compactions"] >= 20
            assert s["records"] < capacity < (s["records"] + s["records_dropped"]) // 8
            # nearly all of the best path lies in the part all paths share, which no compaction looks at again
            _, _, fb, kb = dec.records(c)
            assert kb > 0.9 * len(arcs) and fb - kb < 25_000
            assert plain.best(c)[0] == B.CBD_E_CAPACITY
    finally:
        plain.close()
        dec.close()


def test_compaction_beside_asynchronous_requests_and_parked_channels(torch_cuda):
    """A request begun before a compaction still delivers the result of its own moment (the compaction waits for
    its walk); a request begun after one takes a fresh snapshot; channels in an error state are left alone."""
    torch = torch_cuda
    C, T = 3, 90
    g, L, ctxs, offs = inputs(C, T, seed=33)
    Lh = L.cpu().numpy()
    dec = GH.GpuDecoder(g, C, 12.0, 300, max_frames=T)
    try:
        og = OracleGraph.from_graph(g)
        orcs = GH.oracle_channels(g, C, 12.0, 300, og=og)
        dec.set_contexts(ctxs, offs)
        dec.reset()
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        for t in range(0, T, 30):
            dec.advance(L, t, t + 30)
            for c in range(C):
                orcs[c].advance(Lh[c, t:t + 30])
            t1 = B.cbd_best_paths_begin(dec.dh, dec.all, False, capacity=4 * T)    # walks from the call's own snapshot
            dec.compact()
            t2 = B.cbd_best_paths_begin(dec.dh, dec.all, False, capacity=4 * T)    # after the renumbering
            for tk in (t1, t2):
                st, wl, al, cost, na, nw = B.cbd_best_paths_finish(dec.dh, tk)
                for c in range(C):
                    GH.assert_best_equal((int(st[c]), wl[c], al[c], float(cost[c])), orcs[c].best_path(False),
                                         f"t={t + 30} ticket {tk} ch {c}")
        assert dec.stats(-1)["compactions"] == 3 * C
    finally:
        dec.close()
    # a channel whose record buffer ran full is parked; compacting it is a no-op and the others go on
    small = GH.GpuDecoder(g, C, 12.0, 300, max_frames=4, records_per_frame=64, hash_log2=10)
    try:
        small.set_contexts(ctxs, offs)
        small.reset()
        small.advance(L, 0, 60)
        assert small.best(0)[0] == B.CBD_E_CAPACITY
        before = small.stats(0)
        small.compact()
        after = small.stats(0)
        assert after["compactions"] == 0 and after["records"] == before["records"]
        assert small.best(0)[0] == B.CBD_E_CAPACITY
    finally:
        small.close()


def test_tails_plus_fixed_part_are_the_whole_results(torch_cuda):
    """Results in two parts (Sec. 1 / 3.2: the intermediate result is the best current token's sequence): what the
    compactions have found to be common to all paths, kept by the library in time order, and the rest of the best
    path.  Put together they must be the checker's partial result at every chunk, for channels that are compacted
    every chunk, sometimes, or never; the fixed part only ever grows; requests begun before a compaction are put
    together with the fixed part as it was then."""
    torch = torch_cuda
    C, T, chunk = 4, 400, 10
    g, L, ctxs, offs = inputs(C, T, seed=34, finals=True)
    Lh = L.cpu().numpy()
    dec = GH.GpuDecoder(g, C, 12.0, 250, max_frames=T)
    try:
        og = OracleGraph.from_graph(g)
        orcs = GH.oracle_channels(g, C, 12.0, 250, og=og)
        dec.set_contexts(ctxs, offs)
        dec.reset()
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        fixed = [(np.zeros(0, np.int32), np.zeros(0, np.int32)) for _ in range(C)]

        def whole(c, res, i=None):
            st, wl, al, cost, na, nw, nfw, nfa = res
            i = c if i is None else i
            fw, fa = fixed[c]
            assert nfw[i] <= fw.size and nfa[i] <= fa.size
            return (int(st[i]), np.concatenate([fw[:nfw[i]], wl[i]]), np.concatenate([fa[:nfa[i]], al[i]]), float(cost[i]))

        for k, t in enumerate(range(0, T, chunk)):
            dec.advance(L, t, t + chunk)
            for c in range(C):
                orcs[c].advance(Lh[c, t:t + chunk])
            ticket = B.cbd_best_tails_begin(dec.dh, dec.all, False, capacity=4 * T)   # before this chunk's compaction
            dec.compact(np.array([0], np.int32))
            if k % 7 == 3:
                dec.compact(np.array([2, 3], np.int32))
            for c in range(C):     # the fixed part only grows
                fw, fa = B.cbd_get_fixed(dec.dh, c)
                assert np.array_equal(fw[:fixed[c][0].size], fixed[c][0]) and np.array_equal(fa[:fixed[c][1].size], fixed[c][1])
                more_w, more_a = B.cbd_get_fixed(dec.dh, c, fixed[c][0].size, fixed[c][1].size)   # asking for the rest only
                assert np.array_equal(np.concatenate([fixed[c][0], more_w]), fw)
                assert np.array_equal(np.concatenate([fixed[c][1], more_a]), fa)
                fixed[c] = (fw, fa)
            before = B.cbd_best_tails_finish(dec.dh, ticket)
            after = B.cbd_best_tails(dec.dh, dec.all, False, capacity=4 * T)
            for c in range(C):
                want = orcs[c].best_path(False)
                GH.assert_best_equal(whole(c, before), want, f"t={t + chunk} ch={c} begun before the compaction")
                GH.assert_best_equal(whole(c, after), want, f"t={t + chunk} ch={c} after the compaction")
        final = B.cbd_best_tails(dec.dh, dec.all, True, capacity=4 * T)
        for c in range(C):
            GH.assert_best_equal(whole(c, final), orcs[c].best_path(True), f"final ch={c}")
            GH.assert_best_equal(dec.best(c, True), orcs[c].best_path(True), f"final ch={c}, whole path")
        st, wl, al, cost, na, nw, nfw, nfa = final
        assert nfa[1] == 0 and na[1] >= T                # never compacted: nothing fixed, the tail is the path
        assert nfa[0] > 0.9 * (nfa[0] + na[0])           # compacted every chunk: the tail is what is still open
        assert 0 < nfa[2] and nfa[3] > 0
        # a new utterance starts with an empty fixed part
        dec.reset(np.array([0], np.int32))
        assert B.cbd_get_fixed(dec.dh, 0)[1].size == 0 and B.cbd_get_fixed(dec.dh, 2)[1].size == nfa[2]
    finally:
        dec.close()


def check_one_compaction(dec, c, where):
    arcs, prev, fb, kb = dec.records(c)
    want = mark_and_renumber(arcs, prev, fb, kb, live_mask(dec, c, arcs, fb))
    dec.compact(np.array([c], np.int32))
    arcs2, prev2, fb2, kb2 = dec.records(c)
    assert np.array_equal(arcs2, want[0]) and np.array_equal(prev2, want[1]), where
    assert fb2 == want[2] and arcs2.size == want[3] and kb2 == want[4], where
    # (also: the most records kept within one stretch of 32,768 examined records, the unit the kernel moves by)
    per_stretch = np.add.reduceat(want[5][kb:fb].astype(np.int64), np.arange(0, fb - kb, 32768)) if fb > kb else np.zeros(1)
    return arcs.size, arcs2.size, kb2 - kb, int(per_stretch.max())


def test_compaction_of_a_long_stretch(torch_cuda):
    """One compaction after 4,500 frames: more records than the bitmap the kernel keeps in LDS covers (524,288), and
    a shared beginning longer than what it stages in LDS (4,096 records); then results in two parts."""
    torch = torch_cuda
    T, C = 4500, 2
    w = synth.scaled(synth.WORKLOADS["medium"], channels=C, frames=T, chunk=250, config_id=64)
    g = synth.graph_for(synth.WORKLOADS["medium"])
    og = OracleGraph.from_graph(g)
    L = synth.make_loglikes(C, T, w.num_pdfs, w.sigma, seed_stream=(64,), device="cuda")
    Lh = L.cpu().numpy()
    ctxs, offs = synth.make_contexts(w, g)
    dec = GH.GpuDecoder(g, C, w.beam, w.max_active, max_frames=T, records_per_frame=512,
                        max_context_arcs=max(len(x) for x in ctxs))
    try:
        orcs = GH.oracle_channels(g, C, w.beam, w.max_active, og=og)
        dec.set_contexts(ctxs, offs)
        dec.reset()
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset(); orcs[c].advance(Lh[c])
        for t in range(0, T, w.chunk):
            dec.advance(L, t, t + w.chunk)
        for c in range(C):
            before, after, fixed, _ = check_one_compaction(dec, c, f"ch {c}")
            assert before > 524_288 + 1000 and fixed > 4096 and after < before // 50
        st, wl, al, cost, na, nw, nfw, nfa = B.cbd_best_tails(dec.dh, dec.all, True, capacity=8 * T)
        for c in range(C):
            fw, fa = B.cbd_get_fixed(dec.dh, c)
            assert fa.size == nfa[c] > 4096 and fw.size == nfw[c]
            GH.assert_best_equal((int(st[c]), np.concatenate([fw, wl[c]]), np.concatenate([fa, al[c]]), float(cost[c])),
                                 orcs[c].best_path(True), f"two parts ch {c}")
            GH.assert_best_equal(dec.best(c, True), orcs[c].best_path(True), f"whole path ch {c}")
    finally:
        dec.close()


def test_compaction_of_dense_records(torch_cuda):
    """Flat log-likelihoods and a wide beam: thousands of tokens per frame, and after a dozen frames more records
    of one stretch of the bitmap are still on some token's path than the kernel stages in LDS at a time (4,096)."""
    torch = torch_cuda
    T = 12
    g = synth.make_graph(1_000_000, 500, 2000, 0.10, seed_stream=(41,))
    L = synth.make_loglikes(1, T + 6, 500, 0.5, seed_stream=(41,), device="cuda")
    Lh = L.cpu().numpy()
    dec = GH.GpuDecoder(g, 1, 16.0, 5000, max_frames=T + 6, hash_log2=16, max_context_arcs=4)
    try:
        orc = GH.oracle_channels(g, 1, 16.0, 5000)[0]
        dec.set_contexts([np.zeros(0, np.int32)], [0.0])
        orc.set_context(np.zeros(0, np.int32), 0.0)
        dec.reset(); orc.reset()
        dec.advance(L, 0, T); orc.advance(Lh[0, :T])
        before, after, _, densest = check_one_compaction(dec, 0, "first")
        assert densest > 4096 and before > 2 * 32768
        GH.assert_best_equal(dec.best(0), orc.best_path(False), "after the first compaction")
        dec.advance(L, T, T + 6); orc.advance(Lh[0, T:])
        check_one_compaction(dec, 0, "second")
        GH.assert_best_equal(dec.best(0), orc.best_path(False), "after the second compaction")
        GH.assert_tables_equal(dec.tokens(0), orc.tokens(), "final table")
    finally:
        dec.close()


@pytest.mark.parametrize("seed", [1, 2])
def test_random_schedules(torch_cuda, seed):
    """Seeded random interleaving of everything that touches the records: chunks of 1-17 frames on changing channel
    subsets, compactions of random subsets with random thresholds, new utterances and context changes on single
    channels in between, results asked for whole, in two parts, synchronously and asynchronously.  Every result
    must be the checker's."""
    torch = torch_cuda
    rng = np.random.default_rng(1000 + seed)
    C, T = 6, 260
    g, L, ctxs, offs = inputs(C, T, seed=40 + seed, finals=True)
    Lh = L.cpu().numpy()
    spare, spare_offs = synth.make_contexts(
        synth.scaled(synth.WORKLOADS["large"], channels=C, ctx_min=30, ctx_max=60, config_id=90 + seed), g)
    dec = GH.GpuDecoder(g, C, 12.0, 250, max_frames=T)
    try:
        og = OracleGraph.from_graph(g)
        orcs = GH.oracle_channels(g, C, 12.0, 250, og=og)
        dec.set_contexts(ctxs, offs)
        dec.reset()
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        pos = [0] * C        # frames of L each channel has consumed (its utterance may have restarted since)

        def check(c, res, i, where):
            st, wl, al, cost, na, nw, nfw, nfa = res
            fw, fa = B.cbd_get_fixed(dec.dh, c)
            got = (int(st[i]), np.concatenate([fw[:nfw[i]], wl[i]]), np.concatenate([fa[:nfa[i]], al[i]]), float(cost[i]))
            GH.assert_best_equal(got, orcs[c].best_path(False), where)

        for step in range(60):
            subset = np.sort(rng.choice(C, size=rng.integers(1, C + 1), replace=False)).astype(np.int32)
            n = int(rng.integers(1, 18))
            subset = np.array([c for c in subset if pos[c] + n <= T], np.int32)
            if subset.size == 0:
                break
            # the rows of a call are consecutive in memory: gather this call's frames of the chosen channels
            rows = torch.stack([L[c, pos[c]:pos[c] + n] for c in subset]).contiguous()
            B.cbd_advance(dec.dh, subset, rows.data_ptr(), n * rows.shape[2], n)
            for c in subset:
                orcs[c].advance(Lh[c, pos[c]:pos[c] + n]); pos[c] += n
            ticket = None
            if rng.random() < 0.5:
                ticket = (B.cbd_best_tails_begin(dec.dh, subset, False, capacity=4 * T), subset.copy())
            if rng.random() < 0.6:
                who = np.sort(rng.choice(C, size=rng.integers(1, C + 1), replace=False)).astype(np.int32)
                dec.compact(who, int(rng.choice([0, 0, 300, 3000])))
            if ticket is not None:
                res = B.cbd_best_tails_finish(dec.dh, ticket[0])
                for i, c in enumerate(ticket[1]):
                    check(int(c), res, i, f"seed {seed} step {step} ch {c} (begun before)")
            res = B.cbd_best_tails(dec.dh, dec.all, False, capacity=4 * T)
            for c in range(C):
                check(c, res, c, f"seed {seed} step {step} ch {c}")
            if rng.random() < 0.3:
                c = int(rng.integers(C))
                GH.assert_best_equal(dec.best(c, True), orcs[c].best_path(True), f"seed {seed} step {step} ch {c} whole, final")
            if rng.random() < 0.15:      # a new utterance on one channel, with another context
                c = int(rng.integers(C))
                dec.set_contexts([spare[c]], [spare_offs[c]], np.array([c], np.int32))
                orcs[c].set_context(spare[c], spare_offs[c])
                dec.reset(np.array([c], np.int32)); orcs[c].reset()
            elif rng.random() < 0.15:    # a context change in mid-utterance
                c = int(rng.integers(C))
                dec.set_contexts([ctxs[(c + 1) % C]], [offs[(c + 1) % C]], np.array([c], np.int32))
                orcs[c].set_context(ctxs[(c + 1) % C], offs[(c + 1) % C])
        assert dec.stats(-1)["status"] == 0 and dec.stats(-1)["compactions"] > 10
    finally:
        dec.close()
