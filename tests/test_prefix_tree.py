"""Host-side session prefix tree against brute force (CPU only, no kernel is launched)."""
import numpy as np
import pytest

from paper_2508_11553_amd.prefix_tree import PrefixTree


def lcp(a, b):
    n = min(len(a), len(b))
    i = 0
    while i < n and a[i] == b[i]:
        i += 1
    return i


def random_session(rng, nbranch, base_len, vocab=50):
    """Branches that continue random cut points of earlier branches (a session's trajectories)."""
    trajs = [rng.integers(0, vocab, size=base_len).tolist()]
    for _ in range(nbranch - 1):
        src = trajs[int(rng.integers(len(trajs)))]
        cut = int(rng.integers(1, len(src) + 1))
        trajs.append(src[:cut] + rng.integers(0, vocab, size=int(rng.integers(1, 80))).tolist())
    return trajs


def test_match_is_page_granular_longest_prefix():
    rng = np.random.default_rng(0)
    t = PrefixTree(4096)
    stored = []
    for s in range(6):
        for tr in random_session(rng, 8, 100 + 37 * s):
            # brute force: the best stored trajectory's common prefix, rounded down to whole pages that it stores as full pages
            want = max((min(lcp(tr, o), len(o) // 16 * 16, len(tr) // 16 * 16) // 16 * 16 for o in stored), default=0)
            assert t.match(tr) == want
            tid, m = t.insert(tr)
            assert m == want and t.length(tid) == len(tr)
            stored.append(tr)


def test_pages_are_shared_exactly_when_prefixes_are_equal():
    rng = np.random.default_rng(1)
    t = PrefixTree(4096)
    trajs = random_session(rng, 20, 300)
    ids = [t.insert(tr)[0] for tr in trajs]
    tables = [t.block_table(i) for i in ids]
    for a in range(len(trajs)):
        assert len(tables[a]) == (len(trajs[a]) + 15) // 16
        for b in range(a):
            for j in range(min(len(tables[a]), len(tables[b]))):
                both_full = 16 * (j + 1) <= min(len(trajs[a]), len(trajs[b]))
                same_prefix = both_full and trajs[a][:16 * (j + 1)] == trajs[b][:16 * (j + 1)]
                assert (tables[a][j] == tables[b][j]) == same_prefix
    # every page id is in range and the number of distinct ids is what the tree says is in use
    allp = np.concatenate(tables)
    assert allp.min() >= 0 and allp.max() < 4096 and len(set(allp.tolist())) == t.pages_in_use
    # tokens read back
    for i, tr in zip(ids, trajs):
        for pos in (0, len(tr) // 2, len(tr) - 1):
            assert t.token_at(i, pos) == (tr[pos], 0)


def test_versions_split_pages():
    """The same tokens produced under another model version are different KV: no sharing from that page on."""
    t = PrefixTree(64)
    toks = list(range(48))
    a, _ = t.insert(toks, [0] * 48)
    b, m = t.insert(toks, [0] * 20 + [1] * 28)  # weights were reloaded after token 20
    assert m == 16
    ta, tb = t.block_table(a), t.block_table(b)
    assert ta[0] == tb[0] and ta[1] != tb[1] and ta[2] != tb[2]
    assert t.token_at(b, 19) == (19, 0) and t.token_at(b, 20) == (20, 1)
    assert t.match(toks, [0] * 48) == 48 and t.match(toks, [1] * 48) == 0


def test_release_returns_pages_and_keeps_shared_ones():
    t = PrefixTree(32)
    base = list(range(40))
    a, _ = t.insert(base)                 # 2 full pages + tail = 3 pages
    b, m = t.insert(base[:32] + [99] * 20)  # shares 2, adds 1 full + tail = 2
    assert m == 32 and t.pages_in_use == 5
    t.release(a)
    assert t.pages_in_use == 4            # only a's tail went back
    assert t.match(base) == 32
    t.release(b)
    assert t.pages_in_use == 0 and t.match(base) == 0
    with pytest.raises(Exception):
        t.release(b)
    # the pool can be used up and reports it without changing anything
    t2 = PrefixTree(3)
    t2.insert(list(range(40)))
    with pytest.raises(Exception):
        t2.insert([7] * 17)
    assert t2.pages_in_use == 3


def test_batch_groups_describe_common_pages():
    rng = np.random.default_rng(2)
    t = PrefixTree(8192)
    batch, want_tr = [], []
    for s in range(5):
        trs = random_session(rng, int(rng.integers(1, 7)), 200 + 50 * s, vocab=1000)
        for tr in trs:
            batch.append(t.insert(tr)[0]); want_tr.append(tr)
    batch.append(t.insert([5] * 7)[0]); want_tr.append([5] * 7)  # shorter than a page: never grouped
    gs, sh = t.batch_groups(batch)
    assert gs[0] == 0 and gs[-1] == len(batch) and np.all(np.diff(gs) > 0)
    tables = [t.block_table(i) for i in batch]
    for g in range(len(gs) - 1):
        members = range(gs[g], gs[g + 1])
        common = min(len(tables[m]) for m in members)
        k = 0
        while k < common and all(tables[m][k] == tables[gs[g]][k] and 16 * (k + 1) <= len(want_tr[m]) for m in members):
            k += 1
        want = 16 * k if len(members) > 1 else 0
        assert all(sh[m] == want for m in members)
        # neighbours in different groups do not start with the same page (or one of them has no full page)
        if g + 1 < len(gs) - 1:
            a, b = gs[g], gs[g + 1]
            assert len(want_tr[a]) < 16 or len(want_tr[b]) < 16 or tables[a][0] != tables[b][0]


def test_fork_shares_full_pages_and_copies_the_partial_one():
    t = PrefixTree(64)
    toks = list(range(40))                      # two full pages and a tail of 8
    a, _ = t.insert(toks)
    used = t.pages_in_use
    b, src, dst = t.fork(a)
    ta, tb = t.block_table(a), t.block_table(b)
    assert (ta[:2] == tb[:2]).all() and ta[2] != tb[2]
    assert (src, dst) == (ta[2], tb[2]) and t.pages_in_use == used + 1
    assert t.length(b) == 40 and [t.token_at(b, i)[0] for i in range(40)] == toks
    # a fork at a page boundary has nothing to copy
    c, _ = t.insert(list(range(100, 132)))
    d, src, dst = t.fork(c)
    assert (src, dst) == (-1, -1) and (t.block_table(c) == t.block_table(d)).all()
    # the branches form one group that shares the full pages
    gs, sh = t.batch_groups([a, b])
    assert gs.tolist() == [0, 2] and sh.tolist() == [32, 32]
    t.release(a)
    assert t.block_table(b).tolist() == tb.tolist()     # shared pages survive the release of one branch
    t.release(b); t.release(c); t.release(d)
    assert t.pages_in_use == 0


def test_append_walks_pages_and_fills_the_tree_like_an_insert():
    """Decoding token by token ends in the same state as inserting the final sequence: same sharing, same
    tokens, same page count; the reported (page, slot) is where the block table says the token lives."""
    rng = np.random.default_rng(5)
    t = PrefixTree(256)
    prompt = rng.integers(0, 50, size=21).tolist()
    a, _ = t.insert(prompt)
    b, src, dst = t.fork(a)
    grown = {a: list(prompt), b: list(prompt)}
    for step in range(45):
        for tr in (a, b):
            tok = int(rng.integers(0, 50)) if step > 12 or tr == a else grown[a][len(grown[b])]  # b copies a's next tokens for a while
            page, slot = t.append(tr, tok, version=step // 20)
            grown[tr].append(tok)
            pos = len(grown[tr]) - 1
            assert slot == pos % 16 and t.length(tr) == pos + 1
            assert t.block_table(tr)[pos // 16] == page
            assert t.token_at(tr, pos) == (tok, step // 20)
    # b decoded the same tokens as a up to position 21 + 13 = 34: the page that filled up at 32 tokens is equal in
    # both, but each branch wrote its own copy, so only one of them is listed and the other stays private
    ta, tb = t.block_table(a), t.block_table(b)
    assert ta[0] == tb[0] and ta[1] != tb[1]
    # a later insert of a's tokens finds all of a's full pages
    vers = [0] * 21 + [s // 20 for s in range(45)]
    c, matched = t.insert(grown[a], vers)
    assert matched == len(grown[a]) // 16 * 16
    assert (t.block_table(c)[:matched // 16] == ta[:matched // 16]).all()
    for tr in (a, b, c):
        t.release(tr)
    assert t.pages_in_use == 0


def test_fork_and_append_report_an_exhausted_pool():
    from paper_2508_11553_amd.binding import SeamDecodeError
    t = PrefixTree(3)
    a, _ = t.insert(list(range(40)))            # 3 pages: pool full
    with pytest.raises(SeamDecodeError):
        t.fork(a)                               # needs a page for the tail copy
    for i in range(8):
        t.append(a, i)                          # fills the tail: no new page needed
    with pytest.raises(SeamDecodeError):
        t.append(a, 99)
    assert t.length(a) == 48 and t.pages_in_use == 3
