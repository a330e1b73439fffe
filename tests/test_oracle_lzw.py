"""Pins for the LZW oracle: what the paper and the mathematics fix, independent of the oracle's own code."""
import itertools
import os
import random

import numpy as np
import pytest

from oracle import (LZWStream, ST_BAD_CODE, ST_BAD_TOKEN, ST_OK, ST_OVERFLOW, lzw_decode, lzw_encode,
                    pack_entries)

INF = 10 ** 9


# ---------------------------------------------------------------------------
# P1: the paper's worked example (Fig. 1 / Fig. 2 captions; reconstructed table)
# ---------------------------------------------------------------------------
def _read_cases(path):
    cases, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, _, rest = line.partition(" ")
        if key == "case":
            cur = {"name": rest}
        elif key == "end":
            cases.append(cur)
        elif key in ("V", "M", "cap"):
            cur[key] = int(rest)
        elif key in ("tokens", "codes"):
            cur[key] = [int(t) for t in rest.split()]
        elif key == "entries":
            cur[key] = [tuple(int(t) for t in e.split()) for e in rest.split(";")]
    return cases


def test_fig1_worked_example(golden_dir):
    cases = _read_cases(os.path.join(golden_dir, "fig1_to_be_or_not.txt"))
    assert len(cases) == 3
    for c in cases:
        codes, entries, st = lzw_encode(c["tokens"], c["V"], c["M"], c["cap"])
        assert st == ST_OK
        assert codes == c["codes"], c["name"]
        assert entries == c["entries"], c["name"]
        toks, dentries, st = lzw_decode(c["codes"], c["V"], c["M"], c["cap"])
        assert st == ST_OK and toks == c["tokens"] and dentries == c["entries"], c["name"]
    # the captions' own statements: "to be" and "or not" are created, then reused; "to be or" is nested
    c = cases[1]
    codes, entries, _ = lzw_encode(c["tokens"], c["V"], c["M"], c["cap"])
    to_be, or_not, to_be_or = entries.index((0, 1)), entries.index((2, 3)), entries.index((0, 1, 2))
    assert 6 + to_be in codes and 6 + or_not in codes and 6 + to_be_or in codes
    assert to_be < to_be_or


# ---------------------------------------------------------------------------
# P2: round trip and decoder codebook == encoder codebook (section 2.1, "self-contained")
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("V", [1, 2, 3, 5])
def test_round_trip_small_alphabets(V):
    rnd = random.Random(1234 + V)
    for trial in range(400):
        n = rnd.randint(0, 60)
        x = [rnd.randrange(V) for _ in range(n)]
        M = rnd.choice([1, 2, 3, 4, 5, INF])
        cap = rnd.choice([0, 1, 3, 7, INF])
        codes, entries, st = lzw_encode(x, V, M, cap)
        assert st == ST_OK
        toks, dentries, st = lzw_decode(codes, V, M, cap)
        assert st == ST_OK
        assert toks == x
        assert dentries == entries


# ---------------------------------------------------------------------------
# P3: M = 1 is no compression (merge-size ablation table: "M=1 corresponds to no compression")
# ---------------------------------------------------------------------------
def test_m1_and_cap0_are_identity():
    rnd = random.Random(5)
    x = [rnd.randrange(4) for _ in range(200)]
    for M, cap in [(1, INF), (1, 0), (3, 0), (INF, 0)]:
        codes, entries, st = lzw_encode(x, 4, M, cap)
        assert codes == x and entries == [] and st == ST_OK


# ---------------------------------------------------------------------------
# P4: M = inf, cap = inf is textbook LZW -- compare with an independently written byte-string routine
# ---------------------------------------------------------------------------
def _textbook_lzw_bytes(data: bytes):
    table = {bytes([i]): i for i in range(256)}
    out = []
    cur = b""
    for ch in data:
        nxt = cur + bytes([ch])
        if nxt in table:
            cur = nxt
        else:
            out.append(table[cur])
            table[nxt] = len(table)
            cur = bytes([ch])
    if cur:
        out.append(table[cur])
    return out, table


def test_unbounded_equals_textbook_lzw_on_bytes():
    rnd = random.Random(77)
    texts = [b"", b"a", b"TOBEORNOTTOBEORTOBEORNOT", b"abababababababab", bytes(rnd.choices(b"abc", k=500)),
             bytes(rnd.choices(range(256), k=300)), b"aaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaaa"]
    for t in texts:
        ref_codes, ref_table = _textbook_lzw_bytes(t)
        codes, entries, st = lzw_encode(list(t), 256, INF, INF)
        assert st == ST_OK and codes == ref_codes
        assert len(entries) == len(ref_table) - 256
        for i, e in enumerate(entries):
            assert ref_table[bytes(e)] == 256 + i
    # the classic published instance (Welch-style demo string): 24 symbols -> 16 codes
    codes, _, _ = lzw_encode(list(b"TOBEORNOTTOBEORTOBEORNOT"), 256, INF, INF)
    assert codes == [84, 79, 66, 69, 79, 82, 78, 79, 84, 256, 258, 260, 265, 259, 261, 263]


# ---------------------------------------------------------------------------
# P5: closed form on a constant sequence (also the exact form of the O(sqrt N) proposition)
# ---------------------------------------------------------------------------
def _constant_expected(N, M):
    lens, k, left = [], 1, N
    while left > 0:
        L = min(k, M, left)
        lens.append(L)
        left -= L
        k += 1
    return lens


@pytest.mark.parametrize("N,M,want_lens,want_entries", [
    (20, 3, [1, 2, 3, 3, 3, 3, 3, 2], 2),
    (20, 5, [1, 2, 3, 4, 5, 5], 4),
    (20, INF, [1, 2, 3, 4, 5, 5], 5),
    (21, INF, [1, 2, 3, 4, 5, 6], 5),
])
def test_constant_sequence_closed_form(N, M, want_lens, want_entries):
    codes, entries, _ = lzw_encode([0] * N, 1, M, INF)
    lens = [1 if c < 1 else len(entries[c - 1]) for c in codes]
    assert lens == want_lens
    assert len(entries) == want_entries
    assert entries == [tuple([0] * (i + 2)) for i in range(want_entries)]


def test_constant_sequence_sweep_and_sqrt_bound():
    for N in range(0, 80):
        for M in (1, 2, 3, 4, 7, INF):
            codes, entries, _ = lzw_encode([0] * N, 1, M, INF)
            lens = [1 if c < 1 else len(entries[c - 1]) for c in codes]
            if M != INF:
                assert lens == _constant_expected(N, M)
            assert sum(lens) == N
            # an entry of length L needs N >= L(L-1)/2 + 1 (extremal case of the merge-size proposition)
            for e in entries:
                L = len(e)
                assert N >= L * (L - 1) // 2 + 1


# ---------------------------------------------------------------------------
# P6: structural invariants on random inputs
# ---------------------------------------------------------------------------
def _check_invariants(x, V, M, cap, codes, entries):
    N = len(x)
    assert all(2 <= len(e) <= M for e in entries)
    assert len(set(entries)) == len(entries)
    seen = set()
    for e in entries:                      # prefix closure: unit of size k = earlier unit of size k-1 + one token
        assert len(e) == 2 or e[:-1] in seen
        seen.add(e)
    if N:
        assert len(entries) <= min(cap, len(codes) - 1)
        assert -(-N // M) <= len(codes) <= N
    else:
        assert codes == [] and entries == []
    hyper = [c for c in codes if c >= V]
    saved = sum(len(entries[c - V]) - 1 for c in hyper)
    assert N - len(codes) == saved <= (M - 1) * len(hyper)
    for c in codes:
        assert 0 <= c < V + len(entries)


def test_structural_invariants_random():
    rnd = random.Random(99)
    for trial in range(300):
        V = rnd.choice([2, 3, 8, 50])
        n = rnd.randint(0, 300)
        x = [min(V - 1, int(rnd.paretovariate(1.1)) - 1) for _ in range(n)]
        M = rnd.choice([2, 3, 4, 5])
        cap = rnd.choice([4, 16, 64, INF])
        codes, entries, st = lzw_encode(x, V, M, cap)
        assert st == ST_OK
        _check_invariants(x, V, M, cap, codes, entries)


def test_token_statistics_table_is_consistent(golden_dir):
    """The paper's printed token statistics obey the same accounting the oracle obeys (M = 3)."""
    for line in open(os.path.join(golden_dir, "token_stats_table.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, n_orig, n_zip, n_hyper, ratio, rate = line.split()
        n_orig, n_zip, n_hyper = int(n_orig), int(n_zip), int(n_hyper)
        assert abs(n_hyper / n_zip - float(ratio)) < 6e-4
        assert abs(n_zip / n_orig - float(rate)) < 6e-4
        assert n_hyper <= n_orig - n_zip <= (3 - 1) * n_hyper


# ---------------------------------------------------------------------------
# P7: brute force over ALL tiny inputs against an independent set-of-tuples formulation
# ---------------------------------------------------------------------------
def _greedy_longest_match(x, V, M, cap):
    known = []                                  # list of tuples, creation order
    codes, i, n = [], 0, len(x)
    while i < n:
        best = 1
        for L in range(2, min(M, n - i) + 1):
            if tuple(x[i:i + L]) in known:
                best = L
            else:
                break                           # prefix-closed set: a longer match needs this one
        ph = tuple(x[i:i + best])
        codes.append(ph[0] if best == 1 else V + known.index(ph))
        i += best
        if i < n and best + 1 <= M and len(known) < cap:
            known.append(ph + (x[i],))
    return codes, known


def test_brute_force_all_tiny_sequences():
    for V, maxlen in [(2, 9), (3, 6)]:
        for n in range(0, maxlen + 1):
            for x in itertools.product(range(V), repeat=n):
                for M in (1, 2, 3, 4, INF):
                    for cap in (0, 1, 2, INF):
                        codes, entries, _ = lzw_encode(list(x), V, M, cap)
                        ref_codes, ref_entries = _greedy_longest_match(list(x), V, M, cap)
                        assert codes == ref_codes, (x, M, cap)
                        assert entries == ref_entries, (x, M, cap)


# ---------------------------------------------------------------------------
# decoder: the "not yet defined" code, error paths, capacity
# ---------------------------------------------------------------------------
def test_decoder_kwkwk_case_and_errors():
    # a a a a a a  ->  a, [aa] (just created), [aaa] (just created): codes 0, 1, 2 with V = 1
    codes, entries, _ = lzw_encode([0] * 6, 1, INF, INF)
    assert codes == [0, 1, 2]
    toks, dentries, st = lzw_decode(codes, 1, INF, INF)
    assert toks == [0] * 6 and dentries == entries and st == ST_OK
    # a code two beyond the codebook is not decodable; the prefix before it is still returned
    toks, _, st = lzw_decode([0, 1, 5], 1, INF, INF)
    assert st == ST_BAD_CODE and toks == [0, 0, 0]
    # a hyper code first (no previous phrase) cannot exist
    toks, _, st = lzw_decode([3], 3, 3, INF)
    assert st == ST_BAD_CODE and toks == []
    # the "not yet defined" code is refused when the previous phrase already has M tokens
    codes, _, _ = lzw_encode([0] * 6, 1, 2, INF)        # a, aa, aa, a -> codes 0 1 1 0
    assert codes == [0, 1, 1, 0]
    toks, _, st = lzw_decode([0, 1, 2], 1, 2, INF)
    assert st == ST_BAD_CODE and toks == [0, 0, 0]
    # negative code
    toks, _, st = lzw_decode([0, -1], 2, 3, INF)
    assert st == ST_BAD_CODE and toks == [0]
    # short output buffer: stops before the phrase that does not fit
    toks, _, st = lzw_decode([0, 1, 2], 1, INF, INF, max_tokens=4)
    assert st == ST_OVERFLOW and toks == [0, 0, 0]


def test_encoder_bad_token_stops_sequence():
    x = [0, 1, 0, 1, 7, 0, 1]
    codes, entries, st = lzw_encode(x, 2, 3, INF)
    want_codes, want_entries, _ = lzw_encode(x[:4], 2, 3, INF)
    assert st == ST_BAD_TOKEN and codes == want_codes and entries == want_entries
    codes, entries, st = lzw_encode([-1, 0], 2, 3, INF)
    assert st == ST_BAD_TOKEN and codes == [] and entries == []


def test_capacity_freeze_keeps_matching():
    x = [0, 1] * 20
    codes, entries, _ = lzw_encode(x, 2, 3, 2)
    assert len(entries) == 2
    assert any(c >= 2 for c in codes[4:])            # frozen entries are still used
    toks, dentries, st = lzw_decode(codes, 2, 3, 2)
    assert toks == x and dentries == entries and st == ST_OK


# ---------------------------------------------------------------------------
# streaming form: chunked encode, decoder-style updates on arbitrary (model-generated) codes
# ---------------------------------------------------------------------------
def test_stream_whole_sequence_equals_one_shot():
    rnd = random.Random(3)
    for trial in range(200):
        V = rnd.choice([2, 3, 6])
        x = [rnd.randrange(V) for _ in range(rnd.randint(0, 80))]
        M, cap = rnd.choice([1, 2, 3, 5]), rnd.choice([0, 2, 9, INF])
        s = LZWStream(V, M, cap)
        codes, st = s.encode_chunk(x)
        ref_codes, ref_entries, _ = lzw_encode(x, V, M, cap)
        assert codes == ref_codes and s.entries == ref_entries and st == ST_OK


def test_stream_chunked_encode_is_decodable_with_same_codebook():
    rnd = random.Random(4)
    for trial in range(300):
        V = rnd.choice([2, 3, 6])
        x = [rnd.randrange(V) for _ in range(rnd.randint(1, 90))]
        M, cap = rnd.choice([2, 3, 5]), rnd.choice([2, 9, INF])
        enc = LZWStream(V, M, cap)
        all_codes, i = [], 0
        while i < len(x):
            step = rnd.randint(1, 12)
            c, st = enc.encode_chunk(x[i:i + step])
            assert st == ST_OK
            all_codes += c
            i += step
        toks, dentries, st = lzw_decode(all_codes, V, M, cap)
        assert st == ST_OK and toks == x and dentries == enc.entries
        assert len(set(enc.entries)) == len(enc.entries)
        # feeding the codes one at a time gives the same codebook
        dec = LZWStream(V, M, cap)
        got = []
        for c in all_codes:
            t, st = dec.decode_chunk([c])
            assert st == ST_OK
            got += t
        assert got == x and dec.entries == enc.entries


def test_stream_generated_codes_add_at_most_one_unique_entry():
    """Codes a greedy encoder would not emit (section 2.3, steps 9-10: sampled tokens are merged too)."""
    rnd = random.Random(8)
    for trial in range(100):
        V, M, cap = 4, 3, rnd.choice([5, 50])
        s = LZWStream(V, M, cap)
        s.encode_chunk([rnd.randrange(V) for _ in range(30)])
        total = []
        for step in range(60):
            before = len(s.entries)
            k = rnd.randrange(V + before)
            t, st = s.decode_chunk([k])
            assert st == ST_OK
            total += t
            assert 0 <= len(s.entries) - before <= 1
            assert len(set(s.entries)) == len(s.entries)
            assert all(2 <= len(e) <= M for e in s.entries) and len(s.entries) <= cap
            for e in s.entries:
                assert len(e) == 2 or e[:-1] in s.entries


def test_pack_entries_layout():
    tok, ln, C = pack_entries([(5, 6), (5, 6, 7)], cap=4, M=3)
    assert C == 2 and ln.tolist() == [2, 3, 0, 0]
    assert tok.tolist() == [[5, 6, -1], [5, 6, 7], [-1, -1, -1], [-1, -1, -1]]
    assert tok.dtype == np.int32 and ln.dtype == np.int32


# ---------------------------------------------------------------------------
# codebook prefilling (discussion section, "Codebook Management Strategy", item 2)
# ---------------------------------------------------------------------------
def _greedy_with_seed(x, V, M, cap, seed):
    """The set-of-tuples parse of P7, started from a given list of entries."""
    known = list(seed)
    codes, i, n = [], 0, len(x)
    while i < n:
        best = 1
        for L in range(2, min(M, n - i) + 1):
            if tuple(x[i:i + L]) in known:
                best = L
            else:
                break
        ph = tuple(x[i:i + best])
        codes.append(ph[0] if best == 1 else V + known.index(ph))
        i += best
        cand = ph + (x[i],) if i < n else None
        if cand is not None and best + 1 <= M and len(known) < cap and cand not in known:
            known.append(cand)
    return codes, known


def test_prefill_then_parse_equals_seeded_brute_force_and_round_trips():
    rnd = random.Random(11)
    for trial in range(300):
        V = rnd.choice([2, 3, 5])
        M, cap = rnd.choice([2, 3, 4]), rnd.choice([3, 8, 40])
        warm = [rnd.randrange(V) for _ in range(rnd.randint(0, 40))]
        seed = lzw_encode(warm, V, M, cap)[1][: rnd.randint(0, cap)]       # a prefix of a real codebook: prefix-closed
        x = [rnd.randrange(V) for _ in range(rnd.randint(0, 60))]
        enc = LZWStream(V, M, cap)
        added, st = enc.prefill(seed)
        assert st == ST_OK and added == len(seed) and enc.entries == list(seed)
        codes, st = enc.encode_chunk(x)
        ref_codes, ref_known = _greedy_with_seed(x, V, M, cap, seed)
        assert st == ST_OK and codes == ref_codes and enc.entries == ref_known
        dec = LZWStream(V, M, cap)
        dec.prefill(seed)
        toks, st = dec.decode_chunk(codes)
        assert st == ST_OK and toks == x and dec.entries == enc.entries
        if seed and x:
            assert len(codes) <= len(lzw_encode(x, V, M, cap)[0]) + len(x)      # sanity: still a parse of x
    # an empty prefill changes nothing
    s = LZWStream(4, 3, 10)
    assert s.prefill([]) == (0, ST_OK)
    assert s.encode_chunk([1, 2, 1, 2, 1, 2])[0] == lzw_encode([1, 2, 1, 2, 1, 2], 4, 3, 10)[0]


def test_prefill_rejects_what_would_break_the_codebook():
    def run(phrases, V=5, M=3, cap=4):
        s = LZWStream(V, M, cap)
        return s.prefill(phrases), s.entries
    assert run([(1, 2), (1, 2, 3)]) == ((2, ST_OK), [(1, 2), (1, 2, 3)])
    assert run([(1, 2, 3)]) == ((0, ST_BAD_CODE), [])                         # prefix (1, 2) unknown
    assert run([(1, 2), (1, 2)]) == ((1, ST_BAD_CODE), [(1, 2)])              # duplicate
    assert run([(1,)]) == ((0, ST_BAD_TOKEN), [])                             # too short
    assert run([(1, 2), (1, 2, 3), (1, 2, 3, 4)])[0] == (2, ST_BAD_TOKEN)     # longer than M
    assert run([(1, 7)]) == ((0, ST_BAD_TOKEN), [])                           # token out of range
    assert run([(0, 1), (0, 2), (0, 3), (0, 4), (1, 1)])[0] == (4, ST_OVERFLOW)
    # a pending phrase is dropped: the next chunk starts afresh (no entry from the old phrase)
    s = LZWStream(5, 3, 10)
    s.encode_chunk([1, 2])
    s.prefill([(3, 4)])
    s.encode_chunk([0])
    assert s.entries == [(1, 2), (3, 4)]


# ---------------------------------------------------------------------------
# pruning / selective retention (discussion section, "Codebook Management Strategy", item 1)
# ---------------------------------------------------------------------------
def test_prune_equals_prefill_of_the_survivors_and_round_trips():
    rnd = random.Random(12)
    for trial in range(300):
        V = rnd.choice([2, 3, 5])
        M, cap = rnd.choice([2, 3, 4]), rnd.choice([4, 10, 40])
        warm = [rnd.randrange(V) for _ in range(rnd.randint(0, 60))]
        s = LZWStream(V, M, cap)
        codes, _ = s.encode_chunk(warm)
        old = list(s.entries)
        use = s.usage(codes)
        assert sum(use) == sum(1 for c in codes if c >= V) and len(use) == len(old)
        keep = [rnd.random() < 0.6 for _ in old]
        new_index = s.prune(keep)
        # survivors: flagged, and so is every prefix (computed here from the definition, by fixed point)
        alive = set(i for i, k in enumerate(keep) if k)
        changed = True
        while changed:
            changed = False
            for i in list(alive):
                e = old[i]
                if len(e) > 2 and old.index(e[:-1]) not in alive:
                    alive.discard(i)
                    changed = True
        want = [e for i, e in enumerate(old) if i in alive]
        assert s.entries == want
        assert [i for i, n in enumerate(new_index) if n >= 0] == sorted(alive)
        assert [n for n in new_index if n >= 0] == list(range(len(want)))
        # the pruned codebook is the one a fresh stream gets by prefilling the survivors
        f = LZWStream(V, M, cap)
        assert f.prefill(want) == (len(want), ST_OK) and f.entries == s.entries and f.book == s.book
        # and the parse goes on from it, decodable by a decoder that pruned alike
        x = [rnd.randrange(V) for _ in range(rnd.randint(0, 50))]
        c2, st = s.encode_chunk(x)
        d = LZWStream(V, M, cap)
        d.prefill(want)
        toks, st2 = d.decode_chunk(c2)
        assert st == ST_OK and st2 == ST_OK and toks == x and d.entries == s.entries
    # keep everything: nothing changes; keep nothing: empty
    s = LZWStream(3, 3, 20)
    s.encode_chunk([0, 1, 0, 1, 0, 1, 2, 2, 2, 2])
    e = list(s.entries)
    assert s.prune([True] * len(e)) == list(range(len(e))) and s.entries == e
    assert s.prune([False] * len(e)) == [-1] * len(e) and s.entries == [] and s.book == {}
    # dropping (0, 1) drops its extension (0, 1, 0) although that one is flagged
    s = LZWStream(3, 3, 20)
    s.prefill([(0, 1), (0, 1, 0), (1, 1)])
    assert s.prune([False, True, True]) == [-1, -1, 0] and s.entries == [(1, 1)]


# ---------------------------------------------------------------------------
# entry usage (discussion section: how many of the created hypertokens are ever used again)
# ---------------------------------------------------------------------------
def test_usage_counts_each_entry_by_the_phrases_of_the_parse():
    """usage is pinned per entry, not through its sum: (1) a hand-worked stream; (2) an independent count -- the
    stream is decoded code by code and every decoded phrase of two or more tokens is looked up, as a tuple, in
    the codebook, which names its entry without going through the code's arithmetic; (3) codes that name no
    entry (base tokens, IDs past the codebook) count nothing."""
    # (1) V = 6: "to be or not" three times at M = 3 (Fig. 1's example continued): codes 0 1 2 3 6 8 10 3,
    # entries to-be, be-or, or-not, not-to, to-be-or, or-not-to -> entries 0, 2 and 4 are named once each
    s = LZWStream(6, 3, 100)
    codes, st = s.encode_chunk([0, 1, 2, 3] * 3)
    assert st == ST_OK and codes == [0, 1, 2, 3, 6, 8, 10, 3]
    assert s.entries[:6] == [(0, 1), (1, 2), (2, 3), (3, 0), (0, 1, 2), (2, 3, 0)]
    assert s.usage(codes) == [1, 0, 1, 0, 1, 0][:len(s.entries)] + [0] * (len(s.entries) - 6)
    # (2) random streams over tiny alphabets
    rnd = random.Random(77)
    for trial in range(300):
        V = rnd.choice([2, 3, 5])
        M, cap = rnd.choice([2, 3, 5]), rnd.choice([3, 10, 60])
        toks = [rnd.randrange(V) for _ in range(rnd.randint(0, 80))]
        s = LZWStream(V, M, cap)
        codes, st = s.encode_chunk(toks)
        assert st == ST_OK
        back, entries, dst = lzw_decode(codes, V, M, cap)
        assert dst == ST_OK and back == toks and [tuple(e) for e in entries] == [tuple(e) for e in s.entries]
        # phrases of the parse, recovered from the token stream and the code count alone: walk the tokens with a
        # decoder and record each phrase as a tuple
        d = LZWStream(V, M, cap)
        want = [0] * len(s.entries)
        index = {tuple(e): i for i, e in enumerate(s.entries)}
        for c in codes:
            phrase, dst = d.decode_chunk([c])
            assert dst == ST_OK
            if len(phrase) >= 2:
                want[index[tuple(phrase)]] += 1
        assert s.usage(codes) == want
        # (3) foreign codes count nothing
        assert s.usage(list(range(V)) + [V + len(s.entries), V + len(s.entries) + 5, -1]) == [0] * len(s.entries)
