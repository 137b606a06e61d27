"""Model check of the resident attention kernel's wave-to-wave protocol (host only).

decode_stream.hip runs four waves per workgroup with no barrier in its item loop: item records in
a queue, a rotating ticket drawer, two staging buffers with an arrival counter, a load cursor that
runs into the next item, and a ring of page slots consumed two at a time.  This file restates that
control logic (no arithmetic, no memory) as Python generators, one per wave, which yield wherever
the kernel would poll a flag or finish a step; a seeded random scheduler interleaves the waves of
all workgroups, letting single waves run far ahead.  Checked: every page of every (request,
kv-head) is consumed exactly once, by the slot that holds its page id; no live ring slot is
overwritten; null slots are passed over within the guard; a staging buffer is never written before
its previous item was combined; every item is combined exactly once; every wave terminates.

A second mode models the kernel with every wait expiring at once (the state a broken hand-shake, or
the library's test flag, puts it in): the results are then worthless by design, and what is checked
is that every wave still terminates, that every page it touches lies inside its row's table, and that
every item it would store lies inside the batch -- i.e. that the failure mode is safe to run."""
import random

import numpy as np
import pytest

KW = 4; KQ = 8

def run(seq_lens, block_table, Hkv, pt_arg, max_seq_len, n_wg, S, NB, seed, cshift=0, waits_expire=False,
        clear_expired_items=True):
    rnd = random.Random(seed)
    B = len(seq_lens)
    pt_given = pt_arg if pt_arg > 0 else (1 << 30)
    pt = pt_given << (cshift if pt_arg > 0 else 0)   # items are runs of 1 << cshift partitions
    L = np.clip(seq_lens, 0, max_seq_len)
    f = L // pt; g = ((L % pt != 0) | (L == 0)).astype(int)
    pref_full = np.concatenate([[0], np.cumsum(f)]); pref_rag = np.concatenate([[0], np.cumsum(g)])
    tf, tg = int(pref_full[-1]), int(pref_rag[-1])
    total = (tf + tg) * Hkv
    ppp = pt // 16
    counter = [0]
    def draw():
        counter[0] += 1; return counter[0] - 1
    def find_row(pref, u):
        lo, hi = 0, B
        while hi - lo > 1:
            mid = (lo + hi) >> 1
            if pref[mid] <= u: lo = mid
            else: hi = mid
        return lo
    def decode(ticket):
        it = dict(valid=0 <= ticket < total, b=0, kvh=0, part=0, t1=0, n_parts=1)
        if it["valid"]:
            unit = ticket // Hkv; it["kvh"] = ticket - unit * Hkv
            if unit < tf:
                b = find_row(pref_full, unit); it["part"] = unit - int(pref_full[b]); t1 = (it["part"] + 1) * pt
            else:
                b = find_row(pref_rag, unit - tf); it["part"] = int(pref_full[b + 1] - pref_full[b]); t1 = int(L[b])
            it["b"] = b; it["t1"] = t1
            it["n_parts"] = (int(L[b]) - 1) // pt_given + 1 if L[b] > 0 else 1   # as the caller counts them
        return it
    consumed = {}      # (b, kvh, page_index) -> count
    combined = {}      # (b, kvh, part) -> count
    stats = dict(pairs=0, singles=0, nulls=0, polls=0, expired=0, stored=0)

    def wave_proc(wg, wave):
        sh = wg["sh"]
        def first_page(it): return it["part"] * ppp + wave
        def end_page(it): return (it["t1"] + 15) // 16 if it["valid"] else 0
        def fetch(idx):
            while sh["rec"][idx % KQ]["seq"] != idx:
                stats["polls"] += 1
                if waits_expire:     # the record never came: the wave goes on as if the item were past the end
                    stats["expired"] += 1
                    yield
                    if not clear_expired_items:
                        # what the slot holds then is whatever the LDS held: any bit pattern.  The kernel must
                        # not let it through (clear_expired_items=False plants that mistake)
                        return dict(valid=False, b=rnd.randrange(-2**31, 2**31), kvh=rnd.randrange(-2**31, 2**31),
                                    part=rnd.randrange(-2**31, 2**31), t1=rnd.randrange(-2**31, 2**31), n_parts=1)
                    return dict(valid=False, b=0, kvh=0, part=0, t1=0, n_parts=1)
                yield
            return dict(sh["rec"][idx % KQ]["it"])
        C = yield from fetch(0)
        N = yield from fetch(1)
        cur = dict(in_next=0, pg=first_page(C), end=end_page(C), b=C["b"], kvh=C["kvh"], ok=False, id=0)
        def settle():
            if not cur["in_next"] and cur["pg"] >= cur["end"]:
                cur.update(in_next=1, pg=first_page(N), end=end_page(N), b=N["b"], kvh=N["kvh"])
            cur["ok"] = cur["pg"] < cur["end"]
            if cur["ok"]:
                assert 0 <= cur["pg"] < block_table.shape[1] and 0 <= cur["b"] < B
                cur["id"] = int(block_table[cur["b"], cur["pg"]])
        ring = [None] * S
        st = dict(head=0, tail=0, occ=0)
        def issue():
            t = st["tail"]
            assert ring[t] is None or ring[t] == "null", "overwriting a live slot"
            if cur["ok"]:
                ring[t] = (cur["b"], cur["kvh"], cur["pg"], cur["id"])
                cur["pg"] += KW
                settle()
            else:
                ring[t] = "null"; stats["nulls"] += 1
            st["tail"] = (t + 1) % S; st["occ"] += 1
        settle()
        invalid_run = 0
        k = 0
        P = dict(valid=0)
        while True:
            invalid_run = 0 if C["valid"] else invalid_run + 1
            if invalid_run == KW:
                break
            drawer = (k % KW) == wave
            ticket = draw() if drawer else None
            pg = first_page(C); pg_end = end_page(C)
            while pg < pg_end:
                while st["occ"] < S: issue()
                guard = 0
                while ring[st["head"]] == "null" and guard <= S:
                    ring[st["head"]] = None
                    st["head"] = (st["head"] + 1) % S; st["occ"] -= 1
                    issue(); guard += 1
                assert ring[st["head"]] != "null", "pass-over guard exceeded"
                second = (st["head"] + 1) % S
                pair = pg + KW < pg_end and ring[second] not in (None, "null")
                for slot, want in ((st["head"], pg),) + (((second, pg + KW),) if pair else ()):
                    b_, kvh_, pg_, id_ = ring[slot]
                    if not waits_expire:
                        assert (b_, kvh_, pg_) == (C["b"], C["kvh"], want), ("wrong slot", ring[slot], C, want)
                        assert id_ == int(block_table[C["b"], want])
                    consumed[(b_, kvh_, pg_)] = consumed.get((b_, kvh_, pg_), 0) + 1
                    ring[slot] = None
                if pair:
                    st["head"] = (second + 1) % S; st["occ"] -= 2; pg += 2 * KW; stats["pairs"] += 1
                else:
                    st["head"] = second; st["occ"] -= 1; pg += KW; stats["singles"] += 1
                while st["occ"] < S: issue()
                yield
            if drawer:
                idx = k + 3
                rec = sh["rec"][idx % KQ]
                rec["it"] = decode(ticket); rec["seq"] = idx
            buf = (k % 2) if NB == 2 else 0
            use = (k // 2) if NB == 2 else k
            while sh["gen"][buf] != use:
                stats["polls"] += 1
                if waits_expire:
                    stats["expired"] += 1
                    break
                yield
            if C["valid"]:
                assert waits_expire or sh["stage_owner"][buf][wave] is None, "staging overwritten"
                sh["stage_owner"][buf][wave] = k
            sh["arrive"][buf] += 1
            # The combining goes round the waves.  With two staging buffers it is one item late: at
            # the end of item k the wave whose turn it is combines item k - 1, which the others have
            # most likely delivered already; with one buffer it combines item k and waits for them.
            late = 1 if NB == 2 else 0
            if (k + 2) % KW == wave and k >= late:
                q = k - late
                qbuf = (q % 2) if NB == 2 else 0
                Q = P if late else C
                arrived = True
                while sh["arrive"][qbuf] != KW:
                    stats["polls"] += 1
                    if waits_expire:
                        stats["expired"] += 1
                        arrived = False
                        break
                    yield
                if Q["valid"]:
                    # what the combining wave stores (results, or NaN after an expired wait) goes to the item's place
                    assert 0 <= Q["b"] < B and 0 <= Q["kvh"] < Hkv
                    assert 0 <= (Q["part"] << cshift) < max(1, -(-max_seq_len // pt_given)) or pt_arg == 0
                    stats["stored"] += 1
                    if not waits_expire:
                        assert all(o == q for o in sh["stage_owner"][qbuf]), ("combine mix", sh["stage_owner"][qbuf], q)
                    key = (Q["b"], Q["kvh"], Q["part"]); combined[key] = combined.get(key, 0) + 1
                    sh["stage_owner"][qbuf] = [None] * KW
                if arrived:
                    sh["arrive"][qbuf] = 0; sh["gen"][qbuf] = ((q // 2) if NB == 2 else q) + 1
            P = C
            yield
            C = N
            N = yield from fetch(k + 2)
            cur["in_next"] = 0
            if not cur["ok"]:
                settle()
            k += 1
        wg["done"] += 1

    procs = []
    for w in range(n_wg):
        sh = dict(rec=[dict(seq=-1, it=None) for _ in range(KQ)], gen=[0, 0], arrive=[0, 0],
                  stage_owner=[[None] * KW, [None] * KW])
        for i in range(3):
            sh["rec"][i] = dict(seq=i, it=decode(draw()))
        wg = dict(sh=sh, done=0)
        for wave in range(KW):
            procs.append(wave_proc(wg, wave))
    live = list(procs)
    steps = 0
    while live:
        i = rnd.randrange(len(live))
        # occasionally let one wave run far ahead
        burst = rnd.choice([1, 1, 1, 5, 40])
        for _ in range(burst):
            try:
                next(live[i])
            except StopIteration:
                live.pop(i); break
        steps += 1
        assert steps < 50_000_000, "no progress: deadlock"
    if waits_expire:
        return stats    # no coverage is promised; termination and the range checks above are the point
    # coverage
    exp_pages = {}
    for b in range(B):
        for p_ in range((int(L[b]) + 15) // 16):
            for h in range(Hkv):
                exp_pages[(b, h, p_)] = 1
    assert consumed == exp_pages, ("coverage", len(consumed), len(exp_pages))
    exp_items = {}   # one combined result per run of partitions
    for b in range(B):
        npart = (int(L[b]) - 1) // pt + 1 if L[b] > 0 else 1
        for p_ in range(npart):
            for h in range(Hkv):
                exp_items[(b, h, p_)] = 1
    assert combined == exp_items, ("items", len(combined), len(exp_items))
    return stats


CASES = []
_rng = np.random.default_rng(5)
for _trial in range(24):
    _B = int(_rng.integers(1, 40))
    _kind = _trial % 4
    if _kind == 0:
        _lens = _rng.integers(0, 70, size=_B)
    elif _kind == 1:
        _lens = _rng.integers(0, 1500, size=_B)
    elif _kind == 2:
        _lens = np.where(_rng.random(_B) < 0.2, _rng.integers(2000, 5000, size=_B), _rng.integers(0, 40, size=_B))
    else:
        _lens = _rng.integers(500, 520, size=_B)
    CASES.append((_trial, _lens.astype(np.int32), int(_rng.choice([1, 2, 8])), int(_rng.choice([0, 64, 512])),
                  int(_rng.choice([2, 3, 4, 6])), int(_rng.choice([1, 2])), int(_rng.choice([1, 2, 5, 16])),
                  _trial % 3))


@pytest.mark.parametrize("trial,lens,Hkv,pt,S,NB,n_wg,cshift", CASES, ids=[str(c[0]) for c in CASES])
def test_protocol_covers_every_page_once_and_terminates(trial, lens, Hkv, pt, S, NB, n_wg, cshift):
    rng = np.random.default_rng(100 + trial)
    maxp = max(1, (int(lens.max()) + 15) // 16)
    table = rng.integers(0, 10000, size=(len(lens), maxp)).astype(np.int32)
    stats = run(lens, table, Hkv, pt, int(lens.max()), n_wg, S, NB, trial, cshift)
    assert stats["pairs"] + stats["singles"] > 0 or int(lens.max()) == 0


@pytest.mark.parametrize("trial,lens,Hkv,pt,S,NB,n_wg,cshift", CASES, ids=[str(c[0]) for c in CASES])
def test_with_every_wait_expiring_the_waves_still_terminate_inside_their_rows(trial, lens, Hkv, pt, S, NB, n_wg, cshift):
    rng = np.random.default_rng(300 + trial)
    maxp = max(1, (int(lens.max()) + 15) // 16)
    table = rng.integers(0, 10000, size=(len(lens), maxp)).astype(np.int32)
    stats = run(lens, table, Hkv, pt, int(lens.max()), n_wg, S, NB, trial, cshift, waits_expire=True)
    assert stats["expired"] > 0


def test_an_expired_record_fetch_must_hand_on_a_cleared_item():
    """What a record slot holds when its record never came is arbitrary.  The load cursor starts from the item's
    partition whether the item is valid or not, so stale fields (a negative partition, say) would send it to pages
    outside the row's table: the kernel clears the fields of such an item.  Planting the omission here must trip
    the model's bounds checks for at least one of the schedules."""
    tripped = 0
    for trial, lens, Hkv, pt, S, NB, n_wg, cshift in CASES[:40]:
        rng = np.random.default_rng(300 + trial)
        maxp = max(1, (int(lens.max()) + 15) // 16)
        table = rng.integers(0, 10000, size=(len(lens), maxp)).astype(np.int32)
        try:
            run(lens, table, Hkv, pt, int(lens.max()), n_wg, S, NB, trial, cshift, waits_expire=True,
                clear_expired_items=False)
        except (AssertionError, IndexError, RuntimeError):
            tripped += 1
    assert tripped > 0, "stale fields of an expired fetch went unnoticed"
