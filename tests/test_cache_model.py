"""Pins for the cache / prefetch-queue reference model: hand-worked traces (tests/golden/lru_traces.txt,
derived by hand from the paper's LRU rule and Alg. 1 / Alg. 2) and structural invariants."""
import os
import random

from oracle.cache_model import CacheModel

GOLD = os.path.join(os.path.dirname(__file__), "golden", "lru_traces.txt")


def _parse():
    traces, cur = [], None
    for line in open(GOLD):
        line = line.split("#")[0].rstrip()
        if not line:
            continue
        if line.startswith("trace"):
            parts = line.split()
            kw = dict(p.split("=") for p in parts[2:])
            cur = dict(name=parts[1], slots=int(kw["slots"]), cutoff=int(kw["cutoff"]), steps=[])
        elif line == "end":
            traces.append(cur)
        else:
            lhs, rhs = line.split("->")
            q, st = rhs.split("|")
            op, args = lhs.split()
            cur["steps"].append((op, [int(a) for a in args.split(",")],
                                 [int(a) for a in q.strip().split(",")] if q.strip() else [],
                                 [int(a) for a in st.split()]))
    return traces


def test_hand_worked_traces():
    traces = _parse()
    assert len(traces) == 3
    for tr in traces:
        m = CacheModel(1, 8, tr["slots"], cutoff_layer=tr["cutoff"])
        for op, args, q, (h, mi, ev) in tr["steps"]:
            if op == "P":
                m.prefetch(0, args)
            else:
                m.verify(0, sorted(args))
            assert m.contents(0) == q, (tr["name"], op, args)
            assert (m.stats["hits"], m.stats["misses"], m.stats["evictions"]) == (h, mi, ev), (tr["name"], op, args)


def test_invariants_random_sequences():
    rng = random.Random(3)
    for trial in range(200):
        E, S, Lc = rng.choice([8, 16, 64]), rng.randint(1, 6), rng.randint(-1, 3)
        m = CacheModel(4, E, S, cutoff_layer=Lc)
        for step in range(60):
            layer = rng.randrange(4)
            before = m.contents(layer)
            if rng.random() < 0.5:
                task = [rng.randrange(E) for _ in range(rng.randint(1, 4))]
                loaded = m.prefetch(layer, task)
                after = m.contents(layer)
                if layer > Lc:
                    assert loaded == [] and after == before          # Alg. 1: only l <= L
                else:
                    uniq = list(dict.fromkeys(task))[:S]
                    assert all(e in after for e in uniq)              # a task never evicts its own experts
                    assert [e for e, _ in loaded] == [e for e in uniq if e not in before]
            else:
                need = sorted(rng.sample(range(E), rng.randint(1, min(E, 7))))
                hits, loaded = m.verify(layer, need)
                assert hits == [e for e in need if e in before]       # hit = activated expert found cached
                after = m.contents(layer)
                assert after[-1] == need[-1] if need[-1] not in hits or len(loaded) == 0 else True
            q = m.contents(layer)
            assert len(q) <= S and len(set(q)) == len(q)
        st = m.stats
        assert st["misses"] == st["ondemand_loads"]
        assert st["prefetch_used"] + st["prefetch_wasted"] <= st["prefetch_issued"]
        assert 0.0 <= m.hit_rate() <= 1.0


def test_filter_cached_matches_alg1():
    m = CacheModel(1, 8, 3, cutoff_layer=0)
    m.prefetch(0, [4, 5])
    assert m.filter_cached(0, [5, 1, 4, 1, 2]) == [1, 2]
