"""Pins for the cache / prefetch-queue reference model: hand-worked traces (tests/golden/lru_traces.txt,
derived by hand from the paper's LRU rule and Alg. 1 / Alg. 2), structural invariants, and planted
mistakes in a temporary copy of the model's source, each of which the traces must notice."""
import importlib.util
import os
import random
import tempfile

import pytest

import oracle.cache_model as cache_model
from oracle.cache_model import CacheModel

GOLD = os.path.join(os.path.dirname(__file__), "golden", "lru_traces.txt")
COUNTERS = ("prefetch_issued", "prefetch_used", "prefetch_wasted", "ondemand_loads")


def _ints(text):
    text = text.strip()
    return [int(a) for a in text.replace(",", " ").split()] if text else []


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
            cols = rhs.split("|")
            op, args = lhs.split()
            assert len(cols) == (4 if op == "F" else 3), line
            cur["steps"].append(dict(op=op, args=_ints(args), queue=_ints(cols[0]), hme=_ints(cols[1]),
                                     counters=_ints(cols[2]), returned=_ints(cols[3]) if op == "F" else None))
    return traces


def trace_failures(model_class):
    """Replays every hand-worked trace on `model_class`; returns the list of (trace, step) that disagree."""
    bad = []
    for tr in _parse():
        m = model_class(1, 8, tr["slots"], cutoff_layer=tr["cutoff"])
        for n, st in enumerate(tr["steps"]):
            returned = None
            if st["op"] == "P":
                m.prefetch(0, st["args"])
            elif st["op"] == "F":
                returned = m.filter_cached(0, st["args"])
            else:
                m.verify(0, sorted(st["args"]))
            ok = (m.contents(0) == st["queue"]
                  and [m.stats[key] for key in ("hits", "misses", "evictions")] == st["hme"]
                  and [m.stats[key] for key in COUNTERS] == st["counters"]
                  and returned == st["returned"])
            if not ok:
                bad.append((tr["name"], n, st["op"], st["args"]))
    return bad


def test_hand_worked_traces():
    assert len(_parse()) == 7
    assert trace_failures(CacheModel) == []


def test_invariants_random_sequences():
    rng = random.Random(3)
    for trial in range(200):
        E, S, Lc = rng.choice([8, 16, 64]), rng.randint(1, 6), rng.randint(-1, 3)
        m = CacheModel(4, E, S, cutoff_layer=Lc)
        for step in range(60):
            layer = rng.randrange(4)
            before = m.contents(layer)
            if rng.random() < 0.5:
                task = [rng.randrange(E) for _ in range(rng.randint(1, 8))]
                if rng.random() < 0.5:
                    task = m.filter_cached(layer, task) + [e for e in task if rng.random() < 0.2]
                    before = m.contents(layer)
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


def test_a_task_keeps_the_cached_experts_it_predicted():
    # any ranked prediction, any cache state: after Alg. 1's filter and the task's loads (Alg. 2), the first
    # `slots` experts of the prediction are all resident -- the task never evicted one it had named
    rng = random.Random(11)
    for trial in range(300):
        E, S = rng.choice([8, 16]), rng.randint(1, 5)
        m = CacheModel(1, E, S, cutoff_layer=0)
        for step in range(20):
            m.verify(0, sorted(rng.sample(range(E), rng.randint(1, 3))))
            ranked = rng.sample(range(E), rng.randint(1, E))
            m.prefetch(0, m.filter_cached(0, ranked))
            assert set(ranked[:S]) <= set(m.contents(0)), (trial, step, ranked, m.contents(0))


def test_ranking_of_a_prediction_over_several_draft_states():
    _check_ranking(cache_model)


def _check_ranking(cache_model):
    # hand-worked: three draft states, top-2 each, six experts
    #   state 0 selects 2 (p 0.50) and 5 (p 0.30); state 1 selects 2 (0.40) and 1 (0.35); state 2 selects 5 (0.45) and 1 (0.20)
    #   votes 2 / 2 / 2 for experts 2, 5, 1; summed probabilities 0.90 / 0.75 / 0.55 -> 2, 5, 1
    prob = [[0, 0.10, 0.50, 0.05, 0.05, 0.30], [0.05, 0.35, 0.40, 0.10, 0.05, 0.05], [0.10, 0.20, 0.05, 0.10, 0.10, 0.45]]
    assert cache_model.rank_predicted([[2, 5], [2, 1], [5, 1]], prob, 6) == [2, 5, 1]
    # votes come before probability: expert 0 is named twice with little mass, expert 3 once with a lot
    prob = [[0.10, 0.05, 0.05, 0.80], [0.15, 0.60, 0.20, 0.05]]
    assert cache_model.rank_predicted([[3, 0], [1, 0]], prob, 4) == [0, 3, 1]
    # equal votes and equal mass: the lower index first; one state: TopK_Index's own order survives
    assert cache_model.rank_predicted([[3, 2]], [[0.1, 0.1, 0.4, 0.4]], 4) == [2, 3]
    assert cache_model.rank_predicted([[1, 3]], [[0.05, 0.6, 0.05, 0.3]], 4) == [1, 3]


def test_filter_cached_matches_alg1():
    m = CacheModel(1, 8, 3, cutoff_layer=0)
    m.prefetch(0, [4, 5])
    assert m.filter_cached(0, [5, 1, 4, 1, 2]) == [1]          # task = first three distinct: 5, 1, 4
    assert m.filter_cached(0, [1, 2]) == [1, 2]


# ---- the traces must be able to fail: plausible mistakes planted in a copy of the model ----------------
MUTANTS = {
    "no_touch_in_filter": ("""            if e in self.queue[layer]:
                self._touch(layer, e)
            else:
                out.append(e)""", """            if e in self.queue[layer]:
                pass
            else:
                out.append(e)"""),
    "no_cut_in_filter": ("        task = task[: self.slots]\n", "        task = task[:]\n"),
    "cut_after_filter": ("""        task = task[: self.slots]
        out = []
        for e in task:
            if e in self.queue[layer]:
                self._touch(layer, e)
            else:
                out.append(e)
        return out""", """        out = []
        for e in task:
            if e in self.queue[layer]:
                self._touch(layer, e)
            else:
                out.append(e)
        return out[: self.slots]"""),
    "filter_ignores_cutoff": ("""        if self.cutoff < 0 or layer > self.cutoff:
            return []
        task = []""", """        task = []"""),
    "used_not_counted": ('                self.stats["prefetch_used"] += 1', "                pass"),
    "used_counted_on_every_hit": ("""            if e in self.unused_prefetch[layer]:
                self.unused_prefetch[layer].discard(e)
                self.stats["prefetch_used"] += 1""", """            if True:
                self.stats["prefetch_used"] += 1"""),
    "wasted_not_counted": ('                self.stats["prefetch_wasted"] += 1', "                pass"),
    "wasted_counted_for_used_experts": ("            if victim in self.unused_prefetch[layer]:", "            if True:"),
    "victim_from_tail": ("            victim = q.pop(0)", "            victim = q.pop()"),
    "cutoff_off_by_one": ("""        if self.cutoff < 0 or layer > self.cutoff:
            return []
        uniq = []""", """        if self.cutoff < 0 or layer >= self.cutoff:
            return []
        uniq = []"""),
    "cutoff_ignored": ("""        if self.cutoff < 0 or layer > self.cutoff:
            return []
        uniq = []""", """        uniq = []"""),
    "no_touch_on_verify_hit": ("""        for e in hits:
            self._touch(layer, e)""", """        for e in hits:
            pass"""),
    "no_touch_in_prefetch": ("""            if e in self.queue[layer]:
                self._touch(layer, e)
        loaded = []""", """            if e in self.queue[layer]:
                pass
        loaded = []"""),
    "prefetch_not_cut": ("        uniq = uniq[: self.slots]\n", ""),
    "ondemand_not_counted": ('            self.stats["ondemand_loads"] += 1', "            pass"),
    "issued_not_counted": ('            self.stats["prefetch_issued"] += 1', "            pass"),
    "ranking_ignores_votes": ("    return sorted(chosen, key=lambda e: (-votes[e], -psum[e], e))",
                              "    return sorted(chosen, key=lambda e: (-psum[e], e))"),
    "ranking_ties_to_higher_index": ("    return sorted(chosen, key=lambda e: (-votes[e], -psum[e], e))",
                                     "    return sorted(chosen, key=lambda e: (-votes[e], -psum[e], -e))"),
    "misses_loaded_before_hits_touched": ("""        for e in hits:
            self._touch(layer, e)
            if e in self.unused_prefetch[layer]:
                self.unused_prefetch[layer].discard(e)
                self.stats["prefetch_used"] += 1
        loaded = []
        for e in misses:
            victim = self._insert(layer, e)
            self.stats["ondemand_loads"] += 1
            loaded.append((e, victim))""", """        loaded = []
        for e in misses:
            victim = self._insert(layer, e)
            self.stats["ondemand_loads"] += 1
            loaded.append((e, victim))
        for e in hits:
            if e in self.queue[layer]:
                self._touch(layer, e)
            if e in self.unused_prefetch[layer]:
                self.unused_prefetch[layer].discard(e)
                self.stats["prefetch_used"] += 1"""),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_in_the_cache_model_is_caught(name):
    old, new = MUTANTS[name]
    text = open(cache_model.__file__).read()
    assert text.count(old) == 1, "mutation site for %s not found exactly once" % name
    with tempfile.TemporaryDirectory() as tmp:
        path = os.path.join(tmp, "mutant_%s.py" % name)
        open(path, "w").write(text.replace(old, new))
        spec = importlib.util.spec_from_file_location("mutant_%s" % name, path)
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        if name.startswith("ranking"):
            with pytest.raises(AssertionError):
                _check_ranking(mod)
            return
        assert trace_failures(mod.CacheModel), "the traces did not notice the planted mistake '%s'" % name
