"""Reference model of the per-layer expert cache and prefetch queue.  TEST INFRASTRUCTURE.

Plain Python lists; follows the paper's Alg. 1 (prediction + task-queue management), Alg. 2
(prefetch execution) and the "Cache Implementation" paragraph (LRU queue: a new expert evicts the
head and is pushed to the tail; an expert already in the queue is removed and reinserted at the
back).  Readings of points the paper leaves open:

* one queue per layer with a fixed number of slots (the paper reserves "a fixed number of experts
  per layer");
* a task names at most as many experts as the layer has slots: a ranked prediction (or a raw
  list) longer than that is cut to the slot count, in the given order, BEFORE the cached ones
  are dropped (Alg. 1's task is TopK_Index's k experts, and k never exceeds the per-layer
  budget in the paper);
* a predicted expert that is already cached is removed from the load list (Alg. 1) *and* touched,
  so the task that predicted it cannot pick it as a victim;
* victims are taken from the head of the queue (Alg. 2's "first N entries"); because the task's
  cached experts were moved to the tail first and cached + loaded experts of one task are no
  more than the slot count, a task never evicts one of its own experts;
* at verification, cached experts are used first, then missing ones are loaded on demand in
  ascending expert order, each evicting the current head (which may be an expert this same batch
  has already used, when the batch needs more experts than there are slots);
* layers beyond the cutoff L are not predicted or prefetched (Alg. 1's "l <= L", 0-based, inclusive);
* metadata changes at call time, in program order; only the copies themselves are asynchronous.

The model predicts, for any sequence of prefetch / verify calls, the exact queue order, hits,
misses and evictions that the library must report.
"""


def rank_predicted(pidx, prob, n_experts):
    """Alg. 1's `experts` when one task scores several draft states at once (the paper's hook fires per draft
    token, so it is silent here; with one state this is TopK_Index's own order): every expert some state selected,
    most-voted first, then larger summed gate probability over the states that selected it, then lower index.
    pidx[n][k]: selected experts per state; prob[n][E]: softmax probabilities per state."""
    votes = [0] * n_experts
    psum = [0.0] * n_experts
    for t, row in enumerate(pidx):
        for e in row:
            e = int(e)
            votes[e] += 1
            psum[e] += float(prob[t][e])
    chosen = [e for e in range(n_experts) if votes[e] > 0]
    return sorted(chosen, key=lambda e: (-votes[e], -psum[e], e))


class CacheModel:
    def __init__(self, n_layers, n_experts, slots, cutoff_layer=-1):
        self.n_layers, self.n_experts, self.slots, self.cutoff = n_layers, n_experts, slots, cutoff_layer
        self.reset()

    def reset(self):
        # queue[l]: expert ids, head (index 0) = least recently used
        self.queue = [[] for _ in range(self.n_layers)]
        # experts brought in by prefetch and not yet used by a verify pass
        self.unused_prefetch = [set() for _ in range(self.n_layers)]
        self.stats = dict(hits=0, misses=0, evictions=0, prefetch_issued=0, prefetch_used=0,
                          prefetch_wasted=0, ondemand_loads=0)

    # ---- LRU primitives ("Cache Implementation") ------------------------------------------------
    def _touch(self, layer, e):
        q = self.queue[layer]
        q.remove(e)
        q.append(e)

    def _insert(self, layer, e):
        """Bring expert e in at the tail; if the queue is full the head is evicted.  Returns the victim or None."""
        q = self.queue[layer]
        victim = None
        if len(q) >= self.slots:
            victim = q.pop(0)
            self.stats["evictions"] += 1
            if victim in self.unused_prefetch[layer]:
                self.unused_prefetch[layer].discard(victim)
                self.stats["prefetch_wasted"] += 1
        q.append(e)
        return victim

    # ---- Alg. 1 lines 4-6 + Alg. 2 ---------------------------------------------------------------
    def filter_cached(self, layer, experts):
        """Alg. 1 lines 1 and 4-6 for a ranked prediction: nothing beyond the cutoff layer; duplicates
        dropped (order kept); the list cut to the slot count; predicted experts already in Q_cache
        dropped from it.  The cached ones are touched, so the task built from the rest cannot pick
        them as victims.  Returns the experts left to load."""
        if self.cutoff < 0 or layer > self.cutoff:
            return []
        task = []
        for e in experts:
            if e not in task:
                task.append(e)
        task = task[: self.slots]
        out = []
        for e in task:
            if e in self.queue[layer]:
                self._touch(layer, e)
            else:
                out.append(e)
        return out

    def prefetch(self, layer, experts):
        """One prefetch task for `layer` (Alg. 2).  Returns [(expert, victim_or_None)] actually loaded."""
        if self.cutoff < 0 or layer > self.cutoff:
            return []
        uniq = []
        for e in experts:
            if e not in uniq:
                uniq.append(e)
        uniq = uniq[: self.slots]
        for e in uniq:                           # predicted and cached: touched, not loaded
            if e in self.queue[layer]:
                self._touch(layer, e)
        loaded = []
        for e in uniq:
            if e in self.queue[layer]:
                continue
            victim = self._insert(layer, e)      # head of the queue; never one of this task's experts
            self.unused_prefetch[layer].add(e)
            self.stats["prefetch_issued"] += 1
            loaded.append((e, victim))
        return loaded

    # ---- verification-time use ("Computation Implementation": cached experts first) -------------
    def verify(self, layer, needed):
        """`needed`: distinct routed experts of the verify batch, ascending.  Cached experts are
        used (and touched) first, then each missing one is loaded on demand in ascending order,
        evicting the queue head.  Returns (hits, [(missed_expert, victim_or_None)])."""
        needed = list(needed)
        hits = [e for e in needed if e in self.queue[layer]]
        misses = [e for e in needed if e not in self.queue[layer]]
        self.stats["hits"] += len(hits)
        self.stats["misses"] += len(misses)
        for e in hits:
            self._touch(layer, e)
            if e in self.unused_prefetch[layer]:
                self.unused_prefetch[layer].discard(e)
                self.stats["prefetch_used"] += 1
        loaded = []
        for e in misses:
            victim = self._insert(layer, e)
            self.stats["ondemand_loads"] += 1
            loaded.append((e, victim))
        return hits, loaded

    def contents(self, layer):
        return list(self.queue[layer])

    def hit_rate(self):
        n = self.stats["hits"] + self.stats["misses"]
        return self.stats["hits"] / n if n else 0.0
