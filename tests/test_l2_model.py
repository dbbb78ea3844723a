"""The cache model behind the "why 21 % and not 32 %" argument (studies.py l2model), checked against
what it models: an LRU cache driven by independent references with a skewed popularity."""
from collections import OrderedDict

import numpy as np

from paper_2204_02662_amd.studies import lru_hit_rate_irm


def simulate_lru(prob, places, n_refs, seed):
    rng = np.random.default_rng(seed)
    refs = rng.choice(prob.size, size=n_refs, p=prob)
    cache, hits = OrderedDict(), 0
    warm = n_refs // 5
    for k, i in enumerate(refs.tolist()):
        if i in cache:
            cache.move_to_end(i)
            hits += k >= warm
        else:
            cache[i] = True
            if len(cache) > places:
                cache.popitem(last=False)
    return hits / (n_refs - warm)


def test_che_approximation_matches_a_simulated_lru_cache():
    items = 3000
    weight = 1.0 / np.arange(1, items + 1) ** 0.9  # heavy head, long tail
    prob = weight / weight.sum()
    for places in (30, 150, 600):
        model = lru_hit_rate_irm(weight, places)
        sim = simulate_lru(prob, places, 300_000, seed=places)
        static = float(np.sort(prob)[::-1][:places].sum())  # a cache that held the most popular items for good
        assert abs(model - sim) < 0.01, (places, model, sim)
        assert sim < static - 0.03, (places, sim, static)  # LRU is clearly below the static share


def test_cache_that_holds_everything_always_hits():
    assert lru_hit_rate_irm([5, 1, 1, 3], 4) == 1.0
