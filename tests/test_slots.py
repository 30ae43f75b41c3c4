"""Residency bookkeeping of the adapter slot manager (host logic; a manager without parts owns no
memory and issues no copies, so these run without a GPU) against a model written out here."""
import numpy as np
import pytest

import paper_2605_14217_amd as preft


class _Model:
    """Least-recently-used residency, one tick per acquire call, never evicting a slot the call names."""

    def __init__(self, n_adapters, n_slots):
        self.n_adapters, self.n_slots = n_adapters, min(n_slots, n_adapters)
        self.slot_of, self.adapter_in, self.last = {}, [-1] * self.n_slots, [0] * self.n_slots
        self.tick = self.hits = self.misses = self.evictions = 0

    def acquire(self, ids):
        self.tick += 1
        seen = set()
        for a in ids:
            if 0 <= a < self.n_adapters and a in self.slot_of and a not in seen:
                seen.add(a)
                self.hits += 1
                self.last[self.slot_of[a]] = self.tick
        out = []
        for a in ids:
            if not 0 <= a < self.n_adapters:
                out.append(-1)
                continue
            if a not in self.slot_of:
                free = [s for s in range(self.n_slots) if self.last[s] != self.tick]
                if not free:
                    return None
                victim = min(free, key=lambda s: (self.last[s], s))
                if self.adapter_in[victim] >= 0:
                    del self.slot_of[self.adapter_in[victim]]
                    self.evictions += 1
                self.adapter_in[victim], self.slot_of[a], self.last[victim] = a, victim, self.tick
                self.misses += 1
            out.append(self.slot_of[a])
        return out


@pytest.mark.parametrize("n_adapters,n_slots,batch,seed", [(40, 8, 6, 0), (512, 32, 32, 1), (5, 9, 4, 2), (16, 4, 4, 3)])
def test_residency_follows_the_lru_model(n_adapters, n_slots, batch, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    h = preft.preft_slots_create(n_adapters, n_slots, [])
    model = _Model(n_adapters, n_slots)
    try:
        for step in range(300):
            ids = rng.integers(-1, n_adapters + 1, size=int(rng.integers(0, batch + 1))).tolist()
            want = model.acquire(ids)
            assert want is not None
            got = preft.preft_slots_acquire(h, ids)
            assert got == want, f"step {step}"
            # a batch's adapters sit in distinct slots, and residency queries agree
            named = {a: s for a, s in zip(ids, got) if s >= 0}
            assert len(set(named.values())) == len(named)
            for a, s in named.items():
                assert preft.preft_slots_resident(h, a) == s
        st = preft.preft_slots_stats(h)
        assert (st["hits"], st["misses"], st["evictions"]) == (model.hits, model.misses, model.evictions)
        assert st["bytes_copied"] == 0 and st["n_slots"] == min(n_slots, n_adapters)
    finally:
        preft.preft_slots_destroy(h)


def test_more_distinct_adapters_than_slots_is_an_error_and_leaves_the_manager_usable():
    h = preft.preft_slots_create(10, 3, [])
    try:
        assert preft.preft_slots_acquire(h, [4, 5, 6]) == [0, 1, 2]
        with pytest.raises(preft.PreftError) as e:
            preft.preft_slots_acquire(h, [4, 7, 8, 9, 5])
        assert e.value.code == preft.PREFT_ECAPACITY
        # every slot holds one adapter, every resident adapter one slot
        slots = [preft.preft_slots_resident(h, a) for a in range(10)]
        held = [s for s in slots if s >= 0]
        assert sorted(held) == [0, 1, 2]
        assert preft.preft_slots_acquire(h, [1, 1, 1]) [0] == preft.preft_slots_resident(h, 1)
    finally:
        preft.preft_slots_destroy(h)


def test_bad_arguments():
    lib = preft.load_library()
    import ctypes
    handle = ctypes.c_void_p()
    assert lib.preft_slots_create(None, 4, 2, 0, None) == -1
    assert lib.preft_slots_create(ctypes.byref(handle), 0, 2, 0, None) == -1
    assert lib.preft_slots_create(ctypes.byref(handle), 4, 0, 0, None) == -1
    assert lib.preft_slots_create(ctypes.byref(handle), 4, 2, 2, None) == -1
    assert lib.preft_slots_create(ctypes.byref(handle), 4, 2, 33, None) == -1
    assert lib.preft_slots_acquire(None, None, 0, None, None) == -1
    assert lib.preft_slots_stats(None, None) == -1
    assert lib.preft_slots_resident(None, 0) == -1
    assert lib.preft_slots_pool(None, 0) is None
    assert lib.preft_slots_destroy(None) == 0
    h = preft.preft_slots_create(4, 2, [])
    try:
        assert lib.preft_slots_store(h, 0, 0, None, None) == -1          # a manager without parts stores nothing
        assert lib.preft_slots_pool(h, 0) is None
        assert preft.preft_slots_acquire(h, []) == []
    finally:
        preft.preft_slots_destroy(h)
    assert "slots" in preft.preft_strerror(preft.PREFT_ECAPACITY)
