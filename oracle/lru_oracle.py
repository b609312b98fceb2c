"""CPU model of the LRU cache over a host-memory table -- TEST INFRASTRUCTURE (plain Python).

Section 4.2.2: the parameter server keeps the embedding parameters in an LRU cache, an array list of entries
plus a map from key to the entry's index; when the cache is full the least recently used entry makes room.

Readings (the paper describes a per-item LRU on CPU threads; here a whole batch arrives at once):
  * recency is per call: all rows of one call are equally recent (they share the call's step number);
  * a call that misses M rows replaces the M least recently used slots among those the call itself does not
    use; among slots of equal age the lower slot index goes first, ages of `age_max` - 1 calls and more count
    as equal (everything that cold is equally cold), and empty slots are older than any row;
  * the missing rows, in ascending row order, receive the freed slots in this order: first every slot strictly
    older than the youngest age that has to give, in slot order, then the slots of exactly that age, in slot
    order.
The cache is transparent (what a lookup or an update computes does not depend on it); this model exists to
check the policy: which rows are resident, in which slot, and how many misses and write-backs each call costs.
Parity status: pinned (tests/test_lru_oracle_pins.py: textbook per-item LRU, recency invariant, capacity).
"""


class LruCache:
    def __init__(self, capacity, age_max=1023):
        self.C = int(capacity)
        self.age_max = int(age_max)
        self.slot_row = [None] * self.C     # the array list: row held by each slot
        self.stamp = [0] * self.C           # step of the slot's last use (0 = never)
        self.where = {}                     # the map: row -> slot
        self.step = 0
        self.requested = self.misses = self.written_back = 0

    def access(self, rows):
        """One call touching the given rows (any iterable; duplicates ignored).  Returns (hits, misses)."""
        rows = sorted(set(int(r) for r in rows))
        if not rows:
            return 0, 0
        self.step += 1
        missing = []
        for r in rows:
            s = self.where.get(r)
            if s is None:
                missing.append(r)
            else:
                self.stamp[s] = self.step
        M = len(missing)
        self.requested += len(rows)
        self.misses += M
        if M == 0:
            return len(rows), 0
        # an empty slot is older than any row; rows idle for age_max - 1 calls or more are equally old
        age = lambda s: self.age_max if self.stamp[s] == 0 else min(self.step - self.stamp[s], self.age_max - 1)
        free = [s for s in range(self.C) if self.stamp[s] != self.step]
        if len(free) < M:
            raise ValueError("the call needs more slots than the cache can free")
        # the youngest age that still has to give up slots
        by_age = sorted(free, key=lambda s: -age(s))
        threshold = age(by_age[M - 1])
        older = [s for s in free if age(s) > threshold]                 # slot order
        equal = [s for s in free if age(s) == threshold][:M - len(older)]
        for r, s in zip(missing, older + equal):
            old = self.slot_row[s]
            if old is not None:
                del self.where[old]
                self.written_back += 1
            self.slot_row[s] = r
            self.stamp[s] = self.step
            self.where[r] = s
        return len(rows) - M, M
