"""CPU oracle of the dynamic data pipeline (section 4.3 of the paper): the
leader's bookkeeping that hands data partitions to workers on demand.

TEST INFRASTRUCTURE ONLY, like the rest of this package; it shares no code
with the library's implementation.  Pure integer work, plain Python.

What the section fixes, restated:

* the data set is cut into d partitions at the meta-data level only; the
  leader draws a random permutation of the partition indexes and replies to
  each request with the next unassigned partition;
* every worker keeps an offset into its current partition (where its next
  mini-batch starts);
* a joining worker is simply given unprocessed or partially processed
  partitions; a worker that leaves gracefully reports its current partition
  and offset, and the leader gives the rest of that partition to another
  worker;
* permutation and progress are part of the checkpoint;
* whatever scaling happens, an epoch goes over the data set once, without
  repetition and without omission.

Readings where the section is silent (also listed in the design notes):

R1  partition j covers the samples [j*s, min((j+1)*s, N)), s = ceil(N/d); a
    worker reads its partition front to back (sequential reads are the point
    of partitions).
R2  handed-back remainders are served before unassigned partitions, first
    in first out; the leavers of one adjustment hand back in their old rank
    order.
R3  a global mini-batch is assembled in worker-rank order, B/p samples per
    worker; a worker that the leader cannot serve in full (the epoch's data is
    running out) passes what it lacks on to the workers after it, wrapping
    round, so a mini-batch has B samples as long as the epoch has B left.  The
    shards of such a tail mini-batch can be unequal.
R4  an epoch ends when nothing is left anywhere (no unassigned partition, no
    remainder, every current partition read to its end); the next request
    starts epoch e+1 with the permutation of (seed, e+1).  The permutation is
    the job's own generator applied to d items, so d = N with a fixed worker
    set is the one-sample-partition scheme of the training step's shard
    assignment.

Parity pins: tests/test_oracle_pipeline.py (the shard-assignment oracle at
d = N; brute-force coverage of every epoch under random scaling schedules; the
paper's 10 -> 15 -> 12 worker example scaled down and at full size; hand-back
order; save / load).
"""
from . import oracle as _o


class DataPipeline:
    """The leader's state.  Workers are named by integer ids chosen by the
    caller; the set of ids may change between any two mini-batches."""

    def __init__(self, seed: int, N: int, d: int):
        if N <= 0 or d <= 0 or d > N:
            raise ValueError("need 0 < d <= N")
        self.seed, self.N, self.d = seed, N, d
        self.s = -(-N // d)
        if (d - 1) * self.s >= N:
            raise ValueError("d partitions of ceil(N/d) samples leave some partition empty")
        self.epoch = 0
        self.consumed = 0                      # samples handed out in this epoch
        self.perm = _o.epoch_permutation(seed, 0, d)
        self.cursor = 0                        # next unassigned position of perm
        self.remainders = []                   # handed back: (partition, offset), first in first out
        self.current = {}                      # worker id -> [partition, offset]; absent: holds nothing
        self.ranks = []                        # worker ids of the previous mini-batch, in rank order

    # -- partition geometry (R1)
    def _end(self, part: int) -> int:
        return min((part + 1) * self.s, self.N)

    def _next_piece(self):
        """(partition, offset) of the next piece the leader would hand out, or None (R2)."""
        if self.remainders:
            return self.remainders.pop(0)
        if self.cursor < self.d:
            part = self.perm[self.cursor]
            self.cursor += 1
            return (part, part * self.s)
        return None

    def _draw(self, wid: int, want: int, out: list) -> int:
        """Up to `want` samples for worker `wid`, appended to out; returns how many."""
        got = 0
        while got < want:
            cur = self.current.get(wid)
            if cur is None or cur[1] >= self._end(cur[0]):
                piece = self._next_piece()
                if piece is None:
                    self.current.pop(wid, None)
                    break
                cur = [piece[0], piece[1]]
                self.current[wid] = cur
            take = min(want - got, self._end(cur[0]) - cur[1])
            out.extend(range(cur[1], cur[1] + take))
            cur[1] += take
            got += take
        return got

    def next_batch(self, B: int, workers):
        """The next global mini-batch of B samples for the workers `workers`
        (ids in rank order).  Returns (idx, off): worker k's samples are
        idx[off[k]:off[k+1]]."""
        workers = list(workers)
        p = len(workers)
        if p <= 0 or B <= 0 or B % p or len(set(workers)) != p:
            raise ValueError("bad request")
        if self.N % B:
            raise ValueError("B must divide N")
        if self.consumed == self.N:                              # R4
            self.epoch += 1
            self.consumed = 0
            self.perm = _o.epoch_permutation(self.seed, self.epoch, self.d)
            self.cursor = 0
            self.remainders = []
            self.current = {}
        # graceful exits first, in the leavers' old rank order (R2)
        for wid in self.ranks:
            if wid not in workers:
                cur = self.current.pop(wid, None)
                if cur is not None and cur[1] < self._end(cur[0]):
                    self.remainders.append((cur[0], cur[1]))
        self.ranks = workers
        n = B // p
        shards = [[] for _ in range(p)]
        lacking = 0
        for k, wid in enumerate(workers):                        # R3: rank order, deficits passed on
            got = self._draw(wid, n + lacking, shards[k])
            lacking = n + lacking - got
        k = 0
        while lacking > 0 and k < p:                             # wrap round once: earlier workers may still hold data
            lacking -= self._draw(workers[k], lacking, shards[k])
            k += 1
        if lacking:
            raise RuntimeError("the epoch ran out inside a mini-batch")   # cannot happen while B divides N
        idx, off = [], [0]
        for sh in shards:
            idx.extend(sh)
            off.append(len(idx))
        self.consumed += B
        return idx, off

    # -- checkpoint (the permutation follows from seed and epoch)
    def save(self) -> dict:
        return dict(seed=self.seed, N=self.N, d=self.d, epoch=self.epoch, consumed=self.consumed, cursor=self.cursor,
                    remainders=[tuple(r) for r in self.remainders], ranks=list(self.ranks),
                    current={w: tuple(c) for w, c in self.current.items()})

    @classmethod
    def load(cls, st: dict) -> "DataPipeline":
        p = cls(st["seed"], st["N"], st["d"])
        p.epoch, p.consumed, p.cursor = st["epoch"], st["consumed"], st["cursor"]
        p.perm = _o.epoch_permutation(p.seed, p.epoch, p.d)
        p.remainders = [tuple(r) for r in st["remainders"]]
        p.ranks = list(st["ranks"])
        p.current = {w: list(c) for w, c in st["current"].items()}
        return p
