"""Reference model of the host-to-device copy queue (TEST INFRASTRUCTURE ONLY).

The paper gives cache-miss resolution "the highest priority in the memory
queue" (Sec. 3.4) over one transfer stream (Sec. 4.1).  Reading used here,
since the paper describes no mechanism: experts travel over one link in chunks
of at most ``chunk_bytes``; at most ``depth`` chunks are committed to the link
at a time (they transfer one after the other at ``bandwidth`` bytes per
second); whenever there is room, the next chunk committed belongs to the oldest
priority copy (a miss of the layer being run, or a prefetch that a layer found
still queued and promoted), else to the oldest prefetch.  A priority copy
therefore waits for at most the chunks already committed, never for a whole
queued prefetch.  A copy is complete when its last chunk has transferred.

Plain event-driven simulation; times are floats in seconds.
"""
from __future__ import annotations


class CopyQueue:
    def __init__(self, bandwidth: float, chunk_bytes: int, depth: int):
        self.bw = float(bandwidth)
        self.chunk = int(chunk_bytes)
        self.depth = int(depth)
        self.pending = []        # [job] in arrival order; job = dict(id, left, miss)
        self.committed = []      # [(finish_time, job id)] in commit order
        self.done_at = {}        # job id -> completion time (known once its last chunk is committed)
        self.t = 0.0             # time up to which the queue has been simulated
        self.link_free = 0.0

    # -- internals ---------------------------------------------------------
    def _next(self):
        for j in self.pending:
            if j["miss"]:
                return j
        return self.pending[0] if self.pending else None

    def _fill(self):
        while len(self.committed) < self.depth:
            j = self._next()
            if j is None:
                return
            n = min(self.chunk, j["left"])
            start = max(self.link_free, self.t)
            finish = start + n / self.bw
            self.link_free = finish
            j["left"] -= n
            self.committed.append((finish, j["id"]))
            if j["left"] == 0:
                self.done_at[j["id"]] = finish
                self.pending.remove(j)

    def advance(self, now: float):
        """Simulate up to time `now`."""
        while True:
            self._fill()
            if not self.committed or self.committed[0][0] > now:
                break
            self.t = max(self.t, self.committed[0][0])
            self.committed.pop(0)
        self.t = max(self.t, now)
        self._fill()

    # -- interface ---------------------------------------------------------
    def submit(self, now: float, job_id, nbytes: int, miss: bool):
        self.advance(now)
        self.cancel(job_id)
        self.pending.append(dict(id=job_id, left=int(nbytes), miss=bool(miss)))
        self.done_at.pop(job_id, None)
        self._fill()

    def cancel(self, job_id):
        """A copy still queued for a slot that is handed to another expert is void."""
        self.pending = [j for j in self.pending if j["id"] != job_id]

    def wait(self, now: float, job_ids):
        """The layer being run needs these copies: they become priority copies; returns the time at which
        all of them are complete (never before `now`)."""
        self.advance(now)
        for j in self.pending:
            if j["id"] in job_ids:
                j["miss"] = True
        self._fill()
        while any(j["id"] in job_ids for j in self.pending):
            assert self.committed
            self.t = max(self.t, self.committed[0][0])
            self.committed.pop(0)
            self._fill()
        return max([now] + [self.done_at[i] for i in job_ids if i in self.done_at])
