"""Refresh of the inverse roots on a second stream with bounded staleness (single-GPU form of the
paper's staleness barrier, Sec. III-D, swept over S in Sec. IV-C).

Host orchestration only: every arithmetic step is an entry point of the HIP library.  The loop is
the optimizer side of training: each step updates the statistics of every block and preconditions
every gradient with the PUBLISHED roots; every `pf` steps a refresh of all roots is due.

  - A refresh works on a snapshot of the statistics (one device copy on the step stream at the
    period boundary, so that the steps may go on updating L and R) and writes a private set of
    roots, on its own stream with its own workspace.  At most one refresh is in flight.
  - When a refresh has finished, its roots are published at the next step boundary: one device copy
    on the step stream into the set the steps read, and the version counter (the period index of the
    snapshot) is advanced - on the host and in a device word the steps could read.
  - Staleness bound S: a step of period p may use roots of version >= p - S.  If the published
    version is older, the step waits for the refresh in flight (the paper's rule: wait for the pending
    job when the version age exceeds S).  S = 0 is the synchronous schedule.

On one GPU the refresh and the steps share the same compute units, so asynchrony cannot remove the
refresh's work from the period; what it removes is the stall of a single step by a whole refresh.
`run` reports both: wall time per period, time spent waiting ("exposed" refresh time), and the
longest single step.
"""
from __future__ import annotations

import time


class RefreshPipeline:
    def __init__(self, torch, ast, run, pf: int = 10):
        """`run`: an object with the gradients `Gs`, `shapes`, `Ps` (outputs), `beta`, `eps_rel`, `opts`
        and the refresh workspace `ws` (bench.RootRun)."""
        self.torch, self.ast, self.run_, self.pf, self.S = torch, ast, run, pf, 0
        dev = run.Gs[0].device
        shapes = run.shapes
        # snapshot of the statistics and the private root set, each one flat buffer (one copy kernel)
        sizes = [m * m for m, n in shapes] + [n * n for m, n in shapes]
        total = sum(sizes)
        self.stats_flat = torch.zeros(total, device=dev)         # the live statistics move here (views)
        self.snap_flat = torch.empty(total, device=dev)
        self.pub_flat = torch.empty(total, device=dev)           # roots the steps read
        self.work_flat = torch.empty(total, device=dev)          # roots the refresh writes
        dims = [m for m, n in shapes] + [n for m, n in shapes]
        def views(flat):
            out, off = [], 0
            for d in dims:
                out.append(flat[off:off + d * d].view(d, d))
                off += d * d
            return out
        nb = len(shapes)
        live, snap, pub, work = views(self.stats_flat), views(self.snap_flat), views(self.pub_flat), views(self.work_flat)
        self.blocks = ast.Blocks(list(zip(run.Gs, live[:nb], live[nb:])))
        self.pblocks = ast.PBlocks(list(zip(pub[:nb], run.Gs, pub[nb:], run.Ps)))
        self.factors = ast.Factors(list(zip(snap, work)))
        self.ws_step = torch.empty(int(max(ast.stats_update_workspace_bytes(self.blocks),
                                           ast.precondition_workspace_bytes(self.pblocks))), dtype=torch.uint8, device=dev)
        self.info = torch.zeros(len(dims), dtype=torch.int32, device=dev)
        self.version_dev = torch.full((1,), -1, dtype=torch.int32, device=dev)
        self.refresh_stream = torch.cuda.Stream()               # default priority
        self.main = torch.cuda.current_stream()

    # -- pieces -----------------------------------------------------------------------------------
    def _step(self):
        self.ast.stats_update(self.blocks, self.run_.beta, ws=self.ws_step)
        self.ast.precondition(self.pblocks, ws=self.ws_step)

    def _launch_refresh(self, period):
        torch = self.torch
        self.snap_flat.copy_(self.stats_flat)                    # on the step stream: statistics as of this boundary
        ready = torch.cuda.Event()
        ready.record(self.main)
        with torch.cuda.stream(self.refresh_stream):
            self.refresh_stream.wait_event(ready)
            if self.work_free is not None:
                self.refresh_stream.wait_event(self.work_free)   # the last publish has read the private set
            self.ast.inverse_root(self.factors, self.run_.eps_rel, relative=True, root=4, opts=self.run_.opts,
                                  info=self.info, ws=self.run_.ws, stream=self.refresh_stream)
            done = torch.cuda.Event()
            done.record(self.refresh_stream)
        self.pending = (period, done)

    def _publish(self):
        period, done = self.pending
        self.main.wait_event(done)
        self.pub_flat.copy_(self.work_flat)                      # on the step stream, ordered with the steps
        self.version_dev.fill_(period)
        self.work_free = self.torch.cuda.Event()
        self.work_free.record(self.main)
        self.version, self.pending = period, None

    # -- the loop ---------------------------------------------------------------------------------
    def run(self, periods: int, staleness: int, warm_periods: int = 1):
        torch = self.torch
        self.S = int(staleness)
        self.version, self.pending, self.work_free = -1, None, None
        self.stats_flat.zero_()
        # roots to start from: one synchronous refresh of the initial statistics
        self._step_stats_only()
        self._launch_refresh(-1)
        self.pending[1].synchronize()
        self._publish()
        torch.cuda.synchronize()
        waited, max_age, step_events = 0.0, 0, []
        t_start, launched, n_launched = None, -1, 0
        for p in range(warm_periods + periods):
            if p == warm_periods:
                torch.cuda.synchronize()
                waited, max_age, step_events, n_launched = 0.0, 0, [], 0
                t_start = time.time()
            for s in range(self.pf):
                if self.pending is not None and self.pending[1].query():
                    self._publish()                              # finished: publish at this step boundary
                if self.pending is None and launched < p:
                    self._launch_refresh(p)                      # a refresh is due once per period, as soon as
                    launched = p                                 # the one before it has been published
                    n_launched += 1
                if p - self.version > self.S and self.pending is not None:
                    t = time.time()
                    self.pending[1].synchronize()                # staleness barrier: wait for the refresh in flight
                    waited += time.time() - t
                    self._publish()
                max_age = max(max_age, p - self.version)
                e = torch.cuda.Event(enable_timing=True)
                self._step()
                e.record(self.main)
                step_events.append(e)
        torch.cuda.synchronize()
        wall = time.time() - t_start
        lat = [a.elapsed_time(b) for a, b in zip(step_events[:-1], step_events[1:])]
        if self.pending is not None:                             # drain
            self.pending[1].synchronize()
            self._publish()
            torch.cuda.synchronize()
        # without waiting (large S) the steps of a period can finish before its refresh does: the refresh of
        # the next period then starts late, and fewer than `periods` refreshes fall into the timed window
        return {"period_ms": 1e3 * wall / periods, "refreshes_started": int(n_launched),
                "exposed_ms": 1e3 * waited / periods, "max_age": int(max_age),
                "max_step_ms": max(lat) if lat else 0.0, "median_step_ms": sorted(lat)[len(lat) // 2] if lat else 0.0,
                "not_converged": int((self.info != 0).sum())}

    def _step_stats_only(self):
        self.ast.stats_update(self.blocks, self.run_.beta, ws=self.ws_step)
