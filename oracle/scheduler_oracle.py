"""CPU oracle of the compress-queue scheduler (test infrastructure; shares no
code with the library).

What the paper says (Algorithm 1 and the "Memory-Aware Scheduling" paragraph):
requests are accumulated; when the queue holds at least B_min of them or the
wait time is exceeded, FormBatch(Q, B_max) builds a batch; the scheduler looks
at ALL pending requests, not only the head of the queue, and constructs the
largest batch that fits the memory that is free right now; AdjustBatch adapts
the batch size to runtime conditions.  The paper gives no formulas, so the
readings taken here are:

  * time is an integer number of microseconds; arrivals are non-decreasing;
  * the memory a request needs in the compress stage is the blocks of its
    compressed cache, ceil(budget / 16) (new blocks are popped before the old
    ones are returned);
  * trigger: the queue is non-empty and (|Q| >= b_target or the oldest pending
    request has waited max_wait or longer);
  * FormBatch: requests that have waited max_wait or longer come first, in
    arrival order, each taken if it still fits (memory and B_max), skipped if
    not; then the others in order of (need, arrival, id) while they fit, which
    gives the largest number of requests that fits, with the smallest total
    need among such sets; the batch is returned in arrival order;
  * AdjustBatch: b_target = the number of arrivals expected during one batch
    service time, ceil(service / gap), clamped to [B_min, B_max], where service
    and gap are running averages avg += floor((x - avg) / 4) (the first sample
    sets the average) of the batch service times reported by the caller and of
    the gaps between arrivals; before both have a sample, b_target = B_min.
"""

BLOCK = 16


def blocks(budget):
    return (int(budget) + BLOCK - 1) // BLOCK


class Scheduler:
    def __init__(self, b_min, b_max, max_wait_us):
        assert 1 <= b_min <= b_max and max_wait_us >= 0
        self.b_min, self.b_max, self.max_wait = int(b_min), int(b_max), int(max_wait_us)
        self.b_target = self.b_min
        self.pending = []          # (arrival_us, id, seq_len, budget), arrival order
        self.gap_avg = 0           # 0 = no sample yet
        self.svc_avg = 0
        self.last_arrival = None

    @staticmethod
    def _avg(avg, x):
        if avg == 0:
            return x
        return avg + (x - avg) // 4          # floor division, also for negative differences

    def submit(self, req_id, arrival_us, seq_len, budget):
        """Returns False (and changes nothing) for an arrival before the last one,
        a budget outside 1..seq_len, or an id that is still pending."""
        if self.last_arrival is not None and arrival_us < self.last_arrival:
            return False
        if not (1 <= budget <= seq_len):
            return False
        if any(p[1] == req_id for p in self.pending):
            return False
        if self.last_arrival is not None:
            self.gap_avg = self._avg(self.gap_avg, arrival_us - self.last_arrival)
        self.last_arrival = arrival_us
        self.pending.append((int(arrival_us), int(req_id), int(seq_len), int(budget)))
        return True

    def ready(self, now_us):
        if not self.pending:
            return False
        return len(self.pending) >= self.b_target or now_us - self.pending[0][0] >= self.max_wait

    def form_batch(self, now_us, free_blocks):
        """The batch (list of ids in arrival order), empty if the trigger has not
        fired or nothing fits."""
        if not self.ready(now_us):
            return []
        overdue = [p for p in self.pending if now_us - p[0] >= self.max_wait]
        rest = [p for p in self.pending if now_us - p[0] < self.max_wait]
        rest.sort(key=lambda p: (blocks(p[3]), p[0], p[1]))
        chosen, used = [], 0
        for p in overdue:
            if len(chosen) < self.b_max and used + blocks(p[3]) <= free_blocks:
                chosen.append(p)
                used += blocks(p[3])
        for p in rest:
            if len(chosen) >= self.b_max or used + blocks(p[3]) > free_blocks:
                break
            chosen.append(p)
            used += blocks(p[3])
        ids = set(p[1] for p in chosen)
        batch = [p[1] for p in self.pending if p[1] in ids]
        self.pending = [p for p in self.pending if p[1] not in ids]
        return batch

    def adjust(self, service_us):
        self.svc_avg = self._avg(self.svc_avg, int(service_us))
        if self.gap_avg > 0 and self.svc_avg > 0:
            want = (self.svc_avg + self.gap_avg - 1) // self.gap_avg
            self.b_target = min(max(want, self.b_min), self.b_max)
        else:
            self.b_target = self.b_min
        return self.b_target
