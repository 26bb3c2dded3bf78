"""Plain event-order model of the asynchronous swap policy (TEST INFRASTRUCTURE ONLY).

Paper section 4.3: the moves of a query run asynchronously; a query whose blocks are still in flight waits
while the queries that are ready run.  The model keeps the waiting queries in a list in order of arrival and,
at every poll, hands out those whose moves have completed (oldest first, at most `max_ready`), leaving the rest
where they are.  Completion is told to it from outside, as a set of finished ids.
"""


class PolicyModel:
    def __init__(self):
        self.waiting = []          # ids in order of arrival
        self.done = set()          # ids whose moves have completed
        self.handed_out = []

    def submit(self, req_id, has_moves):
        assert req_id not in self.waiting
        self.waiting.append(req_id)
        if not has_moves:
            self.done.add(req_id)

    def complete(self, req_id):
        assert req_id in self.waiting
        self.done.add(req_id)

    def poll(self, max_ready):
        out = []
        for r in list(self.waiting):
            if len(out) >= max_ready:
                break
            if r in self.done:
                out.append(r)
        for r in out:
            self.waiting.remove(r)
            self.done.discard(r)
        self.handed_out.extend(out)
        return out
