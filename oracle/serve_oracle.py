"""CPU oracle of the continuous-batching loop's bookkeeping.  TEST INFRASTRUCTURE.

Only tests may import this file; it shares no code with the package.

Algorithm 3 (ContinuousBatching) with hybrid iteration-level batching: a pass admits requests
FCFS (sched_oracle.Batcher), executes one mini-batch made of one decode row for every batch
member whose prompt is done and a prompt chunk for every other member, and drops the members
that finished.  What the pass computes on the rows is the stage forward (stage_oracle); this
file models which rows run in which pass:
  - decode rows first, then prompt chunks, each group in batch order;
  - a chunk has min(max_chunk, prompt rows left, rows left in the pass) rows; at most 32 chunks
    and max_tokens rows per pass; members that get no row wait for the next pass;
  - KV pages: a request holds ceil(cached tokens / page_size) pages, taken from a free list
    (page 0 first; returned pages are reused last-in first-out) just before the rows that need
    them run.  A request gets its first rows only when the pages of its whole sequence,
    ceil((prompt_len + n_decode) / page_size), can be set aside out of the pages that no started
    request has set aside; until then it waits in the batch.  Started requests therefore always
    find their pages and finish, which returns their pages: the loop cannot stall with the pool
    full of partly served requests.
A request of prompt_len prompt rows and n_decode decode steps is finished after
prompt_len + n_decode rows.
"""
from oracle.sched_oracle import Batcher


class ServeModel:
    def __init__(self, C, T_w, n_pages, page_size, max_chunk, max_tokens):
        self.b = Batcher(C, T_w)
        self.free = list(range(n_pages - 1, -1, -1))
        self.unreserved = n_pages
        self.P, self.max_chunk, self.max_tokens = page_size, max_chunk, max_tokens
        self.req = {}

    def submit(self, rid, prompt_len, n_decode):
        self.b.push(rid, False)
        self.req[rid] = dict(prompt=prompt_len, total=prompt_len + n_decode, done=0, pages=[], reserved=0)

    def _take(self, r, rows):
        if not r["reserved"]:
            whole = -(-r["total"] // self.P)
            if whole > self.unreserved:
                return False
            r["reserved"] = whole
            self.unreserved -= whole
        need = -(-(r["done"] + rows) // self.P) - len(r["pages"])
        assert need <= len(self.free)
        for _ in range(need):
            r["pages"].append(self.free.pop())
        return True

    def run_pass(self, now):
        """Returns (members, finished, pages): members = [(id, first row, rows)], decode rows first;
        pages = the page list of every member as the pass sees it."""
        batch, new, _ = self.b.form(now)
        left = self.max_tokens
        dec, pre = [], []
        for rid in batch:
            r = self.req[rid]
            if r["done"] >= r["prompt"] and left > 0 and self._take(r, 1):
                dec.append((rid, r["done"], 1))
                left -= 1
        for rid in batch:
            r = self.req[rid]
            if r["done"] >= r["prompt"] or len(pre) >= 32:
                continue
            rows = min(self.max_chunk, r["prompt"] - r["done"], left)
            if rows > 0 and self._take(r, rows):
                pre.append((rid, r["done"], rows))
                left -= rows
        members = dec + pre
        pages = {rid: list(self.req[rid]["pages"]) for rid, _, _ in members}
        finished = []
        for rid, _, rows in members:
            r = self.req[rid]
            r["done"] += rows
            if r["done"] >= r["total"]:
                finished.append(rid)
        for rid in finished:
            r = self.req.pop(rid)
            self.free.extend(r["pages"])
            self.unreserved += r["reserved"]
        self.b.finish(finished)
        return members, finished, pages, len(batch), len(new)
