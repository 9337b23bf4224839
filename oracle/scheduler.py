"""FCFS continuous-batching scheduler with paged-KV accounting: an integer state machine.
Oracle code: test infrastructure only.

Follows the scheduler loop of section 4.2 of the paper (persistent scheduler; continuous
batching with inline prefill; ring buffer): scan the ring for submitted prompts, claim
them, run a prefill pass for the newly admitted while running decodes are paused, otherwise
a decode pass over everything running, then publish tokens and retire finished requests.
The paper gives no KV-block algorithm; the reading taken here:

  * Requests carry tickets 0,1,2,.. in submission order; ring slot = ticket mod ring_slots.
  * One iteration = one forward pass. At its start: (1) retire what finished in the previous
    iteration, batch slot ascending, pushing blocks back in block-table order; (2) poll:
    tickets below `tail` are visible; (3) admit strictly in ticket order, no skipping, while
    a batch slot is free, the worst-case reservation ceil((P + max_new - 1)/bs) (at least 1)
    fits in n_blocks - committed, and the prompt tokens admitted this iteration stay within
    max_prefill_tokens (the first admitted request is exempt); (4) any admission makes this
    a prefill iteration over exactly the admitted requests, else a decode iteration over all
    running requests, else idle; (5) allocate physical blocks, batch slot ascending:
    ceil(P/bs) for a prefill, one more for a decode whose context fills its blocks exactly;
    the free list is a stack whose first pops return 0,1,2,..; (6) build the batch metadata.
  * After the forward pass and sampling: append the token, finish a request when it has
    max_new tokens or emitted the end-of-sequence id (which is emitted and counted).

Chunked prefill with mixed iterations (`chunked=True`), the first extension the paper names in its discussion
(section 7: the scheduler already tracks per-request progress). The paper gives no algorithm; the reading taken here
is the usual token-budget one: an iteration carries at most max_prefill_tokens tokens. Every running request that has
its whole prompt cached decodes (one token each, never paused). The remaining budget goes to prompts in ticket order:
first to the one request that may be part-way through its prompt, then to new admissions, each taking
min(prompt tokens left, budget left); a request is admitted only while budget is left (so it processes at least one
token in the iteration that admits it, and at most one request is ever part-way), a batch slot is free and its
reservation fits. A request samples its first token in the iteration that processes the last token of its prompt;
blocks are allocated as the cached length grows. Decodes are not paused in this mode.

On-demand KV growth with preemption (`preempt=True`; the paper's slot life cycle has DECODE_PAUSED "to support
preemption", section 4.2, and says no more). The reading taken here replaces the worst-case reservation: a request is
admitted when the blocks of the tokens it must prefill are free NOW (beside those promised to requests admitted before it
in the same iteration); decoding requests take a block from the free stack when their context fills their blocks. When a
decode iteration needs more blocks than are free, running requests are preempted, the most recently submitted (highest
ticket) first, until the rest fits: a victim gives back all its blocks (in block-table order), leaves its batch slot and
goes to DECODE_PAUSED. Preempted requests are resumed before any new request is admitted, lowest ticket first, by
recomputation: the resumed request prefills its prompt followed by the tokens it has generated so far and samples its
next output token from the last position, so its stream continues where it stopped. The oldest running request is never
short of blocks once the others are gone, because a request that could not fit the pool alone is refused at submission.

Prefix caching (`prefix_cache=True`; section 7 of the paper: the paged cache provides reusable blocks, and a hash
table inside the scheduler can map token prefixes to blocks. It says no more). The reading taken here, for the plain mode:
  * Unit: a full block of PROMPT tokens. Block j of a prompt has the key h_j = mix64(h_{j-1} xor g_j), h_{-1} a constant,
    g_j a hash of the block's 16 token ids (prefix_block_hash, prefix_chain): the key covers the whole prefix up to and
    including block j. The table maps key -> physical block; two prefixes with equal 64-bit keys are taken as equal.
  * Admission of a request matches the leading blocks of its prompt against the table as it stands at the start of the
    iteration, stopping at the first miss and never matching the block that holds the last prompt token (at least one
    token is computed). The m matched blocks head its block table, its prefill computes the tokens from 16 m on, and
    it reserves its worst case minus m. Matched blocks are reference-counted; cached blocks in use count once against
    the pool (pinned), beside the private reservations. In the FCFS admission test a matched block that is idle at
    the start of the iteration is charged to every candidate that matches it (conservative inside one iteration).
    The prefill-token budget counts computed tokens.
  * After the allocation of a prefill iteration every admitted request, in batch-slot order, enters its own full prompt
    blocks beyond the matched ones into the table (reference count 1, moved from its private reservation to the
    pinned count) unless the key is already there; a block whose key is present stays private.
  * The free list is a double-ended queue. Retirement pushes private blocks on top in block-table order as before;
    a cached block whose reference count drops to zero stays in the table and goes to the BOTTOM, the request's
    blocks in reverse block-table order (so the head of a prefix lies deepest). Allocation pops from the top: private
    blocks are reused first, idle cached blocks oldest first, and a prefix loses its tail before its head. Popping
    an idle cached block evicts it from the table. A match on an idle block takes it out of the queue by moving
    the top element into its place.

Speculative decoding (`speculative=k > 0`; section 7: the scheduler runs draft generation followed by target verification
and publishes only accepted tokens. It names no draft source). The reading taken here needs no second model:
  * Drafts by lookup in the request's own tokens (prompt, then outputs), for greedy requests only: with n tokens so far,
    the last of them not yet in the cache, find the most recent earlier place i <= n - 3, not further back than
    SPEC_LOOKBACK positions, where tokens i, i + 1 equal tokens n - 2, n - 1; the up to k tokens that followed there
    (i + 2 ...) are the drafts, never more than the request may still emit minus one.
  * A decode iteration processes, per request, its last token and its m drafts at consecutive positions (blocks for all of
    them are taken from the request's reservation) and computes a logits row at every one of the m + 1 positions.
  * Verification, per request in row order: row j gives token t_j (the request's own sampler at output index gen + j);
    t_j is emitted; the walk goes on to row j + 1 only if t_j equals draft j and the request has not finished. What is
    emitted is exactly what one-token-per-iteration decoding emits; cached entries of rejected drafts lie beyond the
    context length and are overwritten later.
Plain mode only.
"""
import numpy as np

SPEC_LOOKBACK = 1024

MASK64 = (1 << 64) - 1
PREFIX_H0 = 0x243F6A8885A308D3


def mix64(z):
    """The finalizer of splitmix64 (Steele, Lea and Flood's generator) on a 64-bit integer."""
    z &= MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def prefix_block_hash(tokens):
    """g of one block: polynomial in the token ids modulo 2^64, then mixed."""
    a = 0
    for t in tokens:
        a = (a * 0x9E3779B97F4A7C15 + int(t) + 1) & MASK64
    return mix64(a)


def prefix_chain(h_prev, tokens):
    return mix64(h_prev ^ prefix_block_hash(tokens))


EMPTY, PREFILL_PENDING, PREFILL_PROCESSING, DECODE_PROCESSING, DECODE_COMPLETED, DECODE_PAUSED = range(6)

LEGAL_EDGES = {
    (EMPTY, PREFILL_PENDING), (PREFILL_PENDING, PREFILL_PROCESSING),
    (PREFILL_PROCESSING, DECODE_PROCESSING), (PREFILL_PROCESSING, DECODE_COMPLETED),
    (DECODE_PROCESSING, DECODE_PAUSED), (DECODE_PAUSED, DECODE_PROCESSING),
    (DECODE_PROCESSING, DECODE_COMPLETED), (DECODE_PAUSED, DECODE_COMPLETED),
    (DECODE_COMPLETED, EMPTY),
}

IDLE, PREFILL, DECODE = 0, 1, 2


class Running:
    __slots__ = ("ticket", "P", "max_new", "gen", "ctx_len", "reserved", "blocks", "finished", "last_token", "prefilled",
                 "h_end", "n_matched")

    def prefilled_blocks(self, bs):
        return self.n_matched


class Plan:
    """Batch metadata of one iteration (section 4.2: what the scheduler populates before a launch)."""

    def __init__(self):
        self.kind = IDLE
        self.iteration = 0
        self.tail = 0
        self.admitted = []      # tickets admitted this iteration, in order
        self.resumed = []       # preemption mode: tickets resumed this iteration (before the admissions), in order
        self.preempted = []     # preemption mode: tickets preempted this iteration, in order (highest ticket first)
        self.batch_slots = []   # batch slot of each sequence in this iteration, ascending
        self.tickets = []
        self.seq_lens = []      # context length of each sequence after this iteration's tokens
        self.cu_seqlens = [0]   # token offsets per sequence
        self.input_ids = []
        self.positions = []
        self.slot_mapping = []
        self.tok_seq = []
        self.last_idx = []
        self.block_tables = []  # per sequence, list of block ids
        self.gen_index = []     # index of the output token each sampling sequence samples in this iteration
        self.sample_seq = []    # indices (into tickets / batch_slots) of the sequences that sample a token in this iteration;
                                # last_idx and gen_index have one entry per sampling sequence. Without chunked prefill every
                                # sequence of an iteration samples
        self.pos0 = []          # position of the first token each sequence processes in this iteration
        self.row0 = []          # speculative decoding: first logits row (index into last_idx) of each sequence; the rows of a
                                # sequence are consecutive, one per token it processes in a decode iteration (last_idx then has
                                # one entry per row, not per sequence)
        self.free_blocks_after = 0

    @property
    def sample_tickets(self):
        return [self.tickets[i] for i in self.sample_seq]


def blocks_needed(P, max_new, bs):
    return max(1, -(-(P + max_new - 1) // bs))


class Scheduler:
    def __init__(self, n_blocks, block_size, max_batch, max_prefill_tokens, ring_slots, eos_token_id=-1,
                 free_list=None, chunked=False, preempt=False, prefix_cache=False, speculative=0):
        self.chunked, self.preempt, self.prefix_cache = chunked, preempt, prefix_cache
        assert not (prefix_cache and (chunked or preempt)), "prefix caching is defined for the plain mode only"
        self.speculative = int(speculative)
        assert not (self.speculative and (chunked or preempt or prefix_cache)), "speculative decoding is defined for the plain mode only"
        self.greedy = {}            # ticket -> whether the request decodes greedily (only those speculate)
        self.drafted = self.accepted = 0
        self.table = {}             # prefix caching: key -> block
        self.bkey = {}              # block -> key, for the cached blocks
        self.ref = [0] * n_blocks   # running requests that hold the cached block
        self.pinned = 0             # cached blocks with a reference
        self.cache_hits = 0         # blocks matched so far
        self.evictions = 0
        assert not (chunked and preempt), "preemption is defined for the plain (pause-and-resume) mode only"
        self.preempted = []         # Running records of preempted requests (no blocks, no batch slot)
        if chunked:
            assert max_prefill_tokens > max_batch, "the token budget must leave room for a prompt token beside the decodes"
        self.n_blocks, self.bs, self.max_batch = n_blocks, block_size, max_batch
        self.max_prefill_tokens, self.ring_slots, self.eos = max_prefill_tokens, ring_slots, eos_token_id
        # stack: pop from the end. Default order makes the first pops return 0, 1, 2, ...
        self.free = list(range(n_blocks - 1, -1, -1)) if free_list is None else list(free_list)
        self.running = [None] * max_batch
        self.committed = 0
        self.next_ticket = 0
        self.iteration = 0
        self.requests = {}          # ticket -> (prompt, max_new)
        self.state = {}             # ticket -> slot state
        self.transitions = []       # (ticket, from, to)
        self.outputs = {}           # ticket -> list of tokens

    @classmethod
    def from_engine(cls, eng):
        """From an engine configuration dict (synth.configs)."""
        return cls(eng["kv_num_blocks"], eng["kv_block_size"], eng["max_batch"], eng["max_prefill_tokens"], eng["ring_slots"],
                   eng.get("eos_token_id", -1), chunked=bool(eng.get("chunked_prefill", False)), preempt=bool(eng.get("preemption", False)),
                   prefix_cache=bool(eng.get("prefix_cache", False)), speculative=int(eng.get("speculative", 0)))

    # ---- ring side -------------------------------------------------------------------
    def submit(self, prompt, max_new, greedy=True):
        t = len(self.requests)
        self.greedy[t] = bool(greedy)
        self.requests[t] = (np.asarray(prompt, dtype=np.int64), int(max_new))
        self.outputs[t] = []
        self.state[t] = EMPTY
        self._set(t, PREFILL_PENDING)
        return t

    def _set(self, ticket, new):
        old = self.state[ticket]
        self.transitions.append((ticket, old, new))
        self.state[ticket] = new

    # ---- one iteration: steps (1)-(6) -------------------------------------------------
    def step(self, tail):
        if self.chunked:
            return self._step_chunked(tail)
        if self.preempt:
            return self._step_preempt(tail)
        if self.prefix_cache:
            return self._step_cached(tail)
        bs = self.bs
        plan = Plan()
        plan.tail = tail
        # (1) retire
        for b in range(self.max_batch):
            r = self.running[b]
            if r is not None and r.finished:
                self.free.extend(r.blocks)
                self.committed -= r.reserved
                self.running[b] = None
        # (2)+(3) admit in ticket order
        admitted_tokens = 0
        new_slots = []
        while self.next_ticket < tail:
            t = self.next_ticket
            prompt, max_new = self.requests[t]
            P = prompt.size
            need = blocks_needed(P, max_new, bs)
            free_slots = [b for b in range(self.max_batch) if self.running[b] is None]
            if not free_slots:
                break
            if self.committed + need > self.n_blocks:
                break
            if new_slots and admitted_tokens + P > self.max_prefill_tokens:
                break
            r = Running()
            r.ticket, r.P, r.max_new, r.gen, r.ctx_len = t, P, max_new, 0, 0
            r.reserved, r.blocks, r.finished, r.last_token, r.prefilled = need, [], False, -1, P
            b = free_slots[0]
            self.running[b] = r
            self.committed += need
            admitted_tokens += P
            new_slots.append(b)
            plan.admitted.append(t)
            self._set(t, PREFILL_PROCESSING)
            self.next_ticket = t + 1
        # (4) kind
        if new_slots:
            plan.kind = PREFILL
            slots = sorted(new_slots)
            for b in range(self.max_batch):   # running decodes are paused for this iteration
                r = self.running[b]
                if r is not None and b not in new_slots and self.state[r.ticket] == DECODE_PROCESSING:
                    self._set(r.ticket, DECODE_PAUSED)
        else:
            slots = [b for b in range(self.max_batch) if self.running[b] is not None]
            if not slots:
                plan.kind = IDLE
                return plan
            plan.kind = DECODE
            for b in slots:
                r = self.running[b]
                if self.state[r.ticket] == DECODE_PAUSED:
                    self._set(r.ticket, DECODE_PROCESSING)
        plan.iteration = self.iteration
        self.iteration += 1
        # (5) allocate, (6) metadata
        for si, b in enumerate(slots):
            r = self.running[b]
            if plan.kind == PREFILL:
                for _ in range(-(-r.P // bs)):
                    r.blocks.append(self.free.pop())
                toks = list(self.requests[r.ticket][0])
                pos = list(range(r.P))
                r.ctx_len = r.P
            else:
                drafts = self._drafts(r) if self.speculative else []
                toks = [r.last_token] + drafts
                pos = list(range(r.ctx_len, r.ctx_len + len(toks)))
                while len(r.blocks) * bs < r.ctx_len + len(toks):
                    r.blocks.append(self.free.pop())
                r.ctx_len += len(toks)               # provisional: commit() takes back the rejected drafts
            plan.batch_slots.append(b)
            plan.tickets.append(r.ticket)
            plan.seq_lens.append(r.ctx_len)
            first_row = len(plan.input_ids) if (plan.kind == DECODE and self.speculative) else len(plan.input_ids) + len(toks) - 1
            plan.input_ids += [int(x) for x in toks]
            plan.positions += pos
            plan.slot_mapping += [r.blocks[p // bs] * bs + p % bs for p in pos]
            plan.tok_seq += [si] * len(pos)
            plan.cu_seqlens.append(len(plan.input_ids))
            if self.speculative:                      # a logits row at every position of a decoding sequence
                plan.row0.append(len(plan.last_idx))
                plan.last_idx += list(range(first_row, len(plan.input_ids)))
            else:
                plan.last_idx.append(len(plan.input_ids) - 1)
            plan.block_tables.append(list(r.blocks))
            plan.gen_index.append(r.gen)
            plan.sample_seq.append(si)
            plan.pos0.append(pos[0])
        plan.free_blocks_after = len(self.free)
        return plan

    def _tokens_so_far(self, r):
        return [int(x) for x in self.requests[r.ticket][0]] + self.outputs[r.ticket]

    def _drafts(self, r):
        if not self.greedy[r.ticket]:
            return []
        s = self._tokens_so_far(r)
        n = len(s)
        room = min(self.speculative, r.max_new - r.gen - 1)
        if n < 3 or room <= 0:
            return []
        for i in range(n - 3, max(-1, n - 3 - SPEC_LOOKBACK), -1):
            if s[i] == s[n - 2] and s[i + 1] == s[n - 1]:
                return s[i + 2:i + 2 + room]
        return []

    # ---- one iteration with prefix caching ---------------------------------------------------------------------------
    def _pop_block(self):
        blk = self.free.pop()
        if blk in self.bkey:                  # an idle cached block is reused: evicted
            del self.table[self.bkey.pop(blk)]
            self.evictions += 1
        return blk

    def _step_cached(self, tail):
        bs = self.bs
        plan = Plan()
        plan.tail = tail
        # (1) retire
        for b in range(self.max_batch):
            r = self.running[b]
            if r is not None and r.finished:
                idle = []
                for blk in r.blocks:
                    if blk in self.bkey:
                        self.ref[blk] -= 1
                        if self.ref[blk] == 0:
                            self.pinned -= 1
                            idle.append(blk)
                    else:
                        self.free.append(blk)
                for blk in reversed(idle):
                    self.free.insert(0, blk)
                self.committed -= r.reserved
                self.running[b] = None
        # (2)+(3) admit in ticket order against the table and the reference counts of the start of the iteration
        ref0 = list(self.ref)
        load = self.committed + self.pinned
        admitted_tokens = 0
        new_slots = []
        while self.next_ticket < tail:
            t = self.next_ticket
            prompt, max_new = self.requests[t]
            P = prompt.size
            h, matched = PREFIX_H0, []
            for j in range((P - 1) // bs):
                hj = prefix_chain(h, prompt[j * bs:(j + 1) * bs])
                if hj not in self.table:
                    break
                matched.append(self.table[hj])
                h = hj
            m = len(matched)
            need = blocks_needed(P, max_new, bs) - m
            charge = need + sum(1 for blk in matched if ref0[blk] == 0)
            free_slots = [b for b in range(self.max_batch) if self.running[b] is None]
            if not free_slots:
                break
            if load + charge > self.n_blocks:
                break
            if new_slots and admitted_tokens + (P - m * bs) > self.max_prefill_tokens:
                break
            for blk in matched:
                if self.ref[blk] == 0:           # idle: out of the queue, the top element fills its place
                    i = self.free.index(blk)
                    top = self.free.pop()
                    if i < len(self.free):
                        self.free[i] = top
                    self.pinned += 1
                self.ref[blk] += 1
            self.cache_hits += m
            r = Running()
            r.ticket, r.P, r.max_new, r.gen, r.ctx_len = t, P, max_new, 0, 0
            r.reserved, r.blocks, r.finished, r.last_token, r.prefilled = need, list(matched), False, -1, P
            r.h_end, r.n_matched = h, m
            b = free_slots[0]
            self.running[b] = r
            self.committed += need
            load += charge
            admitted_tokens += P - m * bs
            new_slots.append(b)
            plan.admitted.append(t)
            self._set(t, PREFILL_PROCESSING)
            self.next_ticket = t + 1
        # (4) kind
        if new_slots:
            plan.kind = PREFILL
            slots = sorted(new_slots)
            for b in range(self.max_batch):
                r = self.running[b]
                if r is not None and b not in new_slots and self.state[r.ticket] == DECODE_PROCESSING:
                    self._set(r.ticket, DECODE_PAUSED)
        else:
            slots = [b for b in range(self.max_batch) if self.running[b] is not None]
            if not slots:
                plan.kind = IDLE
                return plan
            plan.kind = DECODE
            for b in slots:
                r = self.running[b]
                if self.state[r.ticket] == DECODE_PAUSED:
                    self._set(r.ticket, DECODE_PROCESSING)
        plan.iteration = self.iteration
        self.iteration += 1
        # (5) allocate, (6) metadata
        for si, b in enumerate(slots):
            r = self.running[b]
            if plan.kind == PREFILL:
                p0 = len(r.blocks) * bs                      # the matched prefix is not recomputed
                for _ in range(-(-r.P // bs) - len(r.blocks)):
                    r.blocks.append(self._pop_block())
                toks = list(self.requests[r.ticket][0][p0:])
                pos = list(range(p0, r.P))
                r.ctx_len = r.P
            else:
                if r.ctx_len == len(r.blocks) * bs:
                    r.blocks.append(self._pop_block())
                toks = [r.last_token]
                pos = [r.ctx_len]
                r.ctx_len += 1
            plan.batch_slots.append(b)
            plan.tickets.append(r.ticket)
            plan.seq_lens.append(r.ctx_len)
            plan.input_ids += [int(x) for x in toks]
            plan.positions += pos
            plan.slot_mapping += [r.blocks[p // bs] * bs + p % bs for p in pos]
            plan.tok_seq += [si] * len(pos)
            plan.cu_seqlens.append(len(plan.input_ids))
            plan.last_idx.append(len(plan.input_ids) - 1)
            plan.block_tables.append(list(r.blocks))
            plan.gen_index.append(r.gen)
            plan.sample_seq.append(si)
            plan.pos0.append(pos[0])
        # the admitted requests' own full prompt blocks enter the table, batch slot ascending
        if plan.kind == PREFILL:
            for b in slots:
                r = self.running[b]
                prompt = self.requests[r.ticket][0]
                h = r.h_end
                for j in range(r.prefilled_blocks(bs), r.P // bs):
                    h = prefix_chain(h, prompt[j * bs:(j + 1) * bs])
                    if h not in self.table:
                        blk = r.blocks[j]
                        self.table[h] = blk
                        self.bkey[blk] = h
                        self.ref[blk] = 1
                        r.reserved -= 1
                        self.committed -= 1
                        self.pinned += 1
        plan.free_blocks_after = len(self.free)
        return plan

    # ---- one iteration with on-demand KV growth and preemption ------------------------------------------------------
    def _step_preempt(self, tail):
        bs = self.bs
        plan = Plan()
        plan.tail = tail
        # (1) retire
        for b in range(self.max_batch):
            r = self.running[b]
            if r is not None and r.finished:
                self.free.extend(r.blocks)
                self.running[b] = None
        # (2)+(3) resume the preempted (lowest ticket first), then admit new tickets, strictly in that order: the first that
        # does not fit stops everything behind it. A request fits when a batch slot is free and the blocks of the tokens
        # it prefills are free beside those promised earlier in this iteration; the prefill-token budget as in the plain mode
        promised = admitted_tokens = 0
        new_slots = []
        while True:
            cand = min(self.preempted, key=lambda r: r.ticket) if self.preempted else None
            if cand is None:
                if self.next_ticket >= tail:
                    break
                t = self.next_ticket
                prompt, max_new = self.requests[t]
                cand = Running()
                cand.ticket, cand.P, cand.max_new, cand.gen = t, prompt.size, max_new, 0
                cand.finished, cand.last_token = False, -1
            n_tok = cand.P + cand.gen                       # tokens to prefill: the prompt and what was generated so far
            need = -(-n_tok // bs)
            free_slots = [b for b in range(self.max_batch) if self.running[b] is None]
            if not free_slots or promised + need > len(self.free):
                break
            if new_slots and admitted_tokens + n_tok > self.max_prefill_tokens:
                break
            cand.ctx_len, cand.reserved, cand.blocks, cand.prefilled = 0, 0, [], n_tok
            b = free_slots[0]
            self.running[b] = cand
            promised += need
            admitted_tokens += n_tok
            new_slots.append(b)
            if cand in self.preempted:
                self.preempted.remove(cand)
                plan.resumed.append(cand.ticket)            # stays DECODE_PAUSED until its next token is published
            else:
                plan.admitted.append(cand.ticket)
                self._set(cand.ticket, PREFILL_PROCESSING)
                self.next_ticket = cand.ticket + 1
        # (4) kind
        if new_slots:
            plan.kind = PREFILL
            slots = sorted(new_slots)
            for b in range(self.max_batch):   # running decodes are paused for this iteration
                r = self.running[b]
                if r is not None and b not in new_slots and self.state[r.ticket] == DECODE_PROCESSING:
                    self._set(r.ticket, DECODE_PAUSED)
        else:
            if not any(r is not None for r in self.running):
                plan.kind = IDLE
                return plan
            plan.kind = DECODE
            # preempt, highest ticket first, until the blocks this iteration needs are free
            def needed():
                return sum(1 for r in self.running if r is not None and r.ctx_len == len(r.blocks) * bs)
            while needed() > len(self.free):
                b = max((b for b in range(self.max_batch) if self.running[b] is not None), key=lambda b: self.running[b].ticket)
                r = self.running[b]
                self.free.extend(r.blocks)
                r.blocks = []
                self.running[b] = None
                self.preempted.append(r)
                plan.preempted.append(r.ticket)
                if self.state[r.ticket] == DECODE_PROCESSING:
                    self._set(r.ticket, DECODE_PAUSED)
            slots = [b for b in range(self.max_batch) if self.running[b] is not None]
            assert slots, "the oldest request always fits the pool alone"
            for b in slots:
                r = self.running[b]
                if self.state[r.ticket] == DECODE_PAUSED:
                    self._set(r.ticket, DECODE_PROCESSING)
        plan.iteration = self.iteration
        self.iteration += 1
        # (5) allocate, (6) metadata
        for si, b in enumerate(slots):
            r = self.running[b]
            if plan.kind == PREFILL:
                n_tok = r.P + r.gen
                for _ in range(-(-n_tok // bs)):
                    r.blocks.append(self.free.pop())
                toks = list(self.requests[r.ticket][0]) + list(self.outputs[r.ticket][:r.gen])
                pos = list(range(n_tok))
                r.ctx_len = n_tok
            else:
                if r.ctx_len == len(r.blocks) * bs:
                    r.blocks.append(self.free.pop())
                toks = [r.last_token]
                pos = [r.ctx_len]
                r.ctx_len += 1
            plan.batch_slots.append(b)
            plan.tickets.append(r.ticket)
            plan.seq_lens.append(r.ctx_len)
            plan.input_ids += [int(x) for x in toks]
            plan.positions += pos
            plan.slot_mapping += [r.blocks[p // bs] * bs + p % bs for p in pos]
            plan.tok_seq += [si] * len(pos)
            plan.cu_seqlens.append(len(plan.input_ids))
            plan.last_idx.append(len(plan.input_ids) - 1)
            plan.block_tables.append(list(r.blocks))
            plan.gen_index.append(r.gen)
            plan.sample_seq.append(si)
            plan.pos0.append(pos[0])
        plan.free_blocks_after = len(self.free)
        return plan

    # ---- one iteration with chunked prefill: decodes and prompt chunks share a token budget ---------------------
    def _step_chunked(self, tail):
        bs, budget = self.bs, self.max_prefill_tokens
        plan = Plan()
        plan.tail = tail
        # (1) retire
        for b in range(self.max_batch):
            r = self.running[b]
            if r is not None and r.finished:
                self.free.extend(r.blocks)
                self.committed -= r.reserved
                self.running[b] = None
        # tokens of this iteration per batch slot: one per decoding request, then prompt chunks in ticket order
        chunk = {}
        used = 0
        for b in range(self.max_batch):
            r = self.running[b]
            if r is not None and r.prefilled == r.P:
                chunk[b] = 1
                used += 1
        partway = sorted((r.ticket, b) for b, r in enumerate(self.running) if r is not None and r.prefilled < r.P)
        assert len(partway) <= 1, "at most one request is part-way through its prompt"
        for _, b in partway:
            r = self.running[b]
            chunk[b] = min(r.P - r.prefilled, budget - used)
            used += chunk[b]
        # (2)+(3) admit in ticket order while token budget, a batch slot and the block reservation allow
        while self.next_ticket < tail and used < budget:
            t = self.next_ticket
            prompt, max_new = self.requests[t]
            P = prompt.size
            need = blocks_needed(P, max_new, bs)
            free_slots = [b for b in range(self.max_batch) if self.running[b] is None]
            if not free_slots or self.committed + need > self.n_blocks:
                break
            r = Running()
            r.ticket, r.P, r.max_new, r.gen, r.ctx_len = t, P, max_new, 0, 0
            r.reserved, r.blocks, r.finished, r.last_token, r.prefilled = need, [], False, -1, 0
            b = free_slots[0]
            self.running[b] = r
            self.committed += need
            chunk[b] = min(P, budget - used)
            used += chunk[b]
            plan.admitted.append(t)
            self._set(t, PREFILL_PROCESSING)
            self.next_ticket = t + 1
        slots = sorted(chunk)
        if not slots:
            plan.kind = IDLE
            return plan
        # (4) kind: an iteration with prompt tokens in it counts as a prefill iteration
        plan.kind = PREFILL if any(self.running[b].prefilled < self.running[b].P for b in slots) else DECODE
        plan.iteration = self.iteration
        self.iteration += 1
        # (5) allocate, (6) metadata, batch slot ascending
        for si, b in enumerate(slots):
            r = self.running[b]
            if r.prefilled < r.P:
                n = chunk[b]
                pos = list(range(r.prefilled, r.prefilled + n))
                toks = list(self.requests[r.ticket][0][r.prefilled:r.prefilled + n])
                while len(r.blocks) * bs < r.prefilled + n:
                    r.blocks.append(self.free.pop())
                r.prefilled += n
                r.ctx_len = r.prefilled
                samples = r.prefilled == r.P
            else:
                if r.ctx_len == len(r.blocks) * bs:
                    r.blocks.append(self.free.pop())
                toks = [r.last_token]
                pos = [r.ctx_len]
                r.ctx_len += 1
                samples = True
            plan.batch_slots.append(b)
            plan.tickets.append(r.ticket)
            plan.seq_lens.append(r.ctx_len)
            plan.input_ids += [int(x) for x in toks]
            plan.positions += pos
            plan.slot_mapping += [r.blocks[p // bs] * bs + p % bs for p in pos]
            plan.tok_seq += [si] * len(pos)
            plan.cu_seqlens.append(len(plan.input_ids))
            plan.block_tables.append(list(r.blocks))
            plan.pos0.append(pos[0])
            if samples:
                plan.sample_seq.append(si)
                plan.last_idx.append(len(plan.input_ids) - 1)
                plan.gen_index.append(r.gen)
        assert len(plan.input_ids) <= budget
        plan.free_blocks_after = len(self.free)
        return plan

    # ---- steps (7)-(8): tokens of the iteration ----------------------------------------
    def commit(self, plan, tokens):
        """tokens[i]: sampled token of the i-th sampling sequence of the plan. Returns events
        (ticket, index, token, is_first, is_last) in batch-slot order."""
        if self.speculative:
            return self._commit_speculative(plan, tokens)
        events = []
        assert len(tokens) == len(plan.sample_seq)
        for b, tok in zip([plan.batch_slots[i] for i in plan.sample_seq], tokens):
            r = self.running[b]
            tok = int(tok)
            self.outputs[r.ticket].append(tok)
            idx = r.gen
            r.gen += 1
            r.last_token = tok
            done = r.gen == r.max_new or tok == self.eos
            if self.state[r.ticket] in (PREFILL_PROCESSING, DECODE_PAUSED) and not done:
                self._set(r.ticket, DECODE_PROCESSING)     # (DECODE_PAUSED: a preempted request that has just been recomputed)
            if done:
                r.finished = True
                self._set(r.ticket, DECODE_COMPLETED)
            events.append((r.ticket, idx, tok, idx == 0, done))
        return events

    def rows_of(self, plan, i):
        """Speculative mode: the logits rows (indices into last_idx) of the i-th sequence of the plan."""
        end = plan.row0[i + 1] if i + 1 < len(plan.row0) else len(plan.last_idx)
        return list(range(plan.row0[i], end))

    def _commit_speculative(self, plan, row_tokens):
        """row_tokens[j]: the token the sampler gives for logits row j (every row, whether the walk reaches it or not).
        Emits per sequence row by row while the row's token equals the draft that was fed at the next position."""
        events = []
        assert len(row_tokens) == len(plan.last_idx)
        for i, b in enumerate(plan.batch_slots):
            r = self.running[b]
            rows = self.rows_of(plan, i)
            n_fed = len(rows)                                   # 1 + drafts in a decode iteration; 1 in a prefill iteration
            base = plan.cu_seqlens[i + 1] - n_fed               # index of the first token that has a row
            emitted = 0
            done = False
            for j, row in enumerate(rows):
                tok = int(row_tokens[row])
                self.outputs[r.ticket].append(tok)
                idx = r.gen
                r.gen += 1
                r.last_token = tok
                emitted += 1
                done = r.gen == r.max_new or tok == self.eos
                events.append((r.ticket, idx, tok, idx == 0, done))
                if done or j + 1 == n_fed or tok != plan.input_ids[base + j + 1]:
                    break
            if plan.kind == DECODE:
                self.drafted += n_fed - 1
                self.accepted += emitted - 1
                r.ctx_len -= n_fed - emitted                    # the rejected drafts' cache entries are dead
            if self.state[r.ticket] in (PREFILL_PROCESSING, DECODE_PAUSED) and not done:
                self._set(r.ticket, DECODE_PROCESSING)
            if done:
                r.finished = True
                self._set(r.ticket, DECODE_COMPLETED)
        return events

    # ---- invariants ---------------------------------------------------------------------
    def check_invariants(self):
        held = [blk for r in self.running if r is not None for blk in r.blocks]
        if self.prefix_cache:
            # a cached block in use is held by `ref` requests and counts once; an idle one sits in the queue and in the table
            refs = {}
            for blk in held:
                if blk in self.bkey:
                    refs[blk] = refs.get(blk, 0) + 1
            assert all(self.ref[blk] == n for blk, n in refs.items())
            assert all((self.ref[blk] > 0) == (blk in refs) for blk in self.bkey)
            assert self.pinned == len(refs)
            assert all(self.table[k] == blk for blk, k in self.bkey.items()) and len(self.table) == len(self.bkey)
            assert all(blk in self.bkey for blk in range(self.n_blocks) if self.ref[blk] > 0)
            private = [blk for blk in held if blk not in self.bkey]
            allb = private + list(refs) + self.free
            assert len(allb) == self.n_blocks and len(set(allb)) == self.n_blocks, "block leaked or duplicated"
            assert sum(r.reserved for r in self.running if r is not None) == self.committed
            assert len(private) <= self.committed and self.committed + self.pinned <= self.n_blocks
            for r in self.running:
                if r is not None:
                    assert len([blk for blk in r.blocks if blk not in self.bkey]) <= r.reserved
                    assert len(r.blocks) * self.bs >= r.ctx_len
            for (_, a, b) in self.transitions:
                assert (a, b) in LEGAL_EDGES, (a, b)
            return
        allb = held + self.free
        assert len(allb) == self.n_blocks, "block leaked or duplicated"
        assert len(set(allb)) == self.n_blocks, "block id appears twice"
        if not self.preempt:
            assert sum(r.reserved for r in self.running if r is not None) == self.committed
            assert len(held) <= self.committed <= self.n_blocks
        for r in self.preempted:
            assert not r.blocks and self.state[r.ticket] == DECODE_PAUSED
        for r in self.running:
            if r is not None:
                assert self.preempt or len(r.blocks) <= r.reserved
                assert len(r.blocks) * self.bs >= r.ctx_len
        for (_, a, b) in self.transitions:
            assert (a, b) in LEGAL_EDGES, (a, b)

    def n_running(self):
        return sum(r is not None for r in self.running)
