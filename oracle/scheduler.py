"""Integer model of the fused stage's bookkeeping.  TEST INFRASTRUCTURE ONLY.

The paper fixes the events (Section 4): samples leave the generation stage one by one as
they reach their termination point; once the number of samples still in generation falls
below the trigger R_t (Section 4.2, "Migration triggering"), finished samples flow to the
inference stage as they complete (Section 4.2, end), and the KV-cache budget C bounds how
many long samples an instance may hold (Section 4.2, "Migration destination", second
constraint).  It does not fix an engine's slot order, page order or batch boundaries; the
rules below are this build's reading, stated so that every integer is determined:

* Samples are ids 0..N-1; the waiting queue is FIFO.  Sample i reserves
  ceil((P_i + max_new_i) / page) pages.  At the top of a step the head of the queue is
  admitted while the reservation fits the pool and the active array has room; the first
  sample that does not fit blocks those behind it.
* The free list is a stack that first issues pages 0, 1, 2, ...  A sample takes a page
  exactly when it is about to write a position that is a multiple of the page size.
  Newcomers take their prompt pages in position order, newcomers in id order, before the
  step's decode growth, which goes in slot order.
* A newcomer is prefilled (its first output token), joins the END of the active array,
  and takes part in the same step's decode unless already at its target length.  A sample
  of length L costs one prefill and L-1 decode inputs; its last token is never fed back.
* retire(): scan slots in order; a sample whose generated length equals its target
  leaves; its pages go back in reverse page-table order; survivors keep their order.
* migrate(ids): the second migration mechanism of Section 4.2 ("Migration mechanism"): an
  unfinished sample's KV cache is discarded and only its tokens travel; the receiver reruns
  the prefill phase over prompt + tokens generated so far and goes on decoding.  On one
  instance sender and receiver coincide: the listed active samples give their pages back
  (each in reverse page-table order, samples in the order listed), release their
  reservation, leave the active array (survivors keep their order) and re-enter the waiting
  queue, at its head in the order listed (or at its tail).  When re-admitted, a sample with
  g tokens generated rebuilds positions 0 .. P+g-2 (everything but its newest token, which
  was never fed), emits nothing, and feeds that newest token in the same step's decode.
* optimistic = True replaces the reservation rule (the paper only asks that an instance have
  "sufficient memory", Section 4.2) by admission on present need plus preemption, with
  migrate() as the preemption: the head of the queue is admitted while the pages for the rows
  it rebuilds plus one more token fit in what is free after the newcomers before it, and,
  unless nothing is running, one further free page is left per running sample.  Before the
  step's decode, if the pages the decode is about to take exceed the free ones, the most
  recently admitted unfinished samples are preempted one by one until they fit; the victims
  return to the head of the queue in their admission order.  A single sample always fits
  (the pool holds any one sample at its cap), so every step decodes at least one token.
* Scoring batches: after each step's retire, if scoring is enabled (fused mode and
  remaining = waiting + active < R_t, or generation is over) the un-scored part of the
  retired FIFO is cut, from its head, into consecutive batches of at most
  `score_chunk_tokens` prompt+response tokens: a batch closes when the next retired sample
  would take it past that bound (a single longer sample is a batch of its own); when
  generation is over the remainder is flushed as a last batch.  (The paper's Section 4.2
  leaves the size of the scoring batches to the implementation; a bound from above lets a
  caller pick the pass size that fills its compute tiles.)  Sequential mode (fused = 0) applies the same cut only
  after the last step.
"""
from dataclasses import dataclass, field
from typing import List, Optional, Sequence


@dataclass
class StepInfo:
    step: int
    n_admitted: int
    n_prefill_tokens: int
    n_decoded: int
    n_active: int


class SchedulerModel:
    def __init__(self, prompt_lens: Sequence[int], max_new: Sequence[int],
                 target_len: Sequence[int], pool_pages: int, page_tokens: int = 16,
                 max_active: Optional[int] = None, optimistic: bool = False):
        self.N = len(prompt_lens)
        self.P = [int(p) for p in prompt_lens]
        self.max_new = [int(m) for m in max_new]
        self.target = [int(t) for t in target_len]
        assert all(1 <= t <= m for t, m in zip(self.target, self.max_new))
        self.page = int(page_tokens)
        self.pool_pages = int(pool_pages)
        self.max_active = self.N if max_active is None else int(max_active)
        self.optimistic = bool(optimistic)
        self.n_preempted = 0
        self.reserve = [-(-(p + m) // self.page) for p, m in zip(self.P, self.max_new)]
        if any(r > self.pool_pages for r in self.reserve):
            raise MemoryError("a sample's reservation exceeds the pool")
        self.waiting = list(range(self.N))           # head at index 0
        self.active: List[int] = []                  # slot order
        self.ctx = [0] * self.N                      # tokens whose K/V are cached
        self.gen_len = [0] * self.N
        self.pages: List[List[int]] = [[] for _ in range(self.N)]
        self.free = list(range(self.pool_pages - 1, -1, -1))   # pop() issues 0, 1, 2, ...
        self.reserved = 0
        self.retired: List[int] = []
        self.n_scored = 0                            # retired[:n_scored] are in some batch
        self.batches: List[List[int]] = []
        self.batch_step: List[int] = []              # step after which each batch closed
        self.step = 0
        self.admit_step = [-1] * self.N

    # ----------------------------------------------------------------- generation
    def _write_position(self, i: int):
        """Sample i is about to write K/V at position ctx[i]."""
        if self.ctx[i] % self.page == 0:
            self.pages[i].append(self.free.pop())
        self.ctx[i] += 1

    def _rebuilt_rows(self, i: int) -> int:
        return self.P[i] + max(self.gen_len[i] - 1, 0)

    def _admit(self) -> List[int]:
        newcomers = []
        if not self.optimistic:
            while (self.waiting and len(self.active) + len(newcomers) < self.max_active
                   and self.reserved + self.reserve[self.waiting[0]] <= self.pool_pages):
                i = self.waiting.pop(0)
                self.reserved += self.reserve[i]
                newcomers.append(i)
            return newcomers
        free = len(self.free)
        while self.waiting and len(self.active) + len(newcomers) < self.max_active:
            i = self.waiting[0]
            need = -(-(self._rebuilt_rows(i) + 1) // self.page)
            running = len(self.active) + len(newcomers)
            if need > free or (running > 0 and free - need < running):
                break
            free -= need
            self.waiting.pop(0)
            self.reserved += self.reserve[i]
            newcomers.append(i)
        return newcomers

    def _preempt_for_decode(self) -> None:
        victims = []
        while True:
            dec = [i for i in self.active if self.gen_len[i] < self.target[i]]
            need = sum(1 for i in dec if self.ctx[i] % self.page == 0)
            if need <= len(self.free):
                break
            v = dec[-1]                               # most recently admitted unfinished sample
            for pg in reversed(self.pages[v]):
                self.free.append(pg)
            self.pages[v] = []
            self.ctx[v] = 0
            self.reserved -= self.reserve[v]
            self.active.remove(v)
            victims.append(v)
        self.waiting = victims[::-1] + self.waiting
        self.n_preempted += len(victims)

    def generate_step(self) -> StepInfo:
        newcomers = self._admit()
        n_pre = 0
        for i in newcomers:
            # first admission: prompt positions, then y_1.  After a migration: prompt and all
            # generated tokens but the newest are rebuilt, nothing is emitted.
            rebuilt = self.P[i] + max(self.gen_len[i] - 1, 0)
            for _ in range(rebuilt):
                self._write_position(i)
            n_pre += rebuilt
            self.gen_len[i] = max(self.gen_len[i], 1)
            self.admit_step[i] = self.step
            self.active.append(i)
        if self.optimistic:
            self._preempt_for_decode()
        n_dec = 0
        for i in self.active:                        # decode: feed the last token
            if self.gen_len[i] < self.target[i]:
                self._write_position(i)
                self.gen_len[i] += 1
                n_dec += 1
        info = StepInfo(self.step, len(newcomers), n_pre, n_dec, len(self.active))
        self.step += 1
        return info

    def retire(self) -> List[int]:
        out, keep = [], []
        for i in self.active:
            if self.gen_len[i] == self.target[i]:
                for pg in reversed(self.pages[i]):
                    self.free.append(pg)
                self.pages[i] = []
                self.reserved -= self.reserve[i]
                self.retired.append(i)
                out.append(i)
            else:
                keep.append(i)
        self.active = keep
        return out

    def migrate(self, ids: Sequence[int], to_back: bool = False) -> None:
        ids = [int(i) for i in ids]
        if len(set(ids)) != len(ids):
            raise ValueError("duplicate id")
        for i in ids:
            if i not in self.active or self.gen_len[i] >= self.target[i]:
                raise ValueError(f"sample {i} is not an unfinished active sample")
        for i in ids:
            for pg in reversed(self.pages[i]):
                self.free.append(pg)
            self.pages[i] = []
            self.ctx[i] = 0
            self.reserved -= self.reserve[i]
        self.active = [i for i in self.active if i not in ids]
        self.waiting = self.waiting + ids if to_back else ids + self.waiting

    def generation_done(self) -> bool:
        return not self.waiting and not self.active

    # -------------------------------------------------------------------- scoring
    def seq_tokens(self, i: int) -> int:
        return self.P[i] + self.target[i]

    def form_batches(self, chunk_tokens: int) -> List[List[int]]:
        """Cut the un-scored FIFO into batches of <= chunk_tokens (at least one sample each): a
        batch closes once the next retired sample would not fit; flush when generation is over.
        Returns the batches closed by this call."""
        chunk = max(1, int(chunk_tokens))
        new = []
        while True:
            k, tok = self.n_scored, 0
            while k < len(self.retired):
                t = self.seq_tokens(self.retired[k])
                if k > self.n_scored and tok + t > chunk:
                    break
                tok += t
                k += 1
            full = k < len(self.retired)          # the next sample is there and does not fit
            if k > self.n_scored and (full or self.generation_done()):
                new.append(self.retired[self.n_scored:k])
                self.n_scored = k
            else:
                break
        for b in new:
            self.batches.append(b)
            self.batch_step.append(self.step - 1)
        return new

    def run_stage(self, fused: bool, R_t: int, chunk_tokens: int):
        """Whole stage.  Returns the per-step trace [(StepInfo, retired ids, new batches)]."""
        trace = []
        while not self.generation_done():
            info = self.generate_step()
            gone = self.retire()
            new = []
            remaining = len(self.waiting) + len(self.active)
            if (fused and remaining < R_t) or self.generation_done():
                new = self.form_batches(chunk_tokens)
            trace.append((info, gone, new))
        return trace

    # ------------------------------------------------------------------- snapshot
    def snapshot(self) -> dict:
        return {
            "step": self.step,
            "n_waiting": len(self.waiting),
            "active": list(self.active),
            "ctx": list(self.ctx),
            "gen_len": list(self.gen_len),
            "pages": [list(p) for p in self.pages],
            "free": list(self.free),
            "reserved": self.reserved,
            "retired": list(self.retired),
            "batches": [list(b) for b in self.batches],
            "n_preempted": self.n_preempted,
        }
