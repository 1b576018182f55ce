"""Proof building inside a serving loop with continuous batching: every decode step hands over
the last-layer hidden state of one new token for whichever sequences are running, each at its
own position; a sequence's proof is cut every `chunk_tokens` tokens (Section 5.6 and 5.8 of the
paper: one proof per 32 new tokens, plus one over the prompt) and when it ends.

Bookkeeping only: the positions live in a host array, every step of the method runs in the
library's kernels (toploc_stream_append_rows / toploc_stream_emit_rows keep the running top-k
per sequence on the GPU, so no ring of hidden states is stored or re-read)."""
import numpy as np
import torch

from . import binding


class OnlineProver:
    def __init__(self, n_slots, hidden, k=128, chunk_tokens=32, device="cuda:0"):
        if hidden % 8 or k > chunk_tokens * hidden:
            raise ValueError("hidden must be a multiple of 8 and a full chunk must hold k values")
        self.n_slots, self.hidden, self.k, self.chunk_tokens = n_slots, hidden, k, chunk_tokens
        self.device = torch.device(device)
        self.state = binding.toploc_stream_new_state(n_slots, k, self.device)
        self.rows = np.zeros(n_slots, dtype=np.int64)      # rows in each sequence's open chunk

    def prefill(self, prompt_hidden):
        """The proof over a whole prompt: prompt_hidden [n_tokens, H] bf16 -> (proof uint8 [2+2k], status)."""
        off = np.array([0, prompt_hidden.shape[0]], dtype=np.uint64)
        proofs, status = binding.toploc_build_proofs_segments(prompt_hidden, off, k=self.k)
        return proofs[0], status[0]

    def append(self, step_hidden, slots):
        """One new token for each sequence in `slots` (distinct): step_hidden [len(slots), H] bf16.
        Returns (slots, proofs, status) for the sequences whose chunk this token completed, else None."""
        slots = np.asarray(slots, dtype=np.int64)
        if slots.size != np.unique(slots).size or (slots.size and (slots.min() < 0 or slots.max() >= self.n_slots)):
            raise ValueError("slots must be distinct and inside [0, n_slots)")
        if step_hidden.shape != (slots.size, self.hidden):
            raise ValueError("step_hidden must be [len(slots), hidden]")
        if slots.size == 0:
            return None
        binding.toploc_stream_append_rows(self.state, self.n_slots, step_hidden, slots, self.rows[slots],
                                          k=self.k, chunk_tokens=self.chunk_tokens)
        self.rows[slots] += 1
        full = slots[self.rows[slots] == self.chunk_tokens]
        return self._emit(full) if full.size else None

    def finish(self, slots):
        """The ragged last chunk of sequences that ended: (slots, proofs, status) for those holding rows
        (status CHUNK_SHORT where the rows hold fewer than k values), else None."""
        slots = np.unique(np.asarray(slots, dtype=np.int64))
        open_ = slots[self.rows[slots] > 0]
        return self._emit(open_) if open_.size else None

    def _emit(self, slots):
        proofs, status = binding.toploc_stream_emit_rows(self.state, self.n_slots, slots, k=self.k)
        self.rows[slots] = 0
        return slots, proofs, status
