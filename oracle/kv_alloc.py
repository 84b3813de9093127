"""Model of the paged KV allocator (test oracle).  The paper has no KV cache; this states the
bookkeeping the library is required to reproduce index-for-index:
 - blocks of `block_tokens` positions; a free stack from which the lowest id is taken first at start;
 - before a forward that writes R rows, sequences in ascending order take blocks until they own
   ceil((len + R) / block_tokens);
 - a commit / rollback to `new_len` returns the blocks with table index >= ceil(new_len / block_tokens)
   to the stack, highest table index first, sequences in ascending order."""


class PagedAllocator:
    def __init__(self, n_blocks, block_tokens, max_seqs, max_blocks_per_seq):
        self.bt = block_tokens
        self.free = list(range(n_blocks - 1, -1, -1))      # pop() yields 0 first
        self.table = [[-1] * max_blocks_per_seq for _ in range(max_seqs)]
        self.owned = [0] * max_seqs
        self.length = [0] * max_seqs

    def _need(self, tokens):
        return -(-tokens // self.bt)

    def reserve(self, seq, rows):
        need = self._need(self.length[seq] + rows)
        while self.owned[seq] < need:
            if not self.free:
                raise MemoryError("pool exhausted")
            self.table[seq][self.owned[seq]] = self.free.pop()
            self.owned[seq] += 1

    def set_length(self, seq, new_len):
        keep = self._need(new_len)
        while self.owned[seq] > keep:
            self.owned[seq] -= 1
            self.free.append(self.table[seq][self.owned[seq]])
            self.table[seq][self.owned[seq]] = -1
        self.length[seq] = new_len

    def slot(self, seq, pos):
        """(block id, offset in block) of a position."""
        return self.table[seq][pos // self.bt], pos % self.bt
