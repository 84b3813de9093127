"""Host loop of Alg. 1 over the C ABI: K draft steps, one verification, and the draft cache following the
target's decision - all enqueued on the current stream without reading anything back."""
import torch

from . import binding as B


class SSDSession:
    def __init__(self, target_shape, target_w, draft_shape, draft_w, n_seqs, K, max_positions, cfg, dcfg,
                 block_tokens=16, n_blocks=None, max_rows=None, device="cuda"):
        if max_rows is None:                     # rows per sequence and launch: prefill chunks (the library takes 1024 rows in all)
            max_rows = max(K + 1, 1024 // n_seqs)
        self.K, self.n_seqs = K, n_seqs
        self.cfg, self.dcfg = cfg, dcfg
        self.target = B.Model(target_shape, B.upload_weights(target_shape, target_w, device), max_positions, device)
        mbps = -(-max_positions // block_tokens)
        nb = n_blocks if n_blocks is not None else n_seqs * mbps
        self.kv = B.KVCache(self.target, n_seqs, max(max_rows, K + 1), nb, block_tokens, mbps, 1)
        self.draft = self.kv_d = None
        if draft_shape is not None:
            self.draft = B.Model(draft_shape, B.upload_weights(draft_shape, draft_w, device), max_positions, device)
            self.kv_d = B.KVCache(self.draft, n_seqs, max(max_rows, 2), nb, block_tokens, mbps, 2)
        V = target_shape["vocab"]
        self.V = V
        self.x = torch.zeros((n_seqs, max(K, 1)), dtype=torch.int32, device=device)
        self.pd = torch.zeros((n_seqs, max(K, 1), V), dtype=torch.float32, device=device)
        self.n_acc = torch.zeros(n_seqs, dtype=torch.int32, device=device)
        self.next = torch.zeros(n_seqs, dtype=torch.int32, device=device)

    def prefill(self, seq, tokens):
        B.ssd_prefill(self.target, self.kv, seq, tokens)
        if self.draft is not None:
            B.ssd_prefill(self.draft, self.kv_d, seq, tokens)

    def cycle(self, step, out=None):
        """One SSD cycle.  `out` (optional) = dict(n_accepted, next_token[, probs, logits]) of device tensors."""
        K, n = self.K, self.n_seqs
        for i in range(K):
            B.ssd_draft_step(self.draft, self.kv_d, n, self.dcfg, step, i, self.x[:, i], K, self.pd[:, i], K * self.V)
        if out is None:
            out = dict(n_accepted=self.n_acc, next_token=self.next, probs=None, logits=None)
        B.ssd_verify(self.target, self.kv, n, self.x if K else None, self.pd if K else None, K, self.cfg, step, out=out)
        if K:
            B.ssd_kv_follow(self.kv_d, n, K, out["n_accepted"], out["next_token"], self.x)
        return out

    def graph_cycle(self, first_step=0):
        """The same cycle captured once as a graph (ssd_cycle_create); each launch() of the result replays it with the
        next cycle index.  Results land in self.x, self.pd, self.n_acc, self.next."""
        return B.Cycle(self.target, self.kv, self.draft, self.kv_d, self.n_seqs, self.K, self.cfg, self.dcfg, self.x, self.pd,
                       self.n_acc, self.next, first_step)

    def ar_step(self, step, out=None):
        """Plain autoregressive decoding of the target: a verification with no draft tokens."""
        if out is None:
            out = dict(n_accepted=self.n_acc, next_token=self.next, probs=None, logits=None)
        B.ssd_verify(self.target, self.kv, self.n_seqs, None, None, 0, self.cfg, step, out=out)
        return out
