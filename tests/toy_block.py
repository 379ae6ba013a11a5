"""A tiny packed-sequence transformer block for the hook-harness tests: token
embedding, causal self-attention confined to each sequence, a gated MLP and a
vocabulary head, returning the log-probability of each sequence's tokens."""
import numpy as np
import torch
from torch import nn


class ToyBlock(nn.Module):
    def __init__(self, vocab=48, hidden=32, heads=2, ffn=64, dtype=torch.float32):
        super().__init__()
        self.heads = heads
        self.emb = nn.Embedding(vocab, hidden, dtype=dtype)
        self.q = nn.Linear(hidden, hidden, bias=False, dtype=dtype)
        self.k = nn.Linear(hidden, hidden, bias=False, dtype=dtype)
        self.v = nn.Linear(hidden, hidden, bias=False, dtype=dtype)
        self.o = nn.Linear(hidden, hidden, bias=False, dtype=dtype)
        self.gate = nn.Linear(hidden, ffn, bias=False, dtype=dtype)
        self.up = nn.Linear(hidden, ffn, bias=False, dtype=dtype)
        self.down = nn.Linear(ffn, hidden, bias=False, dtype=dtype)
        self.head = nn.Linear(hidden, vocab, bias=False, dtype=dtype)

    def forward(self, tokens, targets, seq_offsets):
        """tokens, targets: [N] packed; returns per-token log-probabilities [N]."""
        n = tokens.shape[0]
        off = np.asarray(seq_offsets)
        seq_id = torch.from_numpy(np.repeat(np.arange(off.size - 1), np.diff(off))).to(tokens.device)
        pos = torch.arange(n, device=tokens.device)
        allowed = (seq_id[:, None] == seq_id[None, :]) & (pos[None, :] <= pos[:, None])
        x = self.emb(tokens)
        h = self.heads
        q = self.q(x).view(n, h, -1).transpose(0, 1)
        k = self.k(x).view(n, h, -1).transpose(0, 1)
        v = self.v(x).view(n, h, -1).transpose(0, 1)
        att = (q @ k.transpose(1, 2)) / q.shape[-1] ** 0.5
        att = att.masked_fill(~allowed[None], float("-inf")).softmax(-1)
        x = x + self.o((att @ v).transpose(0, 1).reshape(n, -1))
        x = x + self.down(torch.nn.functional.silu(self.gate(x)) * self.up(x))
        logp = torch.log_softmax(self.head(x), dim=-1)
        return logp.gather(1, targets[:, None])[:, 0]


def make_batch(lengths, vocab=48, seed=0, device="cpu"):
    rng = np.random.default_rng(seed)
    n = int(np.sum(lengths))
    off = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)
    tokens = torch.from_numpy(rng.integers(0, vocab, n)).to(device)
    targets = torch.from_numpy(rng.integers(0, vocab, n)).to(device)
    A = rng.standard_normal(len(lengths))
    A = (A - A.mean()) / A.std()
    return tokens, targets, off, A
