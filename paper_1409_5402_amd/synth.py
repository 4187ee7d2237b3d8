"""Seeded synthetic LDA corpora shaped like the paper's workloads.

This module only *generates inputs* (it contains none of the sampler's
arithmetic) and serves both the GPU path and the CPU oracle.  A corpus is drawn
from the LDA generative process: topic-word distributions from a symmetric
Dirichlet (optionally skewed by a Zipf law over word ids), document-topic
distributions from a symmetric Dirichlet, document lengths from a Poisson or a
log-normal law, tokens by ancestral sampling.  The result is a CSC matrix whose
columns are documents: ``colptr`` int32 [D+1], ``rowidx`` int32 [nnz] (word ids,
ascending inside a document), ``val`` float32 [nnz] (integer-valued counts).

The real corpora the paper measures on (a news collection of ~300k documents /
~100k words / ~100M tokens and an abstract collection of ~8M documents / ~140k
words / ~730M tokens, Section 6.1) are not available; the presets below only
take their shapes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch


@dataclass
class Corpus:
    D: int
    V: int
    colptr: torch.Tensor      # int32 [D+1]
    rowidx: torch.Tensor      # int32 [nnz]
    val: torch.Tensor         # float32 [nnz]
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowidx.shape[0])

    @property
    def tokens(self) -> int:
        return int(self.val.sum(dtype=torch.float64).item())

    def to(self, device) -> "Corpus":
        return Corpus(self.D, self.V, self.colptr.to(device), self.rowidx.to(device),
                      self.val.to(device), dict(self.meta))

    def slice_docs(self, lo: int, hi: int) -> "Corpus":
        a, b = int(self.colptr[lo]), int(self.colptr[hi])
        return Corpus(hi - lo, self.V, (self.colptr[lo:hi + 1] - a).contiguous(),
                      self.rowidx[a:b].contiguous(), self.val[a:b].contiguous(), dict(self.meta))

    def stats(self) -> dict:
        word_tokens = torch.zeros(self.V, dtype=torch.float32, device=self.val.device)
        word_tokens.index_add_(0, self.rowidx.long(), self.val)      # informational (float32 sums)
        return {"D": self.D, "V": self.V, "nnz": self.nnz, "tokens": self.tokens,
                "max_count": int(self.val.max().item()) if self.nnz else 0,
                "max_word_tokens": int(word_tokens.max().item()) if self.nnz else 0}


def _dirichlet_rows(rows: int, cols: int, conc: float, gen: torch.Generator, device) -> torch.Tensor:
    """rows x cols matrix of symmetric-Dirichlet(conc) rows (float64) via normalised Gamma draws."""
    shape = torch.full((rows, cols), conc, dtype=torch.float64, device=device)
    g = torch._standard_gamma(shape, generator=gen)
    g = g.clamp_min_(1e-300)
    return g / g.sum(dim=1, keepdim=True)


def generate(D: int, V: int, K: int, alpha: float, beta: float, seed: int,
             length: str = "poisson", mean_len: float = 100.0, sigma: float = 0.6,
             zipf_s: float = 0.0, device="cpu", doc_chunk: int = 50_000) -> Corpus:
    """Draw a corpus from the LDA generative process (see module docstring)."""
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))

    phi = _dirichlet_rows(K, V, beta, gen, device)                      # [K][V]
    if zipf_s > 0.0:
        rank = torch.arange(1, V + 1, dtype=torch.float64, device=device)
        phi = phi * rank.pow(-zipf_s)
        phi = phi / phi.sum(dim=1, keepdim=True)
    # one ascending sequence holding every topic's word cdf: entry k*V+w = k + cdf_k(w)
    word_cdf = phi.cumsum(dim=1)
    word_cdf = word_cdf / word_cdf[:, -1:].clone()
    word_cdf[:, -1] = 1.0
    word_cdf = (word_cdf + torch.arange(K, dtype=torch.float64, device=device)[:, None]).reshape(-1)
    del phi

    if length == "poisson":
        lens = torch.poisson(torch.full((D,), float(mean_len), dtype=torch.float64, device=device), generator=gen)
    elif length == "lognormal":
        mu = math.log(mean_len) - 0.5 * sigma * sigma
        z = torch.randn(D, dtype=torch.float64, device=device, generator=gen)
        lens = torch.exp(mu + sigma * z).round()
    else:
        raise ValueError(length)
    lens = lens.clamp_min(1.0).long()

    keys_parts, counts_parts = [], []
    for lo in range(0, D, doc_chunk):
        hi = min(D, lo + doc_chunk)
        n_docs = hi - lo
        theta = _dirichlet_rows(n_docs, K, alpha, gen, device)
        topic_cdf = theta.cumsum(dim=1)
        topic_cdf = topic_cdf / topic_cdf[:, -1:].clone()
        topic_cdf[:, -1] = 1.0
        topic_cdf = (topic_cdf + torch.arange(n_docs, dtype=torch.float64, device=device)[:, None]).reshape(-1)
        doc_local = torch.repeat_interleave(torch.arange(n_docs, device=device), lens[lo:hi])
        n_tok = doc_local.shape[0]
        u = torch.rand(n_tok, dtype=torch.float64, device=device, generator=gen)
        z = torch.searchsorted(topic_cdf, doc_local.double() + u, right=True) - doc_local * K
        z = z.clamp_(0, K - 1)
        u = torch.rand(n_tok, dtype=torch.float64, device=device, generator=gen)
        w = torch.searchsorted(word_cdf, z.double() + u, right=True) - z * V
        w = w.clamp_(0, V - 1)
        key = (doc_local + lo) * V + w
        uk, cnt = torch.unique(key, sorted=True, return_counts=True)
        keys_parts.append(uk)
        counts_parts.append(cnt)
        del theta, topic_cdf, doc_local, u, z, w, key

    keys = torch.cat(keys_parts)
    counts = torch.cat(counts_parts)
    doc_of = torch.div(keys, V, rounding_mode="floor")
    rowidx = (keys - doc_of * V).to(torch.int32)
    per_doc = torch.bincount(doc_of, minlength=D)
    colptr = torch.zeros(D + 1, dtype=torch.int64, device=device)
    colptr[1:] = per_doc.cumsum(0)
    assert int(colptr[-1]) < 2 ** 31, "nnz must fit int32 column pointers"
    meta = {"K_true": K, "alpha_true": alpha, "beta_true": beta, "seed": seed, "length": length,
            "mean_len": mean_len, "sigma": sigma, "zipf_s": zipf_s}
    return Corpus(D, V, colptr.to(torch.int32), rowidx.contiguous(), counts.to(torch.float32), meta)


def state(corpus: Corpus, K: int, alpha: float, beta: float, seed: int, zipf_s: float = 0.0):
    """A seeded, concentrated parameter state shaped like a trained sampler's: theta [D][K] =
    alpha + document length * Dirichlet(alpha) row, phi [V][K] with every topic a Dirichlet(beta)
    distribution over words (optionally Zipf-skewed).  Returned as float32 tensors on the corpus' device."""
    device = corpus.val.device
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    lens = torch.zeros(corpus.D, dtype=torch.float64, device=device)
    doc_of = torch.repeat_interleave(torch.arange(corpus.D, device=device), (corpus.colptr[1:] - corpus.colptr[:-1]).long())
    lens.index_add_(0, doc_of, corpus.val.double())
    theta = torch.empty(corpus.D, K, dtype=torch.float32, device=device)
    for lo in range(0, corpus.D, 50_000):
        hi = min(corpus.D, lo + 50_000)
        theta[lo:hi] = (alpha + lens[lo:hi, None] * _dirichlet_rows(hi - lo, K, alpha, gen, device)).float()
    phi_kv = _dirichlet_rows(K, corpus.V, beta, gen, device)
    if zipf_s > 0.0:
        rank = torch.arange(1, corpus.V + 1, dtype=torch.float64, device=device)
        phi_kv = phi_kv * rank.pow(-zipf_s)
        phi_kv = phi_kv / phi_kv.sum(dim=1, keepdim=True)
    phi = phi_kv.t().contiguous().float().clamp_min_(1e-30)
    return theta, phi


# Workload presets (shapes of the paper's experiments; K and m are the sampler's settings).
PRESETS = {
    # tiny: the oracle finishes in seconds
    "tiny": dict(gen=dict(D=1_000, V=2_000, K=16, alpha=0.1, beta=0.01, seed=0,
                          length="poisson", mean_len=100.0, zipf_s=0.0),
                 K=16, m=10, sweeps=10, alpha=0.1, beta=0.01),
    "medium": dict(gen=dict(D=50_000, V=20_000, K=64, alpha=0.1, beta=0.01, seed=1,
                            length="poisson", mean_len=200.0, zipf_s=1.1),
                   K=64, m=20, sweeps=20, alpha=0.1, beta=0.01),
    # news-collection shape: ~300k documents, ~100k words, ~100M tokens, K=256, m=100
    "news": dict(gen=dict(D=300_000, V=100_000, K=256, alpha=50.0 / 256, beta=0.01, seed=2,
                          length="lognormal", mean_len=330.0, sigma=0.6, zipf_s=1.1),
                 K=256, m=100, sweeps=50, alpha=50.0 / 256, beta=0.01),
    "news_k1024": dict(gen=dict(D=300_000, V=100_000, K=256, alpha=50.0 / 256, beta=0.01, seed=2,
                                length="lognormal", mean_len=330.0, sigma=0.6, zipf_s=1.1),
                       K=1024, m=100, sweeps=50, alpha=50.0 / 1024, beta=0.01),
    "news_k512": dict(gen=dict(D=300_000, V=100_000, K=256, alpha=50.0 / 256, beta=0.01, seed=2,
                               length="lognormal", mean_len=330.0, sigma=0.6, zipf_s=1.1),
                      K=512, m=100, sweeps=50, alpha=50.0 / 512, beta=0.01),
    # abstract-collection shape, one resident minibatch of 100k documents
    "abstracts_batch": dict(gen=dict(D=100_000, V=140_000, K=256, alpha=0.1, beta=0.01, seed=4,
                                     length="poisson", mean_len=90.0, zipf_s=1.05),
                            K=256, m=100, sweeps=1, alpha=0.1, beta=0.01),
}


def preset(name: str, device="cpu", scale: float = 1.0) -> Corpus:
    """Generate a preset corpus; ``scale`` < 1 shrinks the number of documents only."""
    g = dict(PRESETS[name]["gen"])
    g["D"] = max(1, int(round(g["D"] * scale)))
    return generate(device=device, **g)
