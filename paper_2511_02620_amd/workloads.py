"""Seeded synthetic workloads: logits, per-sequence seeds, positions and claim mutations.

These generators serve the tests, the smoke check and the benchmark.  They hold none of
the scoring method's arithmetic (no Philox noise, no softmax, no sampler): honest claims
are produced by whoever calls them, by running a sampler on the *prover* logits this
module returns, and are then passed back through :meth:`Workload.mutate_claims`.

The paper measured on chat prompts with Llama-3 / Qwen models.  None of that data is
available, so the logits here only take those models' shapes (vocabulary 128,256 and
151,936, up to 1,024 generated tokens per sequence) and a Zipf-like value profile:
each row is a random permutation of -1.1 ln(rank), rank = 1..V, plus N(0,1) noise.
The verifier sees the logits rounded to the storage dtype; the prover sees them with a
small extra drift, which models the benign numerical non-determinism the paper's
scores are meant to tolerate.
"""
from __future__ import annotations

import dataclasses
import math

import torch

MASTER_SEED = 0x251102620
_MASK64 = (1 << 64) - 1


def splitmix64(x: int) -> int:
    """One step of the SplitMix64 mixer (used only to derive distinct per-sequence seeds)."""
    x = (x + 0x9E3779B97F4A7C15) & _MASK64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _as_i64(x: int) -> int:
    return x - (1 << 64) if x >= (1 << 63) else x


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    index: int               # config number c: every RNG stream is derived from MASTER_SEED + c
    S: int                   # sequences
    L: int                   # tokens per sequence (rows of a sequence are contiguous)
    V: int                   # vocabulary
    dtype: torch.dtype       # storage dtype of the verifier logits
    temperature: float
    profile: str             # "gauss" (iid N(0, 2^2)) or "zipf"
    drift_sigma: float       # std of the prover's extra logit noise
    prover_bf16: bool        # prover logits re-rounded to bf16 (else kept fp32)
    chunk_rows: int          # rows generated per call of logits_chunk
    mutation: str            # "uniform" | "topk" | "stego" | "none"
    mutation_frac: float = 0.0
    mutation_k: int = 0

    @property
    def N(self) -> int:
        return self.S * self.L

    @property
    def n_chunks(self) -> int:
        assert self.N % self.chunk_rows == 0
        return self.N // self.chunk_rows

    def with_temperature(self, T: float) -> "Workload":
        return dataclasses.replace(self, temperature=float(T))

    # ---- per-row bookkeeping -------------------------------------------------------
    def seeds(self):
        """[S] int64 tensor holding the uint64 sampling seed of each sequence (CPU)."""
        vals = [_as_i64(splitmix64(MASTER_SEED + 1000 * self.index + s)) for s in range(self.S)]
        return torch.tensor(vals, dtype=torch.int64)

    def seq_ids(self):
        return torch.arange(self.S, dtype=torch.int32).repeat_interleave(self.L)

    def positions(self):
        return torch.arange(self.L, dtype=torch.int32).repeat(self.S)

    def seq_offsets(self):
        return torch.arange(self.S + 1, dtype=torch.int64) * self.L

    def stego_sequences(self):
        """Sequences whose claims carry hidden message bits (mutation == "stego")."""
        if self.mutation != "stego":
            return []
        g = torch.Generator().manual_seed(MASTER_SEED + self.index + 7_000_000)
        n = max(1, int(round(self.mutation_frac * self.S)))
        return sorted(torch.randperm(self.S, generator=g)[:n].tolist())

    # ---- logits --------------------------------------------------------------------
    def _gen(self, device, chunk: int, salt: int):
        g = torch.Generator(device=device)
        g.manual_seed(MASTER_SEED + self.index + 10_000 * (chunk + 1) + salt)
        return g

    def logits_chunk(self, chunk: int, device):
        """Rows [chunk*chunk_rows, (chunk+1)*chunk_rows): (verifier, prover) logits on `device`.

        verifier: [rows, V] in the storage dtype.  prover: the verifier's exact values plus
        N(0, drift_sigma^2), fp32 or re-rounded to bf16."""
        device = torch.device(device)
        R, V = self.chunk_rows, self.V
        g = self._gen(device, chunk, 1)
        if self.profile == "gauss":
            z = torch.randn(R, V, generator=g, device=device, dtype=torch.float32) * 2.0
        elif self.profile == "zipf":
            keys = torch.rand(R, V, generator=g, device=device, dtype=torch.float32)
            # a random permutation of the profile: entry v gets the profile value of the rank of its key
            order = torch.argsort(keys, dim=1)                       # order[r, j] = index of j-th smallest key
            del keys
            profile = -1.1 * torch.log(torch.arange(1, V + 1, device=device, dtype=torch.float32))
            z = torch.empty(R, V, device=device, dtype=torch.float32)
            z.scatter_(1, order, profile.expand(R, V))
            del order
            z += torch.randn(R, V, generator=g, device=device, dtype=torch.float32)
        else:
            raise ValueError(self.profile)
        verifier = z.to(self.dtype)
        drift = torch.randn(R, V, generator=g, device=device, dtype=torch.float32) * self.drift_sigma
        if self.prover_bf16:
            prover = (z + drift).to(torch.bfloat16)
        else:
            prover = verifier.to(torch.float32) + drift
        return verifier, prover

    # ---- claims --------------------------------------------------------------------
    def mutate_claims(self, chunk: int, honest, verifier):
        """Apply the config's dishonest-token recipe to the honest claims of one chunk.

        honest: int32 [rows] tokens sampled by the caller from the prover logits.
        verifier: the chunk's verifier logits (needed for top-k recipes).
        Returns int32 [rows] on honest's device."""
        dev = honest.device
        R = self.chunk_rows
        assert honest.shape == (R,)
        g = torch.Generator().manual_seed(MASTER_SEED + self.index + 10_000 * (chunk + 1) + 2)
        claims = honest.clone()
        if self.mutation == "none":
            return claims
        if self.mutation == "uniform":          # a fraction of rows replaced by a uniform-random token
            pick = torch.rand(R, generator=g) < self.mutation_frac
            repl = torch.randint(0, self.V, (R,), generator=g, dtype=torch.int32)
            return torch.where(pick.to(dev), repl.to(dev), claims)
        if self.mutation == "topk":             # a fraction swapped to a random one of the row's top-k tokens
            pick = torch.rand(R, generator=g) < self.mutation_frac
            col = torch.randint(0, self.mutation_k, (R,), generator=g)
            rows = torch.nonzero(pick).flatten()
            if rows.numel():
                top = verifier[rows.to(verifier.device)].float().topk(self.mutation_k, dim=1).indices
                repl = top.gather(1, col[rows].to(top.device).unsqueeze(1)).flatten().to(torch.int32)
                claims[rows.to(dev)] = repl.to(dev)
            return claims
        if self.mutation == "stego":            # chosen sequences encode 2 message bits per token
            stego = set(self.stego_sequences())
            row0 = chunk * R
            seq_of_row = (torch.arange(R) + row0) // self.L
            pick = torch.tensor([int(s) in stego for s in seq_of_row.tolist()])
            rows = torch.nonzero(pick).flatten()
            if rows.numel():
                bits = torch.randint(0, self.mutation_k, (R,), generator=g)
                top = verifier[rows.to(verifier.device)].float().topk(self.mutation_k, dim=1).indices
                repl = top.gather(1, bits[rows].to(top.device).unsqueeze(1)).flatten().to(torch.int32)
                claims[rows.to(dev)] = repl.to(dev)
            return claims
        raise ValueError(self.mutation)


@dataclasses.dataclass(frozen=True)
class LmHeadWorkload:
    """Inputs of the fused LM-head path: final hidden states and the LM-head matrix instead of logits.

    hidden [N, d] bf16 ~ N(0, 1); weight [V, d] bf16 ~ N(0, w_sigma^2); the prover's hidden states are
    the verifier's plus N(0, drift_sigma^2), re-rounded to bf16 (benign numerical drift upstream of
    the LM head)."""
    name: str
    index: int
    S: int
    L: int
    V: int
    d: int
    temperature: float
    w_sigma: float
    drift_sigma: float

    @property
    def N(self) -> int:
        return self.S * self.L

    seeds = Workload.seeds
    seq_ids = Workload.seq_ids
    positions = Workload.positions
    seq_offsets = Workload.seq_offsets

    def _gen(self, device, salt: int):
        g = torch.Generator(device=device)
        g.manual_seed(MASTER_SEED + self.index + 10_000 * salt)
        return g

    def weight(self, device, rows_per_chunk: int = 8192):
        device = torch.device(device)
        g = self._gen(device, 1)
        W = torch.empty(self.V, self.d, dtype=torch.bfloat16, device=device)
        for r0 in range(0, self.V, rows_per_chunk):
            r1 = min(self.V, r0 + rows_per_chunk)
            W[r0:r1] = (torch.randn(r1 - r0, self.d, generator=g, device=device, dtype=torch.float32)
                        * self.w_sigma).to(torch.bfloat16)
        return W

    def hidden(self, device):
        """(verifier, prover) hidden states, both [N, d] bf16 on `device`."""
        device = torch.device(device)
        g = self._gen(device, 2)
        h = torch.randn(self.N, self.d, generator=g, device=device, dtype=torch.float32)
        drift = torch.randn(self.N, self.d, generator=g, device=device, dtype=torch.float32) * self.drift_sigma
        return h.to(torch.bfloat16), (h + drift).to(torch.bfloat16)


# The configurations named in the benchmark spec, in its order (index 4, the fused LM head, takes
# hidden states instead of logits: C4_LMHEAD below).
C1_TINY = Workload("c1_tiny", 1, S=4, L=16, V=1024, dtype=torch.float32, temperature=1.0, profile="gauss",
                   drift_sigma=1e-3, prover_bf16=False, chunk_rows=64, mutation="uniform", mutation_frac=0.10)
C2_3B = Workload("c2_3b_class", 2, S=32, L=128, V=128256, dtype=torch.bfloat16, temperature=0.7, profile="zipf",
                 drift_sigma=2e-3, prover_bf16=False, chunk_rows=256, mutation="topk", mutation_frac=0.02,
                 mutation_k=8)
C3_30B = Workload("c3_30b_moe_class", 3, S=64, L=1024, V=151936, dtype=torch.bfloat16, temperature=1.0,
                  profile="zipf", drift_sigma=4e-3, prover_bf16=True, chunk_rows=512, mutation="none")
C5_STEGO = Workload("c5_stego_audit", 5, S=256, L=1024, V=151936, dtype=torch.bfloat16, temperature=0.8,
                    profile="zipf", drift_sigma=4e-3, prover_bf16=True, chunk_rows=512, mutation="stego",
                    mutation_frac=0.01, mutation_k=4)

C4_LMHEAD = LmHeadWorkload("c4_fused_lm_head", 4, S=16, L=1024, V=151936, d=4096, temperature=1.0, w_sigma=0.02,
                           drift_sigma=4e-3)

WORKLOADS = {w.name: w for w in (C1_TINY, C2_3B, C3_30B, C5_STEGO)}


def scaled(w: Workload, S: int = None, L: int = None, V: int = None, chunk_rows: int = None) -> Workload:
    """A smaller instance of a workload with the same recipe (for tests that run the oracle on every row)."""
    S = w.S if S is None else S
    L = w.L if L is None else L
    V = w.V if V is None else V
    if chunk_rows is None:
        chunk_rows = math.gcd(w.chunk_rows, S * L)
    return dataclasses.replace(w, S=S, L=L, V=V, chunk_rows=chunk_rows)
