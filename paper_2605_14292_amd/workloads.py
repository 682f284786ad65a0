"""Seeded synthetic compression events with the shapes of the five benchmark
configurations.

This module only draws inputs (K, V, Q or scores); it holds none of the
method's arithmetic.  The same tensors are handed to the HIP library and, after
an exact widening to float64, to the CPU oracle by the tests.

One "head" is one independent selection problem: a (sequence, layer, KV-head)
triple.  Heads are generated in fixed-size chunks, each from its own generator
seeded by (seed, config, chunk index), so that any chunk can be regenerated on
its own and a run on the GPU fills HBM chunk by chunk without a host copy.
The bits depend on the device the generator runs on (torch's CPU and GPU
generators are different streams); tests that check a GPU-generated workload
copy the heads they sample back to the host.

They stand in for decode-time KV caches of the 7-8B distilled reasoning models
the paper evaluates; no trace, prompt or weight of those is used.
"""
from __future__ import annotations

import dataclasses
import zlib

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    kv_heads: int
    seqs: int
    n: int            # candidates per head
    b: int            # retained budget (the paper's k)
    d: int
    dtype: str        # "bf16" | "f32"
    lam: float
    v_kind: str       # "clustered" | "dup_normal" | "dup_student_t" | "mixed"
    centres: int = 0
    sigma: float = 0.0
    dup_frac: float = 0.0
    dup_sigma: float = 0.0
    scores: str = "computed"      # "computed" (Q given, G queries) | "given"
    G: int = 1
    what: str = ""

    @property
    def heads(self) -> int:
        return self.layers * self.kv_heads * self.seqs

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    def algorithmic_bytes_per_head(self, b=None, lam=None) -> int:
        """Bytes the method must move once per head: all of V (only the b
        retained rows when lambda == 0), all of K when scores are computed
        from it (else the b retained rows), Q or s, the 2*b retained rows
        written, b int32 indices."""
        b = self.b if b is None else b
        lam = self.lam if lam is None else lam
        e, n, d = self.elem_bytes, self.n, self.d
        v = (n if lam != 0.0 else b) * d * e
        if self.scores == "computed":
            k, q = n * d * e, self.G * d * e
        else:
            k, q = b * d * e, 4 * n
        return v + k + q + 2 * b * d * e + 4 * b


WORKLOADS = {
    "c1": Workload("c1", 1, 1, 1, 192, 64, 128, "f32", 0.5, "clustered",
                   centres=16, sigma=0.1, scores="computed", G=1,
                   what="single head, b=64 retained + 128 recent, fp32"),
    "c2": Workload("c2", 28, 4, 1, 256, 128, 128, "bf16", 0.5, "dup_normal",
                   dup_frac=0.25, dup_sigma=0.05, scores="computed", G=7,
                   what="Qwen-7B-shaped decode-time event, batch 1"),
    "c3": Workload("c3", 32, 8, 32, 192, 64, 128, "bf16", 0.5, "clustered",
                   centres=32, sigma=0.1, scores="given",
                   what="Llama-8B-shaped batched event, 32 sequences"),
    "c4": Workload("c4", 32, 8, 8, 4096, 128, 128, "bf16", 0.5,
                   "dup_student_t", dup_frac=0.2, dup_sigma=0.05,
                   scores="computed", G=4,
                   what="long-prefill one-shot compression, 8 sequences"),
    "c5": Workload("c5", 28, 4, 64, 1024, 128, 128, "bf16", 0.5, "mixed",
                   centres=32, sigma=0.1, scores="computed", G=7,
                   what="lambda sweep, 64 sequences"),
}

CHUNK_HEADS = 64


def _gen(device, seed: int, name: str, chunk: int) -> torch.Generator:
    g = torch.Generator(device=device)
    mix = zlib.crc32(f"{name}/{chunk}".encode()) & 0x7FFFFFFF
    g.manual_seed((int(seed) * 1000003 + mix) % (2**63 - 1))
    return g


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _student_t3(shape, g, device):
    z = _randn(shape, g, device)
    chi = torch.zeros(shape, device=device, dtype=torch.float32)
    for _ in range(3):
        w = _randn(shape, g, device)
        chi.addcmul_(w, w)
    return z / torch.sqrt(chi / 3.0)


def _clustered(h, n, d, centres, sigma, g, device):
    c = _randn((h, centres, d), g, device)
    which = torch.randint(0, centres, (h, n), generator=g, device=device)
    rows = torch.gather(c, 1, which.unsqueeze(-1).expand(h, n, d))
    return rows + sigma * _randn((h, n, d), g, device)


def _apply_duplicates(K, V, frac, sigma, g, device):
    """A random `frac` of the tokens of each head become near-copies (K and V
    rows both) of a random token outside that subset, plus independent noise."""
    h, n, d = V.shape
    n_dup = int(round(frac * n))
    if n_dup == 0:
        return K, V
    perm = torch.argsort(torch.rand((h, n), generator=g, device=device), dim=1)
    dup = perm[:, :n_dup]                       # tokens that become copies
    keep = perm[:, n_dup:]                      # possible sources
    pick = torch.randint(0, n - n_dup, (h, n_dup), generator=g, device=device)
    src = torch.gather(keep, 1, pick)
    e_src = src.unsqueeze(-1).expand(h, n_dup, d)
    e_dup = dup.unsqueeze(-1).expand(h, n_dup, d)
    for X in (K, V):
        rows = torch.gather(X, 1, e_src) + sigma * _randn((h, n_dup, d), g, device)
        X.scatter_(1, e_dup, rows)
    return K, V


def generate_chunk(w: Workload, chunk: int, heads_in_chunk: int, seed=0,
                   device="cpu"):
    """One chunk of heads: dict with K, V [h,n,d] in the workload dtype and
    either Q [h,G,d] (same dtype) or s [h,n] float32."""
    g = _gen(device, seed, w.name, chunk)
    h, n, d = heads_in_chunk, w.n, w.d
    K = _randn((h, n, d), g, device)
    if w.v_kind == "clustered":
        V = _clustered(h, n, d, w.centres, w.sigma, g, device)
    elif w.v_kind == "dup_normal":
        V = _randn((h, n, d), g, device)
        K, V = _apply_duplicates(K, V, w.dup_frac, w.dup_sigma, g, device)
    elif w.v_kind == "dup_student_t":
        V = _student_t3((h, n, d), g, device)
        K, V = _apply_duplicates(K, V, w.dup_frac, w.dup_sigma, g, device)
    elif w.v_kind == "mixed":
        V = _randn((h, n, d), g, device)
        Vc = _clustered(h, n, d, w.centres, w.sigma, g, device)
        perm = torch.argsort(torch.rand((h, n), generator=g, device=device), dim=1)
        is_cl = torch.zeros((h, n), dtype=torch.bool, device=device)
        is_cl.scatter_(1, perm[:, : n // 2], True)
        V = torch.where(is_cl.unsqueeze(-1), Vc, V)
    else:
        raise ValueError(w.v_kind)
    out = {"K": K.to(w.torch_dtype).contiguous(),
           "V": V.to(w.torch_dtype).contiguous()}
    if w.scores == "computed":
        out["Q"] = _randn((h, w.G, d), g, device).to(w.torch_dtype).contiguous()
    else:
        out["s"] = torch.exp(_randn((h, n), g, device)).contiguous()
    return out


def generate(w: Workload, heads=None, seed=0, device="cpu"):
    """The first `heads` heads of the workload (all of them by default),
    concatenated chunk by chunk into preallocated tensors on `device`."""
    H = w.heads if heads is None else int(heads)
    out = None
    done = 0
    chunk = 0
    while done < H:
        hc = min(CHUNK_HEADS, H - done)
        part = generate_chunk(w, chunk, hc, seed=seed, device=device)
        if out is None:
            out = {k: torch.empty((H,) + tuple(v.shape[1:]), dtype=v.dtype,
                                  device=device) for k, v in part.items()}
        for k, v in part.items():
            out[k][done:done + hc].copy_(v)
        done += hc
        chunk += 1
    return out


def to_f64(t: torch.Tensor):
    """Exact widening of a bf16/f32 tensor to a float64 numpy array."""
    return t.detach().to("cpu").to(torch.float64).numpy()
