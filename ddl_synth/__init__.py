"""Seeded synthetic inputs for the synchronizer hot path.

This module only *draws inputs*: tensor shapes, random fragments, token counters and
quorum masks shaped like the five benchmark workloads.  It holds none of the method's
arithmetic (no weights, no merge, no optimiser step) and is the one module that both the
CPU oracle's tests and the HIP path's tests/benchmark use.

Seed scheme: every random stream is keyed by the tuple
``(workload, fragment, tensor, role[, learner])`` hashed with BLAKE2b to a 63-bit seed, so
streams are independent and any single tensor can be regenerated on its own.

Recipe (all workloads): theta ~ N(0, 0.02^2) fp32; v ~ N(0, (1e-4)^2) fp32 (zero in the
tiny workload); learner m = theta + sigma_m * N(0, 1), computed in fp32 and, for bf16
learners, rounded to nearest-even bf16 -- that rounded value is the input to both sides.
Absent learners' buffers can be poisoned with NaN to show they are never read.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

LR_DEFAULT = 0.7
MU_DEFAULT = 0.9


def seed_for(*key) -> int:
    """63-bit seed from an arbitrary key tuple (ints / strings)."""
    h = hashlib.blake2b(repr(tuple(key)).encode(), digest_size=8).digest()
    return int.from_bytes(h, "little") & ((1 << 63) - 1)


@dataclass
class TensorSpec:
    name: str
    shape: Tuple[int, ...]

    @property
    def numel(self) -> int:
        n = 1
        for s in self.shape:
            n *= s
        return n


@dataclass
class FragmentSpec:
    index: int
    tensors: List[TensorSpec]
    M: int
    learner_dtype: str                  # "bf16" or "f32"
    token_counts: List[int]
    quorum_mask: List[int]
    drift: List[float]                  # per-learner sigma of theta_m - theta
    lr: float = LR_DEFAULT
    mu: float = MU_DEFAULT
    v_sigma: float = 1e-4

    @property
    def numel(self) -> int:
        return sum(t.numel for t in self.tensors)

    @property
    def Mq(self) -> int:
        """Learners that actually contribute: in the quorum and with a non-zero counter."""
        return sum(1 for q, n in zip(self.quorum_mask, self.token_counts) if q and n > 0)

    @property
    def bytes_per_param(self) -> int:
        """Algorithmic HBM bytes per parameter: present learners read once, theta and v
        read once and written once."""
        b = 2 if self.learner_dtype == "bf16" else 4
        return self.Mq * b + 16


@dataclass
class Workload:
    name: str
    fragments: List[FragmentSpec]
    arrival_order: List[int] = field(default_factory=list)

    @property
    def numel(self) -> int:
        return sum(f.numel for f in self.fragments)

    @property
    def algorithmic_bytes(self) -> int:
        return sum(f.numel * f.bytes_per_param for f in self.fragments)

    @property
    def num_segments(self) -> int:
        return sum(len(f.tensors) for f in self.fragments)


def _choose_quorum(rng: np.random.Generator, M: int, k: int) -> List[int]:
    mask = np.zeros(M, dtype=np.int64)
    mask[rng.choice(M, size=k, replace=False)] = 1
    return mask.tolist()


def _uniform_tokens(rng: np.random.Generator, M: int, scale: int) -> List[int]:
    return [int(round(x)) for x in rng.uniform(0.5, 1.5, size=M) * scale]


def _dense_block(d_model: int, d_ff: int, gated: bool, prefix: str) -> List[TensorSpec]:
    t = [TensorSpec(f"{prefix}W{n}", (d_model, d_model)) for n in ("q", "k", "v", "o")]
    if gated:
        t += [TensorSpec(f"{prefix}W_gate", (d_model, d_ff)),
              TensorSpec(f"{prefix}W_up", (d_model, d_ff)),
              TensorSpec(f"{prefix}W_down", (d_ff, d_model))]
    else:
        t += [TensorSpec(f"{prefix}W_up", (d_model, d_ff)),
              TensorSpec(f"{prefix}W_down", (d_ff, d_model))]
    return t


def tiny(n: int = 1 << 20) -> Workload:
    """One flat fp32 fragment, M=2 both present, tokens [1000, 3000], v = 0."""
    f = FragmentSpec(0, [TensorSpec("flat", (n,))], M=2, learner_dtype="f32",
                     token_counts=[1000, 3000], quorum_mask=[1, 1], drift=[1e-3, 1e-3],
                     v_sigma=0.0)
    return Workload("tiny", [f], [0])


def dense_block(d_model: int = 2048, d_ff: int = 8192) -> Workload:
    """One transformer block (Wq, Wk, Wv, Wo, W_up, W_down) as six tensors; M=4 bf16
    learners, 3 of 4 in the quorum, tokens U[0.5,1.5] * 2^20."""
    rng = np.random.default_rng(seed_for("dense_block", "meta"))
    M = 4
    f = FragmentSpec(0, _dense_block(d_model, d_ff, False, "blk0."), M=M, learner_dtype="bf16",
                     token_counts=_uniform_tokens(rng, M, 1 << 20),
                     quorum_mask=_choose_quorum(rng, M, 3), drift=[1e-3] * M)
    return Workload("dense_block", [f], [0])


def large_dense(d_model: int = 4096, d_ff: int = 14336, blocks: int = 4) -> Workload:
    """Four gated-FFN transformer blocks as ONE fragment of 28 tensors; M=8 bf16 learners,
    6 of 8 in the quorum, per-learner drift sigma ~ U[5e-4, 2e-3], tokens U * 2^22."""
    rng = np.random.default_rng(seed_for("large_dense", "meta"))
    M = 8
    tensors: List[TensorSpec] = []
    for b in range(blocks):
        tensors += _dense_block(d_model, d_ff, True, f"blk{b}.")
    f = FragmentSpec(0, tensors, M=M, learner_dtype="bf16",
                     token_counts=_uniform_tokens(rng, M, 1 << 22),
                     quorum_mask=_choose_quorum(rng, M, 6),
                     drift=rng.uniform(5e-4, 2e-3, size=M).tolist())
    return Workload("large_dense", [f], [0])


def moe(d_model: int = 2048, d_ff: int = 1408, experts: int = 64,
        stacked: bool = False) -> Workload:
    """64 experts, each three separate d_model x d_ff matrices, plus the router matrix: one
    fragment of 193 tensors; M=16 bf16 learners, 11 of 16 present, heavy-tailed lognormal
    token counters (median 2^20, sigma 1).  ``stacked`` keeps the same parameters in the other
    common storage layout: the experts' matrices stacked into three [experts, ., .] tensors,
    4 tensors in all."""
    rng = np.random.default_rng(seed_for("moe", "meta"))
    M = 16
    tensors: List[TensorSpec] = []
    if stacked:
        tensors += [TensorSpec("experts.W_gate", (experts, d_model, d_ff)),
                    TensorSpec("experts.W_up", (experts, d_model, d_ff)),
                    TensorSpec("experts.W_down", (experts, d_ff, d_model))]
    for e in range(0 if stacked else experts):
        tensors += [TensorSpec(f"expert{e}.W_gate", (d_model, d_ff)),
                    TensorSpec(f"expert{e}.W_up", (d_model, d_ff)),
                    TensorSpec(f"expert{e}.W_down", (d_ff, d_model))]
    tensors.append(TensorSpec("router", (d_model, experts)))
    tokens = [max(1, int(round(x))) for x in rng.lognormal(np.log(2.0 ** 20), 1.0, size=M)]
    f = FragmentSpec(0, tensors, M=M, learner_dtype="bf16", token_counts=tokens,
                     quorum_mask=_choose_quorum(rng, M, 11), drift=[1e-3] * M)
    return Workload("moe_stacked" if stacked else "moe", [f], [0])


def streaming_model(d_model: int = 4096, d_ff: int = 14336, blocks: int = 32,
                    vocab: int = 128256) -> Workload:
    """A dense decoder split into one fragment per block plus the embedding; M=6 bf16
    learners; each fragment has its own seeded quorum (4, 5 or 6 of 6) and token counters;
    fragments arrive in a seeded random order."""
    M = 6
    frags: List[FragmentSpec] = []
    for b in range(blocks + 1):
        rng = np.random.default_rng(seed_for("streaming_model", b, "meta"))
        if b < blocks:
            tensors = _dense_block(d_model, d_ff, True, f"blk{b}.")
        else:
            tensors = [TensorSpec("embedding", (vocab, d_model))]
        k = int(rng.integers(4, M + 1))
        frags.append(FragmentSpec(b, tensors, M=M, learner_dtype="bf16",
                                  token_counts=_uniform_tokens(rng, M, 1 << 22),
                                  quorum_mask=_choose_quorum(rng, M, k), drift=[1e-3] * M))
    order = np.random.default_rng(seed_for("streaming_model", "arrival")).permutation(
        blocks + 1).tolist()
    return Workload("streaming_model", frags, order)


def small_fragments(d_model: int = 512, d_ff: int = 2048, blocks: int = 64) -> Workload:
    """Many small fragments due at the same time: 64 transformer blocks of 3.1 M parameters
    (6 tensors each), one fragment per block; M=4 bf16 learners, per-fragment seeded quorum
    of 3 or 4.  The case for the multi-fragment launch: one kernel covers up to sixteen
    fragments, so small fragments need not each pay a launch."""
    M = 4
    frags: List[FragmentSpec] = []
    for b in range(blocks):
        rng = np.random.default_rng(seed_for("small_fragments", b, "meta"))
        k = int(rng.integers(3, M + 1))
        frags.append(FragmentSpec(b, _dense_block(d_model, d_ff, False, f"blk{b}."), M=M,
                                  learner_dtype="bf16",
                                  token_counts=_uniform_tokens(rng, M, 1 << 20),
                                  quorum_mask=_choose_quorum(rng, M, k), drift=[1e-3] * M))
    order = np.random.default_rng(seed_for("small_fragments", "arrival")).permutation(
        blocks).tolist()
    return Workload("small_fragments", frags, order)


def regroup(wl: Workload, fragment_of: Sequence[int], num_fragments: int) -> Workload:
    """The same tensors regrouped into ``num_fragments`` fragments: tensor i (numbered across
    the fragments of ``wl`` in order) goes to fragment ``fragment_of[i]``.  The partition is an
    input (it comes from the fragmentation routine under test); each new fragment draws its
    own quorum (at least 2/3 of the learners) and token counters, and the arrival order is a
    seeded permutation."""
    tensors = [t for f in wl.fragments for t in f.tensors]
    assert len(fragment_of) == len(tensors)
    base = wl.fragments[0]
    name = f"{wl.name}/regrouped{num_fragments}"
    frags: List[FragmentSpec] = []
    for p in range(num_fragments):
        rng = np.random.default_rng(seed_for(name, p, "meta"))
        mine = [t for t, q in zip(tensors, fragment_of) if q == p]
        k = int(rng.integers(-(-2 * base.M // 3), base.M + 1))
        frags.append(FragmentSpec(p, mine, M=base.M, learner_dtype=base.learner_dtype,
                                  token_counts=_uniform_tokens(rng, base.M, 1 << 22),
                                  quorum_mask=_choose_quorum(rng, base.M, k),
                                  drift=list(base.drift), lr=base.lr, mu=base.mu,
                                  v_sigma=base.v_sigma))
    order = np.random.default_rng(seed_for(name, "arrival")).permutation(num_fragments).tolist()
    return Workload(name, frags, order)


WORKLOADS = {
    "tiny": tiny,
    "dense_block": dense_block,
    "large_dense": large_dense,
    "moe": moe,
    "moe_stacked": lambda: moe(stacked=True),
    "streaming_model": streaming_model,
    "small_fragments": small_fragments,
}


def reduced(name: str) -> Workload:
    """The same structure (tensor count, M, quorum, counters, dtype) at sizes a CPU oracle
    finishes in seconds.  Dimensions are chosen odd-ish so tensors end in ragged tails."""
    if name == "tiny":
        return tiny(1 << 16)
    if name == "dense_block":
        return dense_block(d_model=120, d_ff=499)
    if name == "large_dense":
        return large_dense(d_model=72, d_ff=251, blocks=4)
    if name == "moe":
        return moe(d_model=64, d_ff=45, experts=64)
    if name == "moe_stacked":
        return moe(d_model=64, d_ff=45, experts=64, stacked=True)
    if name == "small_fragments":
        return small_fragments(d_model=40, d_ff=131, blocks=64)
    if name == "streaming_model":
        return streaming_model(d_model=48, d_ff=163, blocks=32, vocab=1003)
    raise KeyError(name)


# ---------------------------------------------------------------------------------------
# tensor generation
# ---------------------------------------------------------------------------------------

def _gen(device, *key) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed_for(*key))
    return g


_CHUNK = 1 << 26  # elements generated at a time: bounds the temporaries on huge tensors


def _randn_into(out: torch.Tensor, sigma: float, g: torch.Generator,
                base: Optional[torch.Tensor] = None) -> None:
    """out[i] = (base[i] if base is given else 0) + sigma * N(0,1), drawn chunk by chunk in
    fp32 and cast to out's dtype (round-to-nearest-even for bf16)."""
    n = out.numel()
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        z = torch.randn(hi - lo, generator=g, device=out.device, dtype=torch.float32)
        z.mul_(sigma)
        if base is not None:
            z.add_(base[lo:hi])
        out[lo:hi] = z.to(out.dtype)


@dataclass
class SegmentData:
    """Device (or host) tensors of one tensor of one fragment."""
    theta: torch.Tensor
    v: torch.Tensor
    learners: List[Optional[torch.Tensor]]


def make_segment(wl: Workload, frag: FragmentSpec, tensor_index: int, device="cpu",
                 absent: str = "valid", numel: Optional[int] = None) -> SegmentData:
    """Draw theta, v and the M learner copies of one tensor.

    ``absent`` says what absent learners' buffers hold: "valid" (a normal drifted copy, as
    when a learner merely missed the deadline), "nan" (poisoned) or "none" (no buffer).
    ``numel`` overrides the tensor's element count (for sampling a prefix)."""
    spec = frag.tensors[tensor_index]
    n = spec.numel if numel is None else numel
    dt = torch.bfloat16 if frag.learner_dtype == "bf16" else torch.float32
    key = (wl.name, frag.index, tensor_index)
    theta = torch.empty(n, dtype=torch.float32, device=device)
    _randn_into(theta, 0.02, _gen(device, *key, "theta"))
    v = torch.zeros(n, dtype=torch.float32, device=device)
    if frag.v_sigma > 0:
        _randn_into(v, frag.v_sigma, _gen(device, *key, "v"))
    learners: List[Optional[torch.Tensor]] = []
    for m in range(frag.M):
        present = bool(frag.quorum_mask[m]) and frag.token_counts[m] > 0
        if not present and absent == "none":
            learners.append(None)
            continue
        x = torch.empty(n, dtype=dt, device=device)
        if not present and absent == "nan":
            x.fill_(float("nan"))
        else:
            _randn_into(x, frag.drift[m], _gen(device, *key, "learner", m), base=theta)
        learners.append(x)
    return SegmentData(theta, v, learners)


def make_fragment(wl: Workload, frag: FragmentSpec, device="cpu",
                  absent: str = "valid") -> List[SegmentData]:
    return [make_segment(wl, frag, i, device, absent) for i in range(len(frag.tensors))]


# ---------------------------------------------------------------------------------------
# host views for the oracle (pure data movement)
# ---------------------------------------------------------------------------------------

def to_host_array(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """fp32 tensor -> float32 array; bf16 tensor -> uint16 array of the raw bit patterns."""
    if t is None:
        return None
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    assert t.dtype == torch.float32
    return t.numpy()


def sample_windows(n: int, num: int, width: int, seed: int) -> List[Tuple[int, int]]:
    """Seeded [lo, hi) windows into a tensor of n elements: always the first and the last
    ``width`` elements (the ragged tail lives there), the rest at random, unaligned offsets."""
    if n <= width * max(num, 2):
        return [(0, n)]
    rng = np.random.default_rng(seed)
    wins = [(0, width), (n - width, n)]
    for _ in range(max(0, num - 2)):
        lo = int(rng.integers(0, n - width))
        wins.append((lo, lo + width))
    return wins
