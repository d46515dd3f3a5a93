"""Seeded synthetic inputs for the bucket-wise clip + Adam path.

This module only *describes* inputs: BERT-shaped tensor lists, how a flat
gradient stream is cut into buckets, and seeded random values for gradients,
parameters and moments.  It contains none of the method's arithmetic (no
norm, no clip coefficient, no Adam) so that both the CPU oracle's tests and the
GPU path's tests can draw the very same host arrays from it.

Shapes follow BERT (Devlin et al.) as the paper trains it (Sec. 2.4: MLPerf
BERT, max sequence 512); buckets follow the paper's description of bucketed
all-reduce (Sec. 2.1: gradients are grouped into fixed-size buckets, 25 MB by
default, ordered by when backward produces them, i.e. last layer first, which
is also the b = B..1 loop of Alg. 1).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

MIB = 1 << 20

# ----------------------------------------------------------------------------
# tensor lists
# ----------------------------------------------------------------------------


def bert_tensor_list(vocab: int, hidden: int, n_layers: int, ffn: int,
                     max_pos: int) -> List[Tuple[str, int]]:
    """(name, numel) in registration order for a BERT encoder with pooler."""
    H, F = hidden, ffn
    out: List[Tuple[str, int]] = [
        ("emb.word", vocab * H), ("emb.pos", max_pos * H), ("emb.type", 2 * H),
        ("emb.ln.g", H), ("emb.ln.b", H),
    ]
    for l in range(n_layers):
        pre = f"l{l}."
        out += [
            (pre + "q.w", H * H), (pre + "q.b", H),
            (pre + "k.w", H * H), (pre + "k.b", H),
            (pre + "v.w", H * H), (pre + "v.b", H),
            (pre + "o.w", H * H), (pre + "o.b", H),
            (pre + "ln1.g", H), (pre + "ln1.b", H),
            (pre + "ffn1.w", H * F), (pre + "ffn1.b", F),
            (pre + "ffn2.w", F * H), (pre + "ffn2.b", H),
            (pre + "ln2.g", H), (pre + "ln2.b", H),
        ]
    out += [("pooler.w", H * H), ("pooler.b", H)]
    return out


def bert_base_numels() -> List[int]:
    return [n for _, n in bert_tensor_list(30522, 768, 12, 3072, 512)]


def bert_large_numels() -> List[int]:
    return [n for _, n in bert_tensor_list(30522, 1024, 24, 4096, 512)]


# ----------------------------------------------------------------------------
# bucket layouts
# ----------------------------------------------------------------------------


@dataclass
class Layout:
    """A bucket layout: every element of every tensor lies in exactly one
    segment of exactly one bucket.  Segment s covers elements
    [seg_begin[s], seg_begin[s] + seg_len[s]) of tensor seg_tensor[s]; bucket b
    owns segments bucket_seg_off[b] .. bucket_seg_off[b+1]-1, in that order.
    Bucket 0 is the first one backward completes (the model's last tensors)."""
    tensor_numel: np.ndarray        # uint64 [n_tensors]
    bucket_seg_off: np.ndarray      # uint64 [n_buckets + 1]
    seg_tensor: np.ndarray          # uint32 [n_segments]
    seg_begin: np.ndarray           # uint64 [n_segments]
    seg_len: np.ndarray             # uint64 [n_segments]

    @property
    def n_tensors(self) -> int:
        return int(self.tensor_numel.shape[0])

    @property
    def n_buckets(self) -> int:
        return int(self.bucket_seg_off.shape[0]) - 1

    @property
    def n_segments(self) -> int:
        return int(self.seg_tensor.shape[0])

    @property
    def n_elements(self) -> int:
        return int(self.tensor_numel.sum())

    def bucket_numel(self) -> np.ndarray:
        cs = np.concatenate([[0], np.cumsum(self.seg_len.astype(np.int64))])
        off = self.bucket_seg_off.astype(np.int64)
        return cs[off[1:]] - cs[off[:-1]]

    def segments_of(self, b: int):
        lo, hi = int(self.bucket_seg_off[b]), int(self.bucket_seg_off[b + 1])
        for s in range(lo, hi):
            yield int(self.seg_tensor[s]), int(self.seg_begin[s]), int(self.seg_len[s])

    def tensors_split(self) -> int:
        """Number of tensors that appear in more than one bucket."""
        owner: Dict[int, set] = {}
        for b in range(self.n_buckets):
            for t, _, _ in self.segments_of(b):
                owner.setdefault(t, set()).add(b)
        return sum(1 for s in owner.values() if len(s) > 1)


def _mk_layout(numels: Sequence[int], buckets: List[List[Tuple[int, int, int]]]) -> Layout:
    off = [0]
    st, sb, sl = [], [], []
    for segs in buckets:
        for (t, b, l) in segs:
            st.append(t), sb.append(b), sl.append(l)
        off.append(len(st))
    return Layout(np.asarray(numels, dtype=np.uint64), np.asarray(off, dtype=np.uint64),
                  np.asarray(st, dtype=np.uint32), np.asarray(sb, dtype=np.uint64),
                  np.asarray(sl, dtype=np.uint64))


def layout_one_tensor_per_bucket(numels: Sequence[int]) -> Layout:
    return _mk_layout(numels, [[(t, 0, int(n))] for t, n in enumerate(numels)])


def layout_flat_split(numels: Sequence[int], cap_elems: int, reverse: bool = True) -> Layout:
    """Concatenate the tensors (last-registered first when `reverse`) into one
    flat stream and cut it every `cap_elems` elements.  Tensors that straddle a
    cut are split into several segments."""
    assert cap_elems > 0
    order = range(len(numels) - 1, -1, -1) if reverse else range(len(numels))
    buckets: List[List[Tuple[int, int, int]]] = [[]]
    room = cap_elems
    for t in order:
        pos, left = 0, int(numels[t])
        while left > 0:
            if room == 0:
                buckets.append([])
                room = cap_elems
            take = min(left, room)
            buckets[-1].append((t, pos, take))
            pos += take
            left -= take
            room -= take
    return _mk_layout(numels, buckets)


def layout_whole_tensors(numels: Sequence[int], cap_elems: int, reverse: bool = True) -> Layout:
    """DDP-style packing: whole tensors are appended to the current bucket and a
    new bucket is opened once the current one has reached `cap_elems`."""
    order = range(len(numels) - 1, -1, -1) if reverse else range(len(numels))
    buckets: List[List[Tuple[int, int, int]]] = [[]]
    fill = 0
    for t in order:
        if fill >= cap_elems and buckets[-1]:
            buckets.append([])
            fill = 0
        buckets[-1].append((t, 0, int(numels[t])))
        fill += int(numels[t])
    return _mk_layout(numels, buckets)


# ----------------------------------------------------------------------------
# seeded values
# ----------------------------------------------------------------------------

_KIND = {"p": 1, "m": 2, "v": 3, "g": 4, "aux": 5}


def _rng(seed: int, kind: str, tensor: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, _KIND[kind], tensor])))


def _fill(numels: Sequence[int], fn, threads: int = 8) -> List[np.ndarray]:
    idx = list(range(len(numels)))
    if threads <= 1 or len(idx) < 4:
        return [fn(t, int(numels[t])) for t in idx]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda t: fn(t, int(numels[t])), idx))


def normal_tensors(numels, seed: int, kind: str, sigma: float, threads: int = 8) -> List[np.ndarray]:
    def one(t, n):
        a = _rng(seed, kind, t).standard_normal(n, dtype=np.float32)
        a *= np.float32(sigma)
        return a
    return _fill(numels, one, threads)


def zeros_tensors(numels) -> List[np.ndarray]:
    return [np.zeros(int(n), dtype=np.float32) for n in numels]


def warm_second_moment(numels, seed: int, threads: int = 8) -> List[np.ndarray]:
    """v = 1e-6 * (0.5 + U[0,1)): a strictly positive second moment of the size
    gradients of scale 1e-3 would have built up."""
    def one(t, n):
        a = _rng(seed, "v", t).random(n, dtype=np.float32)
        a += np.float32(0.5)
        a *= np.float32(1e-6)
        return a
    return _fill(numels, one, threads)


def student_t_fp16_tensors(numels, seed: int, scale: float, threads: int = 8) -> List[np.ndarray]:
    """Student-t (3 degrees of freedom) times `scale`, rounded to fp16."""
    def one(t, n):
        a = _rng(seed, "g", t).standard_t(3.0, n).astype(np.float32)
        a *= np.float32(scale)
        return a.astype(np.float16)
    return _fill(numels, one, threads)


def float32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Input preparation only: the bfloat16 bit patterns (uint16) nearest to fp32 values,
    ties to even; NaN stays NaN.  bfloat16 is the upper half of a binary32."""
    u = np.ascontiguousarray(a, np.float32).view(np.uint32).astype(np.uint64)
    rounded = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        rounded[nan] = ((u[nan] >> 16) | 0x40).astype(np.uint16)
    return rounded


def bf16_bits_to_float32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal_bf16_tensors(numels, seed: int, sigma: float, threads: int = 8) -> List[np.ndarray]:
    """N(0, sigma^2) rounded to bfloat16, as uint16 bit patterns."""
    return [float32_to_bf16_bits(x) for x in normal_tensors(numels, seed, "g", sigma, threads)]


def bert_decay_mask(vocab: int, hidden: int, n_layers: int, ffn: int, max_pos: int) -> np.ndarray:
    """The usual BERT exemption: weight decay on weight matrices and embeddings,
    none on biases and LayerNorm gains/offsets.  uint8 [n_tensors], 1 = decay."""
    names = [n for n, _ in bert_tensor_list(vocab, hidden, n_layers, ffn, max_pos)]
    return np.asarray([0 if (n.endswith(".b") or ".ln" in n) else 1 for n in names], np.uint8)


def scale_buckets_inplace(layout: Layout, tensors: List[np.ndarray], which: Sequence[int], factor: float):
    for b in which:
        for t, beg, ln in layout.segments_of(b):
            tensors[t][beg:beg + ln] *= tensors[t].dtype.type(factor)


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------


@dataclass
class Hyper:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-6
    weight_decay: float = 0.01


@dataclass
class Workload:
    name: str
    layout: Layout
    grad_dtype: str                 # "f32" | "f16"
    thresholds: np.ndarray          # float32 [n_buckets]: the per-bucket value actually compared
    hyper: Hyper
    first_step: int
    n_steps: int = 1
    seed: int = 0
    sigma_g: float = 1e-3
    warm: bool = False
    hot_buckets: List[int] = field(default_factory=list)   # buckets whose gradients are x100

    # -- value generators (host arrays; same bits go to oracle and to the GPU) --
    def params(self, threads: int = 8) -> List[np.ndarray]:
        return normal_tensors(self.layout.tensor_numel, self.seed, "p", 0.02, threads)

    def exp_avg(self, threads: int = 8) -> List[np.ndarray]:
        if not self.warm:
            return zeros_tensors(self.layout.tensor_numel)
        return normal_tensors(self.layout.tensor_numel, self.seed, "m", 3e-4, threads)

    def exp_avg_sq(self, threads: int = 8) -> List[np.ndarray]:
        if not self.warm:
            return zeros_tensors(self.layout.tensor_numel)
        return warm_second_moment(self.layout.tensor_numel, self.seed, threads)

    def grads(self, step_index: int = 0, threads: int = 8) -> List[np.ndarray]:
        """Gradients for the step_index-th step of this workload (0-based)."""
        seed = self.seed if self.n_steps == 1 else 1000 + self.first_step + step_index
        if self.grad_dtype == "f16":
            return student_t_fp16_tensors(self.layout.tensor_numel, seed, self.sigma_g, threads)
        g = normal_tensors(self.layout.tensor_numel, seed, "g", self.sigma_g, threads)
        if self.hot_buckets:
            scale_buckets_inplace(self.layout, g, self.hot_buckets, 100.0)
        return g


def config_tiny() -> Workload:
    lay = layout_one_tensor_per_bucket([1000, 4096, 12345])
    return Workload("tiny", lay, "f32", np.asarray([0.1, 1.0, 10.0], np.float32), Hyper(),
                    first_step=1, seed=0, sigma_g=1e-2)


def config_bert_base(numels: Optional[Sequence[int]] = None, bucket_bytes: int = 25 * MIB) -> Workload:
    lay = layout_flat_split(numels or bert_base_numels(), bucket_bytes // 4)
    return Workload("bert_base_25MiB", lay, "f32", np.full(lay.n_buckets, 1.0, np.float32), Hyper(),
                    first_step=100, seed=0)


def config_bert_large(numels: Optional[Sequence[int]] = None, bucket_bytes: int = 50 * MIB) -> Workload:
    lay = layout_flat_split(numels or bert_large_numels(), bucket_bytes // 4)
    hot = [b for b in range(lay.n_buckets) if b % 10 == 3]      # 10 % of the buckets get gradients x100
    return Workload("bert_large_50MiB", lay, "f32", np.full(lay.n_buckets, 1.0, np.float32), Hyper(),
                    first_step=1000, seed=0, warm=True, hot_buckets=hot)


def config_bert_large_fp16(numels: Optional[Sequence[int]] = None, bucket_bytes: int = 1 * MIB) -> Workload:
    # Bucket capacity is counted at 4 bytes per element whatever the gradient
    # type, so that 1 MiB gives the ~1300 buckets the configuration names.
    lay = layout_flat_split(numels or bert_large_numels(), bucket_bytes // 4)
    thr = np.full(lay.n_buckets, 1.0 / np.sqrt(float(lay.n_buckets)), np.float32)
    return Workload("bert_large_fp16_1MiB", lay, "f16", thr, Hyper(), first_step=1000, seed=0,
                    sigma_g=1e-4, warm=True)


def config_bert_large_multistep(numels: Optional[Sequence[int]] = None, bucket_bytes: int = 4 * MIB,
                                n_steps: int = 20) -> Workload:
    lay = layout_flat_split(numels or bert_large_numels(), bucket_bytes // 4)
    u = np.random.Generator(np.random.Philox(np.random.SeedSequence([0, _KIND["aux"], 5])))
    thr = (0.01 + (2.0 - 0.01) * u.random(lay.n_buckets)).astype(np.float32)
    return Workload("bert_large_4MiB_20steps", lay, "f32", thr, Hyper(), first_step=1, n_steps=n_steps,
                    seed=0)


def scaled_bert_numels(hidden: int, n_layers: int, ffn: int, vocab: int = 3052, max_pos: int = 64) -> List[int]:
    """A BERT-shaped tensor list shrunk so that the CPU oracle finishes in well
    under a second; same structure (391-tensor pattern for 24 layers)."""
    return [n for _, n in bert_tensor_list(vocab, hidden, n_layers, ffn, max_pos)]


# ----------------------------------------------------------------------------
# sequence-length histograms for the load-balancing simulation
# ----------------------------------------------------------------------------

# Sec. 4.1: four strata by length; Sec. 3.1: share of the Wikipedia samples in each.
LENGTH_STRATUM_END = (128, 256, 384, 512)
LENGTH_STRATUM_SHARE = (0.373, 0.197, 0.117, 0.314)


def length_histogram_piecewise_uniform(n_samples: int = 10_000_000, stratum_end: Sequence[int] = LENGTH_STRATUM_END,
                                       share: Sequence[float] = LENGTH_STRATUM_SHARE) -> np.ndarray:
    """Cumulative length histogram cum[0..L] (uint32, cum[l] = number of samples of length <= l)
    of a synthetic dataset that has the printed share of samples in every stratum and, inside a
    stratum, equally many samples of every length.  Stands in for the Wikipedia histogram, which
    the paper does not print."""
    L = int(stratum_end[-1])
    hist = np.zeros(L + 1, np.int64)
    lo = 0
    for end, sh in zip(stratum_end, share):
        n = int(round(sh / sum(share) * n_samples))
        width = end - lo
        hist[lo + 1:end + 1] = n // width
        hist[lo + 1:lo + 1 + n % width] += 1
        lo = end
    cum = np.cumsum(hist)
    assert cum[-1] < 2 ** 32
    return cum.astype(np.uint32)


def stratum_quota(cum: np.ndarray, stratum_end: Sequence[int], local_batch: int) -> np.ndarray:
    """Samples per stratum in a local batch, in proportion to the strata's sizes
    (largest-remainder rounding so that they add up to local_batch)."""
    ends = [0] + [int(e) for e in stratum_end]
    sizes = np.asarray([int(cum[b]) - int(cum[a]) for a, b in zip(ends[:-1], ends[1:])], np.float64)
    ideal = sizes / sizes.sum() * local_batch
    q = np.floor(ideal).astype(np.int64)
    for i in np.argsort(-(ideal - q), kind="stable")[:local_batch - int(q.sum())]:
        q[i] += 1
    return q.astype(np.uint32)


CONFIGS = {
    1: config_tiny,
    2: config_bert_base,
    3: config_bert_large,
    4: config_bert_large_fp16,
    5: config_bert_large_multistep,
}
