"""Seeded synthetic workloads for the OSP synchronization step.

This module holds tensor-shape tables and random input generators only; it
contains none of the method's arithmetic.  It serves the CPU oracle and the
HIP library alike (both are handed the same host arrays), and imports neither.

The paper evaluates on real CNNs trained on CIFAR / ImageNet (Sec. 5.1.2,
"Workloads").  Those datasets and weights are not used here: each workload
takes only the *parameter-tensor shapes* of the corresponding CNN, in the
order PyTorch enumerates them, and fills parameters and per-worker gradients
from seeded distributions.

Arena layout: every buffer (PS parameters, PS momentum, each worker's
parameter replica, each worker's gradient set) is one flat fp32 array of
``arena_elems`` elements; tensor ``l`` occupies
``[offset[l], offset[l] + numel[l])``.  Offsets are multiples of ``align``
elements.  Elements outside every tensor are padding.
"""
from __future__ import annotations

import dataclasses
import threading
from typing import Callable, List, Sequence

import numpy as np


# ----------------------------------------------------------------------------
# shape rules
# ----------------------------------------------------------------------------

def _conv(cout: int, cin: int, k: int) -> int:
    return cout * cin * k * k


def _bn(c: int) -> List[int]:
    return [c, c]                        # weight vector, bias vector


def tiny_shapes() -> List[int]:
    # odd sizes and a one-element tensor on purpose: exercises ragged tails
    return [432, 16, 4608, 32, 18432, 64, 36864, 64, 38400, 600, 487, 1]


def resnet_basic_shapes(blocks: Sequence[int], n_classes: int) -> List[int]:
    """Basic-block ResNet with a 3x3 stem (the CIFAR variant)."""
    out = [_conv(64, 3, 3)] + _bn(64)
    cin = 64
    for stage, (width, nb) in enumerate(zip((64, 128, 256, 512), blocks)):
        for b in range(nb):
            out += [_conv(width, cin, 3)] + _bn(width)
            out += [_conv(width, width, 3)] + _bn(width)
            if b == 0 and stage > 0:
                out += [_conv(width, cin, 1)] + _bn(width)
            cin = width
    out += [cin * n_classes, n_classes]
    return out


def resnet_bottleneck_shapes(blocks: Sequence[int], n_classes: int) -> List[int]:
    """Bottleneck ResNet (1x1 / 3x3 / 1x1, expansion 4) with a 7x7 stem."""
    out = [_conv(64, 3, 7)] + _bn(64)
    cin = 64
    for width, nb in zip((64, 128, 256, 512), blocks):
        for b in range(nb):
            out += [_conv(width, cin, 1)] + _bn(width)
            out += [_conv(width, width, 3)] + _bn(width)
            out += [_conv(width * 4, width, 1)] + _bn(width * 4)
            if b == 0:
                out += [_conv(width * 4, cin, 1)] + _bn(width * 4)
            cin = width * 4
    out += [cin * n_classes, n_classes]
    return out


def vgg16_shapes(n_classes: int = 1000) -> List[int]:
    out: List[int] = []
    cin = 3
    for c in (64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512):
        out += [_conv(c, cin, 3), c]
        cin = c
    for fin, fout in ((512 * 7 * 7, 4096), (4096, 4096), (4096, n_classes)):
        out += [fin * fout, fout]
    return out


def bert_base_shapes(vocab: int = 30522, hidden: int = 768, layers: int = 12,
                     intermediate: int = 3072, max_pos: int = 512, type_vocab: int = 2) -> List[int]:
    """BERT-base encoder with pooler, parameter tensors in PyTorch order."""
    out = [vocab * hidden, max_pos * hidden, type_vocab * hidden, hidden, hidden]
    for _ in range(layers):
        for _ in range(4):                       # query, key, value, attention output
            out += [hidden * hidden, hidden]
        out += [hidden, hidden]                  # LayerNorm
        out += [hidden * intermediate, intermediate, intermediate * hidden, hidden]
        out += [hidden, hidden]                  # LayerNorm
    out += [hidden * hidden, hidden]             # pooler
    return out


# ----------------------------------------------------------------------------
# gradient distributions (one call fills one tensor of one worker)
# ----------------------------------------------------------------------------

def _grad_normal(std: float) -> Callable:
    def fill(rng: np.random.Generator, out: np.ndarray, tensor_scale: float) -> None:
        rng.standard_normal(out.shape[0], dtype=np.float32, out=out)
        out *= np.float32(std)
    return fill


def _grad_per_tensor_scale(rng: np.random.Generator, out: np.ndarray, tensor_scale: float) -> None:
    rng.standard_normal(out.shape[0], dtype=np.float32, out=out)
    out *= np.float32(tensor_scale)


def _grad_student_t(rng: np.random.Generator, out: np.ndarray, tensor_scale: float) -> None:
    n = out.shape[0]
    step = 1 << 22                       # bounded fp64 temporaries
    for a in range(0, n, step):
        b = min(n, a + step)
        out[a:b] = (1e-3 * rng.standard_t(3.0, b - a)).astype(np.float32)


def _grad_outliers(rng: np.random.Generator, out: np.ndarray, tensor_scale: float) -> None:
    n = out.shape[0]
    rng.standard_normal(n, dtype=np.float32, out=out)
    out *= np.float32(1e-3)
    step = 1 << 22
    for a in range(0, n, step):
        b = min(n, a + step)
        hit = rng.random(b - a, dtype=np.float32) < np.float32(0.01)
        out[a:b][hit] *= np.float32(100.0)


# ----------------------------------------------------------------------------
# bfloat16 storage of gradients (input preparation only)
# ----------------------------------------------------------------------------

def to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest even; NaN stays NaN."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    nan = np.isnan(a)
    if nan.any():
        r[nan] = (u[nan] >> 16) | 0x40
    return r.astype(np.uint16)


def from_bf16(h: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> the fp32 with the same value (exact)."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    n_workers: int
    numel: tuple
    stage2_fraction: float
    grad_fill: Callable
    per_tensor_scale: bool = False
    lr: float = 0.1
    momentum: float = 0.9
    param_std: float = 0.05
    align: int = 1024                    # elements; 1024 fp32 = 4 KiB (measured 1.5-2 % faster than 256 B)

    # ---- layout --------------------------------------------------------
    @property
    def n_tensors(self) -> int:
        return len(self.numel)

    @property
    def n_params(self) -> int:
        return int(sum(self.numel))

    @property
    def budget(self) -> int:
        # floor(f * M), evaluated in exact integer arithmetic on f = p/1000
        return (int(round(self.stage2_fraction * 1000)) * self.n_params) // 1000

    def offsets(self, align: int | None = None) -> np.ndarray:
        a = self.align if align is None else align
        off = np.zeros(self.n_tensors, dtype=np.int64)
        cur = 0
        for i, n in enumerate(self.numel):
            off[i] = cur
            cur = -(-(cur + n) // a) * a
        return off

    def arena_elems(self, align: int | None = None) -> int:
        a = self.align if align is None else align
        off = self.offsets(a)
        end = int(off[-1] + self.numel[-1])
        return -(-end // a) * a

    def _stride(self, align: int | None, pad: int) -> int:
        m = self.arena_elems(align)
        unit = (1 << 18) if m >= (1 << 20) else 1024          # 1 MiB, or 4 KiB for small arenas
        return -(-m // unit) * unit + pad

    def replica_stride(self, align: int | None = None) -> int:
        """Distance in elements between consecutive workers' parameter replicas: the arena
        rounded up to 1 MiB, plus 1 KiB.  Measured on MI355X: rows that are not a multiple of
        1 KiB apart (the earlier 4 KiB + 768 B) cost the kernels that write all N replicas from
        one wavefront 1.5-3 %; an exact multiple of 8 MiB costs the install 5 %."""
        return self._stride(align, 256)

    def worker_stride(self, align: int | None = None) -> int:
        """Distance in elements between consecutive workers' gradient arenas: the arena rounded
        up to 1 MiB, plus 8 KiB (measured against 4 KiB + 768 B: the kernels that read all N
        arenas at once 1-3 % faster; +4 KiB to +32 KiB measure the same)."""
        return self._stride(align, 2048)

    # ---- seeded inputs ---------------------------------------------------
    def _rng(self, seed: int, *path: int) -> np.random.Generator:
        ss = np.random.SeedSequence([seed, self.config_id, *path])
        return np.random.Generator(np.random.PCG64(ss))

    def make_params(self, seed: int = 0, align: int | None = None) -> np.ndarray:
        """PS parameters ~ N(0, param_std); padding is zero."""
        off = self.offsets(align)
        p = np.zeros(self.arena_elems(align), dtype=np.float32)
        for l, n in enumerate(self.numel):
            rng = self._rng(seed, 0x50, l)
            v = p[off[l]:off[l] + n]
            rng.standard_normal(n, dtype=np.float32, out=v)
            v *= np.float32(self.param_std)
        return p

    def tensor_scales(self, seed: int = 0) -> np.ndarray:
        if not self.per_tensor_scale:
            return np.ones(self.n_tensors)
        rng = self._rng(seed, 0x53)
        return 10.0 ** rng.uniform(-4.0, -2.0, self.n_tensors)

    def make_grads(self, seed: int = 0, step: int = 0, align: int | None = None,
                   stride: int | None = None, threads: int = 1,
                   out: np.ndarray | None = None) -> np.ndarray:
        """All workers' gradients for one iteration, shape [N, stride] fp32
        (only the first arena_elems of each row are meaningful; padding = 0)."""
        off = self.offsets(align)
        m_pad = self.arena_elems(align)
        stride = m_pad if stride is None else stride
        assert stride >= m_pad
        if out is None:
            out = np.zeros((self.n_workers, stride), dtype=np.float32)
        assert out.shape == (self.n_workers, stride) and out.dtype == np.float32
        scales = self.tensor_scales(seed)

        def fill_worker(w: int) -> None:
            row = out[w]
            for l, n in enumerate(self.numel):
                rng = self._rng(seed, 0x47, step, w, l)
                self.grad_fill(rng, row[off[l]:off[l] + n], float(scales[l]))

        if threads <= 1:
            for w in range(self.n_workers):
                fill_worker(w)
        else:
            # numpy's generators release the GIL while filling
            pending = list(range(self.n_workers))
            lock = threading.Lock()

            def run() -> None:
                while True:
                    with lock:
                        if not pending:
                            return
                        w = pending.pop()
                    fill_worker(w)

            ts = [threading.Thread(target=run) for _ in range(min(threads, self.n_workers))]
            for t in ts:
                t.start()
            for t in ts:
                t.join()
        return out


def _mk(name, cid, n, numel, f, fill, **kw) -> Workload:
    return Workload(name=name, config_id=cid, n_workers=n, numel=tuple(int(x) for x in numel),
                    stage2_fraction=f, grad_fill=fill, **kw)


WORKLOADS = {
    "tiny": _mk("tiny", 0, 4, tiny_shapes(), 0.3, _grad_normal(1e-3), align=4),
    "resnet18": _mk("resnet18", 1, 8, resnet_basic_shapes((2, 2, 2, 2), 10), 0.5,
                    _grad_per_tensor_scale, per_tensor_scale=True),
    "resnet50": _mk("resnet50", 2, 8, resnet_bottleneck_shapes((3, 4, 6, 3), 1000), 0.5,
                    _grad_student_t),
    "resnet152": _mk("resnet152", 3, 8, resnet_bottleneck_shapes((3, 8, 36, 3), 1000), 0.7,
                     _grad_outliers),
    "vgg16": _mk("vgg16", 4, 16, vgg16_shapes(), 0.5, _grad_normal(5e-4)),
    # not one of the five stated configurations: the paper's NLP model (Sec. 5.1.2), same
    # recipe as resnet18 (8 workers, per-tensor gradient scale)
    "bert_base": _mk("bert_base", 5, 8, bert_base_shapes(), 0.5, _grad_per_tensor_scale,
                     per_tensor_scale=True),
}

# exact tensor and parameter counts of the shape rules above
EXPECTED_COUNTS = {
    "tiny": (12, 100_000),
    "resnet18": (62, 11_173_962),
    "resnet50": (161, 25_557_032),
    "resnet152": (467, 60_192_808),
    "vgg16": (32, 138_357_544),
    "bert_base": (199, 109_482_240),
}


def get(name: str) -> Workload:
    return WORKLOADS[name]


def custom(numel: Sequence[int], n_workers: int, stage2_fraction: float = 0.5,
           align: int = 4, config_id: int = 99, grad_std: float = 1e-3, **kw) -> Workload:
    """Small ad-hoc workload for tests."""
    return _mk("custom", config_id, n_workers, numel, stage2_fraction,
               _grad_normal(grad_std), align=align, **kw)
