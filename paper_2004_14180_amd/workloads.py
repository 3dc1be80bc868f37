"""Seeded synthetic inputs: layer lists and gradient generators of the five workloads.

This module serves both the GPU path and the CPU oracle (tests, smoke, benchmark) and holds none
of the optimizer's arithmetic: it only produces flat fp32 vectors.  The paper's own workloads
(ResNet-101 / CIFAR100 and VGG16 / CIFAR10, Sec. 5.1) need datasets and training that are not
available; what the optimizer step sees of them is "one gradient vector per worker per step over a
list of layers", which is what is synthesised here with the shapes of public architectures.

Randomness comes from ``torch.Generator`` objects seeded from (seed, workload, step, worker,
purpose); a workload is generated on one device and copied wherever else it is needed (CPU and
GPU generators produce different streams).
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field
from typing import List, Sequence

import torch


# ------------------------------------------------------------------------------------ layer lists
def resnet18_layers() -> List[int]:
    """ResNet-18 (ImageNet head): conv / bn weight+bias / fc weight+bias, 62 segments, 11 689 512."""
    sizes: List[int] = []

    def conv(cout, cin, k):
        sizes.append(cout * cin * k * k)

    def bn(c):
        sizes.extend([c, c])

    conv(64, 3, 7); bn(64)
    cin = 64
    for stage, cout in enumerate([64, 128, 256, 512]):
        for block in range(2):
            first = block == 0 and stage > 0
            conv(cout, cin if block == 0 else cout, 3); bn(cout)
            conv(cout, cout, 3); bn(cout)
            if first:
                conv(cout, cin, 1); bn(cout)
        cin = cout
    sizes.extend([512 * 1000, 1000])
    return sizes


def gpt_layers(n_blocks: int, d: int, vocab: int, ctx: int) -> List[int]:
    """GPT-2-style decoder with tied output head: token and position embeddings, per block
    ln1(w,b), qkv(w,b), proj(w,b), ln2(w,b), fc(w,b), proj(w,b); final ln(w,b)."""
    sizes = [vocab * d, ctx * d]
    for _ in range(n_blocks):
        sizes += [d, d, d * 3 * d, 3 * d, d * d, d, d, d, d * 4 * d, 4 * d, 4 * d * d, d]
    sizes += [d, d]
    return sizes


def offsets(sizes: Sequence[int]) -> List[int]:
    out = [0]
    for s in sizes:
        out.append(out[-1] + int(s))
    return out


# --------------------------------------------------------------------------------------- workload
@dataclass
class Workload:
    """One of the five configurations (``config`` = 1..5), optionally shrunk for quick tests."""
    config: int
    name: str
    sizes: List[int]
    num_workers: int
    steps: int
    k_g: int = 2
    k_x: int = 6
    weight_ef: int = 1
    weight_quant: bool = True
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8
    seed: int = 0
    embedding_rows: int = 0        # config 3: rows of the first segment that may be zeroed
    embedding_dim: int = 0
    _layer_std: torch.Tensor = field(default=None, repr=False)
    _block_scale: torch.Tensor = field(default=None, repr=False)

    @property
    def seg_offsets(self) -> List[int]:
        return offsets(self.sizes)

    @property
    def num_params(self) -> int:
        return sum(self.sizes)

    # ---- generators ---------------------------------------------------------------------------
    def _gen(self, device, *key) -> torch.Generator:
        g = torch.Generator(device=device)
        h = zlib.crc32(repr((self.seed, self.config, self.name) + tuple(key)).encode())
        g.manual_seed(h)
        return g

    def layer_std(self) -> torch.Tensor:
        """Per-layer gradient scale s_l = 10^U(-4,-1), drawn once per workload (CPU, fp64)."""
        if self._layer_std is None:
            g = self._gen("cpu", "layer_std")
            u = torch.rand(len(self.sizes), generator=g, dtype=torch.float64)
            self._layer_std = 10.0 ** (-4.0 + 3.0 * u)
        return self._layer_std

    def init_weights(self, device) -> torch.Tensor:
        """x_1 ~ N(0, 0.02^2)."""
        g = self._gen(device, "x0")
        x = torch.empty(self.num_params, dtype=torch.float32, device=device)
        return x.normal_(0.0, 0.02, generator=g)

    def synthetic_state(self, device, num_workers=None):
        """A plausible mid-training optimizer state, so that a single step exercises every input:
        error buffers e_i ~ N(0, (0.2 s_l)^2), m ~ N(0, (0.3 s_l)^2), v = (N(0, s_l^2))^2 and a weight
        residual uniform within half a grid step of Q_x.  Returns dict(errs, m, v, werr)."""
        N = self.num_workers if num_workers is None else num_workers
        P = self.num_params
        mk = lambda: torch.empty(P, dtype=torch.float32, device=device)
        errs = []
        for i in range(N):
            e = mk()
            self._fill_layered_normal(e, self._gen(device, "state_e", i), 0.2)
            errs.append(e)
        m = mk()
        self._fill_layered_normal(m, self._gen(device, "state_m"), 0.3)
        v = mk()
        self._fill_layered_normal(v, self._gen(device, "state_v"), 1.0)
        v.square_()
        werr = torch.rand(P, generator=self._gen(device, "state_w"), device=device, dtype=torch.float32)
        werr.sub_(0.5).mul_(2.0 ** -(self.k_x + 1))
        return dict(errs=errs, m=m, v=v, werr=werr)

    def _fill_layered_normal(self, out: torch.Tensor, gen: torch.Generator, rel: float):
        offs = self.seg_offsets
        std = self.layer_std()
        for l, n in enumerate(self.sizes):
            if n:
                out[offs[l]:offs[l + 1]].normal_(0.0, float(std[l]) * rel, generator=gen)

    def fill_gradients(self, step: int, grads: Sequence[torch.Tensor]):
        """Write the step's gradient of every worker into the preallocated flat tensors."""
        assert len(grads) == self.num_workers
        device = grads[0].device
        P = self.num_params
        if self.config == 1:
            for i, g in enumerate(grads):
                g.normal_(0.0, 0.01, generator=self._gen(device, "g", step, i))
        elif self.config in (2, 5):
            # shared mean N(0, s_l^2) + per-worker noise N(0, (0.5 s_l)^2)
            shared = torch.empty(P, dtype=torch.float32, device=device)
            self._fill_layered_normal(shared, self._gen(device, "shared", step), 1.0)
            for i, g in enumerate(grads):
                self._fill_layered_normal(g, self._gen(device, "noise", step, i), 0.5)
                g.add_(shared)
            del shared
        elif self.config == 3:
            # Student-t with 3 degrees of freedom, Z / sqrt((Z1^2+Z2^2+Z3^2)/3), times s_l;
            # 10 % of the embedding rows exactly zero per (step, worker)
            offs = self.seg_offsets
            std = self.layer_std()
            for i, g in enumerate(grads):
                gen = self._gen(device, "t", step, i)
                for l, n in enumerate(self.sizes):
                    if not n:
                        continue
                    z = torch.randn(4, n, generator=gen, device=device, dtype=torch.float32)
                    den = (z[1:].square().sum(0) / 3.0).sqrt_()
                    g[offs[l]:offs[l + 1]] = z[0] / den * float(std[l])
                    del z, den
                if self.embedding_rows:
                    keep = torch.rand(self.embedding_rows, generator=gen, device=device) >= 0.10
                    emb = g[: self.embedding_rows * self.embedding_dim].view(self.embedding_rows, self.embedding_dim)
                    emb.mul_(keep.to(torch.float32).unsqueeze(1))
        elif self.config == 4:
            # N(0,1) times a per-4096-block factor 10^U(-6,2) (drawn once), then a fraction 1e-3 of
            # the entries set to +-1e3
            if self._block_scale is None or self._block_scale.device != device:
                nb = (P + 4095) // 4096
                u = torch.rand(nb, generator=self._gen("cpu", "block_scale"), dtype=torch.float64)
                self._block_scale = (10.0 ** (-6.0 + 8.0 * u)).to(torch.float32).to(device)
            for i, g in enumerate(grads):
                gen = self._gen(device, "adv", step, i)
                g.normal_(0.0, 1.0, generator=gen)
                nb = self._block_scale.numel()
                full = (P // 4096) * 4096
                if full:
                    g[:full].view(-1, 4096).mul_(self._block_scale[: full // 4096].unsqueeze(1))
                if full < P:
                    g[full:].mul_(self._block_scale[nb - 1])
                r = torch.rand(P, generator=gen, device=device)
                g[r < 0.5e-3] = 1e3
                g[r > 1.0 - 0.5e-3] = -1e3
                del r
        else:
            raise ValueError("unknown config %r" % self.config)


def make_workload(config: int, shrink: int = 1, seed: int = 0, misalign: bool = False) -> Workload:
    """The configuration `config` (1..5).  shrink > 1 divides the model dimensions (not the number
    of layers) for quick parity runs that keep the layer structure.  misalign: put one 1001-element
    layer in front, so that every layer of the configuration starts off a 16-byte boundary (the odd
    layer itself is aligned; everything behind it starts at flat index = 1 mod 4)."""
    if misalign:
        wl = make_workload(config, shrink=shrink, seed=seed)
        wl.sizes = [1001] + wl.sizes
        wl.name += "+odd-first-layer"
        if wl.embedding_rows:
            wl.embedding_rows = 0      # the zeroed-row pattern addresses the first segment: not used here
        return wl
    if config == 1:
        return Workload(1, "flat-1M", [max(1, (1 << 20) // shrink)], 1, 10, k_g=2, weight_quant=False,
                        weight_ef=0, seed=seed)
    if config == 2:
        sizes = resnet18_layers()
        if shrink > 1:
            sizes = [max(1, s // shrink) for s in sizes]
        return Workload(2, "resnet18", sizes, 4, 50, seed=seed)
    if config == 3:
        d, vocab, ctx = 768 // shrink, max(1, 50257 // shrink), max(1, 1024 // shrink)
        return Workload(3, "gpt2-small", gpt_layers(12, d, vocab, ctx), 8, 20, seed=seed,
                        embedding_rows=vocab, embedding_dim=d)
    if config == 4:
        return Workload(4, "adversarial-256M", [(1 << 28) // shrink], 16, 10, seed=seed)
    if config == 5:
        d, vocab, ctx = 2048 // shrink, max(1, 50257 // shrink), max(1, 2048 // shrink)
        return Workload(5, "gpt-1.3b", gpt_layers(24, d, vocab, ctx), 8, 5, seed=seed)
    raise ValueError("config must be 1..5")
