"""Seeded synthetic inputs shaped like multi-image prompts.

This module only *makes inputs*: interleaved text / image token layouts, clustered image
keys and values, Gaussian text keys / values and queries.  It contains none of the
compression method's arithmetic, so both the HIP path and the independent CPU oracle can be
fed from it.  The benchmark suites, models and weights the paper evaluates on are not
available offline; these inputs take their shape statistics (hundreds of image tokens per
image, many images, short text spans, interleaving as in Section 3.1) and stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np
import torch

BASE_SEED = 240618139


@dataclass(frozen=True)
class Workload:
    name: str
    config: int               # which of the five named configurations this belongs to
    H: int                    # heads
    d: int                    # head dim
    dtype: str                # "bf16" or "f32"
    spans: Tuple[int, ...]    # text span lengths; images sit between consecutive spans
    img_tokens: int           # tokens per image
    C: int                    # image-token centroids per head
    sigma: float              # std of the noise added to a centroid
    rho: float                # fraction of evictable image tokens that survive
    M: int                    # recent window
    modes: Tuple[str, ...]    # merge modes run on this workload
    prompt: int = 0           # prompt index (config 5 has four)
    total_budget: int = -1    # if >= 0: absolute budget B instead of the rho mapping
    text_prior: bool = True   # False: the method is handed an all-ones mask (Table 1's rows without text prior)

    @property
    def n_img(self) -> int:
        return len(self.spans) - 1

    @property
    def L(self) -> int:
        return sum(self.spans) + self.n_img * self.img_tokens

    def mask(self) -> np.ndarray:
        """uint8 [L], the modality mask handed to the method: 1 = image token (evictable), 0 = text token; all ones
        when the text prior is switched off."""
        m = self.layout_mask()
        return m if self.text_prior else np.ones_like(m)

    def layout_mask(self) -> np.ndarray:
        """uint8 [L]: 1 = image token, 0 = text token (text, image, text, ..., text): where the tokens really are."""
        parts = []
        for i, s in enumerate(self.spans):
            parts.append(np.zeros(s, np.uint8))
            if i < self.n_img:
                parts.append(np.ones(self.img_tokens, np.uint8))
        return np.concatenate(parts)

    def n_protected(self) -> int:
        """Positions that are text or inside the last M positions, each counted once."""
        m = self.mask()
        tail = np.arange(self.L) >= self.L - self.M
        return int(np.count_nonzero((m == 0) | tail))

    def n_evictable(self) -> int:
        return self.L - self.n_protected()

    def k_img(self) -> int:
        if self.total_budget >= 0:
            return self.total_budget - self.n_protected()
        return int(np.floor(self.rho * self.n_evictable() + 0.5))

    def budget(self) -> int:
        """Total rows kept per head: every protected position plus k_img image tokens."""
        return self.n_protected() + self.k_img()

    def seed(self, layer: int = 0) -> int:
        return BASE_SEED + 1_000_003 * self.config + 10_007 * self.prompt + layer

    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


def generate(w: Workload, layer: int = 0, heads: Sequence[int] | None = None):
    """Returns (q, k, v, mask): CPU torch tensors [H', L, d] in the workload's dtype and a
    uint8 [L] mask.  ``heads`` restricts generation to a subset of heads; every head draws
    from its own stream so a subset equals the matching slice of the full tensors."""
    L, d = w.L, w.d
    mask = w.mask()
    img = w.layout_mask() == 1
    n_image_tok = int(img.sum())
    # one cluster id per image token, shared by heads and by K / V
    cluster = np.random.default_rng([w.seed(layer), 0xC1]).integers(0, w.C, size=n_image_tok)
    hs = list(range(w.H)) if heads is None else list(heads)
    q = np.empty((len(hs), L, d), np.float32)
    k = np.empty((len(hs), L, d), np.float32)
    v = np.empty((len(hs), L, d), np.float32)
    for n, h in enumerate(hs):
        rng = np.random.default_rng([w.seed(layer), 0xA0, h])
        q[n] = rng.standard_normal((L, d), dtype=np.float32)
        k[n] = rng.standard_normal((L, d), dtype=np.float32)
        v[n] = rng.standard_normal((L, d), dtype=np.float32)
        ck = rng.standard_normal((w.C, d), dtype=np.float32)
        cv = rng.standard_normal((w.C, d), dtype=np.float32)
        k[n][img] = ck[cluster] + np.float32(w.sigma) * k[n][img]
        v[n][img] = cv[cluster] + np.float32(w.sigma) * v[n][img]
    dt = w.torch_dtype()
    to = lambda a: torch.from_numpy(a).to(dt)
    return to(q), to(k), to(v), torch.from_numpy(mask)


def generate_on_device(w: Workload, layer: int = 0, device="cuda:0"):
    """Same recipe as ``generate`` but drawn with a seeded torch generator on the GPU (different values, same
    distribution): for timing many layers without minutes of host-side random number generation.  Not used
    for parity (the oracle is fed from ``generate``)."""
    g = torch.Generator(device=device)
    g.manual_seed(w.seed(layer))
    L, d, H = w.L, w.d, w.H
    mask = torch.from_numpy(w.mask()).to(device)
    img = torch.from_numpy(w.layout_mask()).to(device) == 1
    n_image_tok = int(img.sum())
    cluster = torch.randint(0, w.C, (n_image_tok,), generator=g, device=device)
    q = torch.randn((H, L, d), generator=g, device=device)
    k = torch.randn((H, L, d), generator=g, device=device)
    v = torch.randn((H, L, d), generator=g, device=device)
    ck = torch.randn((H, w.C, d), generator=g, device=device)
    cv = torch.randn((H, w.C, d), generator=g, device=device)
    k[:, img] = ck[:, cluster] + w.sigma * k[:, img]
    v[:, img] = cv[:, cluster] + w.sigma * v[:, img]
    dt = w.torch_dtype()
    return q.to(dt), k.to(dt), v.to(dt), mask


_SP4 = (64, 16, 32, 48, 128, 24, 40, 56, 80, 16, 96, 32, 64, 20, 112, 28, 36, 44, 72, 52, 64)

TINY = Workload("tiny", 1, 2, 64, "f32", (32, 32, 64), 64, 8, 0.1, 0.20, 16,
                ("averaged", "pivotal", "weighted", "none"))
LLAVA7B = Workload("llava7b_4img", 2, 32, 128, "bf16", (96, 64, 160, 128, 144), 576, 64, 0.2, 0.20, 32,
                   ("averaged", "pivotal", "weighted"))


def llava13b(rho: float) -> Workload:
    return Workload(f"llava13b_8img_rho{int(round(rho * 100))}", 3, 40, 128, "bf16",
                    (128, 32, 256, 96, 192, 64, 224, 160, 144), 576, 64, 0.2, rho, 32, ("weighted",))


LONG = Workload("long_20img", 4, 32, 128, "bf16", _SP4, 576, 64, 0.2, 0.10, 64, ("pivotal",))
# the same prompt with the paper-style total budget round(0.1 * L)
LONG_TOTAL = Workload("long_20img_total10", 4, 32, 128, "bf16", _SP4, 576, 64, 0.2, 0.10, 64, ("pivotal",),
                      total_budget=int(np.floor(0.1 * (sum(_SP4) + 20 * 576) + 0.5)))

# the same prompt without the text prior: the method sees an all-ones mask, so only the window is protected and
# text tokens compete with image tokens by score (10 % of everything before the window survives)
LONG_NOPRIOR = Workload("long_20img_noprior", 4, 32, 128, "bf16", _SP4, 576, 64, 0.2, 0.10, 64, ("pivotal",),
                        text_prior=False)

STACK_LAYERS = 32


def stack_prompts() -> List[Workload]:
    """Config 5: four ragged prompts (4K, 6K, 9K, 12K tokens); each is compressed for 32 layers."""
    shapes = [((96,) * 6 + (64,), 6), ((96,) * 10, 9), ((76,) * 14 + (88,), 14), ((36,) * 20 + (48,), 20)]
    out = []
    for p, (spans, n_img) in enumerate(shapes):
        assert len(spans) == n_img + 1
        out.append(Workload(f"stack_p{p}", 5, 32, 128, "bf16", tuple(spans), 576, 64, 0.2, 0.20, 32,
                            ("weighted",), prompt=p))
    return out
