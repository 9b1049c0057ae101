"""Seeded synthetic workloads: logit rows shaped like those an image-token AR model emits.

This module holds *only* input generation (random draws and their arrangement on the token
grid).  It contains none of the method's arithmetic: no softmax, no interval, no accept test.
The drafted token of a row is drawn from the distribution its centre logits define by the
Gumbel-max construction (argmax of logits plus Gumbel noise), which needs no normalisation.

Both the HIP path and the CPU oracle are fed the very same bytes produced here; nothing is
regenerated independently on either side.

The five workloads are the ones the benchmark definition names (rows = images x token grid):

  1  "tiny"      1 x 16x16, V=16384, fp32, K=4;  row scale s~U(0.5,3); 60 % of rows get +8 on one
                 random token; target = draft + N(0, 0.5^2)
  2  "img256"    8 x 16x16, V=16384, fp32, K=8;  as 1, but peaked rows come in aligned 4x4 blocks
                 (each block peaked w.p. 0.6, one shared peak token per block); target sigma 0.3
  3  "img512"    16 x 32x32, V=16384, bf16, K=8; random rectangles are drawn on each image until
                 >= 70 % of its cells are covered; covered cells are peaked on the token of the
                 last rectangle that covers them; target sigma 0.5
  4  "codebook8k" 32 x 32x32, V=8192, fp32, K=16; s~LogUniform(0.25, 8), no peaks; target is an
                 exact copy of the draft row for 90 % of rows, and an independent redraw for the
                 rest (forced rejections)
  5  "vocab64k"  8 x 64x64, V=65536, bf16, K=8;  logits = -1.1*ln(1+rank) over one seeded token
                 permutation (a Zipf(1.1) profile) + N(0,1); 50 % of rows peaked; target sigma 0.4;
                 run at interval confidence 0.8, 0.9 and 0.95
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace

import numpy as np
import torch

_CHUNK = 256  # rows per independently seeded block of noise


@dataclass(frozen=True)
class Spec:
    cfg: int
    name: str
    images: int
    grid: int          # token grid is grid x grid
    vocab: int
    dtype: torch.dtype
    window: int
    sigma: float       # std of the target noise
    confidences: tuple = (0.9,)

    @property
    def rows(self) -> int:
        return self.images * self.grid * self.grid


SPECS = {
    1: Spec(1, "tiny", 1, 16, 16384, torch.float32, 4, 0.5),
    2: Spec(2, "img256", 8, 16, 16384, torch.float32, 8, 0.3),
    3: Spec(3, "img512", 16, 32, 16384, torch.bfloat16, 8, 0.5),
    4: Spec(4, "codebook8k", 32, 32, 8192, torch.float32, 16, 0.0),
    5: Spec(5, "vocab64k", 8, 64, 65536, torch.bfloat16, 8, 0.4, (0.8, 0.9, 0.95)),
}


@dataclass
class Workload:
    spec: Spec
    draft: torch.Tensor       # [N, V] centre logits of the device model
    target: torch.Tensor      # [N, V] logits of the cloud verifier
    ids: torch.Tensor         # [N] int32 drafted token ids
    u_accept: torch.Tensor    # [N] float32 in [0,1)
    u_resample: torch.Tensor  # [N] float32 in [0,1)
    peaked: np.ndarray        # [N] bool (structure only; not an input of the method)
    meta: dict = field(default_factory=dict)

    @property
    def rows(self) -> int:
        return self.draft.shape[0]

    def input_bytes(self) -> int:
        return 2 * self.draft.numel() * self.draft.element_size()


def base_seed(cfg: int) -> int:
    return 0xC1A20000 + cfg


# ---- structure on the token grid (small, host side) ---------------------------------------

def _row_structure(spec: Spec, rng: np.random.Generator):
    """Per-row scale, peak mask, peak token, redraw mask."""
    N, V, g = spec.rows, spec.vocab, spec.grid
    scale = np.ones(N, dtype=np.float64)
    peaked = np.zeros(N, dtype=bool)
    peak_id = np.zeros(N, dtype=np.int64)
    redraw = np.zeros(N, dtype=bool)
    scale2 = np.ones(N, dtype=np.float64)

    if spec.cfg in (1, 2, 3):
        scale = rng.uniform(0.5, 3.0, size=N)
    if spec.cfg == 1:
        peaked = rng.random(N) < 0.6
        peak_id = rng.integers(0, V, size=N)
    elif spec.cfg == 2:
        for img in range(spec.images):
            for by in range(g // 4):
                for bx in range(g // 4):
                    on = rng.random() < 0.6
                    tok = int(rng.integers(0, V))
                    for dy in range(4):
                        for dx in range(4):
                            r = img * g * g + (by * 4 + dy) * g + (bx * 4 + dx)
                            peaked[r] = on
                            peak_id[r] = tok
    elif spec.cfg == 3:
        for img in range(spec.images):
            cover = np.zeros((g, g), dtype=bool)
            tok = np.zeros((g, g), dtype=np.int64)
            while cover.mean() < 0.70:
                x0, y0 = int(rng.integers(0, g)), int(rng.integers(0, g))
                w, h = int(rng.integers(2, 17)), int(rng.integers(2, 17))
                cover[y0:y0 + h, x0:x0 + w] = True
                tok[y0:y0 + h, x0:x0 + w] = int(rng.integers(0, V))
            sl = slice(img * g * g, (img + 1) * g * g)
            peaked[sl] = cover.reshape(-1)
            peak_id[sl] = tok.reshape(-1)
    elif spec.cfg == 4:
        scale = np.exp(rng.uniform(np.log(0.25), np.log(8.0), size=N))
        scale2 = np.exp(rng.uniform(np.log(0.25), np.log(8.0), size=N))
        redraw = rng.random(N) < 0.10
    elif spec.cfg == 5:
        peaked = rng.random(N) < 0.5
        peak_id = rng.integers(0, V, size=N)
    return scale, peaked, peak_id, redraw, scale2


def _uniform24(n: int, gen: torch.Generator, device) -> torch.Tensor:
    bits = torch.randint(0, 1 << 24, (n,), generator=gen, device=device, dtype=torch.int32)
    return bits.to(torch.float32) * (1.0 / (1 << 24))


def make(cfg: int, device="cpu", rows: int | None = None, seed: int | None = None,
         images: int | None = None) -> Workload:
    """Generate workload ``cfg`` (1..5).  ``rows`` truncates to the first rows (whole chunks of
    noise are still drawn per 256-row block, so a truncated workload is a prefix of the full one).
    ``images`` replaces the number of images of the recipe (a larger or smaller batch of the same kind of rows:
    another seeded batch, not an extension of the named one)."""
    spec = SPECS[cfg]
    if images is not None and int(images) != spec.images:
        spec = replace(spec, images=int(images), name=f"{spec.name}x{int(images)}img")
    seed = base_seed(cfg) if seed is None else seed
    device = torch.device(device)
    N_full, V = spec.rows, spec.vocab
    N = N_full if rows is None else min(int(rows), N_full)
    rng = np.random.default_rng(seed)
    scale, peaked, peak_id, redraw, scale2 = _row_structure(spec, rng)

    offset = None
    if spec.cfg == 5:
        perm = torch.from_numpy(rng.permutation(V))
        offset = (-1.1 * torch.log1p(perm.to(torch.float64))).to(torch.float32).to(device)

    draft = torch.empty((N, V), dtype=spec.dtype, device=device)
    target = torch.empty((N, V), dtype=spec.dtype, device=device)
    ids = torch.empty(N, dtype=torch.int32, device=device)
    u_acc = torch.empty(N, dtype=torch.float32, device=device)
    u_res = torch.empty(N, dtype=torch.float32, device=device)

    for lo in range(0, N, _CHUNK):
        hi = min(lo + _CHUNK, N)
        n = hi - lo
        gen = torch.Generator(device=device)
        gen.manual_seed((seed * 1000003 + lo // _CHUNK) & 0x7FFFFFFFFFFFFFFF)
        rows_idx = torch.arange(n, device=device)
        s = torch.from_numpy(scale[lo:hi]).to(torch.float32).to(device)[:, None]
        c = torch.randn((_CHUNK, V), generator=gen, device=device, dtype=torch.float32)[:n] * s
        if offset is not None:
            c = c + offset[None, :]
        pk = torch.from_numpy(peaked[lo:hi]).to(device)
        pid = torch.from_numpy(peak_id[lo:hi]).to(device)
        c[rows_idx[pk], pid[pk]] += 8.0
        noise = torch.randn((_CHUNK, V), generator=gen, device=device, dtype=torch.float32)[:n]
        if spec.cfg == 4:
            t = c.clone()
            rd = torch.from_numpy(redraw[lo:hi]).to(device)
            s2 = torch.from_numpy(scale2[lo:hi]).to(torch.float32).to(device)[:, None]
            t[rd] = (noise * s2)[rd]
        else:
            t = c + noise * spec.sigma
        c_st = c.to(spec.dtype)
        draft[lo:hi] = c_st
        target[lo:hi] = t.to(spec.dtype)
        # drafted token ~ distribution of the stored centre logits, by Gumbel-max
        u = torch.rand((_CHUNK, V), generator=gen, device=device, dtype=torch.float32)[:n]
        u = u.clamp_(min=1e-30)
        gumbel = -torch.log((-torch.log(u)).clamp_(min=1e-30))
        ids[lo:hi] = torch.argmax(c_st.to(torch.float32) + gumbel, dim=1).to(torch.int32)
        u_acc[lo:hi] = _uniform24(_CHUNK, gen, device)[:n]
        u_res[lo:hi] = _uniform24(_CHUNK, gen, device)[:n]
        del c, t, noise, u, gumbel, c_st

    return Workload(spec, draft, target, ids, u_acc, u_res, peaked[:N].copy(),
                    {"seed": seed, "redraw": redraw[:N].copy()})


def make_radius(w: Workload, device=None, seed: int | None = None) -> torch.Tensor:
    """Raw radius tensor for the tensor-radius mode: what the radius half of an Interval Head would emit
    before its Softplus.  No trained head is available, so the stand-in is raw ~ N(mu_row, 1) with one
    mean per row, mu_row ~ U(-1, 1) (Softplus then gives radii of about 0.3 ... 2.5), in the dtype and
    shape of the workload's logits.  Seeded per 256-row block like the logits."""
    device = w.draft.device if device is None else torch.device(device)
    seed = (int(w.meta["seed"]) ^ 0x5AD105) if seed is None else seed
    N, V = w.draft.shape
    mu = np.random.default_rng(seed).uniform(-1.0, 1.0, size=w.spec.rows).astype(np.float32)
    out = torch.empty((N, V), dtype=w.draft.dtype, device=device)
    for lo in range(0, N, _CHUNK):
        hi = min(lo + _CHUNK, N)
        gen = torch.Generator(device=device)
        gen.manual_seed((seed * 1000003 + lo // _CHUNK) & 0x7FFFFFFFFFFFFFFF)
        raw = torch.randn((_CHUNK, V), generator=gen, device=device, dtype=torch.float32)[:hi - lo]
        raw += torch.from_numpy(mu[lo:hi]).to(device)[:, None]
        out[lo:hi] = raw.to(w.draft.dtype)
    return out


def take_rows(w: Workload, index) -> Workload:
    """Row subset (e.g. whole sampled windows) on the same device."""
    idx_np = np.asarray(index, dtype=np.int64)
    idx = torch.as_tensor(idx_np, device=w.draft.device)
    return Workload(w.spec, w.draft[idx].contiguous(), w.target[idx].contiguous(), w.ids[idx].contiguous(),
                    w.u_accept[idx].contiguous(), w.u_resample[idx].contiguous(), w.peaked[idx_np],
                    dict(w.meta))


def to_host(w: Workload) -> Workload:
    """Byte-identical copy in host memory (what the oracle reads)."""
    return Workload(w.spec, w.draft.cpu(), w.target.cpu(), w.ids.cpu(), w.u_accept.cpu(),
                    w.u_resample.cpu(), w.peaked, dict(w.meta))
