"""Seeded synthetic checkpoints (inputs only; none of the codec's arithmetic lives here).

The paper's measurements use trained Megatron GPT checkpoints (Evaluation, "Settings");
those are not available, so every test and benchmark input is generated here from a seed.
The tensor lists follow the public architectures of the named models.  Both the CPU oracle's
tests and the HIP path's tests draw their inputs from this module and from nowhere else.

Two generators:

* ``make_tensor_np``  - numpy, bit-reproducible on any machine; used for the tiny config and
  for every stored golden value.
* ``make_tensor_torch`` - the same recipes written with torch ops so that the multi-billion
  element configs can be produced directly in device memory.  Its random stream differs from
  numpy's; only its distribution and structure are the same.

bf16 values are handled as raw ``uint16`` bit patterns (numpy has no bf16); conversion from
fp32 is round-to-nearest-even.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Iterator, List, Optional, Tuple

import numpy as np

SEED_BASE = 20251112

Shape = Tuple[int, ...]


# ----------------------------------------------------------------------------------------------
# tensor lists
# ----------------------------------------------------------------------------------------------
def _gpt_list(layers: int, d: int, ffn: int, vocab: int, positions: int) -> List[Tuple[str, Shape]]:
    out: List[Tuple[str, Shape]] = [("tok_emb", (vocab, d)), ("pos_emb", (positions, d))]
    for i in range(layers):
        p = f"h{i}."
        out += [
            (p + "ln1_g", (d,)), (p + "ln1_b", (d,)),
            (p + "qkv_w", (3 * d, d)), (p + "qkv_b", (3 * d,)),
            (p + "o_w", (d, d)), (p + "o_b", (d,)),
            (p + "ln2_g", (d,)), (p + "ln2_b", (d,)),
            (p + "fc1_w", (ffn, d)), (p + "fc1_b", (ffn,)),
            (p + "fc2_w", (d, ffn)), (p + "fc2_b", (d,)),
        ]
    out += [("lnf_g", (d,)), ("lnf_b", (d,))]
    return out


def _llama_list(layers: int, d: int, ffn: int, vocab: int, tp: int = 1, kv_heads_frac: float = 1.0
                ) -> List[Tuple[str, Shape]]:
    """Llama-style list.  ``tp`` > 1 gives one rank's tensor-parallel slice (column-parallel
    q/k/v/gate/up and vocab, row-parallel o/down, replicated norms)."""
    kv = int(round(d * kv_heads_frac))
    out: List[Tuple[str, Shape]] = [("embed", (vocab // tp, d)), ("lm_head", (vocab // tp, d))]
    for i in range(layers):
        p = f"l{i}."
        out += [
            (p + "q", (d // tp, d)), (p + "k", (kv // tp, d)), (p + "v", (kv // tp, d)),
            (p + "o", (d, d // tp)),
            (p + "gate", (ffn // tp, d)), (p + "up", (ffn // tp, d)), (p + "down", (d, ffn // tp)),
            (p + "norm1", (d,)), (p + "norm2", (d,)),
        ]
    out += [("norm_f", (d,))]
    return out


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    recipe: str            # "bernoulli" | "adam" | "runs"
    p: float               # change probability (bernoulli / runs); ignored for "adam"
    run: int               # run length for "runs"
    tensors: Tuple[Tuple[str, Shape], ...]

    @property
    def n_params(self) -> int:
        return sum(math.prod(s) for _, s in self.tensors)


def config(index: int, p: Optional[float] = None) -> Config:
    """The five workloads.  ``p`` overrides the default change fraction (config 1 sweeps it)."""
    if index == 0:
        c = Config(0, "tiny-gpt-2l-d256", "bernoulli", 0.06, 0, tuple(_gpt_list(2, 256, 1024, 8192, 512)))
    elif index == 1:
        c = Config(1, "gpt2-xl", "bernoulli", 0.06, 0, tuple(_gpt_list(48, 1600, 6400, 50257, 1024)))
    elif index == 2:
        c = Config(2, "llama2-7b", "adam", 0.0, 0, tuple(_llama_list(32, 4096, 11008, 32000)))
    elif index == 3:
        c = Config(3, "llama2-13b", "runs", 0.06, 4096, tuple(_llama_list(40, 5120, 13824, 32000)))
    elif index == 4:
        c = Config(4, "llama2-70b-tp8-slice", "bernoulli", 0.06, 0,
                   tuple(_llama_list(80, 8192, 28672, 32000, tp=8, kv_heads_frac=8 / 64)))
    else:
        raise ValueError(f"no config {index}")
    if p is not None:
        c = Config(c.index, c.name, c.recipe, float(p), c.run, c.tensors)
    return c


def seed_for(cfg_index: int, tensor_index: int) -> int:
    return SEED_BASE + 100000 * cfg_index + tensor_index


# ----------------------------------------------------------------------------------------------
# numpy generator
# ----------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


ADAM = dict(lr=1e-5, beta1=0.9, beta2=0.999, eps=1e-8, steps=100, grad_std=1e-3)


def make_tensor_np(cfg: Config, t: int, n_limit: Optional[int] = None, adam_steps: Optional[int] = None
                   ) -> Dict[str, np.ndarray]:
    """One tensor of ``cfg`` as flat numpy arrays.

    Returns ``base``/``cur`` (uint16 bf16 patterns), ``master``/``m``/``v`` (fp32) and
    ``n_changed`` (the generator's own count of elements whose pattern differs).
    ``n_limit`` truncates the flat tensor (for quick tests on big shapes).
    """
    _, shape = cfg.tensors[t]
    n = math.prod(shape)
    if n_limit is not None:
        n = min(n, n_limit)
    rng = np.random.default_rng(seed_for(cfg.index, t))
    w = (rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)).astype(np.float32)
    base = f32_to_bf16_bits(w)
    if cfg.recipe == "adam":
        steps = ADAM["steps"] if adam_steps is None else adam_steps
        master = w.copy()
        m = np.zeros(n, np.float32)
        v = np.zeros(n, np.float32)
        b1, b2 = np.float32(ADAM["beta1"]), np.float32(ADAM["beta2"])
        for s in range(1, steps + 1):
            g = rng.standard_normal(n, dtype=np.float32) * np.float32(ADAM["grad_std"])
            m = b1 * m + (np.float32(1) - b1) * g
            v = b2 * v + (np.float32(1) - b2) * g * g
            mhat = m / np.float32(1 - ADAM["beta1"] ** s)
            vhat = v / np.float32(1 - ADAM["beta2"] ** s)
            master = (master - np.float32(ADAM["lr"]) * mhat / (np.sqrt(vhat) + np.float32(ADAM["eps"]))
                      ).astype(np.float32)
        cur = f32_to_bf16_bits(master)
    else:
        if cfg.recipe == "bernoulli":
            sel = rng.random(n) < cfg.p
        elif cfg.recipe == "runs":
            nruns = (n + cfg.run - 1) // cfg.run
            sel = np.repeat(rng.random(nruns) < cfg.p, cfg.run)[:n]
        else:
            raise ValueError(cfg.recipe)
        master = w.copy()
        pert = (w + rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)).astype(np.float32)
        master[sel] = pert[sel]
        cur = base.copy()
        new = f32_to_bf16_bits(master)
        same = sel & (new == base)
        new[same] ^= np.uint16(1)          # a replaced value that rounds back: flip the mantissa LSB
        cur[sel] = new[sel]
        m = (rng.standard_normal(n, dtype=np.float32) * np.float32(1e-4)).astype(np.float32)
        ln = np.exp(rng.standard_normal(n, dtype=np.float32)).astype(np.float32)
        v = (m * m * ln).astype(np.float32)
    return dict(base=base, cur=cur, master=master.astype(np.float32), m=m, v=v,
                n_changed=np.int64(np.count_nonzero(base != cur)))


# ----------------------------------------------------------------------------------------------
# torch generator (CPU or device)
# ----------------------------------------------------------------------------------------------
def make_tensor_torch(cfg: Config, t: int, device, n_limit: Optional[int] = None,
                      adam_steps: Optional[int] = None, want: Tuple[str, ...] = ("base", "cur", "master", "m", "v")):
    """Same recipes as ``make_tensor_np`` with torch ops on ``device``.

    ``base``/``cur`` are returned as torch.bfloat16; ``master``/``m``/``v`` as float32.
    """
    import torch

    _, shape = cfg.tensors[t]
    n = math.prod(shape)
    if n_limit is not None:
        n = min(n, n_limit)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed_for(cfg.index, t))
    w = torch.randn(n, device=device, dtype=torch.float32, generator=gen).mul_(0.02)
    base = w.to(torch.bfloat16)
    out = {}
    if cfg.recipe == "adam":
        steps = ADAM["steps"] if adam_steps is None else adam_steps
        master = w
        m = torch.zeros_like(w)
        v = torch.zeros_like(w)
        g = torch.empty_like(w)
        den = torch.empty_like(w)
        b1, b2 = ADAM["beta1"], ADAM["beta2"]
        for s in range(1, steps + 1):
            g.normal_(0.0, ADAM["grad_std"], generator=gen)
            m.lerp_(g, 1.0 - b1)
            v.mul_(b2).addcmul_(g, g, value=1.0 - b2)
            torch.sqrt(v, out=den)
            den.div_(math.sqrt(1.0 - b2 ** s)).add_(ADAM["eps"])
            master.addcdiv_(m, den, value=-ADAM["lr"] / (1.0 - b1 ** s))
        del g, den
        cur = master.to(torch.bfloat16)
    else:
        if cfg.recipe == "bernoulli":
            sel = torch.rand(n, device=device, generator=gen) < cfg.p
        elif cfg.recipe == "runs":
            nruns = (n + cfg.run - 1) // cfg.run
            sel = (torch.rand(nruns, device=device, generator=gen) < cfg.p).repeat_interleave(cfg.run)[:n]
        else:
            raise ValueError(cfg.recipe)
        pert = torch.randn(n, device=device, dtype=torch.float32, generator=gen).mul_(1e-3).add_(w)
        master = torch.where(sel, pert, w)
        del pert
        new = master.to(torch.bfloat16).view(torch.int16)
        b16 = base.view(torch.int16)
        new = torch.where(sel & (new == b16), new ^ 1, new)
        cur = torch.where(sel, new, b16).view(torch.bfloat16)
        del new, sel
        if "m" in want or "v" in want:
            m = torch.randn(n, device=device, dtype=torch.float32, generator=gen).mul_(1e-4)
            v = torch.randn(n, device=device, dtype=torch.float32, generator=gen).exp_().mul_(m).mul_(m)
        else:
            m = v = None
    out["base"], out["cur"], out["master"], out["m"], out["v"] = base, cur, master, m, v
    return {k: out[k] for k in want}


def make_checkpoint_torch(cfg: Config, device, tensors=None, adam_steps: Optional[int] = None,
                          want: Tuple[str, ...] = ("base", "cur", "master", "m", "v"), on_step=None):
    """The tensors of ``cfg`` (all of them, or the listed indices) as a list of dicts like ``make_tensor_torch``'s.

    The Bernoulli and runs recipes go tensor by tensor.  The Adam recipe simulates the whole list at once in flat
    buffers - the recipe is element-wise, so per element nothing changes; the checkpoint then has one random
    stream (seeded like its first tensor) instead of one per tensor - and hands out views: a few hundred large
    kernel launches instead of a few hundred thousand small ones.  Every tensor starts at a multiple of 64
    elements of the flat buffer, so views keep the alignment a fresh allocation would have.  ``on_step(s, steps)``
    is called every tenth simulated step (progress for the caller).
    """
    import torch

    idx = list(range(len(cfg.tensors))) if tensors is None else list(tensors)
    if cfg.recipe != "adam":
        return [make_tensor_torch(cfg, t, device, adam_steps=adam_steps, want=want) for t in idx]
    sizes = [math.prod(cfg.tensors[t][1]) for t in idx]
    starts, total = [], 0
    for n in sizes:
        starts.append(total)
        total += (n + 63) // 64 * 64
    gen = torch.Generator(device=device)
    gen.manual_seed(seed_for(cfg.index, idx[0] if idx else 0))
    steps = ADAM["steps"] if adam_steps is None else adam_steps
    master = torch.randn(total, device=device, dtype=torch.float32, generator=gen).mul_(0.02)
    base = master.to(torch.bfloat16)
    m = torch.zeros_like(master)
    v = torch.zeros_like(master)
    g = torch.empty_like(master)
    den = torch.empty_like(master)
    b1, b2 = ADAM["beta1"], ADAM["beta2"]
    for s in range(1, steps + 1):
        g.normal_(0.0, ADAM["grad_std"], generator=gen)
        m.lerp_(g, 1.0 - b1)
        v.mul_(b2).addcmul_(g, g, value=1.0 - b2)
        torch.sqrt(v, out=den)
        den.div_(math.sqrt(1.0 - b2 ** s)).add_(ADAM["eps"])
        master.addcdiv_(m, den, value=-ADAM["lr"] / (1.0 - b1 ** s))
        if on_step is not None and s % 10 == 0:
            on_step(s, steps)
    del g, den
    cur = master.to(torch.bfloat16)
    flat = dict(base=base, cur=cur, master=master, m=m, v=v)
    return [{k: flat[k][a:a + n] for k in want} for a, n in zip(starts, sizes)]


def iter_tensors(cfg: Config) -> Iterator[Tuple[int, str, int]]:
    for t, (name, shape) in enumerate(cfg.tensors):
        yield t, name, math.prod(shape)


def qmap_table(kind: str = "linear") -> np.ndarray:
    """A 256-entry map Q (fp32, non-decreasing, Q[0] = 0, Q[255] = 1) to pass to the quantiser's table variant:
    an input like any tensor, none of the codec's arithmetic.

    * ``linear``   j/255: the levels the plain entry points use.
    * ``square``   (j/255)^2: levels dense near the cluster minimum.
    * ``normal``   levels at equal steps of probability of a normal distribution cut off at +-2.5 sigma, rescaled
      to [0, 1]: dense in the middle of the range.
    * ``steps``    a coarse staircase with repeated entries (64 distinct levels, each four times).
    """
    j = np.arange(256, dtype=np.float64)
    if kind == "linear":
        q = j / 255.0
    elif kind == "square":
        q = (j / 255.0) ** 2
    elif kind == "normal":
        cdf = lambda z: 0.5 * (1.0 + math.erf(z / math.sqrt(2.0)))
        lo, hi = cdf(-2.5), cdf(2.5)
        q = np.empty(256)
        for i in range(256):
            p = lo + (hi - lo) * i / 255.0
            a, b = -2.5, 2.5
            for _ in range(80):
                mid = 0.5 * (a + b)
                if cdf(mid) < p:
                    a = mid
                else:
                    b = mid
            q[i] = (0.5 * (a + b) + 2.5) / 5.0
        q[0], q[255] = 0.0, 1.0
    elif kind == "steps":
        q = np.floor(j / 4.0) / 63.0
    else:
        raise ValueError(kind)
    return q.astype(np.float32)
