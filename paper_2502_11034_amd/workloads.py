"""Seeded synthetic inputs: parameter-tensor lists and gradient streams.

This module holds NO arithmetic of the clipping method or of the optimizers.
It only produces inputs: shapes of model-like parameter lists, initial
parameter values, and per-step gradients.  Both the GPU library's tests and the
CPU oracle's tests consume the same generated bits (a tensor is generated once,
on whatever device is asked for, and copied to the other side).

The paper trains real language models (Sec. 5.1); their gradients are not
available here, so per-tensor Gaussian gradients with a wide spread of scales,
plus injected spikes, stand in for them.  Tensor enumeration follows the
paper's own count for a dense decoder: four attention tensors, three FFN
tensors and two norm weights per layer, plus embedding, final norm and LM head
(Sec. 4.3, "Memory").
"""
from dataclasses import dataclass, field
import math

import numpy as np
import torch

MASTER_SEED = 0x5EED


@dataclass(frozen=True)
class TensorSpec:
    name: str
    shape: tuple
    kind: str  # "matrix" (N(0, 0.02^2) init), "norm" (ones), "bias" (zeros)

    @property
    def numel(self):
        n = 1
        for s in self.shape:
            n *= s
        return n


# --------------------------------------------------------------------------- lists

def gpt2_like_list(layers, d, ffn, vocab, n_pos):
    """LayerNorm + fused-QKV decoder, 12 tensors per layer."""
    specs = [TensorSpec("wte", (vocab, d), "matrix")]
    if n_pos:
        specs.append(TensorSpec("wpe", (n_pos, d), "matrix"))
    for l in range(layers):
        p = "h%d." % l
        specs += [
            TensorSpec(p + "ln1.w", (d,), "norm"), TensorSpec(p + "ln1.b", (d,), "bias"),
            TensorSpec(p + "qkv.w", (3 * d, d), "matrix"), TensorSpec(p + "qkv.b", (3 * d,), "bias"),
            TensorSpec(p + "proj.w", (d, d), "matrix"), TensorSpec(p + "proj.b", (d,), "bias"),
            TensorSpec(p + "ln2.w", (d,), "norm"), TensorSpec(p + "ln2.b", (d,), "bias"),
            TensorSpec(p + "fc.w", (ffn, d), "matrix"), TensorSpec(p + "fc.b", (ffn,), "bias"),
            TensorSpec(p + "fc_proj.w", (d, ffn), "matrix"), TensorSpec(p + "fc_proj.b", (d,), "bias"),
        ]
    specs += [TensorSpec("ln_f.w", (d,), "norm"), TensorSpec("ln_f.b", (d,), "bias")]
    return specs


def llama_like_list(layers, d, n_q_heads, n_kv_heads, ffn, vocab):
    """RMSNorm + GQA + SwiGLU decoder, 9 tensors per layer + 3."""
    head = d // n_q_heads
    kv = head * n_kv_heads
    specs = [TensorSpec("embed", (vocab, d), "matrix")]
    for l in range(layers):
        p = "l%d." % l
        specs += [
            TensorSpec(p + "attn_norm", (d,), "norm"),
            TensorSpec(p + "q", (d, d), "matrix"), TensorSpec(p + "k", (kv, d), "matrix"),
            TensorSpec(p + "v", (kv, d), "matrix"), TensorSpec(p + "o", (d, d), "matrix"),
            TensorSpec(p + "ffn_norm", (d,), "norm"),
            TensorSpec(p + "gate", (ffn, d), "matrix"), TensorSpec(p + "up", (ffn, d), "matrix"),
            TensorSpec(p + "down", (d, ffn), "matrix"),
        ]
    specs += [TensorSpec("final_norm", (d,), "norm"), TensorSpec("lm_head", (vocab, d), "matrix")]
    return specs


def tiny_transformer_list():
    """2 layers, d=128, FFN 512, vocab 1024, tied embedding: 27 tensors, 527 872 params."""
    return gpt2_like_list(2, 128, 512, 1024, 0)


def gpt2_small_list():
    """12 layers, d=768, FFN 3072, vocab 50257, 1024 positions: 148 tensors, 124 439 808 params."""
    return gpt2_like_list(12, 768, 3072, 50257, 1024)


def llama3_8b_list():
    """32 layers, d=4096, 32 q / 8 kv heads, FFN 14336, vocab 128256: 291 tensors, 8 030 261 248 params."""
    return llama_like_list(32, 4096, 32, 8, 14336, 128256)


def ragged_stress_list(n_tensors=20000, max_elems=4194304, embed_shape=(128256, 4096),
                       seed=MASTER_SEED):
    """n_tensors sizes drawn log-uniform on [1, max_elems] plus one large embedding."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0xA11CE))
    u = rng.random(n_tensors)
    sizes = np.floor(np.exp(u * math.log(max_elems))).astype(np.int64)
    sizes = np.clip(sizes, 1, max_elems)
    specs = [TensorSpec("r%d" % i, (int(s),), "matrix") for i, s in enumerate(sizes)]
    if embed_shape is not None:
        specs.append(TensorSpec("embed", tuple(embed_shape), "matrix"))
    return specs


# --------------------------------------------------------------------------- spike schedules

def forced_spike_schedule(n_tensors, steps, spike_steps, n_spiked, factor, seed=MASTER_SEED,
                          bernoulli_p=0.0, frac=None):
    """{step: (tensor_indices, factor)}.  spike_steps are forced; every other step
    additionally spikes with probability bernoulli_p (seeded)."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5B1CE))
    if frac is not None:
        n_spiked = max(1, int(round(frac * n_tensors)))
    sched = {}
    for t in range(1, steps + 1):
        draw = rng.random()
        idx = np.sort(rng.choice(n_tensors, size=min(n_spiked, n_tensors), replace=False))
        if t in spike_steps or draw < bernoulli_p:
            sched[t] = (idx.astype(np.int64), float(factor))
    return sched


# --------------------------------------------------------------------------- workload

def _mix(seed, a, b):
    """Integer-only stream id for (seed, tensor, step)."""
    seed, a, b = int(seed), int(a), int(b)
    x = (seed * 0x9E3779B97F4A7C15 + a * 0xBF58476D1CE4E5B9 + b * 0x94D049BB133111EB + 0x2545F491)
    x &= (1 << 63) - 1
    return x


@dataclass
class Workload:
    specs: list
    seed: int = MASTER_SEED
    sigma_lo: float = 1e-4
    sigma_hi: float = 1e-1
    spikes: dict = field(default_factory=dict)      # step -> (tensor idx array, factor)
    heavy_tail_frac: float = 0.0                    # fraction of elements replaced by sigma*t(nu=2)
    grad_dtype: torch.dtype = torch.float32
    bf16_copy: bool = False

    def __post_init__(self):
        rng = np.random.Generator(np.random.PCG64(self.seed))
        u = rng.random(len(self.specs))
        lo, hi = math.log(self.sigma_lo), math.log(self.sigma_hi)
        self.sigma = np.exp(lo + u * (hi - lo))
        self.numels = [s.numel for s in self.specs]

    @property
    def n_tensors(self):
        return len(self.specs)

    @property
    def total_params(self):
        return int(sum(self.numels))

    def _gen(self, device, a, b):
        g = torch.Generator(device=device)
        g.manual_seed(_mix(self.seed, a, b))
        return g

    def init_param(self, i, device):
        spec = self.specs[i]
        if spec.kind == "norm":
            return torch.ones(spec.numel, dtype=torch.float32, device=device)
        if spec.kind == "bias":
            return torch.zeros(spec.numel, dtype=torch.float32, device=device)
        t = torch.empty(spec.numel, dtype=torch.float32, device=device)
        t.normal_(0.0, 0.02, generator=self._gen(device, i, 0))
        return t

    def grad_scale(self, i, step):
        s = float(self.sigma[i])
        if step in self.spikes:
            idx, factor = self.spikes[step]
            if i in set(int(k) for k in idx):
                s *= factor
        return s

    def fill_grad(self, out, i, step):
        """Write tensor i's gradient for 1-based step into `out` (fp32 or bf16, on its device)."""
        device = out.device
        gen = self._gen(device, i, step)
        if out.dtype == torch.float32:
            buf = out
        else:
            buf = torch.empty(out.numel(), dtype=torch.float32, device=device)
        buf.normal_(0.0, self.grad_scale(i, step), generator=gen)
        if self.heavy_tail_frac > 0.0:
            sel = torch.rand(buf.numel(), generator=gen, device=device) < self.heavy_tail_frac
            k = int(sel.sum().item())
            if k:
                u = torch.rand(k, generator=gen, device=device, dtype=torch.float64)
                u = u.clamp_(1e-12, 1.0 - 1e-12)
                t2 = (2.0 * u - 1.0) / torch.sqrt(2.0 * u * (1.0 - u))   # inverse CDF of Student-t, nu=2
                buf[sel] = (float(self.sigma[i]) * t2).to(torch.float32)
        if buf is not out:
            out.copy_(buf)
        return out

    def make_grad(self, i, step, device):
        out = torch.empty(self.numels[i], dtype=self.grad_dtype, device=device)
        return self.fill_grad(out, i, step)

    def make_state(self, device, optimizer="adamw"):
        """Fresh state lists: params, exp_avg, exp_avg_sq (None for Lion), bf16 copies (or None)."""
        params = [self.init_param(i, device) for i in range(self.n_tensors)]
        exp_avg = [torch.zeros(n, dtype=torch.float32, device=device) for n in self.numels]
        exp_avg_sq = None
        if optimizer == "adamw":
            exp_avg_sq = [torch.zeros(n, dtype=torch.float32, device=device) for n in self.numels]
        copies = None
        if self.bf16_copy:
            copies = [p.to(torch.bfloat16) for p in params]
        return params, exp_avg, exp_avg_sq, copies

    def make_grads(self, step, device):
        return [self.make_grad(i, step, device) for i in range(self.n_tensors)]


def to_numpy(t):
    """Host numpy copy of a tensor; bf16 becomes its uint16 bit pattern."""
    if t.dtype == torch.bfloat16:
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16).copy()
    return t.detach().cpu().numpy().copy()


# --------------------------------------------------------------------------- the five named workloads

def config1():
    specs = tiny_transformer_list()
    spikes = forced_spike_schedule(len(specs), 20, {7, 13}, 3, 100.0)
    return Workload(specs, spikes=spikes)


def config2():
    specs = gpt2_small_list()
    spikes = forced_spike_schedule(len(specs), 10, {4}, 0, 50.0, bernoulli_p=0.01, frac=0.05)
    return Workload(specs, spikes=spikes)


def config3(specs=None, steps=5):
    specs = specs or llama3_8b_list()
    spikes = forced_spike_schedule(len(specs), steps, {3}, 0, 50.0, bernoulli_p=0.01, frac=0.05)
    return Workload(specs, spikes=spikes, bf16_copy=True)


def config4(specs=None, steps=5):
    specs = specs or llama3_8b_list()
    spikes = forced_spike_schedule(len(specs), steps, {3}, 0, 50.0, bernoulli_p=0.01, frac=0.05)
    return Workload(specs, spikes=spikes, bf16_copy=True, grad_dtype=torch.bfloat16)


def config5(specs=None):
    specs = specs or ragged_stress_list()
    return Workload(specs, heavy_tail_frac=1e-3)
