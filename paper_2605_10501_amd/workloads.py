"""Seeded synthetic workloads: shapes, length mixes and tensors.

This module only describes and generates inputs; it holds none of the
method's arithmetic and is the one module that both the tests' CPU oracle and
the HIP path are fed from.  The workloads stand in for the paper's proprietary
distillation / multimodal data and model weights (Sec. 4, experimental setup):
same shapes, same length structure, random values.

Generator: counter based.  Element i of the tensor named `tag` under `seed` is
a pure function of (seed, tag, i): a 64-bit mix of the counter gives a uniform,
two uniforms give a normal by Box-Muller.  It is written with torch integer ops
so it runs on the CPU and on the GPU.
"""
import math
import zlib
from dataclasses import dataclass, field, asdict

import torch

_M64 = (1 << 64) - 1


def _s64(c):
    c &= _M64
    return c - (1 << 64) if c >= (1 << 63) else c


_C1, _C2, _GAMMA = _s64(0xBF58476D1CE4E5B9), _s64(0x94D049BB133111EB), _s64(0x9E3779B97F4A7C15)


def _lsr(x, s):
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x):
    x = (x ^ _lsr(x, 30)) * _C1
    x = (x ^ _lsr(x, 27)) * _C2
    return x ^ _lsr(x, 31)


def _mix64_int(x):
    x &= _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def _stream_key(seed, tag):
    return _s64(_mix64_int((seed & _M64) ^ ((zlib.crc32(tag.encode()) + 1) * 0xD1342543DE82EF95)))


def _uniform_counters(key, ctr):
    """ctr: int64 tensor of counters -> float32 uniforms in (0, 1)."""
    h = _mix64(key + (ctr + 1) * _GAMMA)
    return (_lsr(h, 40).to(torch.float32) + 0.5) * (1.0 / (1 << 24))


def uniform(seed, tag, n, device="cpu"):
    ctr = torch.arange(n, dtype=torch.int64, device=device)
    return _uniform_counters(_stream_key(seed, tag), ctr)


def normal(seed, tag, shape, std=1.0, mean=0.0, dtype=torch.float32, device="cpu", chunk=1 << 24):
    """N(mean, std) tensor of `shape`, generated in fp32 and rounded to `dtype`."""
    n = int(math.prod(shape))
    out = torch.empty(n, dtype=dtype, device=device)
    key = _stream_key(seed, tag)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        i = torch.arange(s, e, dtype=torch.int64, device=device)
        u1 = _uniform_counters(key, 2 * i)
        u2 = _uniform_counters(key, 2 * i + 1)
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[s:e] = (z * std + mean).to(dtype)
    return out.reshape(shape)


def randint(seed, tag, n, lo, hi, device="cpu"):
    """n integers uniform in [lo, hi) as int32."""
    u = uniform(seed, tag, n, device).to(torch.float64)
    return (lo + torch.floor(u * (hi - lo))).clamp(lo, hi - 1).to(torch.int32)


# --------------------------------------------------------------------- shapes
@dataclass
class SectionConfig:
    arch: str = "decoder"        # "decoder": RMSNorm, RoPE, SwiGLU, causal, no bias
    dtype: str = "bf16"          # "encoder": LayerNorm, GELU, bidirectional, biases
    n_layers: int = 1
    d_model: int = 128
    n_q_heads: int = 2
    n_kv_heads: int = 2
    head_dim: int = 64
    d_ffn: int = 344
    vocab: int = 0               # 0: fed embeddings, else token ids
    norm_eps: float = 1e-6
    rope_base: float = 1e4

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def d_qkv(self):
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def d_up(self):
        return 2 * self.d_ffn if self.arch == "decoder" else self.d_ffn

    def layer_params(self):
        d, f = self.d_model, self.d_ffn
        return d * self.d_qkv + self.n_q_heads * self.head_dim * d + d * self.d_up + f * d


@dataclass
class KDConfig:
    vocab: int
    h_teacher: int
    h_student: int
    temperature: float = 1.0
    chunk: int = 8192
    dtype: str = "bf16"
    token_block: int = 0         # > 0: keep a token block's teacher logits across the two KD passes (variant)


@dataclass
class Workload:
    name: str
    dtype: str
    teacher: SectionConfig = None
    student: SectionConfig = None
    kd: KDConfig = None
    n_tokens: int = 0            # fixed token budget, 0 = sum of sampled lengths
    lengths: list = field(default_factory=list)


def _fill_budget(draws, budget):
    """Take draws in order; the draw that would overflow is truncated to the remainder."""
    out, tot = [], 0
    for v in draws:
        v = int(v)
        if tot + v >= budget:
            out.append(budget - tot)
            return out
        out.append(v)
        tot += v
    raise ValueError("not enough draws to fill the token budget")


def _lengths_c1(seed):
    return [int(v) for v in randint(seed, "c1.lengths", 4, 16, 129)]


def _lengths_lognormal(seed, budget, median=1024.0, sigma=1.0, lo=64, hi=4096, tag="c2.lengths"):
    z = normal(seed, tag, (4 * budget // lo,), std=sigma).to(torch.float64)
    ln = torch.round(torch.exp(math.log(median) + z)).clamp(lo, hi)
    return _fill_budget(ln.tolist(), budget)


def _lengths_c4(seed, n_samples=64, frac_text=0.3, lo=256, hi=4096):
    n_text = int(frac_text * n_samples)
    perm = torch.argsort(uniform(seed, "c4.shuffle", n_samples)).tolist()
    patches = randint(seed, "c4.patches", n_samples, lo, hi + 1).tolist()
    text = set(perm[:n_text])
    return [0 if i in text else int(patches[i]) for i in range(n_samples)]


def _lengths_c5(seed, budget):
    m = 4 * budget // 128
    coin = uniform(seed, "c5.coin", m)
    short = randint(seed, "c5.short", m, 128, 1025)
    long_ = randint(seed, "c5.long", m, 4096, 16385)
    draws = torch.where(coin < 0.5, short, long_).tolist()
    return _fill_budget(draws, budget)


def workload(name, seed=0):
    """The five workload configurations (c1..c5) with their sampled sequence lengths."""
    if name == "c1":
        w = Workload("c1", "fp32",
                     teacher=SectionConfig("decoder", "fp32", 2, 256, 4, 4, 64, 688, 1024),
                     student=SectionConfig("decoder", "fp32", 1, 128, 2, 2, 64, 344, 1024),
                     kd=KDConfig(1024, 256, 128, 1.0, 8192, "fp32"))
        w.lengths = _lengths_c1(seed)
    elif name == "c2":
        w = Workload("c2", "bf16",
                     teacher=SectionConfig("decoder", "bf16", 8, 2048, 16, 4, 128, 5504, 32000),
                     student=SectionConfig("decoder", "bf16", 4, 1024, 8, 2, 128, 2816, 32000),
                     kd=KDConfig(32000, 2048, 1024, 2.0, 8192), n_tokens=16384)
        w.lengths = _lengths_lognormal(seed, 16384)
    elif name == "c3":
        w = Workload("c3", "bf16", kd=KDConfig(151936, 4096, 2048, 2.0, 8192), n_tokens=8192)
        w.lengths = [8192]
    elif name == "c4":
        w = Workload("c4", "bf16",
                     student=SectionConfig("encoder", "bf16", 8, 1280, 16, 16, 80, 5120, 0))
        w.lengths = _lengths_c4(seed)
    elif name == "c5":
        w = Workload("c5", "bf16",
                     teacher=SectionConfig("decoder", "bf16", 4, 4096, 32, 8, 128, 11008, 151936),
                     student=SectionConfig("decoder", "bf16", 4, 1536, 12, 2, 128, 8960, 151936),
                     kd=KDConfig(151936, 4096, 1536, 1.0, 8192), n_tokens=32768)
        w.lengths = _lengths_c5(seed, 32768)
    else:
        raise KeyError(name)
    if not w.n_tokens:
        w.n_tokens = sum(w.lengths)
    return w


def scaled(cfg, **over):
    """Copy of a config with some fields replaced (reduced-size parity cases)."""
    d = asdict(cfg)
    d.update(over)
    return type(cfg)(**d)


# --------------------------------------------------------------------- tensors
def section_weights(cfg, seed, tag, device="cpu"):
    """Every matrix, embedding and bias ~ N(0, 0.02); norm gains 1 + N(0, 0.02)."""
    dt, enc = cfg.torch_dtype, cfg.arch == "encoder"
    d, f = cfg.d_model, cfg.d_ffn

    def mat(name, shape):
        return normal(seed, f"{tag}.{name}", shape, 0.02, 0.0, dt, device)

    def gain(name):
        return normal(seed, f"{tag}.{name}", (d,), 0.02, 1.0, dt, device)

    w = {"embedding": mat("embedding", (cfg.vocab, d)) if cfg.vocab > 0 else None, "layers": []}
    for li in range(cfg.n_layers):
        p = f"l{li}"
        lw = {"norm1_g": gain(p + ".norm1_g"), "w_qkv": mat(p + ".w_qkv", (cfg.d_qkv, d)),
              "w_o": mat(p + ".w_o", (d, cfg.n_q_heads * cfg.head_dim)),
              "norm2_g": gain(p + ".norm2_g"), "w_up": mat(p + ".w_up", (cfg.d_up, d)),
              "w_down": mat(p + ".w_down", (d, f))}
        if enc:
            lw.update({"norm1_b": mat(p + ".norm1_b", (d,)), "b_qkv": mat(p + ".b_qkv", (cfg.d_qkv,)),
                       "b_o": mat(p + ".b_o", (d,)), "norm2_b": mat(p + ".norm2_b", (d,)),
                       "b_up": mat(p + ".b_up", (cfg.d_up,)), "b_down": mat(p + ".b_down", (d,))})
        w["layers"].append(lw)
    w["final_norm_g"] = gain("final_norm_g")
    if enc:
        w["final_norm_b"] = mat("final_norm_b", (d,))
    return w


def cu_seqlens_of(lengths):
    cu = [0]
    for n in lengths:
        if n > 0:
            cu.append(cu[-1] + int(n))
    return cu


def to_f64(obj):
    """Nested dict / list of torch tensors -> same structure of float64 (or int64) ndarrays."""
    if obj is None:
        return None
    if isinstance(obj, dict):
        return {k: to_f64(v) for k, v in obj.items() if v is not None}
    if isinstance(obj, (list, tuple)):
        return [to_f64(v) for v in obj]
    if isinstance(obj, torch.Tensor):
        t = obj.detach().cpu()
        return t.to(torch.float64).numpy() if t.is_floating_point() else t.to(torch.int64).numpy()
    return obj
