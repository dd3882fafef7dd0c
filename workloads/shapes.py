"""Parameter lists (names, shapes, roles) of the models whose optimizer step is measured.

Only public architecture dimensions are used; no weights or data.  `role` decides
the synthetic initial value and the weight-decay exemption:
  "matrix": ~N(0, 0.02), weight decay applies (>= 2-D weights, embeddings)
  "gain":   exactly 1.0, no weight decay (LayerNorm / BatchNorm / RMSNorm scales)
  "bias":   exactly 0.0, no weight decay
"""
from dataclasses import dataclass
from math import prod
from typing import List, Tuple


@dataclass(frozen=True)
class ParamSpec:
    name: str
    shape: Tuple[int, ...]
    role: str

    @property
    def numel(self) -> int:
        return int(prod(self.shape))


def flat_tensor(n: int = 1 << 20) -> List[ParamSpec]:
    """One flat tensor of n parameters."""
    return [ParamSpec("flat", (n,), "matrix")]


def llama31_8b_flat() -> List[ParamSpec]:
    """The Llama-3.1-8B parameter count as ONE flat tensor: the shape a flattened (FSDP-style)
    parameter buffer of the whole model presents to the optimizer step."""
    return flat_tensor(sum(s.numel for s in llama31_8b()))


def odd_sizes() -> List[ParamSpec]:
    """Small tensors whose sizes straddle the group (32), vector and chunk boundaries."""
    sizes = [1, 2, 7, 8, 15, 16, 17, 31, 32, 33, 63, 64, 65, 255, 257, 1000, 1023, 1025,
             4095, 4097, 8191, 8193, 16385, 40000, 65537]
    out = []
    for i, n in enumerate(sizes):
        role = "matrix" if i % 3 != 2 else ("gain" if i % 2 else "bias")
        out.append(ParamSpec(f"odd{i}_{n}", (n,), role))
    return out


def gpt2_small() -> List[ParamSpec]:
    """GPT-2 124M: 12 layers, d=768, ffn=3072, vocab 50257, ctx 1024, tied head (148 tensors)."""
    d, ff, vocab, ctx, layers = 768, 3072, 50257, 1024, 12
    p = [ParamSpec("wte", (vocab, d), "matrix"), ParamSpec("wpe", (ctx, d), "matrix")]
    for i in range(layers):
        h = f"h{i}."
        p += [ParamSpec(h + "ln_1.weight", (d,), "gain"), ParamSpec(h + "ln_1.bias", (d,), "bias"),
              ParamSpec(h + "attn.c_attn.weight", (d, 3 * d), "matrix"),
              ParamSpec(h + "attn.c_attn.bias", (3 * d,), "bias"),
              ParamSpec(h + "attn.c_proj.weight", (d, d), "matrix"),
              ParamSpec(h + "attn.c_proj.bias", (d,), "bias"),
              ParamSpec(h + "ln_2.weight", (d,), "gain"), ParamSpec(h + "ln_2.bias", (d,), "bias"),
              ParamSpec(h + "mlp.c_fc.weight", (d, ff), "matrix"),
              ParamSpec(h + "mlp.c_fc.bias", (ff,), "bias"),
              ParamSpec(h + "mlp.c_proj.weight", (ff, d), "matrix"),
              ParamSpec(h + "mlp.c_proj.bias", (d,), "bias")]
    p += [ParamSpec("ln_f.weight", (d,), "gain"), ParamSpec("ln_f.bias", (d,), "bias")]
    return p


def resnet50() -> List[ParamSpec]:
    """ResNet-50 ([3,4,6,3] bottlenecks, widths 64..2048, 1000 classes; 161 tensors)."""
    p = [ParamSpec("conv1.weight", (64, 3, 7, 7), "matrix"),
         ParamSpec("bn1.weight", (64,), "gain"), ParamSpec("bn1.bias", (64,), "bias")]

    def conv_bn(prefix, cname, bname, cout, cin, k):
        return [ParamSpec(f"{prefix}{cname}.weight", (cout, cin, k, k), "matrix"),
                ParamSpec(f"{prefix}{bname}.weight", (cout,), "gain"),
                ParamSpec(f"{prefix}{bname}.bias", (cout,), "bias")]

    inplanes = 64
    for li, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3)), start=1):
        for b in range(blocks):
            pre = f"layer{li}.{b}."
            p += conv_bn(pre, "conv1", "bn1", planes, inplanes, 1)
            p += conv_bn(pre, "conv2", "bn2", planes, planes, 3)
            p += conv_bn(pre, "conv3", "bn3", planes * 4, planes, 1)
            if b == 0:
                p += conv_bn(pre, "downsample.0", "downsample.1", planes * 4, inplanes, 1)
            inplanes = planes * 4
    p += [ParamSpec("fc.weight", (1000, 2048), "matrix"), ParamSpec("fc.bias", (1000,), "bias")]
    return p


def llama31_8b(layers: int = 32) -> List[ParamSpec]:
    """Llama-3.1-8B: hidden 4096, FFN 14336 (SwiGLU), 32 q / 8 kv heads of 128, vocab 128256,
    untied embeddings (291 tensors at 32 layers).  `layers` < 32 gives a truncated list of the
    same per-layer shapes for tests that cannot hold the full model."""
    d, ff, kv, vocab = 4096, 14336, 8 * 128, 128256
    p = [ParamSpec("embed_tokens.weight", (vocab, d), "matrix")]
    for i in range(layers):
        h = f"layers.{i}."
        p += [ParamSpec(h + "input_layernorm.weight", (d,), "gain"),
              ParamSpec(h + "self_attn.q_proj.weight", (d, d), "matrix"),
              ParamSpec(h + "self_attn.k_proj.weight", (kv, d), "matrix"),
              ParamSpec(h + "self_attn.v_proj.weight", (kv, d), "matrix"),
              ParamSpec(h + "self_attn.o_proj.weight", (d, d), "matrix"),
              ParamSpec(h + "post_attention_layernorm.weight", (d,), "gain"),
              ParamSpec(h + "mlp.gate_proj.weight", (ff, d), "matrix"),
              ParamSpec(h + "mlp.up_proj.weight", (ff, d), "matrix"),
              ParamSpec(h + "mlp.down_proj.weight", (d, ff), "matrix")]
    p += [ParamSpec("norm.weight", (d,), "gain"), ParamSpec("lm_head.weight", (vocab, d), "matrix")]
    return p
