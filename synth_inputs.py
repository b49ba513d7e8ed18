"""Seeded synthetic inputs for the MTAD/MMTAD hot path: model shapes, random-init
weights and random prompts.

This module is the only code the CPU oracle and the HIP path have in common.  It
holds none of the method's arithmetic: it draws numbers, rounds weights to their
storage type and names the workload shapes.  Nothing here imports the oracle or
the HIP package.

Weight storage format (an input format, read by both sides):
  * dtype "fp32": every matrix is a float32 array.
  * dtype "bf16": every matrix is a uint16 array of bfloat16 bit patterns
    (float32 rounded to nearest-even, upper 16 bits kept).
  * norm gains are always float32.
Tensor set of one decoder (all matrices are [out_features, in_features], i.e.
each output feature's weights are contiguous):
  embed  [V, d]
  per layer l: g_attn [d], w_qkv [(H + 2*KVH)*hd, d] (query heads, then key heads,
               then value heads), w_o [d, H*hd], g_ffn [d],
               w_gu [2*f, d] (gate rows, then up rows), w_d [d, f]
  g_final [d], unembed [V, d]
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str = "bf16"          # "fp32" | "bf16"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    def with_layers(self, n_layers: int) -> "ModelShape":
        return dataclasses.replace(self, n_layers=n_layers)

    @property
    def qkv_rows(self) -> int:
        return (self.n_heads + 2 * self.n_kv_heads) * self.head_dim

    def n_params(self) -> int:
        d, f = self.d_model, self.d_ffn
        per_layer = self.qkv_rows * d + d * self.n_heads * self.head_dim + 2 * f * d + d * f + 2 * d
        return self.n_layers * per_layer + 2 * self.vocab * d + d


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    target: ModelShape
    draft: ModelShape
    seed: int
    batch: int
    prompt_len: int
    new_tokens: int
    gamma: int
    beam: int
    mode: str                     # "mtad" (verify the output beam) | "mmtad" (verify the whole beam tree)
    tau: float = 0.3

    @property
    def tree_rows(self) -> int:
        """Rows of one target pass: the root plus gamma (chain) or beam*gamma (tree) nodes."""
        return 1 + (self.gamma if self.mode == "mtad" else self.gamma * self.beam)


def _m(L, d, H, KVH, hd, f, V, dtype):
    return ModelShape(L, d, H, KVH, hd, f, V, dtype)


# The five workloads.  The draft FFN width of C1 (344) keeps the target's 2.6875 ratio.
WORKLOADS = {
    "C1": Workload("C1", _m(4, 256, 4, 4, 64, 688, 1024, "fp32"), _m(2, 128, 2, 2, 64, 344, 1024, "fp32"),
                   seed=0, batch=1, prompt_len=32, new_tokens=64, gamma=4, beam=2, mode="mtad"),
    "C2": Workload("C2", _m(12, 768, 12, 12, 64, 2048, 32000, "bf16"), _m(4, 512, 8, 8, 64, 1376, 32000, "bf16"),
                   seed=1, batch=1, prompt_len=128, new_tokens=256, gamma=4, beam=4, mode="mtad"),
    "C3": Workload("C3", _m(32, 4096, 32, 32, 128, 11008, 32000, "bf16"), _m(2, 768, 12, 12, 64, 3072, 32000, "bf16"),
                   seed=2, batch=1, prompt_len=512, new_tokens=256, gamma=4, beam=4, mode="mtad"),
    "C4": Workload("C4", _m(32, 4096, 32, 32, 128, 11008, 32000, "bf16"), _m(2, 768, 12, 12, 64, 3072, 32000, "bf16"),
                   seed=3, batch=1, prompt_len=2048, new_tokens=512, gamma=4, beam=4, mode="mmtad"),
    "C5": Workload("C5", _m(40, 5120, 40, 40, 128, 13824, 32000, "bf16"), _m(22, 2048, 32, 4, 64, 5632, 32000, "bf16"),
                   seed=4, batch=4, prompt_len=4096, new_tokens=512, gamma=5, beam=8, mode="mmtad"),
}


def reduced(w: Workload, target_layers: int, draft_layers: int | None = None, prompt_len: int | None = None,
            new_tokens: int | None = None, batch: int | None = None) -> Workload:
    """Same widths, heads, FFN and vocabulary, fewer layers / shorter run (for parity at full shape)."""
    return dataclasses.replace(
        w, name=f"{w.name}-L{target_layers}",
        target=w.target.with_layers(target_layers),
        draft=w.draft.with_layers(min(w.draft.n_layers, draft_layers if draft_layers is not None else w.draft.n_layers)),
        prompt_len=prompt_len if prompt_len is not None else w.prompt_len,
        new_tokens=new_tokens if new_tokens is not None else w.new_tokens,
        batch=batch if batch is not None else w.batch)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Storage conversion: float32 -> bfloat16 bit patterns, round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def tensor_names(shape: ModelShape):
    names = ["embed"]
    for l in range(shape.n_layers):
        names += [f"L{l}.g_attn", f"L{l}.w_qkv", f"L{l}.w_o", f"L{l}.g_ffn", f"L{l}.w_gu", f"L{l}.w_d"]
    names += ["g_final", "unembed"]
    return names


def tensor_shape(shape: ModelShape, name: str):
    d, f, V = shape.d_model, shape.d_ffn, shape.vocab
    kind = name.split(".")[-1]
    return {
        "embed": (V, d), "unembed": (V, d), "g_final": (d,), "g_attn": (d,), "g_ffn": (d,),
        "w_qkv": (shape.qkv_rows, d), "w_o": (d, shape.n_heads * shape.head_dim),
        "w_gu": (2 * f, d), "w_d": (d, f),
    }[kind]


_KIND_ID = {"embed": 1, "unembed": 2, "g_final": 3, "g_attn": 4, "w_qkv": 5, "w_o": 6, "g_ffn": 7, "w_gu": 8, "w_d": 9}
_ROLE_ID = {"target": 0, "draft": 1}


def _tensor_key(seed: int, role: str, name: str):
    layer = int(name.split(".")[0][1:]) if name.startswith("L") else 0xFFFF
    kind = _KIND_ID[name.split(".")[-1]]
    return [np.uint64(seed), np.uint64((_ROLE_ID[role] << 40) | (layer << 8) | kind)]


def make_tensor(shape: ModelShape, seed: int, role: str, name: str) -> np.ndarray:
    """One tensor: N(0, 0.02^2); the unembedding N(0, (3/sqrt(d))^2) so that logits of a
    unit-RMS hidden state have standard deviation about 3; norm gains are ones."""
    shp = tensor_shape(shape, name)
    kind = name.split(".")[-1]
    if kind.startswith("g_"):
        return np.ones(shp, dtype=np.float32)
    gen = np.random.Generator(np.random.Philox(key=_tensor_key(seed, role, name)))
    std = 3.0 / np.sqrt(shape.d_model) if kind == "unembed" else 0.02
    x = gen.standard_normal(shp, dtype=np.float32)
    x *= np.float32(std)
    return f32_to_bf16_bits(x) if shape.dtype == "bf16" else x


def make_weights(shape: ModelShape, seed: int, role: str, threads: int = 8) -> dict:
    names = tensor_names(shape)
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        arrs = list(ex.map(lambda n: make_tensor(shape, seed, role, n), names))
    return dict(zip(names, arrs))


def make_prompt(w: Workload) -> np.ndarray:
    """Uniform random token ids, int32 [batch, prompt_len]."""
    gen = np.random.Generator(np.random.Philox(key=[np.uint64(w.seed), np.uint64(0xABCD << 40)]))
    return gen.integers(0, w.target.vocab, size=(w.batch, w.prompt_len), dtype=np.int32)


def tied_pair_weights(shape: ModelShape, seed: int) -> dict:
    """Weights for the special case 'draft model == target model' (acceptance probability 1)."""
    return make_weights(shape, seed, "target")
