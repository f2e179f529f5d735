"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path.

This module only *draws numbers*: model shapes, N(0, 0.02) weights, uniform
prompts, uniforms on the 2^-24 grid, router matrices and synthetic KV / draft
distributions.  It contains none of the method's arithmetic (no forward pass,
no softmax-over-logits acceptance, no RoPE table), so that the oracle and the
kernels share inputs and nothing else.

Stand-in statement: the paper evaluates on natural-language prompt sets with
trained LLaMA-2-13B / LLaMA-68M weights (Section 3.1).  Neither is available
here; uniform random token ids and random weights of the same *shapes* stand in.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional

import numpy as np

FP32 = 0
BF16 = 1


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """Llama-style decoder shape (Section 3.1 names LLaMA for target and draft)."""

    name: str
    n_layers: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: int = BF16
    rope_base: float = 10000.0
    rms_eps: float = 1e-5

    def n_streamed_params(self) -> int:
        """Linear-layer + LM-head parameters read once per forward."""
        d, f = self.d_model, self.d_ffn
        return self.n_layers * (4 * d * d + 3 * d * f) + self.vocab * d

    def kv_bytes_per_token(self) -> int:
        esz = 4 if self.dtype == FP32 else 2
        return 2 * self.n_layers * self.n_heads * self.head_dim * esz


SHAPES: Dict[str, ModelShape] = {
    # config 1: tiny fp32 pair
    "tiny_target": ModelShape("tiny_target", 2, 256, 4, 64, 688, 1024, FP32),
    "tiny_draft": ModelShape("tiny_draft", 1, 128, 2, 64, 344, 1024, FP32),
    # bf16 clones of the tiny pair (fast full-trajectory bf16 parity)
    "tiny_target_bf16": ModelShape("tiny_target_bf16", 2, 256, 4, 64, 688, 1024, BF16),
    "tiny_draft_bf16": ModelShape("tiny_draft_bf16", 1, 128, 2, 64, 344, 1024, BF16),
    # small bf16 pair whose dimensions satisfy the MFMA kernels' alignment (head_dim 128 and 64)
    "small_target_bf16": ModelShape("small_target_bf16", 2, 256, 2, 128, 768, 2048, BF16),
    "small_draft_bf16": ModelShape("small_draft_bf16", 1, 128, 2, 64, 384, 2048, BF16),
    # config 2/3/5 target, config 4 target
    "t7b": ModelShape("t7b", 32, 4096, 32, 128, 11008, 32000, BF16),
    "t13b": ModelShape("t13b", 40, 5120, 40, 128, 13824, 32000, BF16),
    # heterogeneous drafts of config 3 (A is also config 2's 68M-shape draft)
    "draft_a": ModelShape("draft_a", 2, 768, 12, 64, 3072, 32000, BF16),
    "draft_b": ModelShape("draft_b", 4, 1024, 16, 64, 4096, 32000, BF16),
    "draft_c": ModelShape("draft_c", 6, 1024, 16, 64, 4096, 32000, BF16),
    "draft_d": ModelShape("draft_d", 2, 2048, 32, 64, 8192, 32000, BF16),
}


def with_layers(shape: ModelShape, n_layers: int) -> ModelShape:
    """Same widths, reduced depth (for parity runs the oracle can finish)."""
    return dataclasses.replace(shape, n_layers=n_layers, name=f"{shape.name}_L{n_layers}")


def _rng(seed: int, *stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), *map(int, stream)])))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_tensor(seed: int, tid: int, shape, std: float, dtype: int, scale: float = 1.0) -> np.ndarray:
    g = _rng(seed, tid)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if dtype == FP32 else np.uint16)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        blk = g.standard_normal(e - s, dtype=np.float32)
        blk *= np.float32(std * scale)
        out[s:e] = blk if dtype == FP32 else f32_to_bf16_bits(blk)
    return out.reshape(shape)


def make_weights(shape: ModelShape, seed: int, lm_head_scale: float = 1.0, threads: int = 8) -> Dict[str, object]:
    """Random weights, N(0, 0.02), row-major [out][in].

    Matrices are float32 arrays (fp32 shapes) or uint16 bf16 bit patterns (bf16
    shapes).  RMSNorm gains are float32 in both cases, drawn as 1 + N(0, 0.02) so
    that the gain multiply is exercised.  `lm_head_scale` multiplies the LM head
    after sampling (config 1 uses 20 to make the distributions peaked).
    """
    d, f, v, L = shape.d_model, shape.d_ffn, shape.vocab, shape.n_layers
    hd_all = shape.n_heads * shape.head_dim
    jobs = [("embed", 1, (v, d), 1.0), ("lm_head", 2, (v, d), lm_head_scale)]
    per_layer = [("wq", (hd_all, d)), ("wk", (hd_all, d)), ("wv", (hd_all, d)), ("wo", (d, hd_all)),
                 ("wgate", (f, d)), ("wup", (f, d)), ("wdown", (d, f))]
    for l in range(L):
        for j, (nm, shp) in enumerate(per_layer):
            jobs.append((f"{nm}.{l}", 100 + 16 * l + j, shp, 1.0))

    def run(job):
        nm, tid, shp, sc = job
        return nm, _normal_tensor(seed, tid, shp, 0.02, shape.dtype, sc)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = dict(ex.map(run, jobs))
    w: Dict[str, object] = {"embed": res["embed"], "lm_head": res["lm_head"]}
    for nm, _ in per_layer:
        w[nm] = [res[f"{nm}.{l}"] for l in range(L)]

    def gain(tid):
        return (1.0 + 0.02 * _rng(seed, tid).standard_normal(d)).astype(np.float32)

    w["final_norm"] = gain(3)
    w["norm_attn"] = [gain(100 + 16 * l + 8) for l in range(L)]
    w["norm_ffn"] = [gain(100 + 16 * l + 9) for l in range(L)]
    return w


LORA_PROJ = ("q", "k", "v", "o")


def make_lora(shape: ModelShape, seed: int, n_adapters: int, rank: int, std_a: float = 0.02,
              std_b: float = 0.02) -> Dict[str, object]:
    """Random low-rank adapters on the attention projections (Section 2.3: the heterogeneous drafts are
    LoRA fine-tunes of one base model): per layer and projection P in q, k, v, o
    "a_P": [n_adapters][rank][in] and "b_P": [n_adapters][out][rank], in the model's dtype
    (float32 arrays or bf16 bit patterns).  Both factors are random - a trained adapter has B != 0."""
    d, hd_all = shape.d_model, shape.n_heads * shape.head_dim
    dims = {"q": (hd_all, d), "k": (hd_all, d), "v": (hd_all, d), "o": (d, hd_all)}
    w: Dict[str, object] = {"n_adapters": n_adapters, "rank": rank}
    for j, pnm in enumerate(LORA_PROJ):
        n_out, n_in = dims[pnm]
        w["a_" + pnm] = [_normal_tensor(seed, 5000 + 16 * l + 2 * j, (n_adapters, rank, n_in), std_a, shape.dtype, 1.0)
                         for l in range(shape.n_layers)]
        w["b_" + pnm] = [_normal_tensor(seed, 5001 + 16 * l + 2 * j, (n_adapters, n_out, rank), std_b, shape.dtype, 1.0)
                         for l in range(shape.n_layers)]
    return w


def perturbed_copy(weights: Dict[str, object], shape: ModelShape, seed: int, rel: float) -> Dict[str, object]:
    """A draft that is the same model with every matrix perturbed by rel * N(0, 0.02).

    Random independent drafts almost never agree with the target under greedy
    decoding; a perturbed copy gives acceptance rates strictly between 0 and 1.
    """
    out: Dict[str, object] = {}
    tid = [1000]

    def pert(a: np.ndarray) -> np.ndarray:
        tid[0] += 1
        g = _rng(seed, tid[0])
        base = a if shape.dtype == FP32 else bf16_bits_to_f32(a)
        noisy = base + np.float32(rel * 0.02) * g.standard_normal(base.shape, dtype=np.float32)
        return noisy.astype(np.float32) if shape.dtype == FP32 else f32_to_bf16_bits(noisy)

    for k, v in weights.items():
        if k in ("final_norm", "norm_attn", "norm_ffn"):
            out[k] = v
        elif isinstance(v, list):
            out[k] = [pert(a) for a in v]
        else:
            out[k] = pert(v)
    return out


def make_prompt(seed: int, seq: int, length: int, vocab: int) -> np.ndarray:
    return _rng(seed, 7, seq).integers(0, vocab, size=length, dtype=np.int32)


def make_prompt_lengths(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """Lengths uniform in [lo, hi] inclusive."""
    return _rng(seed, 8).integers(lo, hi + 1, size=n, dtype=np.int32)


DRAFT_STREAM = 11
VERIFY_STREAM = 12


def make_uniforms(seed: int, stream: int, seq: int, step: int, n: int) -> np.ndarray:
    """n uniforms in [0,1) on the 2^-24 grid (exact in fp32), indexed by
    (seed, stream, sequence, step) so that batching or grouping never changes them."""
    k = _rng(seed, stream, seq, step).integers(0, 1 << 24, size=n, dtype=np.int64)
    return (k.astype(np.float64) * 2.0 ** -24).astype(np.float32)


def make_router(seed: int, n_drafts: int = 4, emb_dim: int = 256):
    """Random linear prompt classifier: W ~ N(0,1) [n_drafts][emb], b ~ N(0,1)."""
    g = _rng(seed, 20)
    return (g.standard_normal((n_drafts, emb_dim)).astype(np.float32),
            g.standard_normal(n_drafts).astype(np.float32))


def make_prompt_embeddings(seed: int, n: int, emb_dim: int = 256) -> np.ndarray:
    return _rng(seed, 21).standard_normal((n, emb_dim)).astype(np.float32)


def make_kv_rows(seed: int, layer: int, seq: int, length: int, n_heads: int, head_dim: int, dtype: int):
    """Synthetic cache contents for long-context cases: K, V ~ N(0,1), laid out
    [length][n_heads][head_dim]; fp32 arrays or bf16 bit patterns."""
    g = _rng(seed, 30, layer, seq)
    k = g.standard_normal((length, n_heads, head_dim), dtype=np.float32)
    v = g.standard_normal((length, n_heads, head_dim), dtype=np.float32)
    if dtype == BF16:
        return f32_to_bf16_bits(k), f32_to_bf16_bits(v)
    return k, v


def make_logit_noise(seed: int, seq: int, pos: int, vocab: int) -> np.ndarray:
    """N(0,1) noise row used to build synthetic draft logits (verify stress case)."""
    return _rng(seed, 40, seq, pos).standard_normal(vocab, dtype=np.float32)


@dataclasses.dataclass(frozen=True)
class ClassifierShape:
    """Prompt classifier (Sections 2.4, 3.3.3): embedding, one selective state-space layer,
    average pooling, a fully connected layer.  The paper gives no widths; the defaults put the
    model near the size Table 2 reports with a 30522-entry word-piece vocabulary."""

    name: str = "classifier"
    vocab: int = 30522
    d_model: int = 96
    d_inner: int = 192
    d_state: int = 16
    dt_rank: int = 6
    d_conv: int = 4
    n_classes: int = 4


CLASSIFIER_TINY = ClassifierShape("classifier_tiny", vocab=97, d_model=24, d_inner=64, d_state=5, dt_rank=3,
                                  d_conv=3, n_classes=3)


def make_classifier(shape: ClassifierShape, seed: int) -> Dict[str, np.ndarray]:
    """Random fp32 classifier weights, each matrix stored [in features][out features] except
    w_fc, which is [n_classes][d_model].  Step sizes start between about 1e-3 and 0.1 and the
    state matrix is negative, as such layers are usually initialised."""
    g = _rng(seed, 50)
    s = shape
    n = lambda *dims, std=1.0: (g.standard_normal(dims) * std).astype(np.float32)
    return {
        "emb": n(s.vocab, s.d_model),
        "w_in": n(s.d_model, 2 * s.d_inner, std=s.d_model ** -0.5),
        "conv_w": g.uniform(-0.5, 0.5, (s.d_inner, s.d_conv)).astype(np.float32),
        "conv_b": n(s.d_inner, std=0.1),
        "w_x": n(s.d_inner, s.dt_rank + 2 * s.d_state, std=s.d_inner ** -0.5),
        "w_dt": n(s.dt_rank, s.d_inner, std=s.dt_rank ** -0.5),
        "b_dt": g.uniform(-6.0, -2.0, s.d_inner).astype(np.float32),
        "a_log": g.uniform(0.0, np.log(s.d_state), (s.d_inner, s.d_state)).astype(np.float32),
        "d": (1.0 + 0.1 * g.standard_normal(s.d_inner)).astype(np.float32),
        "w_out": n(s.d_inner, s.d_model, std=s.d_inner ** -0.5),
        "w_fc": n(s.n_classes, s.d_model),
        "b_fc": n(s.n_classes, std=0.1),
    }


def make_classifier_prompts(seed: int, n: int, vocab: int, max_len: int, median: float = 24.0):
    """n prompts after stop-word removal: lengths log-normal around `median` tokens, clipped to
    [1, max_len]; ids uniform.  Returns (tokens int32 [n][max_len], zero padded, lens int32 [n])."""
    g = _rng(seed, 51)
    lens = np.clip(np.rint(median * np.exp(0.6 * g.standard_normal(n))), 1, max_len).astype(np.int32)
    tokens = g.integers(0, vocab, size=(n, max_len), dtype=np.int32)
    tokens[np.arange(max_len)[None, :] >= lens[:, None]] = 0
    return tokens, lens
