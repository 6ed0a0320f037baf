"""Seeded synthetic inputs and the workload table.

This module holds no arithmetic of the method: only shapes, random draws and
rounding of the drawn values to the storage type.  Both the HIP path and the
test oracle are fed from here (the oracle receives the rounded values widened
to float64), so neither depends on the other.

The paper trains BERT-Large and GPT-2 on real corpora (Section 7, Table 1);
a stage's forward/backward cost depends only on shapes, so seeded normal
tensors of the same shapes stand in for them.  Matrices ~ N(0, 0.02^2), stage
inputs ~ N(0, 1).  Not fixed by the paper (chosen so that no gradient path is
trivially zero): biases and LayerNorm shifts ~ N(0, 0.02^2), LayerNorm gains
1 + N(0, 0.02^2), upstream gradients ~ N(0, 1) / sqrt(T*H).
"""
from dataclasses import dataclass, asdict

import numpy as np

ARCH_POST_LN_ENCODER = 0
ARCH_PRE_LN_CAUSAL = 1
DTYPE_FP32 = 0
DTYPE_BF16 = 1


@dataclass(frozen=True)
class StageConfig:
    name: str
    arch: int
    dtype: int
    hidden: int
    heads: int
    ffn: int
    seq: int
    micro_batch: int
    n_own: int
    n_shadow: int
    P: int
    stage_id: int
    M: int
    seed: int

    @property
    def tokens(self):
        return self.micro_batch * self.seq

    @property
    def layer_params(self):
        H, F = self.hidden, self.ffn
        return 4 * H * H + 2 * H * F + 9 * H + F

    def replace(self, **kw):
        d = asdict(self)
        d.update(kw)
        return StageConfig(**d)


CONFIGS = {
    # tiny 2-stage pipeline, fp32
    "tiny": StageConfig("tiny", ARCH_POST_LN_ENCODER, DTYPE_FP32, 64, 2, 256, 16, 2, 1, 1, 2, 0, 4, 0),
    # BERT-large-shaped stage: 24 layers over 4 stages -> 6 own + 6 shadow
    "bert_large_stage": StageConfig("bert_large_stage", ARCH_POST_LN_ENCODER, DTYPE_BF16,
                                    1024, 16, 4096, 512, 8, 6, 6, 4, 1, 8, 2),
    # GPT-2 1.5B-shaped stage: 48 layers over 8 stages -> 6 own + 6 shadow
    "gpt2_1p5b_stage": StageConfig("gpt2_1p5b_stage", ARCH_PRE_LN_CAUSAL, DTYPE_BF16,
                                   1600, 25, 6400, 1024, 4, 6, 6, 8, 3, 16, 3),
    # large-layer stage sized for 288 GB of HBM
    "large_layer_stage": StageConfig("large_layer_stage", ARCH_PRE_LN_CAUSAL, DTYPE_BF16,
                                     12288, 96, 49152, 2048, 1, 2, 2, 8, 3, 16, 5),
}
# the failover workload is the BERT-large-shaped stage with the successor lost
# while micro-batch 5 (0-indexed) is being handed over
FAILOVER_K = 5
FAILOVER_SEED = 4

PARAM_NAMES = ("Wqkv", "bqkv", "Wo", "bo", "g1", "be1", "W1", "b1", "W2", "b2", "g2", "be2")


def param_shapes(H, F):
    return {"Wqkv": (H, 3 * H), "bqkv": (3 * H,), "Wo": (H, H), "bo": (H,),
            "g1": (H,), "be1": (H,), "W1": (H, F), "b1": (F,),
            "W2": (F, H), "b2": (H,), "g2": (H,), "be2": (H,)}


def param_offsets(H, F):
    """name -> (offset, shape) inside one layer's flat vector."""
    out, off = {}, 0
    for n in PARAM_NAMES:
        shp = param_shapes(H, F)[n]
        out[n] = (off, shp)
        off += int(np.prod(shp))
    return out


# ------------------------------------------------------------- bf16 storage

def f32_to_bf16_bits(a):
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(a, dtype):
    """Values as the device will hold them, returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == DTYPE_BF16:
        return bf16_bits_to_f32(f32_to_bf16_bits(a)).reshape(a.shape)
    return a


# ---------------------------------------------------------------- generators

def _draw_layer(rng, H, F):
    parts = []
    for n in PARAM_NAMES:
        shp = param_shapes(H, F)[n]
        v = rng.standard_normal(int(np.prod(shp)), dtype=np.float32) * np.float32(0.02)
        if n in ("g1", "g2"):
            v = v + np.float32(1.0)
        parts.append(v)
    return np.concatenate(parts)


def make_stage_inputs(cfg, n_microbatches=None):
    """Draw, in a fixed order, own layers, shadow layers, x_k, g_z_k.

    Returns float32 arrays already rounded to the storage type:
      own_w    [n_own,    layer_params]
      shadow_w [n_shadow, layer_params]
      x        [M, T, H]   inputs from the previous stage
      gz       [M, T, H]   gradients arriving at the successor's output
    """
    M = cfg.M if n_microbatches is None else n_microbatches
    rng = np.random.default_rng(cfg.seed)
    H, F, T = cfg.hidden, cfg.ffn, cfg.tokens
    own = np.stack([_draw_layer(rng, H, F) for _ in range(cfg.n_own)]) if cfg.n_own else \
        np.zeros((0, cfg.layer_params), np.float32)
    shadow = np.stack([_draw_layer(rng, H, F) for _ in range(cfg.n_shadow)]) if cfg.n_shadow else \
        np.zeros((0, cfg.layer_params), np.float32)
    x = rng.standard_normal((M, T, H), dtype=np.float32)
    gz = rng.standard_normal((M, T, H), dtype=np.float32) / np.float32(np.sqrt(T * H))
    r = lambda a: round_to_storage(a, cfg.dtype)
    return {"own_w": r(own), "shadow_w": r(shadow), "x": r(x), "gz": r(gz)}


# ---- the two ends of the model (wrap-around stage) ------------------------------
# Vocabulary sizes of the paper's language models, padded up to a multiple of 64 as is usual so that the
# head's matrices tile evenly: BERT's 30522 WordPiece entries, GPT-2's 50257 BPE entries.
VOCAB = {"bert_large_stage": 30528, "gpt2_1p5b_stage": 50304}


def front_param_count(arch, V, S, H):
    """E_tok [V,H] | E_pos [S,H] | gain [H] | shift [H] (the last two only for the post-LN encoder)."""
    return V * H + S * H + (2 * H if arch == ARCH_POST_LN_ENCODER else 0)


def back_param_count(arch, V, H):
    """gain [H] | shift [H] (only for the pre-LN decoder: its final LayerNorm) | W_head [H,V]."""
    return (2 * H if arch == ARCH_PRE_LN_CAUSAL else 0) + H * V


def zipf_ids(rng, V, shape):
    """Token ids with Zipf's rank-frequency law (probability of id r proportional to 1/(r+1)): text corpora
    such as the paper's Wikipedia dump repeat a few tokens very often, which is what the embedding gradient
    has to add up."""
    p = 1.0 / np.arange(1, V + 1, dtype=np.float64)
    p /= p.sum()
    return rng.choice(V, size=shape, p=p).astype(np.int32)


def make_ends_inputs(cfg, V, n_microbatches=None):
    """Draw the front and back parameters, token ids, labels and the gradients arriving at the front
    stage's output, in a fixed order (its own seed stream, so the stage inputs do not move).

      front_w [front_param_count]  back_w [back_param_count]   float32, rounded to the storage type
      ids, labels [M, T] int32     g1 [M, T, H] gradients from the stage after the front stage
    """
    M = cfg.M if n_microbatches is None else n_microbatches
    rng = np.random.default_rng([cfg.seed, 77])
    H, S, T = cfg.hidden, cfg.seq, cfg.tokens
    nrm = lambda n: rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
    front = [nrm(V * H), nrm(S * H)]
    if cfg.arch == ARCH_POST_LN_ENCODER:
        front += [nrm(H) + np.float32(1.0), nrm(H)]
    back = []
    if cfg.arch == ARCH_PRE_LN_CAUSAL:
        back += [nrm(H) + np.float32(1.0), nrm(H)]
    back.append(nrm(H * V))
    ids = zipf_ids(rng, V, (M, T))
    labels = zipf_ids(rng, V, (M, T))
    g1 = rng.standard_normal((M, T, H), dtype=np.float32) / np.float32(np.sqrt(T * H))
    r = lambda a: round_to_storage(a, cfg.dtype)
    return {"front_w": r(np.concatenate(front)), "back_w": r(np.concatenate(back)), "ids": ids, "labels": labels,
            "g1": r(g1)}
