"""Seeded synthetic inputs for the chunk-plan executor and for its CPU checker.

This module holds no arithmetic of the method itself: it only draws numbers,
rounds them once to a storage type and names the tensors of each workload.
Both the GPU binding's callers and the tests of the CPU oracle take their
arrays from here, so both sides read identical bits.

Generator: a counter-based stream.  Element ``i`` of the tensor with stream
key ``s`` is a standard normal obtained by the Box-Muller transform from two
uniforms, each the top 53 bits of one splitmix64 output (Steele, Lea & Flood,
"Fast splittable pseudorandom number generators", 2014) at counters
``s * 2**40 + 2*i`` and ``s * 2**40 + 2*i + 1``.  No state is carried, so any
sub-range of a tensor can be regenerated on its own.

Workload recipes (shapes and value distributions of the paper's evaluated
model families, section 4: GPT prefill, ViT, AlphaFold pair stack): activations
N(0, 1); weights N(0, std) with std = 0.02 or 1/sqrt(fan_in); LayerNorm gain 1
and shift 0; biases 0 unless ``bias_std`` is given.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 240110652

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def splitmix64(counter: np.ndarray) -> np.ndarray:
    """splitmix64 output function applied to an array of uint64 counters."""
    with np.errstate(over="ignore"):
        z = (counter.astype(np.uint64) + np.uint64(0x9E3779B97F4A7C15)) & _M64
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
        z = z ^ (z >> np.uint64(31))
    return z


def standard_normal(stream: int, n: int, start: int = 0) -> np.ndarray:
    """``n`` standard normals (fp64), elements ``start .. start+n`` of ``stream``."""
    out = np.empty(n, dtype=np.float64)
    step = 1 << 22
    base = np.uint64((int(stream) << 40) & 0xFFFFFFFFFFFFFFFF)
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        idx = np.arange(start + lo, start + hi, dtype=np.uint64)
        c0 = base + idx * np.uint64(2)
        u1 = (splitmix64(c0) >> np.uint64(11)).astype(np.float64)
        u2 = (splitmix64(c0 + np.uint64(1)) >> np.uint64(11)).astype(np.float64)
        # u1 in (0, 1], u2 in [0, 1)
        u1 = (u1 + 1.0) * (1.0 / 9007199254740992.0)
        u2 = u2 * (1.0 / 9007199254740992.0)
        out[lo:hi] = np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2)
    return out


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32/fp64 values to bfloat16 (nearest, ties to even); returned as fp32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    r = (b + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) of values already representable in bf16."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    return (f.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round once to the storage type; result held as fp32 (exact for both types)."""
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


class _Streams:
    """Hands out one stream key per tensor: seed + 1000*config + tensor index."""

    def __init__(self, config_index: int, seed: int = BASE_SEED):
        self.base = int(seed) + 1000 * int(config_index)
        self.k = 0

    def normal(self, shape, std: float, dtype: str) -> np.ndarray:
        n = int(np.prod(shape))
        v = standard_normal(self.base + self.k, n) * float(std)
        self.k += 1
        return round_to_storage(v, dtype).reshape(shape)

    def skip(self):
        self.k += 1


@dataclass
class TransformerConfig:
    name: str
    index: int
    layers: int
    seq: int
    d_model: int
    heads: int
    d_ffn: int
    causal: bool
    dtype: str            # "f32" | "bf16"
    weight_std: float | None  # None -> 1/sqrt(fan_in)
    batch: int = 1
    activation: str = "gelu_erf"
    ln_eps: float = 1e-5
    chunk_len: int = 0    # rows per segment named by the workload (0: from budget)
    act_budget: int = 0   # bytes per layer (0: none)

    @property
    def head_dim(self) -> int:
        return self.d_model // self.heads

    @property
    def tokens(self) -> int:
        return self.batch * self.seq


@dataclass
class PairConfig:
    name: str
    index: int
    n_res: int
    c_z: int
    c_hidden: int
    heads: int
    head_dim: int
    transition_factor: int
    dtype: str
    chunk_len: int = 64
    activation: str = "relu"
    ln_eps: float = 1e-5

    @property
    def tokens(self) -> int:
        return self.n_res * self.n_res


GIB = 1 << 30

# The five synthetic workloads (shapes of the paper's model families).
C1 = TransformerConfig("C1_block_f32", 0, 1, 256, 64, 4, 256, False, "f32", None, chunk_len=64)
C2 = TransformerConfig("C2_gpt_4l_s8192", 1, 4, 8192, 1024, 16, 4096, True, "bf16", 0.02,
                       act_budget=1 * GIB)
C3 = TransformerConfig("C3_vit_12l_t4096", 2, 12, 4096, 768, 12, 3072, False, "bf16", 0.02,
                       chunk_len=512)
C4 = PairConfig("C4_pair_n1024", 3, 1024, 128, 128, 4, 32, 4, "bf16", chunk_len=64)
C5 = TransformerConfig("C5_gpt_2l_s65536", 4, 2, 65536, 2048, 16, 8192, True, "bf16", 0.02,
                       act_budget=4 * GIB)

CONFIGS = {c.name.split("_")[0]: c for c in (C1, C2, C3, C4, C5)}


# Tensor order of one transformer layer's weights (also the bind order of the executor).
TRANSFORMER_LAYER_TENSORS = (
    "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
    "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2",
)


def transformer_layer_shapes(cfg: TransformerConfig) -> dict:
    d, f = cfg.d_model, cfg.d_ffn
    return {
        "ln1_g": (d,), "ln1_b": (d,),
        "w_qkv": (3 * d, d), "b_qkv": (3 * d,),
        "w_o": (d, d), "b_o": (d,),
        "ln2_g": (d,), "ln2_b": (d,),
        "w_1": (f, d), "b_1": (f,),
        "w_2": (d, f), "b_2": (d,),
    }


def transformer_inputs(cfg: TransformerConfig, seed: int = BASE_SEED, bias_std: float = 0.0,
                       ln_jitter: float = 0.0):
    """Returns (x, layers): x [batch*seq, d_model]; layers = list of dicts of weights.

    Every weight matrix is [out_features, in_features].  ``w_qkv`` stacks the query,
    key and value projections (rows [0,d), [d,2d), [2d,3d)).  ``bias_std`` > 0 draws
    biases N(0, bias_std) and ``ln_jitter`` > 0 perturbs gain/shift, so that tests can
    exercise every epilogue; the benchmark recipe leaves both at 0.
    """
    st = _Streams(cfg.index, seed)
    x = st.normal((cfg.batch * cfg.seq, cfg.d_model), 1.0, cfg.dtype)
    shapes = transformer_layer_shapes(cfg)
    layers = []
    for _ in range(cfg.layers):
        w = {}
        for name in TRANSFORMER_LAYER_TENSORS:
            shp = shapes[name]
            if name.startswith("w_"):
                std = cfg.weight_std if cfg.weight_std is not None else 1.0 / math.sqrt(shp[1])
                w[name] = st.normal(shp, std, cfg.dtype)
            elif name.startswith("b_"):
                if bias_std > 0:
                    w[name] = st.normal(shp, bias_std, cfg.dtype)
                else:
                    st.skip()
                    w[name] = np.zeros(shp, np.float32)
            elif name.endswith("_g"):
                if ln_jitter > 0:
                    w[name] = round_to_storage(1.0 + st.normal(shp, ln_jitter, "f32"), cfg.dtype)
                else:
                    st.skip()
                    w[name] = np.ones(shp, np.float32)
            else:
                if ln_jitter > 0:
                    w[name] = st.normal(shp, ln_jitter, cfg.dtype)
                else:
                    st.skip()
                    w[name] = np.zeros(shp, np.float32)
        layers.append(w)
    return x, layers


# Tensor order of the pair-stack block's weights (also the bind order of the executor).
@dataclass(frozen=True)
class ResStackConfig:
    """UNet residual blocks one after another on channels-last images [batch, height, width, channels]."""
    name: str
    index: int
    layers: int
    batch: int
    height: int
    width: int
    channels: int
    groups: int
    dtype: str = "bf16"
    eps: float = 1e-5
    chunk_len: int = 1    # images per segment
    heads: int = 0        # > 0: every residual block is followed by an attention block with this many heads
    d_ffn: int = 0        # ... and a feed-forward of this width
    activation: str = "gelu_erf"
    context_tokens: int = 0   # > 0: the attention block has a cross-attention to this many context tokens per image
    context_dim: int = 0      # ... of this width
    gated: bool = False       # the feed-forward's hidden rows are value * activation(gate)

    @property
    def tokens(self) -> int:
        return self.batch * self.height * self.width      # pixels


# a latent-diffusion stage: 64 x 64 latents, 320 channels, 32 groups
U1 = ResStackConfig("U1_unet_res_b8_c320_64x64", 5, 2, 8, 64, 64, 320, 32, chunk_len=2)

# the same stage at an attention resolution: every residual block followed by an attention block over the
# 4096 positions of an image (5 heads of 64 channels; cross-attention to 77 context tokens of width 768 per image;
# gated feed-forward 4 x 320)
U2 = ResStackConfig("U2_unet_res_attn_b8_c320_64x64", 6, 1, 8, 64, 64, 320, 32, chunk_len=2, heads=5, d_ffn=1280,
                    context_tokens=77, context_dim=768, gated=True)

CONFIGS["U1"] = U1
CONFIGS["U2"] = U2

RES_BLOCK_TENSORS = ("gn1_g", "gn1_b", "w1", "b1", "gn2_g", "gn2_b", "w2", "b2", "temb")
ATTN_BLOCK_TENSORS = ("gn_g", "gn_b", "w_in", "b_in", "ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                      "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2", "w_out", "b_out")
CROSS_ATTN_TENSORS = ("lnc_g", "lnc_b", "w_qc", "w_kvc", "w_oc", "b_oc", "context")


def attn_block_tensors(cfg) -> tuple:
    """The attention block's tensors in bind order: the cross-attention's sit behind the self-attention's."""
    if cfg.heads <= 0:
        return ()
    if cfg.context_tokens <= 0:
        return ATTN_BLOCK_TENSORS
    return ATTN_BLOCK_TENSORS[:10] + CROSS_ATTN_TENSORS + ATTN_BLOCK_TENSORS[10:]


def res_stack_inputs(cfg: ResStackConfig, seed: int = BASE_SEED, bias_std: float = 0.0, gn_jitter: float = 0.0):
    """Returns (x, layers): x [batch, height, width, channels]; layers = list of dicts with the tensors of
    RES_BLOCK_TENSORS: convolution weights [C, 3, 3, C] ~ N(0, 1 / sqrt(9 C)), the time embedding of every image
    [batch, C] ~ N(0, 0.5), GroupNorm gain 1 and shift 0 (jittered on request), biases 0 (or N(0, bias_std))."""
    st = _Streams(cfg.index, seed)
    c = cfg.channels
    x = st.normal((cfg.batch, cfg.height, cfg.width, c), 1.0, cfg.dtype)
    layers = []
    for _ in range(cfg.layers):
        w = {}
        for name in RES_BLOCK_TENSORS:
            if name in ("w1", "w2"):
                w[name] = st.normal((c, 3, 3, c), 1.0 / math.sqrt(9 * c), cfg.dtype)
            elif name == "temb":
                w[name] = st.normal((cfg.batch, c), 0.5, cfg.dtype)
            elif name.endswith("_g"):
                if gn_jitter > 0:
                    w[name] = round_to_storage(1.0 + st.normal((c,), gn_jitter, "f32"), cfg.dtype)
                else:
                    st.skip()
                    w[name] = np.ones((c,), np.float32)
            else:
                std = gn_jitter if name.startswith("gn") else bias_std
                if std > 0:
                    w[name] = st.normal((c,), std, cfg.dtype)
                else:
                    st.skip()
                    w[name] = np.zeros((c,), np.float32)
        if cfg.heads > 0:
            f = cfg.d_ffn
            shapes = {"w_in": (c, c), "w_qkv": (3 * c, c), "w_o": (c, c), "w_1": ((2 if cfg.gated else 1) * f, c), "w_2": (c, f),
                      "w_out": (c, c), "w_qc": (c, c), "w_kvc": (2 * c, cfg.context_dim), "w_oc": (c, c)}
            for name in attn_block_tensors(cfg):
                if name == "context":
                    w[name] = st.normal((cfg.batch, cfg.context_tokens, cfg.context_dim), 1.0, cfg.dtype)
                elif name in ("w_qc", "w_kvc"):
                    w[name] = st.normal(shapes[name], 1.0 / math.sqrt(shapes[name][1]), cfg.dtype)
                elif name.startswith("w_"):
                    w[name] = st.normal(shapes[name], 1.0 / math.sqrt(shapes[name][1]), cfg.dtype)
                elif name.startswith("b_"):
                    n = shapes["w_" + name[2:]][0]
                    if bias_std > 0:
                        w[name] = st.normal((n,), bias_std, cfg.dtype)
                    else:
                        st.skip()
                        w[name] = np.zeros((n,), np.float32)
                elif name.endswith("_g"):
                    if gn_jitter > 0:
                        w[name] = round_to_storage(1.0 + st.normal((c,), gn_jitter, "f32"), cfg.dtype)
                    else:
                        st.skip()
                        w[name] = np.ones((c,), np.float32)
                else:
                    if gn_jitter > 0:
                        w[name] = st.normal((c,), gn_jitter, cfg.dtype)
                    else:
                        st.skip()
                        w[name] = np.zeros((c,), np.float32)
        layers.append(w)
    return x, layers


def pair_tensor_shapes(cfg: PairConfig) -> "list[tuple[str, tuple]]":
    cz, ch, hd = cfg.c_z, cfg.c_hidden, cfg.heads * cfg.head_dim
    ft = cfg.transition_factor * cz
    out = []
    for m in ("tmo", "tmi"):      # triangle multiplication outgoing / incoming
        out += [
            (f"{m}.ln_in_g", (cz,)), (f"{m}.ln_in_b", (cz,)),
            (f"{m}.w_ap", (ch, cz)), (f"{m}.b_ap", (ch,)),
            (f"{m}.w_ag", (ch, cz)), (f"{m}.b_ag", (ch,)),
            (f"{m}.w_bp", (ch, cz)), (f"{m}.b_bp", (ch,)),
            (f"{m}.w_bg", (ch, cz)), (f"{m}.b_bg", (ch,)),
            (f"{m}.w_g", (cz, cz)), (f"{m}.b_g", (cz,)),
            (f"{m}.ln_out_g", (ch,)), (f"{m}.ln_out_b", (ch,)),
            (f"{m}.w_o", (cz, ch)), (f"{m}.b_o", (cz,)),
        ]
    for m in ("tas", "tae"):      # triangle attention starting / ending node
        out += [
            (f"{m}.ln_g", (cz,)), (f"{m}.ln_b", (cz,)),
            (f"{m}.w_q", (hd, cz)), (f"{m}.w_k", (hd, cz)), (f"{m}.w_v", (hd, cz)),
            (f"{m}.w_bias", (cfg.heads, cz)),
            (f"{m}.w_g", (hd, cz)), (f"{m}.b_g", (hd,)),
            (f"{m}.w_o", (cz, hd)), (f"{m}.b_o", (cz,)),
        ]
    out += [
        ("pt.ln_g", (cz,)), ("pt.ln_b", (cz,)),
        ("pt.w_1", (ft, cz)), ("pt.b_1", (ft,)),
        ("pt.w_2", (cz, ft)), ("pt.b_2", (cz,)),
    ]
    return out


def pair_inputs(cfg: PairConfig, seed: int = BASE_SEED, bias_std: float = 0.0,
                ln_jitter: float = 0.0):
    """Returns (z, weights): z [n_res, n_res, c_z]; weights = dict name -> array."""
    st = _Streams(cfg.index, seed)
    z = st.normal((cfg.n_res, cfg.n_res, cfg.c_z), 1.0, cfg.dtype)
    w = {}
    for name, shp in pair_tensor_shapes(cfg):
        leaf = name.split(".")[1]
        if leaf.startswith("w_"):
            w[name] = st.normal(shp, 1.0 / math.sqrt(shp[1]), cfg.dtype)
        elif leaf.startswith("b_"):
            if bias_std > 0:
                w[name] = st.normal(shp, bias_std, cfg.dtype)
            else:
                st.skip()
                w[name] = np.zeros(shp, np.float32)
        elif leaf.endswith("_g"):
            if ln_jitter > 0:
                w[name] = round_to_storage(1.0 + st.normal(shp, ln_jitter, "f32"), cfg.dtype)
            else:
                st.skip()
                w[name] = np.ones(shp, np.float32)
        else:
            if ln_jitter > 0:
                w[name] = st.normal(shp, ln_jitter, cfg.dtype)
            else:
                st.skip()
                w[name] = np.zeros(shp, np.float32)
    return z, w
