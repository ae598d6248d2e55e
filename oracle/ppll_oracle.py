"""CPU oracle for one gradient-isolated block's local training step (PPLL).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the HIP
library is checked against.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does.  It shares no
code with the HIP path and imports nothing from it.

What it computes (paper: Section 3.2, Algorithm 1, the body of process P_j):
take (x_{j-1}, y); forward the module M_j; (the output is what gets pushed to
the next buffer); gradient of the local loss w.r.t. the module parameters
theta_j and the auxiliary-network parameters gamma_j, nothing for x_{j-1}
(gradient isolation, Sections 3.1-3.2); update (theta_j, gamma_j).

The method reaches exactly the plain definition of forward evaluation, reverse
mode differentiation and optimizer arithmetic, so each function below is that
definition written out with numpy in float64 (dtype selectable), a matmul or an
erf being the only library steps.  No blocking, fusion or reordering.

Model identity (Section 4.1-4.2): ViT encoder layers with an auxiliary net of
"N attention blocks followed by a classifier"; ResNet basic blocks.  Details the
paper leaves open are fixed as documented at each function (pre-LN, exact GELU,
biased variance, ...).

Weights are stored [in, out]; rows of activation matrices are tokens/pixels.
Images and ResNet activations are NHWC.

Mixed precision: the oracle itself is float64 throughout.  For the ReLU network
only, block_init(storage="bf16") rounds the tensors stored between layers to bf16
values, because a ReLU mask is a binary decision that both sides of a comparison
have to take on values of the same precision; the ViT path has no such switch.

Parity pins for every function live in tests/test_oracle_*.py (finite
differences in float64, torch.autograd on library ops, scipy routines, closed
forms, brute-force loops, invariants).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

ARCH_VIT = 0
ARCH_RESNET = 1
IN_IMAGE = 0
IN_ACTIVATION = 1
OPT_SGD = 0
OPT_ADAMW = 1


@dataclass
class BlockConfig:
    """Shape and hyper-parameters of one local block (module + auxiliary net)."""
    arch: int = ARCH_VIT
    input_kind: int = IN_IMAGE
    batch: int = 8
    num_classes: int = 10
    # ViT
    img_h: int = 32
    img_w: int = 32
    img_c: int = 3
    patch: int = 4
    tokens: int = 65
    dim: int = 64
    heads: int = 4
    mlp_dim: int = 128
    depth: int = 2
    aux_depth: int = 0
    # ResNet
    channels: int = 32
    height: int = 16
    width: int = 16
    n_basic_blocks: int = 5
    aux_channels: int = 64
    # 0: every basic block keeps the shape; i+1: basic block i halves the resolution and doubles the
    # channels, so the block input is [batch, 2*height, 2*width, channels/2] (ResNet-32 of Section 4.1:
    # 16 -> 32 -> 64 channels on 32 -> 16 -> 8 pixel maps).  input_kind = IN_IMAGE puts the network's
    # stem (conv3x3 img_c -> input channels, BatchNorm, ReLU) in front of the basic blocks.
    transition_block: int = 0
    # optimizer (Section 4.1: SGD, Nesterov momentum 0.9, L2 weight decay 1e-4)
    optimizer: int = OPT_SGD
    momentum: float = 0.0
    nesterov: int = 0
    weight_decay: float = 0.0
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    ln_eps: float = 1e-6
    bn_eps: float = 1e-5
    bn_momentum: float = 0.1


# --------------------------------------------------------------------------
# parameter tables
# --------------------------------------------------------------------------

def _encoder_layer_spec(prefix: str, D: int, F: int) -> List[Tuple[str, Tuple[int, ...]]]:
    return [
        (f"{prefix}.ln1.g", (D,)), (f"{prefix}.ln1.b", (D,)),
        (f"{prefix}.qkv.w", (D, 3 * D)), (f"{prefix}.qkv.b", (3 * D,)),
        (f"{prefix}.proj.w", (D, D)), (f"{prefix}.proj.b", (D,)),
        (f"{prefix}.ln2.g", (D,)), (f"{prefix}.ln2.b", (D,)),
        (f"{prefix}.fc1.w", (D, F)), (f"{prefix}.fc1.b", (F,)),
        (f"{prefix}.fc2.w", (F, D)), (f"{prefix}.fc2.b", (D,)),
    ]


def resnet_layout(cfg: BlockConfig) -> List[Tuple[int, int, int]]:
    """(input channels, output channels, stride of the first convolution) of every basic block."""
    C, t = cfg.channels, cfg.transition_block - 1
    out = []
    for i in range(cfg.n_basic_blocks):
        if t >= 0 and i < t:
            out.append((C // 2, C // 2, 1))
        elif i == t:
            out.append((C // 2, C, 2))
        else:
            out.append((C, C, 1))
    return out


def resnet_input_shape(cfg: BlockConfig) -> Tuple[int, int, int]:
    """(height, width, channels) of the activation the first basic block reads."""
    if cfg.transition_block > 0:
        return 2 * cfg.height, 2 * cfg.width, cfg.channels // 2
    return cfg.height, cfg.width, cfg.channels


def param_spec(cfg: BlockConfig) -> List[Tuple[str, Tuple[int, ...]]]:
    """Ordered (name, shape) list of theta_j (module) then gamma_j (auxiliary)."""
    spec: List[Tuple[str, Tuple[int, ...]]] = []
    if cfg.arch == ARCH_VIT:
        D, F = cfg.dim, cfg.mlp_dim
        if cfg.input_kind == IN_IMAGE:
            spec += [("pe.w", (cfg.patch * cfg.patch * cfg.img_c, D)), ("pe.b", (D,)),
                     ("cls", (D,)), ("pos", (cfg.tokens, D))]
        for l in range(cfg.depth):
            spec += _encoder_layer_spec(f"blk{l}", D, F)
        for a in range(cfg.aux_depth):
            spec += _encoder_layer_spec(f"aux{a}", D, F)
        spec += [("head.ln.g", (D,)), ("head.ln.b", (D,)),
                 ("head.w", (D, cfg.num_classes)), ("head.b", (cfg.num_classes,))]
    elif cfg.arch == ARCH_RESNET:
        C, A = cfg.channels, cfg.aux_channels
        if cfg.input_kind == IN_IMAGE:
            c0 = resnet_input_shape(cfg)[2]
            spec += [("stem.conv.w", (3, 3, cfg.img_c, c0)), ("stem.bn.g", (c0,)), ("stem.bn.b", (c0,))]
        for i, (ci, co, _) in enumerate(resnet_layout(cfg)):
            spec += [(f"rb{i}.conv1.w", (3, 3, ci, co)), (f"rb{i}.bn1.g", (co,)), (f"rb{i}.bn1.b", (co,)),
                     (f"rb{i}.conv2.w", (3, 3, co, co)), (f"rb{i}.bn2.g", (co,)), (f"rb{i}.bn2.b", (co,))]
        spec += [("aux.conv.w", (3, 3, C, A)), ("aux.bn.g", (A,)), ("aux.bn.b", (A,)),
                 ("head.w", (A, cfg.num_classes)), ("head.b", (cfg.num_classes,))]
    else:
        raise ValueError("unknown arch")
    return spec


def bn_stat_spec(cfg: BlockConfig) -> List[Tuple[str, int]]:
    """BatchNorm layers carrying running statistics, in forward order."""
    if cfg.arch != ARCH_RESNET:
        return []
    out = []
    if cfg.input_kind == IN_IMAGE:
        out.append(("stem.bn", resnet_input_shape(cfg)[2]))
    for i, (_, co, _) in enumerate(resnet_layout(cfg)):
        out += [(f"rb{i}.bn1", co), (f"rb{i}.bn2", co)]
    out.append(("aux.bn", cfg.aux_channels))
    return out


def param_count(cfg: BlockConfig) -> int:
    return sum(int(np.prod(s)) for _, s in param_spec(cfg))


def unflatten(cfg: BlockConfig, flat: np.ndarray, dtype=np.float64) -> Dict[str, np.ndarray]:
    flat = np.asarray(flat).reshape(-1)
    out, off = {}, 0
    for name, shape in param_spec(cfg):
        n = int(np.prod(shape))
        out[name] = np.array(flat[off:off + n], dtype=dtype).reshape(shape)
        off += n
    if off != flat.size:
        raise ValueError(f"parameter blob has {flat.size} values, spec needs {off}")
    return out


def flatten(cfg: BlockConfig, tensors: Dict[str, np.ndarray]) -> np.ndarray:
    return np.concatenate([np.asarray(tensors[name]).reshape(-1) for name, _ in param_spec(cfg)])


# --------------------------------------------------------------------------
# elementary operations: forward and reverse-mode derivative
# --------------------------------------------------------------------------

def linear_fwd(x, w, b):
    """y = x w + b, w stored [in, out] (leading axes of x are flattened to rows)."""
    return (x.reshape(-1, x.shape[-1]) @ w + b).reshape(x.shape[:-1] + (w.shape[1],))


def linear_bwd(dy, x, w):
    """dx = dy w^T, dw = x^T dy, db = sum over rows of dy."""
    x2 = x.reshape(-1, x.shape[-1])
    dy2 = dy.reshape(-1, dy.shape[-1])
    return (dy2 @ w.T).reshape(x.shape), x2.T @ dy2, dy2.sum(axis=0)


def layernorm_fwd(x, g, b, eps):
    """Per-row normalisation over the last axis with biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd)


def layernorm_bwd(dy, cache, g):
    xhat, rstd = cache
    dyh = dy * g
    dx = rstd * (dyh - dyh.mean(axis=-1, keepdims=True)
                 - xhat * (dyh * xhat).mean(axis=-1, keepdims=True))
    red = tuple(range(dy.ndim - 1))
    return dx, (dy * xhat).sum(axis=red), dy.sum(axis=red)


def gelu_fwd(h):
    """Exact GELU: h * Phi(h), Phi the standard normal CDF."""
    return h * 0.5 * (1.0 + _erf(h / math.sqrt(2.0)))


def gelu_bwd(dg, h):
    """d/dh [h Phi(h)] = Phi(h) + h phi(h)."""
    cdf = 0.5 * (1.0 + _erf(h / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * h * h) / math.sqrt(2.0 * math.pi)
    return dg * (cdf + h * pdf)


def softmax_rows(s):
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention_fwd(qkv, heads):
    """Multi-head self-attention core on qkv [B, T, 3D] laid out [Q | K | V],
    head h owning columns h*dh .. (h+1)*dh of each third.  Scale 1/sqrt(dh)."""
    B, T, D3 = qkv.shape
    D = D3 // 3
    dh = D // heads
    q, k, v = (qkv[:, :, i * D:(i + 1) * D].reshape(B, T, heads, dh).transpose(0, 2, 1, 3)
               for i in range(3))
    scale = 1.0 / math.sqrt(dh)
    s = (q @ k.transpose(0, 1, 3, 2)) * scale
    p = softmax_rows(s)
    o = p @ v                                           # [B, H, T, dh]
    out = o.transpose(0, 2, 1, 3).reshape(B, T, D)
    return out, (q, k, v, p, scale)


def attention_bwd(dout, cache):
    q, k, v, p, scale = cache
    B, H, T, dh = q.shape
    do = dout.reshape(B, T, H, dh).transpose(0, 2, 1, 3)
    dv = p.transpose(0, 1, 3, 2) @ do
    dp = do @ v.transpose(0, 1, 3, 2)
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = (ds @ k) * scale
    dk = (ds.transpose(0, 1, 3, 2) @ q) * scale
    back = lambda t: t.transpose(0, 2, 1, 3).reshape(B, T, H * dh)
    return np.concatenate([back(dq), back(dk), back(dv)], axis=-1)


def patchify(img, patch):
    """NHWC image -> [B, (H/P)*(W/P), P*P*C]; patches row-major over the grid,
    each flattened in (row, col, channel) order."""
    B, H, W, C = img.shape
    gh, gw = H // patch, W // patch
    x = img.reshape(B, gh, patch, gw, patch, C).transpose(0, 1, 3, 2, 4, 5)
    return x.reshape(B, gh * gw, patch * patch * C)


def cross_entropy(logits, labels):
    """Mean softmax cross-entropy (natural log) and its gradient w.r.t. logits."""
    B = logits.shape[0]
    z = logits - logits.max(axis=-1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(axis=-1, keepdims=True))
    loss = -logp[np.arange(B), labels].mean()
    d = np.exp(logp)
    d[np.arange(B), labels] -= 1.0
    return loss, d / B


def _pad1(x):
    return np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))


def conv3x3_fwd(x, w, stride):
    """y[b,oy,ox,co] = sum_{ky,kx,ci} xpad[b, oy*s+ky, ox*s+kx, ci] w[ky,kx,ci,co];
    zero padding 1, no bias, x NHWC, w [3,3,Cin,Cout]."""
    B, H, W, Ci = x.shape
    Ho, Wo = (H + 2 - 3) // stride + 1, (W + 2 - 3) // stride + 1
    xp = _pad1(x)
    y = np.zeros((B, Ho, Wo, w.shape[3]), dtype=x.dtype)
    for ky in range(3):
        for kx in range(3):
            xs = xp[:, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride, :]
            y += xs @ w[ky, kx]
    return y


def conv3x3_bwd_weight(dy, x, stride):
    B, Ho, Wo, Co = dy.shape
    xp = _pad1(x)
    dw = np.zeros((3, 3, x.shape[3], Co), dtype=x.dtype)
    dy2 = dy.reshape(-1, Co)
    for ky in range(3):
        for kx in range(3):
            xs = xp[:, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride, :]
            dw[ky, kx] = xs.reshape(-1, x.shape[3]).T @ dy2
    return dw


def conv3x3_bwd_input(dy, w, stride, in_shape):
    B, H, W, Ci = in_shape
    _, Ho, Wo, _ = dy.shape
    dxp = np.zeros((B, H + 2, W + 2, Ci), dtype=dy.dtype)
    for ky in range(3):
        for kx in range(3):
            dxp[:, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride, :] += dy @ w[ky, kx].T
    return dxp[:, 1:-1, 1:-1, :]


def batchnorm_fwd(x, g, b, eps):
    """Training-mode BatchNorm over (B,H,W) per channel, biased variance."""
    red = tuple(range(x.ndim - 1))
    mu = x.mean(axis=red)
    var = ((x - mu) ** 2).mean(axis=red)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * g + b, (xhat, rstd, mu, var)


def batchnorm_bwd(dy, cache, g):
    xhat, rstd = cache[0], cache[1]
    red = tuple(range(dy.ndim - 1))
    n = dy.size // dy.shape[-1]
    sdy = dy.sum(axis=red)
    sdyx = (dy * xhat).sum(axis=red)
    dx = (g * rstd / n) * (n * dy - sdy - xhat * sdyx)
    return dx, sdyx, sdy


# --------------------------------------------------------------------------
# optimizers (Algorithm 1, the update line; Section 4.1 names SGD with Nesterov
# momentum and L2 weight decay; AdamW is the workload definition's choice)
# --------------------------------------------------------------------------

def shortcut_fwd(x, c_out, stride):
    """Parameter-free shortcut of a basic block (the CIFAR ResNet the paper trains, Section 4.1): the
    identity where the shapes agree; where the block halves the map and widens it, every `stride`-th
    pixel with zero channels appended after the original ones."""
    if stride == 1 and x.shape[-1] == c_out:
        return x
    sub = x[:, ::stride, ::stride, :]
    y = np.zeros(sub.shape[:-1] + (c_out,), dtype=x.dtype)
    y[..., :x.shape[-1]] = sub
    return y


def shortcut_bwd(dy, in_shape, stride):
    if stride == 1 and in_shape[-1] == dy.shape[-1]:
        return dy
    dx = np.zeros(in_shape, dtype=dy.dtype)
    dx[:, ::stride, ::stride, :] = dy[..., :in_shape[-1]]
    return dx


def sgd_update(p, g, buf, lr, momentum, nesterov, weight_decay, first):
    """Coupled L2 decay, then momentum buffer (first step: buffer = gradient),
    then plain or Nesterov step.  Returns (new_p, new_buf)."""
    g = g + weight_decay * p
    if momentum != 0.0:
        buf = g.copy() if first else momentum * buf + g
        g = g + momentum * buf if nesterov else buf
    return p - lr * g, buf


def adamw_update(p, g, m, v, t, lr, beta1, beta2, eps, weight_decay):
    """Decoupled weight decay, bias-corrected moments; t is the 1-based step."""
    p = p * (1.0 - lr * weight_decay)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return p - lr * mhat / (np.sqrt(vhat) + eps), m, v


# --------------------------------------------------------------------------
# block = module M_j + auxiliary network A_j
# --------------------------------------------------------------------------

@dataclass
class BlockState:
    cfg: BlockConfig
    dtype: type
    params: Dict[str, np.ndarray]
    mom1: Dict[str, np.ndarray]
    mom2: Dict[str, np.ndarray]
    steps: int = 0
    bn_mean: Dict[str, np.ndarray] = field(default_factory=dict)
    bn_var: Dict[str, np.ndarray] = field(default_factory=dict)
    grads: Optional[Dict[str, np.ndarray]] = None
    logits: Optional[np.ndarray] = None
    storage: Optional[str] = None

    def act(self, a):
        """A stored activation, in the storage precision being emulated."""
        return bf16_values(a) if self.storage == "bf16" else a

    def wmat(self, w):
        """A weight matrix / filter as the contractions read it (bf16 shadow of the
        fp32 master when bf16 storage is emulated)."""
        return bf16_values(w) if self.storage == "bf16" else w


def bf16_values(a):
    """Values of `a` rounded to the nearest bfloat16 (8-bit significand, ties to
    even), kept in a's dtype.  Used only to emulate where a mixed-precision run
    stores activations and weight shadows, so that sign decisions (ReLU masks)
    are taken on the same stored values; all arithmetic stays in a's dtype.
    (Normal range only: no subnormal or overflow handling is needed here.)"""
    a = np.asarray(a)
    m, e = np.frexp(a)                       # a = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e).astype(a.dtype)


def block_init(cfg: BlockConfig, flat_params: np.ndarray, dtype=np.float64,
               storage: Optional[str] = None) -> BlockState:
    """storage=None: everything in `dtype`; this is the definition and the gate.
    storage="bf16" exists for the ReLU network only, where floating point takes a
    binary decision (the ReLU mask): every tensor a mixed-precision run hands from
    one layer to the next in bf16 (convolution outputs, post-ReLU activations,
    pooled features, and in the backward pass the gradients with respect to those
    same tensors) and the filters its contractions read are rounded to bf16 values,
    so that the masks are decided on values of that precision and cancelling sums
    over such tensors carry that precision's noise (arithmetic, norm statistics,
    loss, parameter gradients and the optimizer stay in `dtype`).  The ViT block
    has no such decision and takes no storage mode."""
    if storage is not None and (storage != "bf16" or cfg.arch != ARCH_RESNET):
        raise ValueError("storage emulation is defined for the ResNet block only, as storage='bf16'")
    params = unflatten(cfg, flat_params, dtype)
    st = BlockState(cfg, dtype, params,
                    {k: np.zeros_like(v) for k, v in params.items()},
                    {k: np.zeros_like(v) for k, v in params.items()}, storage=storage)
    for name, c in bn_stat_spec(cfg):
        st.bn_mean[name] = np.zeros(c, dtype=dtype)
        st.bn_var[name] = np.ones(c, dtype=dtype)
    return st


def _encoder_fwd(x, p, pre, st):
    cfg = st.cfg
    u, c_ln1 = layernorm_fwd(x, p[pre + ".ln1.g"], p[pre + ".ln1.b"], cfg.ln_eps)
    qkv = linear_fwd(u, p[pre + ".qkv.w"], p[pre + ".qkv.b"])
    o, c_att = attention_fwd(qkv, cfg.heads)
    x1 = x + linear_fwd(o, p[pre + ".proj.w"], p[pre + ".proj.b"])
    u2, c_ln2 = layernorm_fwd(x1, p[pre + ".ln2.g"], p[pre + ".ln2.b"], cfg.ln_eps)
    h = linear_fwd(u2, p[pre + ".fc1.w"], p[pre + ".fc1.b"])
    gl = gelu_fwd(h)
    x2 = x1 + linear_fwd(gl, p[pre + ".fc2.w"], p[pre + ".fc2.b"])
    return x2, (c_ln1, u, c_att, o, c_ln2, u2, h, gl)


def _encoder_bwd(dx2, cache, p, pre, grads, st):
    c_ln1, u, c_att, o, c_ln2, u2, h, gl = cache
    dgl, grads[pre + ".fc2.w"], grads[pre + ".fc2.b"] = linear_bwd(dx2, gl, p[pre + ".fc2.w"])
    dh = gelu_bwd(dgl, h)
    du2, grads[pre + ".fc1.w"], grads[pre + ".fc1.b"] = linear_bwd(dh, u2, p[pre + ".fc1.w"])
    d, grads[pre + ".ln2.g"], grads[pre + ".ln2.b"] = layernorm_bwd(du2, c_ln2, p[pre + ".ln2.g"])
    dx1 = dx2 + d
    do, grads[pre + ".proj.w"], grads[pre + ".proj.b"] = linear_bwd(dx1, o, p[pre + ".proj.w"])
    dqkv = attention_bwd(do, c_att)
    du, grads[pre + ".qkv.w"], grads[pre + ".qkv.b"] = linear_bwd(dqkv, u, p[pre + ".qkv.w"])
    d, grads[pre + ".ln1.g"], grads[pre + ".ln1.b"] = layernorm_bwd(du, c_ln1, p[pre + ".ln1.g"])
    return dx1 + d


def vit_forward(st: BlockState, x_in):
    """Module forward x_j = M_j(x_{j-1}) followed by the auxiliary forward.
    Returns (x_out, logits, caches)."""
    cfg, p = st.cfg, st.params
    x_in = np.asarray(x_in, dtype=st.dtype)
    caches = {}
    if cfg.input_kind == IN_IMAGE:
        pt = patchify(x_in, cfg.patch)
        e = linear_fwd(pt, p["pe.w"], p["pe.b"])
        x = np.concatenate([np.broadcast_to(p["cls"], (cfg.batch, 1, cfg.dim)), e], axis=1) + p["pos"]
        caches["patches"] = pt
    else:
        x = x_in
    for l in range(cfg.depth):
        x, caches[f"blk{l}"] = _encoder_fwd(x, p, f"blk{l}", st)
    x_out = x
    for a in range(cfg.aux_depth):
        x, caches[f"aux{a}"] = _encoder_fwd(x, p, f"aux{a}", st)
    z, caches["head.ln"] = layernorm_fwd(x[:, 0, :], p["head.ln.g"], p["head.ln.b"], cfg.ln_eps)
    caches["z"] = z
    logits = linear_fwd(z, p["head.w"], p["head.b"])
    return x_out, logits, caches


def vit_backward(st: BlockState, dlogits, caches):
    """Gradients of the local loss for every tensor of gamma_j and theta_j.
    The chain stops at the block input: nothing is produced for x_{j-1}."""
    cfg, p = st.cfg, st.params
    g: Dict[str, np.ndarray] = {}
    dz, g["head.w"], g["head.b"] = linear_bwd(dlogits, caches["z"], p["head.w"])
    dcls, g["head.ln.g"], g["head.ln.b"] = layernorm_bwd(dz, caches["head.ln"], p["head.ln.g"])
    dx = np.zeros((cfg.batch, cfg.tokens, cfg.dim), dtype=st.dtype)
    dx[:, 0, :] = dcls
    for a in reversed(range(cfg.aux_depth)):
        dx = _encoder_bwd(dx, caches[f"aux{a}"], p, f"aux{a}", g, st)
    for l in reversed(range(cfg.depth)):
        dx = _encoder_bwd(dx, caches[f"blk{l}"], p, f"blk{l}", g, st)
    if cfg.input_kind == IN_IMAGE:
        g["pos"] = dx.sum(axis=0)
        g["cls"] = dx[:, 0, :].sum(axis=0)
        _, g["pe.w"], g["pe.b"] = linear_bwd(dx[:, 1:, :], caches["patches"], p["pe.w"])
    return g


def _bn_track(st: BlockState, name, cache, n):
    """Running statistics (kept, never used inside the step)."""
    m = st.cfg.bn_momentum
    mu, var = cache[2], cache[3]
    st.bn_mean[name] = (1 - m) * st.bn_mean[name] + m * mu
    st.bn_var[name] = (1 - m) * st.bn_var[name] + m * var * (n / (n - 1.0))


def resnet_forward(st: BlockState, x_in, track=True):
    """[stem conv3x3 -> BN -> ReLU when the input is the image] -> n basic blocks
    relu(shortcut(x) + bn2(conv2(relu(bn1(conv1(x)))))) -> x_out, then the auxiliary head
    conv3x3/s2 -> BN -> ReLU -> global average -> Linear."""
    cfg, p, S, W = st.cfg, st.params, st.act, st.wmat
    x = np.asarray(x_in, dtype=st.dtype)
    caches = {}
    if cfg.input_kind == IN_IMAGE:
        c0 = S(conv3x3_fwd(x, W(p["stem.conv.w"]), 1))
        b0, cb0 = batchnorm_fwd(c0, p["stem.bn.g"], p["stem.bn.b"], cfg.bn_eps)
        if track:
            _bn_track(st, "stem.bn", cb0, c0.size // c0.shape[-1])
        caches["stem"] = (x, cb0, b0)
        x = S(np.maximum(b0, 0))
    for i, (_, co, stride) in enumerate(resnet_layout(cfg)):
        pre = f"rb{i}"
        c1 = S(conv3x3_fwd(x, W(p[pre + ".conv1.w"]), stride))
        b1, cb1 = batchnorm_fwd(c1, p[pre + ".bn1.g"], p[pre + ".bn1.b"], cfg.bn_eps)
        y1 = S(np.maximum(b1, 0))
        c2 = S(conv3x3_fwd(y1, W(p[pre + ".conv2.w"]), 1))
        b2, cb2 = batchnorm_fwd(c2, p[pre + ".bn2.g"], p[pre + ".bn2.b"], cfg.bn_eps)
        s = shortcut_fwd(x, co, stride) + b2
        caches[pre] = (x, cb1, b1, y1, cb2, s)
        if track:
            n = c1.size // c1.shape[-1]
            _bn_track(st, pre + ".bn1", cb1, n)
            _bn_track(st, pre + ".bn2", cb2, n)
        x = S(np.maximum(s, 0))
    x_out = x
    ca = S(conv3x3_fwd(x_out, W(p["aux.conv.w"]), 2))
    ba, cba = batchnorm_fwd(ca, p["aux.bn.g"], p["aux.bn.b"], cfg.bn_eps)
    if track:
        _bn_track(st, "aux.bn", cba, ca.size // ca.shape[-1])
    ya = S(np.maximum(ba, 0))
    pooled = S(ya.mean(axis=(1, 2)))
    logits = linear_fwd(pooled, p["head.w"], p["head.b"])
    caches["aux"] = (x_out, cba, ba, ya, pooled)
    return x_out, logits, caches


def resnet_backward(st: BlockState, dlogits, caches):
    cfg, p, S = st.cfg, st.params, st.act
    g: Dict[str, np.ndarray] = {}
    x_out, cba, ba, ya, pooled = caches["aux"]
    dpool, g["head.w"], g["head.b"] = linear_bwd(dlogits, pooled, p["head.w"])
    dpool = S(dpool)
    hw = ya.shape[1] * ya.shape[2]
    dya = S(np.broadcast_to(dpool[:, None, None, :] / hw, ya.shape))
    dba = dya * (ba > 0)
    dca, g["aux.bn.g"], g["aux.bn.b"] = batchnorm_bwd(dba, cba, p["aux.bn.g"])
    dca = S(dca)
    g["aux.conv.w"] = conv3x3_bwd_weight(dca, x_out, 2)
    dx = S(conv3x3_bwd_input(dca, st.wmat(p["aux.conv.w"]), 2, x_out.shape))
    stem = cfg.input_kind == IN_IMAGE
    layout = resnet_layout(cfg)
    for i in reversed(range(cfg.n_basic_blocks)):
        pre = f"rb{i}"
        stride = layout[i][2]
        x, cb1, b1, y1, cb2, s = caches[pre]
        ds = dx * (s > 0)
        dc2, g[pre + ".bn2.g"], g[pre + ".bn2.b"] = batchnorm_bwd(ds, cb2, p[pre + ".bn2.g"])
        dc2 = S(dc2)
        g[pre + ".conv2.w"] = conv3x3_bwd_weight(dc2, y1, 1)
        dy1 = S(conv3x3_bwd_input(dc2, st.wmat(p[pre + ".conv2.w"]), 1, y1.shape))
        db1 = dy1 * (b1 > 0)
        dc1, g[pre + ".bn1.g"], g[pre + ".bn1.b"] = batchnorm_bwd(db1, cb1, p[pre + ".bn1.g"])
        dc1 = S(dc1)
        g[pre + ".conv1.w"] = conv3x3_bwd_weight(dc1, x, stride)
        if i > 0 or stem:   # without a stem the first block's input is the detached x_{j-1}
            dx = S(shortcut_bwd(ds, x.shape, stride) + conv3x3_bwd_input(dc1, st.wmat(p[pre + ".conv1.w"]), stride, x.shape))
    if stem:
        img, cb0, b0 = caches["stem"]
        db0 = dx * (b0 > 0)
        dc0, g["stem.bn.g"], g["stem.bn.b"] = batchnorm_bwd(db0, cb0, p["stem.bn.g"])
        dc0 = S(dc0)
        g["stem.conv.w"] = conv3x3_bwd_weight(dc0, img, 1)
    return g


def batchnorm_eval(x, g, b, mean, var, eps):
    """Evaluation-mode BatchNorm: the affine map fixed by the running statistics."""
    return (x - mean) / np.sqrt(var + eps) * g + b


def block_forward_eval(st: BlockState, x_in):
    """Evaluation-mode forward: (x_j, class scores of the auxiliary network).  No loss, no state
    change; BatchNorm normalises with its running statistics.  A ViT block has no mode-dependent
    layer (no dropout, LayerNorm only), so its evaluation forward is its training forward."""
    if st.cfg.arch == ARCH_VIT:
        x_out, logits, _ = vit_forward(st, x_in)
        return x_out, logits
    cfg, p, S, W = st.cfg, st.params, st.act, st.wmat
    x = np.asarray(x_in, dtype=st.dtype)

    def bn(t, name):
        return batchnorm_eval(t, p[name + ".g"], p[name + ".b"], st.bn_mean[name], st.bn_var[name], cfg.bn_eps)

    if cfg.input_kind == IN_IMAGE:
        x = S(np.maximum(bn(S(conv3x3_fwd(x, W(p["stem.conv.w"]), 1)), "stem.bn"), 0))
    for i, (_, co, stride) in enumerate(resnet_layout(cfg)):
        pre = f"rb{i}"
        c1 = S(conv3x3_fwd(x, W(p[pre + ".conv1.w"]), stride))
        y1 = S(np.maximum(bn(c1, pre + ".bn1"), 0))
        c2 = S(conv3x3_fwd(y1, W(p[pre + ".conv2.w"]), 1))
        x = S(np.maximum(shortcut_fwd(x, co, stride) + bn(c2, pre + ".bn2"), 0))
    x_out = x
    ca = S(conv3x3_fwd(x_out, W(p["aux.conv.w"]), 2))
    ya = S(np.maximum(bn(ca, "aux.bn"), 0))
    pooled = S(ya.mean(axis=(1, 2)))
    return x_out, linear_fwd(pooled, p["head.w"], p["head.b"])


def block_forward(st: BlockState, x_in, track=False):
    if st.cfg.arch == ARCH_VIT:
        return vit_forward(st, x_in)
    return resnet_forward(st, x_in, track=track)


def local_loss(st: BlockState, x_in, labels) -> float:
    """Local loss as a function of the current parameters (used by the
    finite-difference pins)."""
    _, logits, _ = block_forward(st, x_in)
    return float(cross_entropy(logits, np.asarray(labels))[0])


def apply_update(st: BlockState, grads: Dict[str, np.ndarray], lr: float) -> None:
    cfg = st.cfg
    st.steps += 1
    for name in st.params:
        if cfg.optimizer == OPT_SGD:
            st.params[name], st.mom1[name] = sgd_update(
                st.params[name], grads[name], st.mom1[name], lr, cfg.momentum,
                bool(cfg.nesterov), cfg.weight_decay, st.steps == 1)
        else:
            st.params[name], st.mom1[name], st.mom2[name] = adamw_update(
                st.params[name], grads[name], st.mom1[name], st.mom2[name], st.steps, lr,
                cfg.beta1, cfg.beta2, cfg.adam_eps, cfg.weight_decay)


def block_step(st: BlockState, x_in, labels, lr: float):
    """One pass of the loop body of Algorithm 1 for module j.  Returns
    (x_out, loss); x_out is computed with the parameters as they were before
    the update, which is what the algorithm pushes to the next buffer."""
    labels = np.asarray(labels)
    if st.cfg.arch == ARCH_VIT:
        x_out, logits, caches = vit_forward(st, x_in)
    else:
        x_out, logits, caches = resnet_forward(st, x_in, track=True)
    loss, dlogits = cross_entropy(logits, labels)
    if st.cfg.arch == ARCH_VIT:
        grads = vit_backward(st, dlogits, caches)
    else:
        grads = resnet_backward(st, dlogits, caches)
    st.grads, st.logits = grads, logits
    apply_update(st, grads, lr)
    return x_out, float(loss)


def chain_step(states: Sequence[BlockState], x0, labels, lr: float):
    """Sequential local learning over K blocks for one batch: block j consumes
    block j-1's output and the same labels (the (x_j, y) tuple of Algorithm 1).
    With blocking FIFO buffers the pipelined schedule computes these same
    values, so this is the oracle of the pipeline."""
    x, losses, outs = x0, [], []
    for st in states:
        x, loss = block_step(st, x, labels, lr)
        losses.append(loss)
        outs.append(x)
    return losses, outs
