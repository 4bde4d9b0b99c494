"""CPU emulation of the GPU path's operand precisions, for the precision study in test_precision_study.py.

The oracle itself stays untouched: this module only *rounds* the oracle's inputs (weights) and the activations that
are stored between layers, then calls the oracle's own layer routines (fp64 accumulation).  That isolates the one
question the GPU design had to answer -- how many mantissa bits the MFMA operands need -- from every other detail
of the kernels.

Operand formats
  "bf16"   one bf16 per operand (8 significant bits): one MFMA product per layer
  "f16"    one IEEE half per operand (11 significant bits): one product per layer (the no-gradient forward)
  "bf16x2" a (hi, lo) pair of bf16 per operand (16 significant bits): the three-product scheme
           hi_w hi_a + lo_w hi_a + hi_w lo_a of the training forward (the dropped lo_w lo_a term is below 2^-16)
"""
import numpy as np

from oracle import nature_cnn as orc


def round_bf16(x):
    """Round to nearest even to 8 significant bits (bfloat16), returned as float64."""
    x32 = np.asarray(x, dtype=np.float32)
    u = x32.view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return r.view(np.float32).astype(np.float64)


def round_f16(x):
    return np.asarray(x, dtype=np.float64).astype(np.float16).astype(np.float64)


def round_bf16x2(x):
    hi = round_bf16(x)
    return hi + round_bf16(np.asarray(x, dtype=np.float64) - hi)


ROUNDERS = {"bf16": round_bf16, "f16": round_f16, "bf16x2": round_bf16x2, "exact": lambda x: np.asarray(x, np.float64)}


def forward_with_rounded_operands(params, obs_u8, spec, fmt):
    """The oracle's forward pass with every weight matrix and every stored activation rounded to `fmt`: one format
    name for the whole network, or {"conv1" | "conv2" | "conv3" | "fc" | "head": (weight format, format of the
    activation the layer stores)} for a mixture
    (pixels are exact in all formats; biases and the 1/255 scale are applied in full precision, as the
    kernels' fp32 epilogues do).  Returns the same cache layout as oracle.forward for the policy/value head."""
    if isinstance(fmt, str):
        fmt = {layer: (fmt, fmt) for layer in ("conv1", "conv2", "conv3", "fc", "head")}
    qw = {layer: ROUNDERS[f[0]] for layer, f in fmt.items()}      # the layer's weights
    qa = {layer: ROUNDERS[f[1]] for layer, f in fmt.items()}      # the activation it stores
    q = qw["head"]
    assert spec.head == "pv"
    cache = {"x": obs_u8.astype(np.float64) / 255.0}
    a = obs_u8.astype(np.float64)
    for i, (co, k, s, p) in enumerate(spec.geometry.convs, start=1):
        pre = orc.conv2d(a, qw[f"conv{i}"](params[f"conv{i}.W"]), None, s, p)
        if i == 1:
            pre = pre / 255.0
        pre = pre + params[f"conv{i}.b"][None, :, None, None]
        a = qa[f"conv{i}"](np.maximum(pre, 0.0))
        cache[f"pre{i}"], cache[f"act{i}"] = pre, a
    B = obs_u8.shape[0]
    pre_fc = a.reshape(B, -1) @ qw["fc"](params["fc.W"]).T + params["fc.b"]
    h = qa["fc"](np.maximum(pre_fc, 0.0))
    cache["pre_fc"], cache["h"] = pre_fc, h
    cache["logits"] = h @ q(params["pi.W"]).T + params["pi.b"]
    cache["value"] = (h @ q(params["v.W"]).T + params["v.b"])[:, 0]
    return cache


def gradient_from_forward(params, cache, batch, spec):
    """fp64 backward pass (the oracle's) on a given forward cache: what the gradient becomes when only the
    forward pass -- and with it the ReLU masks -- is computed at reduced precision."""
    dz, dv = orc.a2c_loss_grad(cache["logits"], cache["value"], batch["action"], batch["adv"].astype(np.float64),
                               batch["ret"].astype(np.float64))
    return orc.flatten(orc.backward(params, cache, spec, dlogits=dz, dvalue=dv), spec)
