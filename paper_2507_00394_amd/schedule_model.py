"""Closed forms of the paper's quantitative analysis, fed with attention times measured on
this kernel: where the attention of a micro batch runs (Section 4.2), how much crosses a
stage boundary (Section 4.2), and the pipeline bubble time and activation memory of 1F1B,
ZB1P and HelixPipe (Equations 1-4, Table 2, Section 4.5).  Host arithmetic only; nothing
here touches the GPU.  Times are in any one unit, memory in elements unless stated.

    python -m paper_2507_00394_amd.schedule_model --help
"""
from __future__ import annotations

import argparse
import json
from dataclasses import dataclass

SCHEDULES = ("1f1b", "zb1p", "helix_naive", "helix_two_fold", "helix")


# ----------------------------------------------------------------- Section 4.2: the helix mapping
def stage_of_pre_attention(layer: int, p: int) -> int:
    """Pre-attention of layer 0 sits on stage 0, that of layer l >= 1 (concatenated with the
    post-attention of layer l-1) on stage l mod p."""
    return layer % p


def stage_of_post_attention(layer: int, n_layers: int, p: int) -> int:
    """Post-attention of layer l < L-1 shares a stage with the pre-attention of layer l+1;
    that of the last layer returns to stage 0."""
    return 0 if layer == n_layers - 1 else (layer + 1) % p


def stage_of_attention(layer: int, micro_batch: int, p: int) -> int:
    """Attention of micro batch i in layer l runs on stage (l + i + 1) mod p, so the p micro
    batches of one loop occupy p different stages at once."""
    return (layer + micro_batch + 1) % p


# ----------------------------------------------------------------- Section 4.2: boundary volumes
def boundary_elements(b: int, s: int, h: int, qkv_linear_on_attention_stage: bool = True) -> dict:
    """Elements crossing the two boundaries of an attention part for one micro batch and layer.
    Attention -> post-attention carries the attention output and the residual input (2bsh).
    Pre-attention -> attention would carry Q, K, V and the residual input A (4bsh); moving the
    QKV linear layer to the attention stage replaces that by A and the layer's weights."""
    bsh = b * s * h
    return {"attention_to_post": 2 * bsh,
            "pre_to_attention": 2 * bsh + 3 * h * h if qkv_linear_on_attention_stage else 4 * bsh}


# ----------------------------------------------------------------- Table 1: matrix FLOPs of a layer
def layer_flops(b: int, s: int, h: int) -> dict:
    """Matrix FLOPs per transformer layer (Table 1; `attention` is the full-score-matrix count)."""
    bsh2 = b * s * h * h
    fwd = {"qkv_linear": 6 * bsh2, "attention": 4 * b * h * s * s, "o_linear": 2 * bsh2,
           "linear1": 8 * bsh2, "linear2": 8 * bsh2}
    bwd_b = dict(fwd, attention=8 * b * h * s * s)
    bwd_w = dict(fwd, attention=0)
    return {"forward": fwd, "backward_b": bwd_b, "backward_w": bwd_w}


# ----------------------------------------------------------------- Equations 1-4, Table 2, Section 4.5
def bubble_time(schedule: str, p: int, n_layers: int, t_pre: float, t_attn: float, t_post: float) -> float:
    """Pipeline bubble time per training iteration.  t_* are FORWARD times of the three parts of
    one layer for one micro batch; the backward pass is taken as twice the forward."""
    if schedule == "1f1b":            # Equation 1
        return 3 * (p - 1) * (t_pre + t_attn + t_post) * n_layers / p
    if schedule == "zb1p":            # Equation 3: backward W fills what it can; attention has none
        return (p - 1) * (t_pre + 3 * t_attn + t_post) * n_layers / p
    if schedule == "helix_naive":     # one micro batch at a time
        return 3 * (p - 1) * (t_pre + t_post)
    if schedule == "helix_two_fold":  # two micro batches at a time to hide the transfers
        return 6 * (p - 1) * (t_pre + t_post)
    if schedule == "helix":           # two-fold, plus the re-run of pre/post before their backward
        return 8 * (p - 1) * (t_pre + t_post)
    raise ValueError(f"unknown schedule {schedule!r}; one of {SCHEDULES}")


def activation_elements(schedule: str, p: int, n_layers: int, b: int, s: int, h: int, m: int = 0, stage: int = 0) -> int:
    """Activation elements stashed on pipeline stage `stage` at the peak (Table 2).  m: micro
    batches per iteration (HelixPipe only; m must be a multiple of p, of 2p for two-fold)."""
    bsh = b * s * h
    if schedule == "1f1b":            # Equation 2: p - i micro batches outstanding on stage i
        return 16 * (p - stage) * bsh * n_layers // p
    if schedule == "zb1p":            # Equation 4
        return 16 * bsh * n_layers
    if schedule in ("helix_naive", "helix_two_fold"):
        return 16 * bsh * m * n_layers // p
    if schedule == "helix":           # recomputation without attention: 4bsh per layer
        return 4 * bsh * m * n_layers // p
    raise ValueError(f"unknown schedule {schedule!r}; one of {SCHEDULES}")


@dataclass
class Prediction:
    schedule: str
    bubble: float
    busy: float

    @property
    def bubble_fraction(self) -> float:
        return self.bubble / (self.bubble + self.busy)


def predict(schedule: str, p: int, n_layers: int, m: int, t_pre: float, t_attn: float, t_post: float) -> Prediction:
    """Bubble fraction of one iteration: bubble / (bubble + busy), with the busy time of a stage
    = m micro batches x L/p layers x (forward + twice that for backward), plus, for `helix`,
    one more forward of pre- and post-attention per layer (the recomputation)."""
    per_layer = 3 * (t_pre + t_attn + t_post) + ((t_pre + t_post) if schedule == "helix" else 0.0)
    return Prediction(schedule, bubble_time(schedule, p, n_layers, t_pre, t_attn, t_post), m * n_layers / p * per_layer)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--p", type=int, default=8, help="pipeline stages")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--hidden", type=int, default=4096)
    ap.add_argument("--seq", type=int, default=131072)
    ap.add_argument("--micro-batches", type=int, default=16, help="per iteration (the paper uses 2p)")
    ap.add_argument("--t-attn-ms", type=float, required=True,
                    help="measured attention FORWARD time of one micro batch and layer on one GPU (its share of the heads)")
    ap.add_argument("--gemm-tflops", type=float, default=1000.0,
                    help="assumed sustained rate of the dense layers per GPU, to turn Table 1 FLOPs into t_pre, t_post")
    ap.add_argument("--sp", type=int, default=8, help="sequence-parallel size inside a stage")
    a = ap.parse_args(argv)
    f = layer_flops(1, a.seq, a.hidden)["forward"]
    rate = a.sp * a.gemm_tflops * 1e9                      # FLOPs per ms of one stage
    t_qkv = f["qkv_linear"] / rate
    t_post = (f["o_linear"] + f["linear1"] + f["linear2"]) / rate
    # LayerNorm has no matrix FLOPs.  Layer-wise schedules keep the QKV linear layer (which has a
    # backward W) in the pre-attention part; HelixPipe runs it on the attention stage (Section 4.2),
    # so there it counts as attention time and leaves the bubble.
    parts = {"layerwise": (t_qkv, a.t_attn_ms, t_post), "helix": (0.0, a.t_attn_ms + t_qkv, t_post)}
    out = {"t_qkv_linear_ms": t_qkv, "t_attention_ms": a.t_attn_ms, "t_post_ms": t_post, "schedules": {}}
    for sch in SCHEDULES:
        t_pre, t_attn, t_post_ = parts["helix" if sch.startswith("helix") else "layerwise"]
        pr = predict(sch, a.p, a.layers, a.micro_batches, t_pre, t_attn, t_post_)
        mem = activation_elements(sch, a.p, a.layers, 1, a.seq, a.hidden, a.micro_batches, 0) * 2 / a.sp / 2 ** 30
        out["schedules"][sch] = {"bubble_ms": pr.bubble, "busy_ms": pr.busy, "bubble_fraction": pr.bubble_fraction,
                                 "stage0_activation_gib_per_gpu_fp16": mem}
    print(json.dumps(out, indent=1))


if __name__ == "__main__":
    main()
