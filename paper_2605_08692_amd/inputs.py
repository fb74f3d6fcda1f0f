"""Seeded synthetic inputs shaped like the benchmark layers.

This module only draws random tensors and lists the five benchmark settings;
it holds none of the method's arithmetic, so both the HIP path and the CPU
checker can be fed from it.  The tensors stand in for real LLM linear weights
and for activations captured on calibration text, which are not available
offline: weights are Gaussian with a sprinkling of heavy-tailed outliers,
activations are Gaussian (or gated, SiLU(a)*b) with a few outlier channels.
"""
import numpy as np
import torch

NVFP4, INT4 = 0, 1

# Ascending 16-entry initial grids: the signed E2M1 values (with +0 and -0 both
# present, hence the duplicated 0) and the symmetric integer grid.
E2M1_GRID = np.array([-6, -4, -3, -2, -1.5, -1, -0.5, 0, 0, 0.5, 1, 1.5, 2, 3, 4, 6], np.float32)
INT4_GRID = np.arange(-8, 8, dtype=np.float32)


def format_grid(fmt):
    """T0 = T1 = the format's own grid, as 32 floats."""
    g = E2M1_GRID if fmt == NVFP4 else INT4_GRID
    return np.concatenate([g, g]).astype(np.float32)


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _student_t(shape, nu, gen, device):
    z = torch.randn(shape, generator=gen, device=device)
    chi2 = torch.zeros(shape, device=device)
    for _ in range(nu):
        chi2 += torch.randn(shape, generator=gen, device=device) ** 2
    return z / torch.sqrt(chi2 / nu)


def make_weight(N, K, dist, seed, device="cpu", chunk_rows=2048):
    """bf16 [N, K].  dist: "gauss_outlier" = N(0, 0.02^2) with 1 % of entries
    replaced by 0.02*StudentT(3); "student5" = 0.015*StudentT(5)."""
    gen = _gen(seed, device)
    out = torch.empty((N, K), dtype=torch.bfloat16, device=device)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        shape = (r1 - r0, K)
        if dist == "gauss_outlier":
            w = 0.02 * torch.randn(shape, generator=gen, device=device)
            mask = torch.rand(shape, generator=gen, device=device) < 0.01
            t = 0.02 * _student_t(shape, 3, gen, device)
            w = torch.where(mask, t, w)
        elif dist == "student5":
            w = 0.015 * _student_t(shape, 5, gen, device)
        else:
            raise ValueError(dist)
        out[r0:r1] = w.to(torch.bfloat16)
    return out


def make_activations(tokens, K, kind, seed, device="cpu", chunk_tokens=4096):
    """bf16 [tokens, K].  kind: ("gauss", n_outlier_channels, "x20") |
    ("gauss", fraction, "u10_50") | ("silu_gate", fraction, "x30")."""
    base, amount, boost = kind
    gen = _gen(seed, device)
    n_out = amount if isinstance(amount, int) else max(1, int(round(amount * K)))
    perm = torch.randperm(K, generator=gen, device=device)[:n_out]
    scale = torch.ones(K, device=device)
    if boost == "x20":
        scale[perm] = 20.0
    elif boost == "x30":
        scale[perm] = 30.0
    elif boost == "u10_50":
        scale[perm] = 10.0 + 40.0 * torch.rand(n_out, generator=gen, device=device)
    else:
        raise ValueError(boost)
    out = torch.empty((tokens, K), dtype=torch.bfloat16, device=device)
    for t0 in range(0, tokens, chunk_tokens):
        t1 = min(tokens, t0 + chunk_tokens)
        shape = (t1 - t0, K)
        if base == "gauss":
            x = torch.randn(shape, generator=gen, device=device)
        elif base == "silu_gate":
            a = torch.randn(shape, generator=gen, device=device)
            b = torch.randn(shape, generator=gen, device=device)
            x = torch.nn.functional.silu(a) * b
        else:
            raise ValueError(base)
        out[t0:t1] = (x * scale).to(torch.bfloat16)
    return out


def bits(t):
    """Host uint16 view (bf16 bit patterns) of a bf16 tensor."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def from_bits(a, device="cpu"):
    """bf16 tensor from a uint16 array of bit patterns."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)


def _layer(name, N, K, dist, seed, x):
    return dict(name=name, N=N, K=K, dist=dist, seed=seed, x=x)


# The five benchmark settings.  "xs" maps an activation key to its recipe; each
# layer names the key of the activations that feed it.
CONFIGS = [
    dict(name="cfg0_small_nvfp4", fmt=NVFP4, g=16, iters=10,
         layers=[_layer("linear", 256, 512, "gauss_outlier", 0, "x512")],
         xs={"x512": dict(tokens=256, K=512, kind=("gauss", 8, "x20"), seed=100)}),
    dict(name="cfg1_llama2_7b_qproj_int4", fmt=INT4, g=128, iters=20,
         layers=[_layer("q_proj", 4096, 4096, "gauss_outlier", 1, "x4096")],
         xs={"x4096": dict(tokens=65536, K=4096, kind=("gauss", 0.01, "u10_50"), seed=101)}),
    dict(name="cfg2_down_proj_nvfp4", fmt=NVFP4, g=16, iters=20,
         layers=[_layer("down_proj", 4096, 11008, "student5", 2, "x11008")],
         xs={"x11008": dict(tokens=65536, K=11008, kind=("silu_gate", 0.005, "x30"), seed=102)}),
    dict(name="cfg3_llama3_8b_block_int4", fmt=INT4, g=128, iters=20,
         layers=[_layer("q_proj", 4096, 4096, "gauss_outlier", 3000, "x4096"),
                 _layer("k_proj", 1024, 4096, "gauss_outlier", 3001, "x4096"),
                 _layer("v_proj", 1024, 4096, "gauss_outlier", 3002, "x4096"),
                 _layer("o_proj", 4096, 4096, "gauss_outlier", 3003, "x4096"),
                 _layer("gate_proj", 14336, 4096, "gauss_outlier", 3004, "x4096"),
                 _layer("up_proj", 14336, 4096, "gauss_outlier", 3005, "x4096"),
                 _layer("down_proj", 4096, 14336, "gauss_outlier", 3006, "x14336")],
         xs={"x4096": dict(tokens=131072, K=4096, kind=("gauss", 0.01, "u10_50"), seed=103),
             "x14336": dict(tokens=131072, K=14336, kind=("gauss", 0.01, "u10_50"), seed=113)}),
    dict(name="cfg4_llama3_70b_mlp_nvfp4", fmt=NVFP4, g=16, iters=30,
         layers=[_layer("gate_proj", 28672, 8192, "gauss_outlier", 4000, "x8192"),
                 _layer("down_proj", 8192, 28672, "gauss_outlier", 4001, "x28672")],
         xs={"x8192": dict(tokens=131072, K=8192, kind=("gauss", 0.01, "u10_50"), seed=104),
             "x28672": dict(tokens=131072, K=28672, kind=("gauss", 0.01, "u10_50"), seed=114)}),
]


def scaled_config(cfg, rows_div=1, tokens_div=1):
    """Copy of a setting with fewer rows / tokens (same widths, same recipe),
    for checks that must finish quickly."""
    out = dict(cfg)
    out["layers"] = [dict(l, N=max(8, l["N"] // rows_div)) for l in cfg["layers"]]
    out["xs"] = {k: dict(v, tokens=max(16, v["tokens"] // tokens_div)) for k, v in cfg["xs"].items()}
    return out


def layer_weights(layer, device="cpu"):
    return make_weight(layer["N"], layer["K"], layer["dist"], layer["seed"], device)


def activations(xrecipe, device="cpu"):
    return make_activations(xrecipe["tokens"], xrecipe["K"], xrecipe["kind"], xrecipe["seed"], device)


def n_weights(cfg):
    return sum(l["N"] * l["K"] for l in cfg["layers"])


__all__ = ["NVFP4", "INT4", "E2M1_GRID", "INT4_GRID", "format_grid", "make_weight",
           "make_activations", "bits", "from_bits", "CONFIGS", "scaled_config", "layer_weights",
           "activations", "n_weights"]
