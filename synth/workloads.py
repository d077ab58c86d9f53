"""Shapes and seeds of the benchmark workloads, and seeded tensors for them.

The five named configurations are the ones the benchmark definition lists: a tiny
two-block model, an SD3-medium-like model, a Flux-like model, a heterogeneous batch of
eight requests on the SD3-like model, and a Wan-like video model.  They stand in for the
image/video pipelines and request-resolution mixes of the paper's evaluation (its trained
weights and traces are not used): weights are N(0, 0.02^2), latent noise and the text
condition are N(0, 1), all from the counter-based generator in `synth.rng`.
"""
import numpy as np

from .rng import gaussian, gaussian_bf16, round_bf16

# Architecture keys mirror the fields of the library's configuration struct.
CONFIGS = {
    "tiny": dict(
        arch=dict(family="J", n_blocks=2, n_single=0, hidden=256, n_heads=4, head_dim=64,
                  mlp_hidden=1024, latent_ch=4, patch=(1, 2, 2), cond_dim=256,
                  rope_axes=(0, 0, 0), rope_theta=10000.0),
        latents=[(1, 16, 16)], n_cond=16, steps=4, shifts=[1.0]),
    "sd3": dict(
        arch=dict(family="J", n_blocks=24, n_single=0, hidden=1536, n_heads=24, head_dim=64,
                  mlp_hidden=6144, latent_ch=16, patch=(1, 2, 2), cond_dim=4096,
                  rope_axes=(0, 0, 0), rope_theta=10000.0),
        latents=[(1, 128, 128)], n_cond=154, steps=28, shifts=[1.0]),
    "flux": dict(
        arch=dict(family="F", n_blocks=19, n_single=38, hidden=3072, n_heads=24, head_dim=128,
                  mlp_hidden=12288, latent_ch=16, patch=(1, 2, 2), cond_dim=4096,
                  rope_axes=(16, 56, 56), rope_theta=10000.0),
        latents=[(1, 128, 128)], n_cond=512, steps=28, shifts=[1.0]),
    "hetero8": dict(
        arch=dict(family="J", n_blocks=24, n_single=0, hidden=1536, n_heads=24, head_dim=64,
                  mlp_hidden=6144, latent_ch=16, patch=(1, 2, 2), cond_dim=4096,
                  rope_axes=(0, 0, 0), rope_theta=10000.0),
        latents=[(1, h, h) for h in (32, 32, 64, 64, 96, 128, 128, 128)], n_cond=154, steps=28,
        shifts=[1.0, 1.0, 1.5, 1.5, 2.0, 3.0, 3.0, 3.0]),
    "wan": dict(
        arch=dict(family="W", n_blocks=40, n_single=0, hidden=5120, n_heads=40, head_dim=128,
                  mlp_hidden=13824, latent_ch=16, patch=(1, 2, 2), cond_dim=4096,
                  rope_axes=(44, 42, 42), rope_theta=10000.0),
        latents=[(21, 60, 104)], n_cond=512, steps=50, shifts=[1.0]),
}


def make_requests(name):
    """List of (frames, height, width, n_cond) in latent units for a named workload."""
    c = CONFIGS[name]
    return [(f, h, w, c["n_cond"]) for (f, h, w) in c["latents"]]


def default_sigmas(steps, shift=1.0):
    """Noise levels sigma_0=1 ... sigma_T=0: sigma = s*u / (1 + (s-1)*u), u = 1 - j/T."""
    u = 1.0 - np.arange(steps + 1, dtype=np.float64) / float(steps)
    return (shift * u / (1.0 + (shift - 1.0) * u)).astype(np.float32)


def make_inputs(reqs, latent_ch, cond_dim, steps, shifts=None, noise_seed=2, cond_seed=100):
    """Seeded latents (float32, N(0,1)), conditions (bf16-valued float32, N(0,1)) and
    per-request sigma schedules for a list of requests (frames, height, width, n_cond)."""
    latents, conds, sigmas = [], [], []
    for r, (f, h, w, nc) in enumerate(reqs):
        n = latent_ch * f * h * w
        latents.append(gaussian(noise_seed + r, "latent", n).reshape(latent_ch, f, h, w))
        conds.append(gaussian_bf16(cond_seed + r, "cond", nc * cond_dim).reshape(nc, cond_dim))
        s = 1.0 if shifts is None else shifts[r]
        sigmas.append(default_sigmas(steps, s))
    return latents, conds, np.stack(sigmas)


def make_params(shapes, seed, std=0.02, bias_std=0.0, gain_std=0.0):
    """Seeded parameter values for a {name: (shape, kind)} table.

    kind "matrix"/"table": N(0, std^2); "bias": zeros, or N(0, bias_std^2) when bias_std > 0;
    "gain": ones, or 1 + N(0, gain_std^2).  Every value is bf16-representable so that a
    bf16 device copy and a float64 reference hold identical numbers.
    """
    out = {}
    for name, (shape, kind) in shapes.items():
        n = int(np.prod(shape))
        if kind in ("matrix", "table"):
            v = gaussian_bf16(seed, name, n, std)
        elif kind == "bias":
            v = gaussian_bf16(seed, name, n, bias_std) if bias_std > 0 else np.zeros(n, np.float32)
        elif kind == "gain":
            v = (round_bf16(1.0 + gaussian(seed, name, n, gain_std)) if gain_std > 0
                 else np.ones(n, np.float32))
        else:
            raise ValueError(kind)
        out[name] = v.reshape(shape)
    return out


# Text encoders of the Encode stage (T5-v1.1-style; the paper's pipelines name T5-XXL, 4.8 B
# parameters, prompts of 30-500 tokens).  Keys mirror the library's encoder configuration.
ENCODERS = {
    "t5_tiny": dict(vocab=1000, d_model=256, n_heads=4, head_dim=64, d_ff=512, n_layers=2),
    "t5_xxl": dict(vocab=32128, d_model=4096, n_heads=64, head_dim=64, d_ff=10240, n_layers=24),
}


def make_tokens(lengths, vocab, seed=7):
    """Seeded token ids for prompts of the given lengths: list of int32 arrays."""
    out = []
    for r, n in enumerate(lengths):
        u = gaussian(seed + r, "tokens", n)                      # any seeded real numbers will do
        out.append((np.floor(np.abs(u) * 1e6).astype(np.int64) % vocab).astype(np.int32))
    return out


# Convolutional decoders of the Decode stage (AutoencoderKL-style).  `channels` are the widths of
# the up levels in execution order; every level but the last ends with a 2x upsampling.
DECODERS = {
    "ae_tiny": dict(latent_ch=16, out_ch=3, channels=(128, 128, 64, 64), n_res=2),
    "ae_kl": dict(latent_ch=16, out_ch=3, channels=(512, 512, 256, 128), n_res=3),
}
# causal video decoders (3x3x3 convolutions; t_up: level transitions that also double the frame rate)
VIDEO_DECODERS = {
    "vae3d_tiny": dict(latent_ch=16, out_ch=3, channels=(128, 64, 64), n_res=1, t_up=1),
    "vae3d": dict(latent_ch=16, out_ch=3, channels=(512, 512, 256, 128), n_res=3, t_up=2),
}
