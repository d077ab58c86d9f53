"""The three stages chained on the GPU, each one's device output feeding the next through the
C ABIs (prompt tokens -> condition -> T denoising steps -> image), against the same chain of
the three float64 oracles.  Tolerances widen along the chain: condition 1e-2, final latent
5e-2 (the denoising bound), image 8e-2 rel-L2."""
import numpy as np
import pytest

import synth
from helpers import rel_l2
from oracle import decoder_oracle as D
from oracle import dit_oracle as O
from oracle import encoder_oracle as E


@pytest.mark.gpu
def test_encode_diffuse_decode_chain_against_the_oracle_chain():
    import torch
    from paper_2510_02838_amd import binding as B, decoder as XD, encoder as XE
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS["tiny"]
    arch, reqs, steps = cfg["arch"], synth.make_requests("tiny"), cfg["steps"]
    f, h, w, n_cond = reqs[0]
    enc_arch = synth.ENCODERS["t5_tiny"]
    dec_arch = dict(latent_ch=arch["latent_ch"], out_ch=3, channels=(128, 64), n_res=1)
    assert enc_arch["d_model"] == arch["cond_dim"] and f == 1

    # parameters and inputs (seeded, bf16-representable)
    pe = synth.make_params(E.param_shapes(enc_arch), 1, 0.05, 0.0, 0.1)
    pe["rel_bias"] = synth.round_bf16(pe["rel_bias"] * 2.0 / 0.05)
    pe["embed"] = synth.round_bf16(pe["embed"] / 0.05)
    pd = synth.make_params(O.param_shapes(arch), 1, 0.06, 0.1, 0.0)
    pc = synth.make_params(D.param_shapes(dec_arch), 1, 0.02, 0.02, 0.1)
    toks = synth.make_tokens([n_cond], enc_arch["vocab"])[0]
    lat, _, sigmas = synth.make_inputs(reqs, arch["latent_ch"], arch["cond_dim"], steps, cfg["shifts"])

    # GPU chain
    enc = XE.Encoder(enc_arch); enc.ensure_workspace([n_cond]); enc.init_weights(0, 0.0); enc.set_params(pe)
    dit = B.DiT(arch); dit.ensure_workspace(reqs, steps); dit.init_weights(0, 0.0); dit.set_params(pd)
    dec = XD.Decoder(dec_arch); dec.ensure_workspace(h, w); dec.init_weights(0, 0.0); dec.set_params(pc)
    cond = torch.empty((n_cond, arch["cond_dim"]), dtype=torch.bfloat16, device="cuda")
    enc.forward([n_cond], torch.from_numpy(toks).cuda(), cond, None)
    x = torch.from_numpy(lat[0].astype(np.float32).ravel()).cuda()
    dit.sample(reqs, x, cond, sigmas)
    up = dec.up_factor()
    img = torch.full((h * up, w * up, 3), float("nan"), dtype=torch.float32, device="cuda")
    dec.forward(h, w, x, img)
    torch.cuda.synchronize()

    # oracle chain
    cond_ref = E.EncoderOracle(enc_arch, pe).forward(toks)
    x_ref = O.DiTOracle(arch, pd).sample(lat[0], cond_ref, sigmas[0])
    img_ref = D.DecoderOracle(dec_arch, pc).forward(np.transpose(x_ref[:, 0], (1, 2, 0)))

    assert rel_l2(cond.to(torch.float32).cpu().numpy(), cond_ref) <= 1e-2
    assert rel_l2(x.cpu().numpy().reshape(x_ref.shape), x_ref) <= 5e-2
    got = img.cpu().numpy()
    assert np.isfinite(got).all()
    assert rel_l2(got, img_ref) <= 8e-2, rel_l2(got, img_ref)
    enc.close(); dec.close()


@pytest.mark.gpu
def test_video_diffuse_decode_chain_against_the_oracle_chain():
    """The video family: T denoising steps of a small model with self- and cross-attention blocks
    leave a [C][F][h][w] latent on the device, which the causal video decoder turns into frames
    (3 latent frames -> 5 frames), against the chain of the two float64 oracles."""
    import torch
    from oracle import video_decoder_oracle as V
    from paper_2510_02838_amd import binding as B, decoder as XD
    torch.cuda.set_device(0)
    arch = dict(family="W", n_blocks=2, n_single=0, hidden=256, n_heads=2, head_dim=128, mlp_hidden=768,
                latent_ch=16, patch=(1, 2, 2), cond_dim=128, rope_axes=(44, 42, 42), rope_theta=10000.0)
    reqs, steps = [(3, 16, 16, 40)], 4
    F, h, w, n_cond = reqs[0]
    dec_arch = synth.VIDEO_DECODERS["vae3d_tiny"]
    assert dec_arch["latent_ch"] == arch["latent_ch"]
    pd = synth.make_params(O.param_shapes(arch), 1, 0.06, 0.1, 0.2)
    pc = synth.make_params(V.param_shapes(dec_arch), 1, 0.012, 0.02, 0.1)
    lat, conds, sigmas = synth.make_inputs(reqs, arch["latent_ch"], arch["cond_dim"], steps, [3.0])

    dit = B.DiT(arch); dit.ensure_workspace(reqs, steps); dit.init_weights(0, 0.0); dit.set_params(pd)
    dec = XD.Decoder(dec_arch); dec.ensure_workspace(h, w, F); dec.init_weights(0, 0.0); dec.set_params(pc)
    x = torch.from_numpy(lat[0].astype(np.float32).ravel()).cuda()
    cond = torch.from_numpy(conds[0]).to(torch.bfloat16).cuda()
    dit.sample(reqs, x, cond, sigmas)
    up, Fo = dec.up_factor(), dec.frames_out(F)
    video = torch.full((Fo, h * up, w * up, 3), float("nan"), dtype=torch.float32, device="cuda")
    dec.forward(h, w, x, video, F)
    torch.cuda.synchronize()

    x_ref = O.DiTOracle(arch, pd).sample(lat[0], conds[0], sigmas[0])
    video_ref = V.VideoDecoderOracle(dec_arch, pc).forward(np.transpose(x_ref, (1, 2, 3, 0)))
    assert rel_l2(x.cpu().numpy().reshape(x_ref.shape), x_ref) <= 5e-2
    got = video.cpu().numpy()
    assert got.shape == video_ref.shape == (5, 64, 64, 3) and np.isfinite(got).all()
    assert rel_l2(got, video_ref) <= 8e-2, rel_l2(got, video_ref)
    dec.close()
