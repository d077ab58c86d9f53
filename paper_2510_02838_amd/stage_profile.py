#!/usr/bin/env python3
"""Offline profiler of the Diffuse stage on one MI355X (k = 1, no sequence parallelism).

Two tables measured through the library's dit_sample on seeded synthetic requests, and one
each for the stages before and after it:

  batch   same-shape dynamic batching (Appendix "Impact of Batch Size" / "Integration with
          Dynamic Batch"): step latency against batch size B per request shape, and the
          optimal batch size by the paper's rule: the largest B whose step latency is less
          than 20 % above that of B = 1.
  grid    per-request metadata of the offline profiler (Section "Profiler": expected running
          time and peak memory per request shape): seconds per denoising step, steps/s, and
          the bytes the stage holds for a request of that shape (weights + workspace), over
          a resolution grid of a workload family.

  encode  the Encode stage (T5-XXL-like text encoder): forward latency against the number of
          prompts per batch, per prompt length, with the same 20 % rule (the paper: the encoder
          "can be run with very large batches almost without slowing down").

    python -m paper_2510_02838_amd.stage_profile batch [--workload sd3] [--res 128,256,512] [--max-batch 32]
    python -m paper_2510_02838_amd.stage_profile grid  [--workload sd3|flux|wan] [--res ...]
  decode  the Decode stage (AutoencoderKL-style decoder): latency against the number of same-size
          latents per call, per image resolution, with the same 20 % rule; product flop rate and
          the bytes held (the paper: Encode and Decode are memory-bound and can reach a higher
          peak memory than Diffuse).

    python -m paper_2510_02838_amd.stage_profile encode [--encoder t5_xxl] [--lens 32,128,500] [--max-batch 64]
    python -m paper_2510_02838_amd.stage_profile decode [--decoder ae_kl] [--res 128,256,512,1024] [--max-batch 8]
    python -m paper_2510_02838_amd.stage_profile decode --decoder vae3d [--res 256x384,512x768] [--frames 1,5,13]
          (the causal video decoder, one video per call: latency against the number of latent frames)
    python -m paper_2510_02838_amd.stage_profile pipeline [--workload sd3|flux] [--res 512,1024] [--steps 28] [--overlap N]
    python -m paper_2510_02838_amd.stage_profile pipeline --workload wan --res 81x512x768 --steps 2   (video: causal video decoder)

  pipeline  one request through all three stages on this GPU, the output of each feeding the next
          (prompt tokens -> condition -> T denoising steps -> image): time per stage and its share
          of the request (the paper's stage-time breakdown: Diffuse dominates, Decode 15-30 %).
          --overlap N: then N requests back to back with the three stages on three HIP streams,
          request i's Decode and request i+2's Encode running beside request i+1's Diffuse
          (events hand the condition and the latent from stream to stream), against the same N
          requests stage after stage on one stream.

Resolutions are pixels; a latent is res/8 on a side and a patch 2x2, so tokens = (res/16)^2
plus the text tokens of the workload.  For the video family `--res` lists
frames x height x width in pixels (latent frames = (frames-1)/4 + 1).  Output: one JSON
line per table row, then a Markdown table on stderr.
"""
import argparse
import json
import sys
import time

import numpy as np


def _latent_dims(family_cfg, spec):
    """'512' -> (1, 32, 32); '81x480x832' -> (21, 60, 104)."""
    parts = [int(p) for p in str(spec).lower().split("x")]
    if len(parts) == 1:
        return (1, parts[0] // 8, parts[0] // 8)
    if len(parts) == 2:
        return (1, parts[0] // 8, parts[1] // 8)
    return ((parts[0] - 1) // 4 + 1, parts[1] // 8, parts[2] // 8)


def _tokens(arch, req):
    f, h, w, nc = req
    pt, ph, pw = arch["patch"]
    return (f // pt) * (h // ph) * (w // pw) + nc


class Stage:
    """One model instance; workspace grows to the largest request list seen."""

    def __init__(self, workload, steps, stream=None):
        import torch
        import synth
        from . import binding as B
        self.torch, self.synth = torch, synth
        self.cfg = synth.CONFIGS[workload]
        self.arch = self.cfg["arch"]
        self.n_cond = self.cfg["n_cond"]
        self.steps = steps
        self.m = B.DiT(self.arch, 0, stream=stream)
        self.ready = False

    def prepare(self, all_req_lists):
        """Binds a workspace large enough for every request list, then fills the weights."""
        need = max(self.m.workspace_bytes(r, self.steps) for r in all_req_lists)
        big = max(all_req_lists, key=lambda r: self.m.workspace_bytes(r, self.steps))
        assert need > 0
        self.m.ensure_workspace(big, self.steps)
        self.m.init_weights(1, 0.02)
        self.ready = True

    def time_steps(self, reqs, reps=3):
        """Best-of-`reps` wall time of one dit_sample of self.steps steps; returns s/step."""
        torch, synth, arch = self.torch, self.synth, self.arch
        lat, cond, _ = synth.make_inputs(reqs, arch["latent_ch"], arch["cond_dim"], 1, None)
        x0 = torch.from_numpy(np.concatenate([a.ravel() for a in lat])).cuda()
        dc = torch.from_numpy(np.concatenate([c.ravel() for c in cond])).cuda().to(torch.bfloat16)
        sg = np.stack([synth.default_sigmas(self.steps, 1.0)] * len(reqs))
        self.m.ensure_workspace(reqs, self.steps)
        x = x0.clone()
        self.m.sample(reqs, x, dc, sg)          # warm-up (plan upload, code load)
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(reps):
            x.copy_(x0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.m.sample(reqs, x, dc, sg)
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0)
        if not bool(torch.isfinite(x).all().item()):
            raise RuntimeError("non-finite latents")
        return best / self.steps


def optimal_batch(latency_by_b, slack=0.20):
    """Largest batch size whose latency is below (1 + slack) x the latency at B = 1."""
    base = latency_by_b[1]
    ok = [b for b, t in sorted(latency_by_b.items()) if t < (1.0 + slack) * base]
    return max(ok) if ok else 1


def run_batch(args):
    st = Stage(args.workload, args.steps)
    shapes = [_latent_dims(st.cfg, r) for r in args.res.split(",")]
    batches = [b for b in (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64) if b <= args.max_batch]
    lists = {(s, b): [(s[0], s[1], s[2], st.n_cond)] * b for s in shapes for b in batches}
    st.prepare(list(lists.values()))
    rows = []
    for s, res in zip(shapes, args.res.split(",")):
        lat = {}
        for b in batches:
            lat[b] = st.time_steps(lists[(s, b)])
            row = {"table": "batch", "workload": args.workload, "res": res, "tokens_per_request": _tokens(st.arch, lists[(s, 1)][0]),
                   "batch": b, "ms_per_step": lat[b] * 1e3, "latency_vs_b1": lat[b] / lat[1],
                   "request_steps_per_s": b / lat[b]}
            rows.append(row)
            print(json.dumps(row), flush=True)
        best = optimal_batch(lat)
        row = {"table": "batch_optimum", "workload": args.workload, "res": res, "optimal_batch": best,
               "rule": "largest B with step latency < 1.2 x latency(B=1)",
               "throughput_gain": (best / lat[best]) / (1 / lat[1])}
        rows.append(row)
        print(json.dumps(row), flush=True)
    hdr = "| res | tokens/request | " + " | ".join(f"B={b}" for b in batches) + " | optimal B |"
    print(hdr, file=sys.stderr)
    print("|" + "---|" * (len(batches) + 3), file=sys.stderr)
    for res in args.res.split(","):
        rr = [r for r in rows if r["table"] == "batch" and r["res"] == res]
        opt = [r for r in rows if r["table"] == "batch_optimum" and r["res"] == res][0]
        cells = " | ".join(f"{r['ms_per_step']:.2f} ms (x{r['latency_vs_b1']:.2f})" for r in rr)
        print(f"| {res} | {rr[0]['tokens_per_request']} | {cells} | {opt['optimal_batch']} |", file=sys.stderr)


def run_grid(args):
    st = Stage(args.workload, args.steps)
    specs = args.res.split(",")
    lists = [[_latent_dims(st.cfg, r) + (st.n_cond,)] for r in specs]
    st.prepare(lists)
    wbytes = st.m.weight_bytes()
    print("| request | tokens | s/step | steps/s | workspace GiB | weights GiB |", file=sys.stderr)
    print("|---|---|---|---|---|---|", file=sys.stderr)
    for spec, reqs in zip(specs, lists):
        t = st.time_steps(reqs, reps=2)
        ws = st.m.workspace_bytes(reqs, args.steps)
        row = {"table": "grid", "workload": args.workload, "request": spec, "latent": list(reqs[0][:3]),
               "tokens": _tokens(st.arch, reqs[0]), "s_per_step": t, "steps_per_s": 1.0 / t,
               "workspace_bytes": ws, "weight_bytes": wbytes, "k": 1}
        print(json.dumps(row), flush=True)
        print(f"| {spec} | {row['tokens']} | {t:.5f} | {1.0 / t:.2f} | {ws / 2**30:.3f} | {wbytes / 2**30:.2f} |", file=sys.stderr)


def run_encode(args):
    import torch
    import synth
    from . import encoder as X
    arch = synth.ENCODERS[args.encoder]
    lens_list = [int(v) for v in args.lens.split(",")]
    batches = [b for b in (1, 2, 4, 8, 16, 32, 64, 128) if b <= args.max_batch]
    m = X.Encoder(arch)
    m.ensure_workspace([max(lens_list)] * max(batches))
    m.init_weights(1, 0.02)
    wbytes = m.weight_bytes()
    floor_ms = wbytes / 8e12 * 1e3
    rows = []
    for n in lens_list:
        lat = {}
        for b in batches:
            lens = [n] * b
            toks = torch.from_numpy(np.concatenate(synth.make_tokens(lens, arch["vocab"]))).cuda()
            out = torch.empty((n * b, arch["d_model"]), dtype=torch.bfloat16, device="cuda")
            m.ensure_workspace(lens)
            m.forward(lens, toks, out, None)
            torch.cuda.synchronize()
            best = float("inf")
            for _ in range(3):
                t0 = time.perf_counter()
                m.forward(lens, toks, out, None)
                torch.cuda.synchronize()
                best = min(best, time.perf_counter() - t0)
            if not bool(torch.isfinite(out.float()).all().item()):
                raise RuntimeError("non-finite encoder output")
            lat[b] = best
            row = {"table": "encode", "encoder": args.encoder, "prompt_tokens": n, "batch": b, "ms": best * 1e3,
                   "latency_vs_b1": best / lat[1], "prompts_per_s": b / best, "tokens_per_s": b * n / best,
                   "weight_read_floor_ms": floor_ms}
            rows.append(row)
            print(json.dumps(row), flush=True)
        print(json.dumps({"table": "encode_optimum", "encoder": args.encoder, "prompt_tokens": n,
                          "optimal_batch": optimal_batch(lat), "rule": "largest B with latency < 1.2 x latency(B=1)"}), flush=True)
    print(f"weights {wbytes / 2**30:.2f} GiB: one pass over them takes {floor_ms:.2f} ms at 8 TB/s", file=sys.stderr)
    print("| prompt tokens | " + " | ".join(f"B={b}" for b in batches) + " | optimal B |", file=sys.stderr)
    print("|" + "---|" * (len(batches) + 2), file=sys.stderr)
    for n in lens_list:
        rr = [r for r in rows if r["prompt_tokens"] == n]
        lat = {r["batch"]: r["ms"] for r in rr}
        cells = " | ".join(f"{r['ms']:.2f} ms (x{r['latency_vs_b1']:.2f})" for r in rr)
        print(f"| {n} | {cells} | {optimal_batch(lat)} |", file=sys.stderr)


def decoder_flops(arch, h, w):
    """Multiply-add flops (2 per MAC) of the products of one decode of an h x w latent."""
    ch = arch["channels"]
    conv = lambda px, cin, cout, k: 2.0 * px * k * k * cin * cout
    res = lambda px, cin, cout: conv(px, cin, cout, 3) + conv(px, cout, cout, 3) + (conv(px, cin, cout, 1) if cin != cout else 0.0)
    px = h * w
    total = conv(px, arch["latent_ch"], ch[0], 3) + 2 * res(px, ch[0], ch[0])
    total += 4 * conv(px, ch[0], ch[0], 1) + 4.0 * px * px * ch[0]          # q, k, v, proj; scores and weighted sum
    prev = ch[0]
    for l, c in enumerate(ch):
        for r in range(arch["n_res"]):
            total += res(px, prev if r == 0 else c, c)
        prev = c
        if l != len(ch) - 1:
            px *= 4
            total += conv(px, c, c, 3)
    return total + conv(px, ch[-1], arch["out_ch"], 3)


def video_decoder_flops(arch, F, h, w):
    """Multiply-add flops (2 per MAC) of the products of one decode of F latent frames of h x w by
    the causal video decoder: 27 taps per 3x3x3 convolution, frame count doubling (2F - 1) at the
    first t_up level transitions."""
    ch = arch["channels"]
    conv = lambda px, cin, cout, taps: 2.0 * px * taps * cin * cout
    res = lambda px, cin, cout: conv(px, cin, cout, 27) + conv(px, cout, cout, 27) + (conv(px, cin, cout, 1) if cin != cout else 0.0)
    px = F * h * w
    total = conv(px, arch["latent_ch"], ch[0], 27) + 2 * res(px, ch[0], ch[0])
    total += 4 * conv(px, ch[0], ch[0], 1) + F * 4.0 * (h * w) ** 2 * ch[0]   # q, k, v, proj; per-frame scores and weighted sum
    prev = ch[0]
    for l, c in enumerate(ch):
        for r in range(arch["n_res"]):
            total += res(px, prev if r == 0 else c, c)
        prev = c
        if l != len(ch) - 1:
            if l < arch["t_up"]:
                F = 2 * F - 1
            h, w = 2 * h, 2 * w
            px = F * h * w
            total += conv(px, c, c, 27)
    return total + conv(px, ch[-1], arch["out_ch"], 27)


def run_decode_video(args):
    """One video per call: latency against the number of latent frames, per frame size."""
    import torch
    import synth
    from . import decoder as X
    arch = synth.VIDEO_DECODERS[args.decoder]
    m = X.Decoder(arch)
    f = m.up_factor()
    sizes = [tuple(int(v) // f for v in r.split("x")) for r in args.res.split(",")]
    frames = [int(v) for v in args.frames.split(",")]
    rows = []
    first = True
    for h, w in sizes:
        for F in frames:
            ws = m.workspace_bytes(h, w, F)
            if ws == 0:                                   # more than 128 output frames or 2^29 output pixels
                continue
            m.ensure_workspace(h, w, F)
            if first:
                m.init_weights(1, 0.02)
                first = False
            Fo = m.frames_out(F)
            z = torch.from_numpy(synth.gaussian(3, "video latent", arch["latent_ch"] * F * h * w).astype(np.float32)).cuda()
            out = torch.empty((Fo, h * f, w * f, arch["out_ch"]), dtype=torch.float32, device="cuda")
            m.forward(h, w, z, out, n=F)
            torch.cuda.synchronize()
            best = float("inf")
            for _ in range(3):
                t0 = time.perf_counter()
                m.forward(h, w, z, out, n=F)
                torch.cuda.synchronize()
                best = min(best, time.perf_counter() - t0)
            if not bool(torch.isfinite(out).all().item()):
                raise RuntimeError("non-finite video")
            fl = video_decoder_flops(arch, F, h, w)
            row = {"table": "decode_video", "decoder": args.decoder, "height": h * f, "width": w * f, "latent_frames": F,
                   "frames": Fo, "ms": best * 1e3, "ms_per_frame": best * 1e3 / Fo, "product_flops": fl,
                   "tflops": fl / best / 1e12, "workspace_bytes": ws, "weight_bytes": m.weight_bytes()}
            rows.append(row)
            print(json.dumps(row), flush=True)
            del z, out
    print("| video | latent frames -> frames | TFLOP | ms | TFLOP/s | ms per frame | workspace GiB |", file=sys.stderr)
    print("|---|---|---|---|---|---|---|", file=sys.stderr)
    for r in rows:
        print(f"| {r['height']}x{r['width']} | {r['latent_frames']} -> {r['frames']} | {r['product_flops'] / 1e12:.1f} | {r['ms']:.1f} | "
              f"{r['tflops']:.0f} | {r['ms_per_frame']:.2f} | {r['workspace_bytes'] / 2**30:.2f} |", file=sys.stderr)
    print(f"weights {m.weight_bytes() / 2**20:.0f} MiB", file=sys.stderr)


def run_decode(args):
    import torch
    import synth
    from . import decoder as X
    if args.decoder in synth.VIDEO_DECODERS:
        return run_decode_video(args)
    arch = synth.DECODERS[args.decoder]
    m = X.Decoder(arch)
    f = m.up_factor()
    sizes = [int(v) // f for v in args.res.split(",")]
    batches = [b for b in (1, 2, 4, 8, 16, 32) if b <= args.max_batch]
    rows = []
    first = True
    for n in sizes:
        lat = {}
        for b in batches:
            ws = m.workspace_bytes(n, n, b)
            if ws == 0:                                   # the batch form needs h*w % 256 == 0 and fewer than 2^29 output pixels
                continue
            m.ensure_workspace(n, n, b)
            if first:
                m.init_weights(1, 0.02)
                first = False
            z = torch.from_numpy(synth.gaussian(3, "latent", b * arch["latent_ch"] * n * n).astype(np.float32)).cuda()
            img = torch.empty((b, n * f, n * f, arch["out_ch"]), dtype=torch.float32, device="cuda")
            m.forward(n, n, z, img, n=b)
            torch.cuda.synchronize()
            best = float("inf")
            for _ in range(3):
                t0 = time.perf_counter()
                m.forward(n, n, z, img, n=b)
                torch.cuda.synchronize()
                best = min(best, time.perf_counter() - t0)
            if not bool(torch.isfinite(img).all().item()):
                raise RuntimeError("non-finite image")
            lat[b] = best
            fl = b * decoder_flops(arch, n, n)
            row = {"table": "decode", "decoder": args.decoder, "image": n * f, "latent": n, "batch": b, "ms": best * 1e3,
                   "latency_vs_b1": best / lat[1], "images_per_s": b / best, "product_flops": fl, "tflops": fl / best / 1e12,
                   "workspace_bytes": ws, "weight_bytes": m.weight_bytes()}
            rows.append(row)
            print(json.dumps(row), flush=True)
            del z, img
        print(json.dumps({"table": "decode_optimum", "decoder": args.decoder, "image": n * f, "optimal_batch": optimal_batch(lat),
                          "rule": "largest B with latency < 1.2 x latency(B=1)"}), flush=True)
    print("| image | latent | GFLOP/image | " + " | ".join(f"B={b}" for b in batches) + " | optimal B | workspace GiB (B=1) |", file=sys.stderr)
    print("|" + "---|" * (len(batches) + 5), file=sys.stderr)
    for n in sizes:
        rr = {r["batch"]: r for r in rows if r["latent"] == n}
        cells = " | ".join((f"{rr[b]['ms']:.2f} ms (x{rr[b]['latency_vs_b1']:.2f}, {rr[b]['tflops']:.0f} TF)" if b in rr else "-") for b in batches)
        print(f"| {n * f}x{n * f} | {n}x{n} | {decoder_flops(arch, n, n) / 1e9:.0f} | {cells} | "
              f"{optimal_batch({b: r['ms'] for b, r in rr.items()})} | {rr[1]['workspace_bytes'] / 2**30:.2f} |", file=sys.stderr)
    print(f"weights {m.weight_bytes() / 2**20:.0f} MiB", file=sys.stderr)


def run_pipeline(args):
    import torch
    import synth
    from . import encoder as XE, decoder as XD
    st = Stage(args.workload, args.steps)
    arch = st.arch
    video = arch["family"] == "W"            # video latents [C][F][h][w] go to the causal video decoder
    enc_arch = synth.ENCODERS["t5_xxl"]
    dec_arch = synth.VIDEO_DECODERS["vae3d"] if video else synth.DECODERS["ae_kl"]
    if arch["cond_dim"] != enc_arch["d_model"] or arch["latent_ch"] != dec_arch["latent_ch"] or arch["patch"][0] != 1:
        raise SystemExit("pipeline: the workload's condition width / latent channels do not match t5_xxl / the decoder")
    specs = args.res.split(",")
    reqs = [[_latent_dims(st.cfg, r) + (st.n_cond,)] for r in specs]
    st.prepare(reqs)
    enc = XE.Encoder(enc_arch)
    lens = [st.n_cond]
    enc.ensure_workspace(lens)
    enc.init_weights(1, 0.02)
    dec = XD.Decoder(dec_arch)
    big = max(reqs, key=lambda r: dec.workspace_bytes(r[0][1], r[0][2], r[0][0]))[0]
    if min(dec.workspace_bytes(r[0][1], r[0][2], r[0][0]) for r in reqs) == 0:
        raise SystemExit("pipeline: a frame size outside the decoder's limits (latent pixels a multiple of 64, of 256 for several frames)")
    dec.ensure_workspace(big[1], big[2], big[0])
    dec.init_weights(1, 0.02)
    f = dec.up_factor()
    nominal = st.cfg["steps"]                 # steps of a full request of this workload
    toks = torch.from_numpy(np.concatenate(synth.make_tokens(lens, enc_arch["vocab"]))).cuda()
    cond = torch.empty((st.n_cond, arch["cond_dim"]), dtype=torch.bfloat16, device="cuda")
    sg = np.stack([synth.default_sigmas(args.steps, 1.0)])

    def timed(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(reps):
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0)
        return best

    print(f"| image | tokens | encode ms | diffuse ms ({args.steps} steps) | decode ms | total ms | shares E / D / C |", file=sys.stderr)
    print("|---|---|---|---|---|---|---|", file=sys.stderr)
    for spec, rq in zip(specs, reqs):
        F, h, w, _ = rq[0]
        n = arch["latent_ch"] * F * h * w
        x0 = torch.from_numpy(synth.gaussian(2, "latent", n).astype(np.float32)).cuda()
        x = x0.clone()
        img = torch.empty((dec.frames_out(F), h * f, w * f, dec_arch["out_ch"]), dtype=torch.float32, device="cuda")
        st.m.ensure_workspace(rq, args.steps)
        t_e = timed(lambda: enc.forward(lens, toks, cond, None))

        def diffuse():
            x.copy_(x0)
            st.m.sample(rq, x, cond, sg)
        t_d = timed(diffuse, reps=1 if video else 3)
        t_c = timed(lambda: dec.forward(h, w, x, img, n=F))
        if not bool(torch.isfinite(img).all().item()):
            raise RuntimeError("non-finite image")
        tot = t_e + t_d + t_c
        row = {"table": "pipeline", "workload": args.workload, "image": spec, "tokens": _tokens(arch, rq[0]),
               "steps": args.steps, "encode_ms": t_e * 1e3, "diffuse_ms": t_d * 1e3, "decode_ms": t_c * 1e3,
               "share_encode": t_e / tot, "share_diffuse": t_d / tot, "share_decode": t_c / tot}
        if args.steps != nominal:             # the same stage times with the workload's own step count
            t_n = t_d * nominal / args.steps
            row.update({"nominal_steps": nominal, "share_encode_nominal": t_e / (t_e + t_n + t_c),
                        "share_diffuse_nominal": t_n / (t_e + t_n + t_c), "share_decode_nominal": t_c / (t_e + t_n + t_c)})
        print(json.dumps(row), flush=True)
        print(f"| {spec} | {row['tokens']} | {t_e * 1e3:.2f} | {t_d * 1e3:.1f} | {t_c * 1e3:.2f} | {tot * 1e3:.1f} | "
              f"{100 * t_e / tot:.1f} % / {100 * t_d / tot:.1f} % / {100 * t_c / tot:.1f} % |", file=sys.stderr)
        if args.steps != nominal:
            print(f"  (at the workload's {nominal} steps, diffuse time scaled from {args.steps}: "
                  f"{100 * row['share_encode_nominal']:.2f} % / {100 * row['share_diffuse_nominal']:.2f} % / {100 * row['share_decode_nominal']:.2f} %)", file=sys.stderr)
    if args.overlap:
        _overlap(args, specs[-1], reqs[-1])


def _overlap(args, spec, rq):
    """N requests of one shape: the three stages on three streams against one stream."""
    import torch
    import synth
    from . import encoder as XE, decoder as XD
    N = args.overlap
    enc_arch, dec_arch = synth.ENCODERS["t5_xxl"], synth.DECODERS["ae_kl"]
    _, h, w, n_cond = rq[0]
    results = {}
    for mode in ("one stream", "three streams"):
        streams = [torch.cuda.Stream() for _ in range(3)] if mode == "three streams" else [torch.cuda.Stream()] * 3
        se, sd, sc = streams
        st = Stage(args.workload, args.steps, stream=sd.cuda_stream)
        st.prepare([rq])
        arch = st.arch
        enc = XE.Encoder(enc_arch, stream=se.cuda_stream)
        enc.ensure_workspace([n_cond]); enc.init_weights(1, 0.02)
        dec = XD.Decoder(dec_arch, stream=sc.cuda_stream)
        dec.ensure_workspace(h, w); dec.init_weights(1, 0.02)
        f = dec.up_factor()
        toks = torch.from_numpy(np.concatenate(synth.make_tokens([n_cond], enc_arch["vocab"]))).cuda()
        sg = np.stack([synth.default_sigmas(args.steps, 1.0)])
        x0 = torch.from_numpy(synth.gaussian(2, "latent", arch["latent_ch"] * h * w).astype(np.float32)).cuda()
        # per-request buffers: a stage may run ahead of the next one
        conds = [torch.empty((n_cond, arch["cond_dim"]), dtype=torch.bfloat16, device="cuda") for _ in range(N)]
        xs = [x0.clone() for _ in range(N)]
        imgs = [torch.empty((h * f, w * f, dec_arch["out_ch"]), dtype=torch.float32, device="cuda") for _ in range(2)]
        torch.cuda.synchronize()

        def run():
            ev_e = [torch.cuda.Event() for _ in range(N)]
            ev_d = [torch.cuda.Event() for _ in range(N)]
            for i in range(N):
                enc.forward([n_cond], toks, conds[i], None)
                ev_e[i].record(se)
            for i in range(N):
                sd.wait_event(ev_e[i])
                st.m.sample(rq, xs[i], conds[i], sg)
                ev_d[i].record(sd)
                sc.wait_event(ev_d[i])
                dec.forward(h, w, xs[i], imgs[i % 2])
            torch.cuda.synchronize()

        run()                                          # warm-up
        for x in xs:
            x.copy_(x0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run()
        results[mode] = time.perf_counter() - t0
        if not bool(torch.isfinite(imgs[(N - 1) % 2]).all().item()):
            raise RuntimeError("non-finite image")
        del st, enc, dec
    row = {"table": "pipeline_overlap", "workload": args.workload, "image": spec, "requests": N,
           "one_stream_ms": results["one stream"] * 1e3, "three_streams_ms": results["three streams"] * 1e3,
           "requests_per_s_one": N / results["one stream"], "requests_per_s_three": N / results["three streams"]}
    print(json.dumps(row), flush=True)
    print(f"{N} requests of {spec}: one stream {results['one stream'] * 1e3:.1f} ms, three streams {results['three streams'] * 1e3:.1f} ms "
          f"({results['one stream'] / results['three streams']:.3f}x)", file=sys.stderr)


DEFAULT_RES = {
    ("batch", "sd3"): "128,256,512",
    ("batch", "flux"): "128,256,512",
    ("grid", "sd3"): "128,256,512,768,1024,1536",
    ("grid", "flux"): "128,256,512,1024,2048,4096",
    ("grid", "wan"): "17x480x832,49x480x832,81x480x832,81x720x1280",
}


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("table", choices=["batch", "grid", "encode", "decode", "pipeline"])
    ap.add_argument("--decoder", default="ae_kl", choices=["ae_kl", "ae_tiny", "vae3d", "vae3d_tiny"])
    ap.add_argument("--frames", default="1,5,13", help="decode with a video decoder: latent frames per video")
    ap.add_argument("--encoder", default="t5_xxl", choices=["t5_xxl", "t5_tiny"])
    ap.add_argument("--lens", default="32,128,500")
    ap.add_argument("--workload", default="sd3", choices=["sd3", "flux", "wan", "tiny"])
    ap.add_argument("--res", default=None)
    ap.add_argument("--steps", type=int, default=None, help="denoising steps per timed sample")
    ap.add_argument("--max-batch", type=int, default=None)
    ap.add_argument("--overlap", type=int, default=0, help="pipeline: also run N requests with the stages on three streams")
    args = ap.parse_args()
    if args.max_batch is None:
        args.max_batch = 64 if args.table == "encode" else 8 if args.table == "decode" else 32
    if args.table == "encode":
        return run_encode(args)
    if args.table == "decode":
        args.res = args.res or ("256x384,512x768" if args.decoder.startswith("vae3d") else "128,256,512,1024")
        return run_decode(args)
    if args.table == "pipeline":
        args.res = args.res or ("81x512x768" if args.workload == "wan" else "512,1024")
        args.steps = args.steps or (2 if args.workload == "wan" else 28)
        return run_pipeline(args)
    if args.res is None:
        args.res = DEFAULT_RES.get((args.table, args.workload))
        if args.res is None:
            ap.error("give --res for this table/workload")
    if args.steps is None:
        args.steps = 8 if args.table == "batch" else (1 if args.workload == "wan" else 4)
    (run_batch if args.table == "batch" else run_grid)(args)


if __name__ == "__main__":
    main()
