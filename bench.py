#!/usr/bin/env python3
"""Benchmark of the XQuant decode hot path on one MI355X.

One step = one decode step of one layer of the Llama-2-7B-shaped workload (config 2:
d=4096, 32x128 MHA, batch 8, context 4096, X cached 3-bit asym, group 128): quantise and
append the new token's X row (xq_quantize_append, T=1), then rematerialise K,V from the
packed cache and attend (xq_remat_attn_decode).  Inputs are seeded synthetic tensors that
are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E, published
# HBM-side bytes of one launch of the fused kernel on this workload: rocprofv3 FETCH_SIZE + WRITE_SIZE,
# each scaled by the factor that makes the counter read 256 MiB for a plain 256 MiB device copy
# (profiles/remat_attn_hbm_traffic.txt; counters cannot be read from inside this process, so this is a
# recorded constant: measured with the library built from the commit named here; remat_attn16.hip's tiling,
# which fixes the figure, has not changed since)
K3_HBM_BYTES_PER_LAUNCH = 2.18e9
K3_HBM_BYTES_MEASURED_AT = "d65b3cd"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--settle", type=int, default=40,
                    help="launches of the fused kernel during set-up, before the warm-up steps: from an idle GPU the clock "
                         "takes some 15 launches to settle (the first ones run 1.8 - 2.2 ms against 1.7), which a short "
                         "--warmup alone would put inside the timed steps; reported as config.settle_launches")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--cpu-pairs", type=int, default=96, help="(sequence, head) pairs the oracle times")
    ap.add_argument("--profile-copy", action="store_true",
                    help="also run one plain device copy of the 256 MiB X tensor (calibrates HBM byte counters)")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary kernels (profiling runs)")
    ap.add_argument("--profile-kernels", action="store_true",
                    help="after the timed loop also launch, three times each, the accumulator-source kernel on the c2 shape and "
                         "the fused kernel on the c4 (GQA) shape, so that one counter run covers all three (profiling runs)")
    ap.add_argument("--other-configs", action="store_true",
                    help="also time the fused kernel on the GQA (c4) and long-context (c5) shapes; reported under extra")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives); "
              f"--gpus {args.gpus} is not supported, use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2508_10395_amd as xq
    import xq_inputs as xi

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    xq.load_library()
    dev = "cuda"
    w = xi.C2
    B, L, d, Hq, Hkv, hd, bits, G = w.B, w.L, w.d, w.Hq, w.Hkv, w.hd, w.bits, w.G

    def dev_bf16(bits_u16):
        return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16)).view(torch.bfloat16).to(dev)

    # ---- seeded synthetic inputs, made on the host, resident in HBM before timing
    x_bits = xi.gen_x(w)                       # [B][L][d]
    wk_bits, wv_bits = xi.gen_weights(w)
    q_bits = xi.gen_q(w)
    x = dev_bf16(x_bits)
    q = dev_bf16(q_bits)
    attn = xq.XQAttn(Hq, Hkv, hd, hd ** -0.5)
    wprep = xq.xq_prepare_weights(attn, d, G, bits, dev_bf16(wk_bits), dev_bf16(wv_bits))
    cache = xq.alloc_cache(B, L, d, G, bits)
    xq.xq_quantize_append(cache, x[:, :L - 1].contiguous(), [0] * B)       # the L-1 cached tokens
    x_new = x[:, L - 1:L].contiguous()                                     # the decode step's token
    lens = [L] * B
    out = torch.empty((B, Hq, hd), dtype=torch.float32, device=dev)
    ws = torch.empty(xq.xq_remat_attn_workspace_bytes(attn, B, L, d, G), dtype=torch.uint8, device=dev)

    def step(ev=None):
        xq.xq_quantize_append(cache, x_new, [L - 1] * B)
        if ev is not None:
            ev[0].record()
        xq.xq_remat_attn_decode(attn, q, wprep, lens, xcache=cache, out=out, workspace=ws)
        if ev is not None:
            ev[1].record()

    for _ in range(args.settle):                 # set-up: bring the GPU to its clock under this load
        xq.xq_remat_attn_decode(attn, q, wprep, lens, xcache=cache, out=out, workspace=ws)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    remat_ms = sum(a.elapsed_time(b) for a, b in evs) / args.steps   # fused kernel + combine, on the launch stream

    from paper_2508_10395_amd import cost_model as cm
    tokens = B * L
    value = tokens / (ms_per_step * 1e-3)
    flops = cm.remat_attn_flops(tokens, d, Hq, Hkv, hd)                    # remat (Sec. 3.4) + attention
    achieved_tflops = flops / (remat_ms * 1e-3) / 1e12

    if args.profile_copy:
        y = torch.empty_like(x)
        y.copy_(x)
        torch.cuda.synchronize()
        del y

    if args.profile_kernels:
        wprep_d = xq.xq_prepare_weights(attn, d, 128, 16, dev_bf16(wk_bits), dev_bf16(wv_bits))
        for _ in range(3):
            xq.xq_remat_attn_decode(attn, q, wprep_d, lens, acc_bf16=x, out=out, workspace=ws)
        torch.cuda.synchronize()
        del wprep_d
        w4p = xi.C4
        a4p = xq.XQAttn(w4p.Hq, w4p.Hkv, w4p.hd, w4p.hd ** -0.5)
        gp = torch.Generator(device=dev).manual_seed(4)
        c4p = xq.alloc_cache(w4p.B, w4p.L, w4p.d, w4p.G, w4p.bits)
        for b0 in range(w4p.B):
            sub = xq.XQCache(c4p.codes[b0:b0 + 1], c4p.scale[b0:b0 + 1], c4p.zero[b0:b0 + 1], 1, w4p.L, w4p.d, w4p.G, w4p.bits)
            xq.xq_quantize_append(sub, torch.randn((1, w4p.L, w4p.d), device=dev, generator=gp).to(torch.bfloat16), [0])
        wk4p, wv4p = xi.gen_weights(w4p)
        wp4p = xq.xq_prepare_weights(a4p, w4p.d, w4p.G, w4p.bits, dev_bf16(wk4p), dev_bf16(wv4p))
        out4p = torch.empty((w4p.B, w4p.Hq, w4p.hd), dtype=torch.float32, device=dev)
        ws4p = torch.empty(xq.xq_remat_attn_workspace_bytes(a4p, w4p.B, w4p.L, w4p.d, w4p.G), dtype=torch.uint8, device=dev)
        q4p = dev_bf16(xi.gen_q(w4p))
        for _ in range(3):
            xq.xq_remat_attn_decode(a4p, q4p, wp4p, [w4p.L] * w4p.B, xcache=c4p, out=out4p, workspace=ws4p)
        torch.cuda.synchronize()
        del c4p, wp4p, ws4p

    # ---- secondary kernels of the path (reported, not part of `value`)
    def timed(fn, n=10, warm=2):
        for _ in range(warm):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    extra = None
    if not args.no_extra:
        n_el = B * L * d
        bulk_cache = xq.alloc_cache(B, L, d, G, bits)
        t_q = timed(lambda: xq.xq_quantize_append(bulk_cache, x, [0] * B))
        q_bytes = n_el * (2 + bits / 8 + 4 / G)
        acc = x.clone()
        t_acc = timed(lambda: xq.xq_cl_accumulate(acc, bulk_cache, lens, False))
        acc_bytes = n_el * (4 + bits / 8 + 4 / G)
        t_dq = timed(lambda: xq.xq_cl_delta_quantize(bulk_cache, x, acc, [0] * B))
        dq_bytes = n_el * (4 + bits / 8 + 4 / G)
        wprep_dense = xq.xq_prepare_weights(attn, d, 128, 16, dev_bf16(wk_bits), dev_bf16(wv_bits))
        t_dense = timed(lambda: xq.xq_remat_attn_decode(attn, q, wprep_dense, lens, acc_bf16=x, out=out, workspace=ws),
                        n=5, warm=1)
        t_app = timed(lambda: xq.xq_quantize_append(cache, x_new, [L - 1] * B), n=20)
        inv = 10000.0 ** (-torch.arange(hd // 2, dtype=torch.float64) * 2.0 / hd)
        ang = torch.arange(L, dtype=torch.float64)[:, None] * inv[None, :]
        rope = torch.stack([torch.cos(ang), torch.sin(ang)], dim=-1).to(torch.float32).to(dev)
        t_rope = timed(lambda: xq.xq_remat_attn_decode(attn, q, wprep, lens, xcache=cache, out=out, workspace=ws,
                                                       rope_cos_sin=rope), n=10, warm=5)
        # a chunk of 32 new tokens per sequence attending causally to the same cache (chunked prefill)
        Tq = 32
        gen_q = torch.Generator(device=dev).manual_seed(32)
        q_chunk = torch.randn((w.B, Tq, w.Hq, w.hd), device=dev, generator=gen_q).to(torch.bfloat16)
        ws_chunk = torch.empty(xq.xq_remat_attn_prefill_workspace_bytes(attn, w.B, Tq, w.L, w.d, w.G), dtype=torch.uint8,
                               device=dev)
        out_chunk = torch.empty((w.B, Tq, w.Hq, w.hd), dtype=torch.float32, device=dev)
        t_chunk = timed(lambda: xq.xq_remat_attn_prefill(attn, q_chunk, wprep, lens, xcache=cache, out=out_chunk,
                                                         workspace=ws_chunk), n=10, warm=5)
        del ws_chunk, out_chunk
        # the same layer from a per-channel cache (groups of 128 tokens per channel, Sec. 3.3.1) with 77 tokens in
        # the bf16 residual window, and the block quantiser that fills it
        pc_cache = xq.alloc_cache_per_channel(w.B, w.L, w.d, 128, w.bits)
        t_pcq = timed(lambda: xq.xq_quantize_blocks_per_channel(pc_cache, x, [0] * w.B), n=10)
        pcq_bytes = w.B * w.L * w.d * (2 + w.bits / 8.0)
        pc_tail = x[:, L - 128:].contiguous()
        wprep_pc = xq.xq_prepare_weights(attn, w.d, 128, w.bits, dev_bf16(wk_bits), dev_bf16(wv_bits))
        ws_pc = torch.empty(xq.xq_remat_attn_per_channel_workspace_bytes(attn, w.B, w.L, w.d, 128), dtype=torch.uint8,
                            device=dev)
        pc_lens = [w.L - 51] * w.B
        t_pc = timed(lambda: xq.xq_remat_attn_decode_per_channel(attn, q, pc_cache, pc_tail, pc_lens, wprep_pc, wprep_dense,
                                                                 out=out, workspace=ws_pc), n=10, warm=5)
        # the per-block terms kept in the caller's buffer: computed by one call, read by the steps between two
        # block completions (127 of 128 steps)
        pc_terms = xq.alloc_per_channel_terms(pc_cache, w.Hkv)
        xq.xq_remat_attn_decode_per_channel(attn, q, pc_cache, pc_tail, pc_lens, wprep_pc, wprep_dense, out=out,
                                            workspace=ws_pc, terms=pc_terms, terms_valid=False)
        t_pc_kept = timed(lambda: xq.xq_remat_attn_decode_per_channel(attn, q, pc_cache, pc_tail, pc_lens, wprep_pc,
                                                                      wprep_dense, out=out, workspace=ws_pc, terms=pc_terms,
                                                                      terms_valid=True), n=10, warm=5)
        del pc_cache, ws_pc, wprep_pc, pc_tail, pc_terms
        extra = {
            "remat_attn_per_channel": {"workload": "c2 shape, per-channel groups of 128 tokens, 3-bit, 31 blocks + 77 window "
                                                   "tokens per sequence; includes the per-step pre-passes", "ms": t_pc,
                                       "tokens/s/layer": w.B * (w.L - 51) / (t_pc * 1e-3),
                                       "ms_with_kept_block_terms": t_pc_kept,
                                       "tokens/s/layer_with_kept_block_terms": w.B * (w.L - 51) / (t_pc_kept * 1e-3)},
            "quantize_blocks_per_channel": {"workload": "xq_quantize_blocks_per_channel, 32 blocks of 128 tokens per sequence",
                                            "ms": t_pcq, "GB/s": pcq_bytes / t_pcq / 1e6,
                                            "frac_hbm_peak": pcq_bytes / t_pcq / 1e6 / PEAK_HBM_GBS},
            "remat_attn_prefill_chunk32_ms": t_chunk,
            "quantize_bulk": {"workload": "xq_quantize_append T=4096 (whole context), c2 shape", "ms": t_q,
                              "GB/s": q_bytes / t_q / 1e6, "frac_hbm_peak": q_bytes / t_q / 1e6 / PEAK_HBM_GBS},
            "quantize_decode_append_us": t_app * 1e3,
            "cl_accumulate": {"workload": "xq_cl_accumulate over [8][4096][4096] bf16 acc, 3-bit deltas", "ms": t_acc,
                              "GB/s": acc_bytes / t_acc / 1e6, "frac_hbm_peak": acc_bytes / t_acc / 1e6 / PEAK_HBM_GBS},
            "cl_delta_quantize_bulk": {"ms": t_dq, "GB/s": dq_bytes / t_dq / 1e6,
                                       "frac_hbm_peak": dq_bytes / t_dq / 1e6 / PEAK_HBM_GBS},
            "remat_attn_with_rope_ms": t_rope,
            "remat_attn_dense_acc": {"workload": "XQuant-CL source (bf16 accumulator), c2 shape", "ms": t_dense,
                                     "TFLOP/s": flops / t_dense / 1e9,
                                     "frac_mfma_peak": flops / t_dense / 1e9 / PEAK_BF16_TFLOPS},
        }

    if extra is not None:
        # ---- the other workloads, compact forms that fit the default run (the long forms are behind --other-configs).
        # Their inputs are drawn on the device (seeded torch generator; N(0,1) with the workload's outlier channels
        # scaled), since only the timing is taken here: parity at these shapes is what the GPU tests cover.
        del bulk_cache, acc
        torch.cuda.empty_cache()
        gen_o = torch.Generator(device=dev).manual_seed(2508)

        def device_x(ow, rows):
            t = torch.randn((1, rows, ow.d), device=dev, generator=gen_o)
            oc = xi.outlier_channels(ow)
            if len(oc):
                t[..., torch.from_numpy(oc).to(dev)] *= ow.outlier_factor
            return t.to(torch.bfloat16)

        def filled_cache(ow, group, bits_):
            c_ = xq.alloc_cache(ow.B, ow.L, ow.d, group, bits_)
            for b0 in range(ow.B):                       # one sequence at a time (the fp32 draw is 4 bytes per element)
                sub = xq.XQCache(c_.codes[b0:b0 + 1], c_.scale[b0:b0 + 1], c_.zero[b0:b0 + 1], 1, ow.L, ow.d, group, bits_)
                xq.xq_quantize_append(sub, device_x(ow, ow.L), [0])
            return c_

        def remat_entry(ms, ow, fl):
            return {"ms": ms, "tokens/s/layer": ow.B * ow.L / (ms * 1e-3), "TFLOP/s": fl / ms / 1e9,
                    "frac_mfma_peak": fl / ms / 1e9 / PEAK_BF16_TFLOPS}

        # config 2 again, cycling through 8 distinct layers (8 X caches + 8 weight streams = 1.0 GB, four times the
        # 256 MB Infinity Cache), so that no layer finds its cache or weights where its last visit left them
        n_rot = 8
        rot_caches, rot_streams = [], []
        for l in range(n_rot):
            c_ = xq.alloc_cache(B, L, d, G, bits)
            xq.xq_quantize_append(c_, torch.roll(x, shifts=l * 37 + 1, dims=1), [0] * B)
            rot_caches.append(c_)
            wk_l, wv_l = xi.gen_weights(w, layer=l + 1)
            rot_streams.append(xq.xq_prepare_weights(attn, d, G, bits, dev_bf16(wk_l), dev_bf16(wv_l)))

        def rotate():
            for l in range(n_rot):
                xq.xq_remat_attn_decode(attn, q, rot_streams[l], lens, xcache=rot_caches[l], out=out, workspace=ws)

        t_rot = timed(rotate, n=5, warm=2) / n_rot
        extra["remat_attn_c2_rotating_8_layers"] = dict(
            remat_entry(t_rot, w, flops),
            workload="c2, xq_remat_attn_decode over 8 distinct layers in turn (caches + weight streams 1.0 GB); ms per layer",
            ratio_to_single_layer=t_rot / remat_ms)
        del rot_caches, rot_streams
        torch.cuda.empty_cache()

        # The same launch (same cache, same instruction stream) with other weight VALUES: all weights zero, and all
        # weights one constant.  The matrix pipe's power draw depends on the bits that toggle in its operands and the
        # GPU lowers its clock under it, so this separates what the kernel's structure allows from what the data costs.
        dep = {}
        for tag, fillv in (("all_zero", 0.0), ("all_equal", 2.0 ** -6)):
            wc = torch.full((d, Hkv * hd), fillv, dtype=torch.bfloat16, device=dev)
            wpc = xq.xq_prepare_weights(attn, d, G, bits, wc, wc)
            t_w = timed(lambda: xq.xq_remat_attn_decode(attn, q, wpc, lens, xcache=cache, out=out, workspace=ws), n=20, warm=10)
            dep[tag + "_ms"] = t_w
            dep[tag + "_frac_mfma_peak"] = flops / t_w / 1e9 / PEAK_BF16_TFLOPS
            del wc, wpc
        dep["workload_weights_ms"] = remat_ms
        dep["note"] = ("xq_remat_attn_decode on c2 with the workload's N(0, 1/d) weights against the same call with constant "
                       "weights: identical work and instruction stream, the time follows the operand data (clock under load)")
        extra["remat_attn_c2_weight_data_dependence"] = dep

        # config 4 (GQA, B=16, L=8192, 2-bit, group 64): the naive X cache, and the latent cache of Sec. 3.3.1
        w4 = xi.C4
        a4 = xq.XQAttn(w4.Hq, w4.Hkv, w4.hd, w4.hd ** -0.5)
        q4 = dev_bf16(xi.gen_q(w4))
        out4 = torch.empty((w4.B, w4.Hq, w4.hd), dtype=torch.float32, device=dev)
        lens4 = [w4.L] * w4.B
        wk4, wv4 = xi.gen_weights(w4)
        wp4 = xq.xq_prepare_weights(a4, w4.d, w4.G, w4.bits, dev_bf16(wk4), dev_bf16(wv4))
        c4 = filled_cache(w4, w4.G, w4.bits)
        ws4 = torch.empty(xq.xq_remat_attn_workspace_bytes(a4, w4.B, w4.L, w4.d, w4.G), dtype=torch.uint8, device=dev)
        t_c4 = timed(lambda: xq.xq_remat_attn_decode(a4, q4, wp4, lens4, xcache=c4, out=out4, workspace=ws4), n=10, warm=5)
        extra["remat_attn_c4_gqa_naive"] = dict(remat_entry(t_c4, w4, cm.remat_attn_flops(w4.B * w4.L, w4.d, w4.Hq, w4.Hkv, w4.hd)),
                                                workload="c4: B=16, L=8192, d=4096, 32 query / 8 KV heads, X cache 2-bit group 64")
        del c4, wp4, ws4
        r4 = w4.Hkv * w4.hd
        lat4 = xq.alloc_cache(w4.B, w4.L, 2 * r4, w4.G, w4.bits)
        for b0 in range(w4.B):
            sub = xq.XQCache(lat4.codes[b0:b0 + 1], lat4.scale[b0:b0 + 1], lat4.zero[b0:b0 + 1], 1, w4.L, 2 * r4, w4.G, w4.bits)
            xq.xq_quantize_append(sub, torch.randn((1, w4.L, 2 * r4), device=dev, generator=gen_o).to(torch.bfloat16), [0])
        wfk4 = (torch.randn((r4, r4), device=dev, generator=gen_o) * r4 ** -0.5).to(torch.bfloat16)
        wfv4 = (torch.randn((r4, r4), device=dev, generator=gen_o) * r4 ** -0.5).to(torch.bfloat16)
        lwp4 = xq.xq_prepare_weights_latent(a4, r4, w4.G, w4.bits, wfk4, wfv4)
        lws4 = torch.empty(xq.xq_remat_attn_latent_workspace_bytes(a4, w4.B, w4.L, r4, w4.G), dtype=torch.uint8, device=dev)
        t_l4 = timed(lambda: xq.xq_remat_attn_decode_latent(a4, q4, lwp4, lens4, lat4, out=out4, workspace=lws4), n=10, warm=5)
        lfl4 = 2.0 * w4.B * w4.L * r4 * (2 * r4) + 4.0 * w4.B * w4.L * w4.Hq * w4.hd
        extra["remat_attn_c4_gqa_latent"] = dict(
            remat_entry(t_l4, w4, lfl4),
            workload="c4 layer served from the latent cache [X Uk | X Uv] (r=1024, width 2048, 2-bit, group 64); random latent "
                     "rows and fused matrices; TFLOP/s counts the latent contraction 2*M*r*2r")
        del lat4, lwp4, lws4, wfk4, wfv4
        torch.cuda.empty_cache()

        # config 5 (B=4, 2-bit, group 128): one decode step at the full context of 32768 rows
        w5 = xi.C5
        a5 = xq.XQAttn(w5.Hq, w5.Hkv, w5.hd, w5.hd ** -0.5)
        c5 = filled_cache(w5, w5.G, w5.bits)
        wk5, wv5 = xi.gen_weights(w5)
        wp5 = xq.xq_prepare_weights(a5, w5.d, w5.G, w5.bits, dev_bf16(wk5), dev_bf16(wv5))
        q5 = dev_bf16(xi.gen_q(w5))
        out5 = torch.empty((w5.B, w5.Hq, w5.hd), dtype=torch.float32, device=dev)
        ws5 = torch.empty(xq.xq_remat_attn_workspace_bytes(a5, w5.B, w5.L, w5.d, w5.G), dtype=torch.uint8, device=dev)
        x5 = device_x(w5, 1).expand(w5.B, 1, w5.d).contiguous()

        def c5_step():
            xq.xq_quantize_append(c5, x5, [w5.L - 1] * w5.B)
            xq.xq_remat_attn_decode(a5, q5, wp5, [w5.L] * w5.B, xcache=c5, out=out5, workspace=ws5)

        t_5 = timed(c5_step, n=5, warm=2)
        extra["decode_step_c5_long_context"] = dict(
            remat_entry(t_5, w5, cm.remat_attn_flops(w5.B * w5.L, w5.d, w5.Hq, w5.Hkv, w5.hd)),
            workload="c5: B=4, context 32768, d=4096 MHA, 2-bit group 128; append 1 token per sequence + attend")
        del c5, wp5, ws5
        torch.cuda.empty_cache()

        # config 3 (XQuant-CL, B=8, L=8192, MHA): 4 of the 32 layers of one decode step -- per layer, merge the layer's
        # 2-bit delta cache into the bf16 accumulator, then attend from the accumulator with the layer's weights
        w3 = xi.C3
        a3 = xq.XQAttn(w3.Hq, w3.Hkv, w3.hd, w3.hd ** -0.5)
        n3 = 4
        acc3 = torch.empty((w3.B, w3.L, w3.d), dtype=torch.bfloat16, device=dev)
        for b0 in range(w3.B):
            acc3[b0:b0 + 1] = device_x(w3, w3.L)
        deltas3, streams3 = [], []
        for l in range(n3):
            dcl = xq.alloc_cache(w3.B, w3.L, w3.d, w3.G, w3.delta_bits)
            for b0 in range(w3.B):                      # the layer's true delta N(0, 0.1), quantised against a zero accumulator
                sub = xq.XQCache(dcl.codes[b0:b0 + 1], dcl.scale[b0:b0 + 1], dcl.zero[b0:b0 + 1], 1, w3.L, w3.d, w3.G, w3.delta_bits)
                step_ = (torch.randn((1, w3.L, w3.d), device=dev, generator=gen_o) * w3.delta_var ** 0.5).to(torch.bfloat16)
                xq.xq_quantize_append(sub, step_, [0])
            deltas3.append(dcl)
            wk3, wv3 = xi.gen_weights(w3, layer=l)
            streams3.append(xq.xq_prepare_weights(a3, w3.d, 0, 16, dev_bf16(wk3), dev_bf16(wv3)))
        q3 = dev_bf16(xi.gen_q(w3))
        out3 = torch.empty((w3.B, w3.Hq, w3.hd), dtype=torch.float32, device=dev)
        ws3 = torch.empty(xq.xq_remat_attn_workspace_bytes(a3, w3.B, w3.L, w3.d, 0), dtype=torch.uint8, device=dev)
        lens3 = [w3.L] * w3.B
        t_a3 = timed(lambda: [xq.xq_cl_accumulate(acc3, deltas3[l], lens3, False) for l in range(n3)], n=3, warm=1) / n3

        def cl_layers():
            for l in range(n3):
                xq.xq_cl_accumulate(acc3, deltas3[l], lens3, False)
                xq.xq_remat_attn_decode(a3, q3, streams3[l], lens3, acc_bf16=acc3, out=out3, workspace=ws3)

        t_3 = timed(cl_layers, n=3, warm=1) / n3
        fl3 = cm.remat_attn_flops(w3.B * w3.L, w3.d, w3.Hq, w3.Hkv, w3.hd)
        acc3_bytes = w3.B * w3.L * w3.d * cm.cl_accumulate_bytes_per_element(w3.delta_bits, w3.G)
        extra["cl_decode_c3_4_layers"] = {
            "workload": "c3: B=8, L=8192, d=4096 MHA, 2-bit deltas group 128; 4 distinct layers of one XQuant-CL decode step "
                        "(accumulate the layer's delta cache, attend from the accumulator); per layer",
            "ms_per_layer": t_3, "tokens/s/layer": w3.B * w3.L / (t_3 * 1e-3),
            "accumulate_ms": t_a3, "accumulate_GB/s": acc3_bytes / t_a3 / 1e6,
            "accumulate_frac_hbm_peak": acc3_bytes / t_a3 / 1e6 / PEAK_HBM_GBS,
            "remat_attn_ms": t_3 - t_a3, "remat_attn_frac_mfma_peak": fl3 / (t_3 - t_a3) / 1e9 / PEAK_BF16_TFLOPS}
        del deltas3, streams3, acc3, ws3
        torch.cuda.empty_cache()

    if args.other_configs and extra is not None:
        del wprep_dense
        torch.cuda.empty_cache()
        for ow in (xi.C4, xi.C5):
            oq = dev_bf16(xi.gen_q(ow))
            owk, owv = xi.gen_weights(ow)
            oattn = xq.XQAttn(ow.Hq, ow.Hkv, ow.hd, ow.hd ** -0.5)
            owp = xq.xq_prepare_weights(oattn, ow.d, ow.G, ow.bits, dev_bf16(owk), dev_bf16(owv))
            ocache = xq.alloc_cache(ow.B, ow.L, ow.d, ow.G, ow.bits)
            for b0 in range(ow.B):                       # fill one sequence at a time (host memory)
                one = ow.scaled(B=1, cfg_id=ow.cfg_id * 100 + b0)
                sub = xq.XQCache(ocache.codes[b0:b0 + 1], ocache.scale[b0:b0 + 1], ocache.zero[b0:b0 + 1],
                                 1, ow.L, ow.d, ow.G, ow.bits)
                xq.xq_quantize_append(sub, dev_bf16(xi.gen_x(one)), [0])
            oout = torch.empty((ow.B, ow.Hq, ow.hd), dtype=torch.float32, device=dev)
            ows = torch.empty(xq.xq_remat_attn_workspace_bytes(oattn, ow.B, ow.L, ow.d, ow.G), dtype=torch.uint8,
                              device=dev)
            olens = [ow.L] * ow.B
            t_o = timed(lambda: xq.xq_remat_attn_decode(oattn, oq, owp, olens, xcache=ocache, out=oout, workspace=ows),
                        n=10, warm=12)    # (from an idle GPU the clock takes some 10 launches to settle)
            oflops = 2.0 * ow.B * ow.L * ow.d * (2 * ow.Hkv * ow.hd) + 4.0 * ow.B * ow.L * ow.Hq * ow.hd
            extra["remat_attn_" + ow.name] = {"ms": t_o, "tokens/s/layer": ow.B * ow.L / (t_o * 1e-3),
                                              "TFLOP/s": oflops / t_o / 1e9,
                                              "frac_mfma_peak": oflops / t_o / 1e9 / PEAK_BF16_TFLOPS}
            del ocache, owp, ows
        # the same GQA layer served from the latent cache [X Uk | X Uv] (Sec. 3.3.1): r = 1024, cache width 2048
        ow = xi.C4
        r = ow.Hkv * ow.hd
        oattn = xq.XQAttn(ow.Hq, ow.Hkv, ow.hd, ow.hd ** -0.5)
        gen = torch.Generator(device=dev).manual_seed(4)
        lat = torch.randn((ow.B, ow.L, 2 * r), device=dev, generator=gen).to(torch.bfloat16)
        lcache = xq.alloc_cache(ow.B, ow.L, 2 * r, ow.G, ow.bits)
        xq.xq_quantize_append(lcache, lat, [0] * ow.B)
        wfk = (torch.randn((r, r), device=dev, generator=gen) * r ** -0.5).to(torch.bfloat16)
        wfv = (torch.randn((r, r), device=dev, generator=gen) * r ** -0.5).to(torch.bfloat16)
        lwp = xq.xq_prepare_weights_latent(oattn, r, ow.G, ow.bits, wfk, wfv)
        lws = torch.empty(xq.xq_remat_attn_latent_workspace_bytes(oattn, ow.B, ow.L, r, ow.G), dtype=torch.uint8, device=dev)
        oq = dev_bf16(xi.gen_q(ow))
        oout = torch.empty((ow.B, ow.Hq, ow.hd), dtype=torch.float32, device=dev)
        olens = [ow.L] * ow.B
        t_l = timed(lambda: xq.xq_remat_attn_decode_latent(oattn, oq, lwp, olens, lcache, out=oout, workspace=lws),
                    n=10, warm=12)    # (from an idle GPU the clock takes some 10 launches to settle)
        lflops = 2.0 * ow.B * ow.L * r * (2 * r) + 4.0 * ow.B * ow.L * ow.Hq * ow.hd
        ut = (torch.randn((2 * r, ow.d), device=dev, generator=gen) * ow.d ** -0.5).to(torch.bfloat16)
        xnew = torch.randn((ow.B, 1, ow.d), device=dev, generator=gen).to(torch.bfloat16)
        t_p = timed(lambda: xq.xq_latent_project(xnew, ut), n=20)
        extra["remat_attn_c4_latent"] = {"workload": "c4 layer from the latent cache (r=1024, width 2048, 2-bit, group 64); "
                                                     "random latent rows and fused matrices (timing only)",
                                         "ms": t_l, "tokens/s/layer": ow.B * ow.L / (t_l * 1e-3),
                                         "useful_TFLOP/s": lflops / t_l / 1e9,
                                         "decode_projection_us": t_p * 1e3}
        # the paper's setting for this layer: X Uk per channel (blocks of 128 tokens, 100 of the newest in the bf16
        # window), X Uv per token
        kc = xq.alloc_cache_per_channel(ow.B, ow.L, r, 128, ow.bits)
        xq.xq_quantize_blocks_per_channel(kc, lat[..., :r].contiguous(), [0] * ow.B)
        vc = xq.alloc_cache(ow.B, ow.L, r, ow.G, ow.bits)
        xq.xq_quantize_append(vc, lat[..., r:].contiguous(), [0] * ow.B)
        ktail = lat[:, ow.L - 128:, :r].contiguous()
        wkc = xq.xq_prepare_weights_pairs(oattn, r, 128, ow.bits, wfk)
        wkd = xq.xq_prepare_weights_pairs(oattn, r, 0, 16, wfk)
        wvc = xq.xq_prepare_weights_pairs(oattn, r, ow.G, ow.bits, wfv)
        pws = torch.empty(xq.xq_remat_attn_latent_per_channel_workspace_bytes(oattn, ow.B, ow.L, r, 128, ow.G),
                          dtype=torch.uint8, device=dev)
        plens = [ow.L - 28] * ow.B
        t_lp = timed(lambda: xq.xq_remat_attn_decode_latent_per_channel(oattn, oq, kc, ktail, vc, wkc, wkd, wvc, plens,
                                                                        out=oout, workspace=pws), n=5, warm=3)
        kterms = xq.alloc_per_channel_terms(kc, ow.Hkv // 2)
        xq.xq_remat_attn_decode_latent_per_channel(oattn, oq, kc, ktail, vc, wkc, wkd, wvc, plens, out=oout, workspace=pws,
                                                   terms=kterms, terms_valid=False)
        t_lpk = timed(lambda: xq.xq_remat_attn_decode_latent_per_channel(oattn, oq, kc, ktail, vc, wkc, wkd, wvc, plens,
                                                                         out=oout, workspace=pws, terms=kterms,
                                                                         terms_valid=True), n=5, warm=3)
        # App. B: the first channel of X Uk in fp16 (its share of the scores is added between the passes; the zeroed row
        # 0 of the key streams does not change the timing, so the same streams serve here)
        k0 = lat[:, :, 0].to(torch.float16).contiguous()
        w_row0 = wfk[0].contiguous()
        t_lpo = timed(lambda: xq.xq_remat_attn_decode_latent_per_channel(oattn, oq, kc, ktail, vc, wkc, wkd, wvc, plens,
                                                                         out=oout, workspace=pws, terms=kterms,
                                                                         terms_valid=True, k0_f16=k0, wk_row0=w_row0),
                      n=5, warm=3)
        extra["remat_attn_c4_latent_keys_per_channel"] = {
            "workload": "c4 layer, X Uk per channel (2-bit, blocks of 128, 100 window tokens), X Uv per token (2-bit, group 64)",
            "ms": t_lp, "tokens/s/layer": ow.B * (ow.L - 28) / (t_lp * 1e-3), "ms_with_kept_block_terms": t_lpk,
            "ms_with_kept_block_terms_and_fp16_outlier_channel": t_lpo}
        del k0, w_row0
        del kc, vc, ktail, wkc, wkd, wvc, pws, kterms
        del lcache, lat, lwp, lws
        # the cross-layer step of the same GQA layer (Sec. 3.3.2): latent delta of the new token, quantise,
        # up-project every cached delta into the accumulator, attend from the accumulator with [Wk | Wv]
        n_lat = 2 * r
        dcache = xq.alloc_cache(ow.B, ow.L, n_lat, ow.G, ow.bits)
        dl = (torch.randn((ow.B, ow.L, n_lat), device=dev, generator=gen) * 0.3).to(torch.bfloat16)
        xq.xq_quantize_append(dcache, dl, [0] * ow.B)
        del dl
        uprep = xq.xq_prepare_upproject(ow.d, ow.G, ow.bits, ut)
        oacc = torch.randn((ow.B, ow.L, ow.d), device=dev, generator=gen).to(torch.bfloat16)
        uws = torch.empty(xq.xq_cl_accumulate_latent_workspace_bytes(ow.B, ow.L, n_lat, ow.G), dtype=torch.uint8,
                          device=dev)
        t_u = timed(lambda: xq.xq_cl_accumulate_latent(oacc, dcache, uprep, olens, workspace=uws), n=5, warm=5)
        dlat = torch.empty((ow.B, 1, n_lat), dtype=torch.bfloat16, device=dev)
        t_d = timed(lambda: xq.xq_cl_latent_delta_project(xnew, oacc, ut, [ow.L - 1] * ow.B, out=dlat), n=20)
        owk, owv = xi.gen_weights(ow)
        dwp = xq.xq_prepare_weights(oattn, ow.d, 0, 16, dev_bf16(owk), dev_bf16(owv))
        dws = torch.empty(xq.xq_remat_attn_workspace_bytes(oattn, ow.B, ow.L, ow.d, 0), dtype=torch.uint8, device=dev)
        t_a = timed(lambda: xq.xq_remat_attn_decode(oattn, oq, dwp, olens, acc_bf16=oacc, out=oout, workspace=dws),
                    n=10, warm=12)    # (from an idle GPU the clock takes some 10 launches to settle)
        # prefill-sized projections on the matrix cores: a chunk of 1024 new tokens per sequence into the latent
        # space, plain (Sec. 3.3.1) and as the cross-layer delta against the accumulator (Sec. 3.3.2)
        Tb = 1024
        xchunk = torch.randn((ow.B, Tb, ow.d), device=dev, generator=gen).to(torch.bfloat16)
        proj = xq.xq_prepare_projection(ut)
        blat = torch.empty((ow.B, Tb, n_lat), dtype=torch.bfloat16, device=dev)
        t_pb = timed(lambda: xq.xq_latent_project_bulk(xchunk.view(ow.B * Tb, ow.d), proj, n_lat,
                                                       out=blat.view(ow.B * Tb, n_lat)), n=10, warm=3)
        t_db = timed(lambda: xq.xq_cl_latent_delta_project_bulk(xchunk, oacc, proj, n_lat, [ow.L - Tb] * ow.B, out=blat),
                     n=10, warm=3)
        pflops = 2.0 * ow.B * Tb * ow.d * n_lat
        extra["latent_projection_bulk_c4"] = {
            "workload": "16 x 1024 new rows of width 4096 into 2048 latent channels (dense-source contraction kernel)",
            "project_ms": t_pb, "project_TFLOP/s": pflops / t_pb / 1e9,
            "delta_project_ms": t_db, "delta_project_TFLOP/s_of_matrix_work": 2.0 * pflops / t_db / 1e9}
        del xchunk, proj, blat
        uflops = 2.0 * ow.B * ow.L * n_lat * ow.d
        extra["cl_gqa_c4"] = {"workload": "c4 shape, cross-layer step of a GQA layer (latent width 2048, 2-bit, group 64); "
                                          "random latent deltas and U_kv (timing only)",
                              "accumulate_latent_ms": t_u, "accumulate_latent_TFLOP/s": uflops / t_u / 1e9,
                              "accumulate_latent_frac_mfma_peak": uflops / t_u / 1e9 / PEAK_BF16_TFLOPS,
                              "delta_projection_us": t_d * 1e3,
                              "remat_attn_from_accumulator_ms": t_a}
        del dcache, oacc, uprep, uws, dwp, dws
        torch.cuda.empty_cache()
        # config 3: one XQuant-CL decode step through 32 layers (B=8, L=8192, d=4096, MHA): per layer, merge the layer's
        # 2-bit delta cache into the accumulator, then attend from the accumulator with the layer's weights.  Random
        # deltas and weights (timing only); the 32 delta caches and weight streams are distinct.
        w3 = xi.C3
        a3 = xq.XQAttn(w3.Hq, w3.Hkv, w3.hd, w3.hd ** -0.5)
        n_layers = 32
        acc3 = torch.randn((w3.B, w3.L, w3.d), device=dev, generator=gen).to(torch.bfloat16)
        deltas, streams = [], []
        for _ in range(n_layers):
            dcl = xq.alloc_cache(w3.B, w3.L, w3.d, w3.G, 2)
            dcl.codes.copy_(torch.randint(0, 256, dcl.codes.shape, device=dev, dtype=torch.uint8, generator=gen))
            dcl.scale.fill_(0.01)
            dcl.zero.fill_(-0.015)
            deltas.append(dcl)
            wk3 = (torch.randn((w3.d, w3.Hkv * w3.hd), device=dev, generator=gen) * w3.d ** -0.5).to(torch.bfloat16)
            wv3 = (torch.randn((w3.d, w3.Hkv * w3.hd), device=dev, generator=gen) * w3.d ** -0.5).to(torch.bfloat16)
            streams.append(xq.xq_prepare_weights(a3, w3.d, 0, 16, wk3, wv3))
            del wk3, wv3
        q3 = dev_bf16(xi.gen_q(w3))
        out3 = torch.empty((w3.B, w3.Hq, w3.hd), dtype=torch.float32, device=dev)
        ws3 = torch.empty(xq.xq_remat_attn_workspace_bytes(a3, w3.B, w3.L, w3.d, 0), dtype=torch.uint8, device=dev)
        lens3 = [w3.L] * w3.B

        def cl_step():
            for l in range(n_layers):
                xq.xq_cl_accumulate(acc3, deltas[l], lens3, False)
                xq.xq_remat_attn_decode(a3, q3, streams[l], lens3, acc_bf16=acc3, out=out3, workspace=ws3)

        t_cl = timed(cl_step, n=2, warm=1)
        extra["cl_decode_step_c3_32_layers"] = {"workload": "c3: B=8, L=8192, d=4096 MHA, 2-bit deltas, 32 layers", "ms": t_cl,
                                                "ms_per_layer": t_cl / n_layers,
                                                "tokens/s/layer": w3.B * w3.L / (t_cl / n_layers * 1e-3)}
        del deltas, streams, acc3, ws3
        torch.cuda.empty_cache()
        # config 5: 64 decode steps of a long context (B=4, 2-bit, group 128), the length growing from 32704 to 32768
        w5 = xi.C5
        a5 = xq.XQAttn(w5.Hq, w5.Hkv, w5.hd, w5.hd ** -0.5)
        c5 = xq.alloc_cache(w5.B, w5.L, w5.d, w5.G, w5.bits)
        for b0 in range(w5.B):
            sub = xq.XQCache(c5.codes[b0:b0 + 1], c5.scale[b0:b0 + 1], c5.zero[b0:b0 + 1], 1, w5.L, w5.d, w5.G, w5.bits)
            xq.xq_quantize_append(sub, torch.randn((1, w5.L, w5.d), device=dev, generator=gen).to(torch.bfloat16), [0])
        wk5, wv5 = xi.gen_weights(w5)
        wp5 = xq.xq_prepare_weights(a5, w5.d, w5.G, w5.bits, dev_bf16(wk5), dev_bf16(wv5))
        q5 = dev_bf16(xi.gen_q(w5))
        out5 = torch.empty((w5.B, w5.Hq, w5.hd), dtype=torch.float32, device=dev)
        ws5 = torch.empty(xq.xq_remat_attn_workspace_bytes(a5, w5.B, w5.L, w5.d, w5.G), dtype=torch.uint8, device=dev)
        x5 = torch.randn((w5.B, 1, w5.d), device=dev, generator=gen).to(torch.bfloat16)

        def c5_steps():
            for i in range(64):
                n = w5.L - 64 + i
                xq.xq_quantize_append(c5, x5, [n] * w5.B)
                xq.xq_remat_attn_decode(a5, q5, wp5, [n + 1] * w5.B, xcache=c5, out=out5, workspace=ws5)

        t_c5 = timed(c5_steps, n=1, warm=1)
        extra["decode_64_steps_c5"] = {"workload": "c5: B=4, context 32704 -> 32768, 2-bit, group 128; 64 x (append 1 token, attend)",
                                       "ms": t_c5, "ms_per_step": t_c5 / 64,
                                       "tokens/s/layer": w5.B * w5.L / (t_c5 / 64 * 1e-3)}
        del c5, wp5, ws5

    traffic = K3_HBM_BYTES_PER_LAUNCH

    result = {
        "metric": "cached tokens rematerialized+attended/sec/layer",
        "value": value,
        "unit": "tokens/s/layer",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "c2 Llama-2-7B-shaped decode step, one layer: d=4096, 32x128 MHA, batch 8, "
                               "context 4096, X cache 3-bit asym group 128; step = quantize+append 1 token/seq "
                               "then fused dequant-remat-attention",
                   "batch": B, "context": L, "d": d, "heads": Hq, "kv_heads": Hkv, "bits": bits, "group": G,
                   "settle_launches": args.settle},
        "roofline": {"bound": "mfma", "kernel": "remat_attn_tile16_kernel<3,128,0> (events bracket xq_remat_attn_decode: + scale pre-pass and combine, ~1%)",
                     "achieved": achieved_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved_tflops / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_measured_at_commit": K3_HBM_BYTES_MEASURED_AT,
                     "avg_ms": remat_ms, "flops_per_launch": flops},
        "extra": extra,
    }

    # ---- CPU baseline: the oracle, as it stands, on a bounded sample of the same workload
    if not args.no_cpu_baseline:
        from oracle import xq_oracle as xo
        pairs = xi.sample_pairs(w, args.cpu_pairs)
        step()                                   # `out` again holds the XQuant step's result
        torch.cuda.synchronize()
        # the oracle's own cache of the sampled sequences, quantised by the oracle from the same seeded X
        # (untimed, like the GPU's prefill of the cache; the step's own append of one token is in it)
        codes_h = np.zeros((B, L, d * bits // 8), np.uint8)
        scale_h = np.zeros((B, L, d // G), np.uint16)
        zero_h = np.zeros((B, L, d // G), np.uint16)
        for b in sorted({b for b, _ in pairs}):
            c_, s_, z_ = xo.quantize_rows(xi.from_bf16_bits(x_bits[b]), G, bits)
            codes_h[b], scale_h[b], zero_h[b] = xo.pack_rows(c_, bits), s_, z_
        c0 = time.perf_counter()
        ref = xo.remat_attn_pairs(q_bf16=q_bits, Wk=wk_bits, Wv=wv_bits, Hq=Hq, Hkv=Hkv, hd=hd,
                                  softmax_scale=hd ** -0.5, lens=lens, pairs=pairs, packed=codes_h,
                                  scale=scale_h, zero=zero_h, G=G, bits=bits)
        c1 = time.perf_counter()
        full_job_s = (c1 - c0) * (B * Hq) / len(pairs)
        got = out.cpu().numpy()
        sel = np.array([got[b, h] for b, h in pairs], np.float64)
        err = float((np.linalg.norm(sel - ref, axis=-1) / np.linalg.norm(ref, axis=-1)).max())
        result["cpu_baseline"] = {
            "value": tokens / full_job_s, "unit": "tokens/s/layer", "cores": xo.max_threads(), "kind": "oracle",
            "sample": f"{len(pairs)} of {B * Hq} (sequence, head) pairs of the same workload, full context; "
                      f"measured {c1 - c0:.1f} s, full-job time extrapolated x{B * Hq / len(pairs):.0f}",
            "gpu_vs_oracle_max_rel_err_on_sample": err,
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
