#!/usr/bin/env python3
"""Benchmark of the batched watermark-detection path on one MI355X.

One step = one pass of the whole hot path (tile crop + normalise fused into the first convolution,
the convolutional extractor, thresholding, symbol packing, Reed-Solomon decoding) over the 4096-image
"tiled detection" configuration, with images, origins and weights already resident in device memory.

Prints ONE JSON line: images/s (whole job), the roofline of the dominant kernel (the fused pair of
C -> C 3x3 convolution blocks on the bf16 matrix cores; duration per launch measured with HIP events on
the launch stream), per-stage figures for the tile-crop and Reed-Solomon kernels, and the CPU oracle timed on
this machine's host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by a
# copy kernel of known size (profiles/conv_pair_c2_hbm_traffic.txt), for the fused pair of C -> C blocks at the
# default micro-batch of 1024 images: 514.41 MiB read + 512.57 MiB written; algorithmic 2 x 512 MiB.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 1076853382


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="C2", help="C2 (headline), C3 or C4")
    ap.add_argument("--images", type=int, default=0, help="override the number of images (0 = the configuration's)")
    ap.add_argument("--micro-batch", type=int, default=0)
    ap.add_argument("--cpu-sample", type=int, default=256, help="images the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--policy", default="random", choices=["random", "random_grid", "fixed"])
    ap.add_argument("--chunks", type=int, default=16, help="C5 only: chunks per step (a full C5 pass is 128)")
    ap.add_argument("--chunk-images", type=int, default=8192, help="C5 only: images per pinned host chunk")
    ap.add_argument("--streams", type=int, default=3, help="C5 only: chunks in flight (staging buffers) of the upload / compute / download pipeline")
    ap.add_argument("--calibration-copy", type=int, default=0,
                    help="MiB of a plain device-to-device copy issued once before the timed region: the kernel of "
                         "known size that rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, one device); --gpus must be 1. "
              "Images are independent, so more GPUs would each run this same path on their own shard.",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import synth
    import paper_2509_02447_amd as q

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    cfg = synth.CONFIGS[args.config]
    if args.config == "C5":
        return bench_stream(args, cfg, torch, np, synth, q)
    N = args.images or cfg.n_images
    if args.config == "C4" and not args.images:
        N = 4096                                   # 16384 x 768 KiB of host staging is needless for timing
    wts = synth.config_weights(cfg)
    ctx = q.Context(weights=wts, rs=dict(m=cfg.m, prim_poly=cfg.prim_poly, n=cfg.n, k=cfg.k, fcr=cfg.fcr))
    if args.micro_batch:
        ctx.qrm_set_micro_batch(args.micro_batch)

    # ---- inputs: seeded, generated on the host in chunks, resident in HBM before the timed region
    d_img = torch.empty((N, 3, cfg.H, cfg.W), dtype=torch.uint8, device="cuda")
    chunk = 256
    for s in range(0, N, chunk):
        c = min(chunk, N - s)
        d_img[s:s + c].copy_(torch.from_numpy(synth.images(cfg, s, c)))
    off = synth.offsets(cfg, 0, N, args.policy)
    d_off = torch.from_numpy(off).cuda()
    d_logits = torch.empty((N, cfg.n_bits), dtype=torch.float32, device="cuda")
    d_bits = torch.empty((N, cfg.n_bits), dtype=torch.uint8, device="cuda")
    d_msg = torch.empty((N, cfg.k), dtype=torch.uint8, device="cuda")
    d_cw = torch.empty((N, cfg.n), dtype=torch.uint8, device="cuda")
    d_ne = torch.empty((N,), dtype=torch.int8, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        ctx.qrm_detect(d_img, N, cfg.H, cfg.W, d_off, cfg.tile, d_logits, d_bits, d_msg, d_cw, d_ne, stream=stream)

    if args.calibration_copy:
        cal_src = torch.zeros(args.calibration_copy << 20, dtype=torch.uint8, device="cuda")
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    value = N * args.steps / dt

    # ---- roofline of the dominant kernel: same steps again, every launch bracketed by HIP events
    ctx.qrm_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    k_ms, k_launches, k_flops, blocks_per_launch = ctx.qrm_profile_read()
    ctx.qrm_profile_enable(False)
    achieved_tflops = k_flops / (k_ms * 1e-3) / 1e12 if k_ms > 0 else 0.0
    kname = ("conv_pair_kernel<64,false,false> (two fused 3x3 conv blocks C->C, bf16 MFMA implicit GEMM, activations between "
             "them in LDS)") if blocks_per_launch >= 2 else "conv_mid_kernel (3x3 conv C->C, bf16 MFMA implicit GEMM)"
    roofline = {"kernel": kname, "bound": "mfma",
                "achieved": round(achieved_tflops, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH if (blocks_per_launch == 2 and args.config == "C2" and not args.micro_batch
                                                                 and not args.images) else None,
                "launches": int(k_launches), "avg_launch_us": round(k_ms * 1e3 / max(1, k_launches), 2),
                "flops_per_launch": k_flops / max(1, k_launches),
                "sustained_on_random_data": None,   # filled in below: pure matrix loop on random operands
                "timing": "HIP events around every launch, second pass of the same steps"}

    # ---- the other two stages on their own (HBM-bound by bytes, in practice latency / ALU bound)
    def timed(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    l2 = cfg.tile * cfg.tile
    mfma_flops_per_image = 2 * 9 * 3 * cfg.channels * l2 + (cfg.n_blocks - 1) * 2 * 9 * cfg.channels ** 2 * l2
    d_tiles = torch.empty((N, 3, cfg.tile, cfg.tile), dtype=torch.uint8, device="cuda")
    t_tile = timed(lambda: ctx.qrm_extract_tiles(d_img, N, cfg.H, cfg.W, d_off, cfg.tile, d_tiles, stream=stream))
    tile_bytes = N * (6 * cfg.tile * cfg.tile + 8)
    # the same crop on 16 x as many images (4096 crops move 100 MB: a launch of ~12 us at the HBM peak, latency bound)
    n_big = 16 * N if args.config == "C2" and not args.images else 0
    t_tile_big = None
    if n_big:
        big = torch.empty((n_big, 3, cfg.H, cfg.W), dtype=torch.uint8, device="cuda")
        big.random_(0, 256)
        big_off = d_off.repeat(16, 1).contiguous()
        big_tiles = torch.empty((n_big, 3, cfg.tile, cfg.tile), dtype=torch.uint8, device="cuda")
        t_tile_big = timed(lambda: ctx.qrm_extract_tiles(big, n_big, cfg.H, cfg.W, big_off, cfg.tile, big_tiles,
                                                         stream=stream), reps=5)
        del big, big_tiles, big_off
    n_cw = 1 << 20
    sym = torch.randint(0, 1 << cfg.m, (n_cw, cfg.n), dtype=torch.uint8, device="cuda")
    m2 = torch.empty((n_cw, cfg.k), dtype=torch.uint8, device="cuda")
    c2 = torch.empty((n_cw, cfg.n), dtype=torch.uint8, device="cuda")
    e2 = torch.empty((n_cw,), dtype=torch.int8, device="cuda")
    t_rs = timed(lambda: ctx.qrm_rs_decode(sym, n_cw, m2, c2, e2, stream=stream))
    rs_bytes = n_cw * (2 * cfg.n + cfg.k + 1)
    # key verification: on stored messages (streaming, k + 5 bytes per word) and inside the decoder's epilogue
    n_vw = 1 << 24
    vmsg = torch.randint(0, 1 << cfg.m, (n_vw, cfg.k), dtype=torch.uint8, device="cuda")
    vmat = torch.empty((n_vw,), dtype=torch.int32, device="cuda")
    vdet = torch.empty((n_vw,), dtype=torch.uint8, device="cuda")
    ctx.qrm_set_key(np.arange(cfg.k, dtype=np.uint8) & ((1 << cfg.m) - 1),
                    q.binding.qrm_key_threshold(cfg.k * cfg.m, 1e-6))
    t_vk = timed(lambda: ctx.qrm_verify_key(vmsg, n_vw, vmat, vdet, stream=stream))
    vk_bytes = n_vw * (cfg.k + 5)
    del vmsg, vmat, vdet
    # variance-based tile selection: reads every pixel once (all of the image lies under some window)
    sel_off = torch.empty((N, 2), dtype=torch.int32, device="cuda")
    t_sel = timed(lambda: ctx.qrm_select_tiles_variance(d_img, N, cfg.H, cfg.W, cfg.tile, cfg.tile // 2, sel_off,
                                                        None, stream=stream))
    sel_bytes = N * (3 * cfg.H * cfg.W + 8)
    # fused pre-processing from raw 2H x 2W interleaved images: the whole image, and only each image's tile
    n_raw = min(N, 2048)
    raw = torch.randint(0, 256, (n_raw, 2 * cfg.H, 2 * cfg.W, 3), dtype=torch.uint8, device="cuda")
    pre_full = torch.empty((n_raw, 3, cfg.H, cfg.W), dtype=torch.uint8, device="cuda")
    pre_tile = torch.empty((n_raw, 3, cfg.tile, cfg.tile), dtype=torch.uint8, device="cuda")
    t_pre_full = timed(lambda: ctx.qrm_preprocess(raw, n_raw, 2 * cfg.H, 2 * cfg.W, cfg.H, None, 0, pre_full, stream=stream))
    t_pre_tile = timed(lambda: ctx.qrm_preprocess(raw, n_raw, 2 * cfg.H, 2 * cfg.W, cfg.H, d_off, cfg.tile, pre_tile,
                                                  stream=stream))
    pre_full_bytes = n_raw * (4 * 3 * cfg.H * cfg.W + 3 * cfg.H * cfg.W)
    pre_tile_bytes = n_raw * (4 * 3 * l2 + 3 * l2 + 8)
    # a yardstick for the stages above: the same box's plain device copy of the raw images' volume (read + write)
    cp_dst = torch.empty_like(raw)
    t_copy = timed(lambda: cp_dst.copy_(raw))
    copy_bytes = 2 * raw.numel()
    del raw, pre_full, pre_tile, cp_dst
    # what the matrix pipes sustain with nothing else running, by operand data (the clock follows the power budget)
    matrix_probe = {"zeros_tflops": round(ctx.qrm_matrix_rate_probe(0), 1),
                    "random_data_tflops": round(ctx.qrm_matrix_rate_probe(2), 1),
                    "note": "back-to-back bf16 32x32x16 matrix instructions, 8 wavefronts per CU, no memory traffic"}
    if isinstance(roofline, dict) and roofline.get("bound") == "mfma":
        roofline["sustained_on_random_data"] = {"tflops": matrix_probe["random_data_tflops"],
                                                 "frac_of_it": round(roofline["achieved"] / matrix_probe["random_data_tflops"], 4)}
    stages = {
        "matrix_pipe_probe": matrix_probe,
        "device_copy": {"us": round(t_copy * 1e6, 2), "GBs_read_plus_write": round(copy_bytes / t_copy / 1e9, 1),
                        "frac_hbm": round(copy_bytes / t_copy / 1e9 / PEAK_HBM_GBS, 4),
                        "note": "torch copy_ of the raw-image buffer: what a plain read + write stream reaches here"},
        "preprocess_whole_image": {"us": round(t_pre_full * 1e6, 2), "images_per_s": round(n_raw / t_pre_full, 0),
                                   "algorithmic_GBs": round(pre_full_bytes / t_pre_full / 1e9, 1),
                                   "frac_hbm": round(pre_full_bytes / t_pre_full / 1e9 / PEAK_HBM_GBS, 4), "images": n_raw},
        "preprocess_tile_only": {"us": round(t_pre_tile * 1e6, 2), "images_per_s": round(n_raw / t_pre_tile, 0),
                                 "algorithmic_GBs": round(pre_tile_bytes / t_pre_tile / 1e9, 1),
                                 "frac_hbm": round(pre_tile_bytes / t_pre_tile / 1e9 / PEAK_HBM_GBS, 4), "images": n_raw},
        "select_tiles_variance": {"us": round(t_sel * 1e6, 2), "images_per_s": round(N / t_sel, 0),
                                  "algorithmic_GBs": round(sel_bytes / t_sel / 1e9, 1),
                                  "frac_hbm": round(sel_bytes / t_sel / 1e9 / PEAK_HBM_GBS, 4), "images": N},
        "verify_key": {"us": round(t_vk * 1e6, 2), "words_per_s": round(n_vw / t_vk, 0),
                       "algorithmic_GBs": round(vk_bytes / t_vk / 1e9, 1),
                       "frac_hbm": round(vk_bytes / t_vk / 1e9 / PEAK_HBM_GBS, 4), "words": n_vw},
        "tile_crop": {"us": round(t_tile * 1e6, 2), "algorithmic_GBs": round(tile_bytes / t_tile / 1e9, 1),
                      "frac_hbm": round(tile_bytes / t_tile / 1e9 / PEAK_HBM_GBS, 4), "images": N},
        "tile_crop_large_batch": None if not t_tile_big else {
            "us": round(t_tile_big * 1e6, 2), "algorithmic_GBs": round(16 * tile_bytes / t_tile_big / 1e9, 1),
            "frac_hbm": round(16 * tile_bytes / t_tile_big / 1e9 / PEAK_HBM_GBS, 4), "images": n_big},
        "rs_decode": {"us": round(t_rs * 1e6, 2), "codewords_per_s": round(n_cw / t_rs, 0),
                      "algorithmic_GBs": round(rs_bytes / t_rs / 1e9, 2),
                      "frac_hbm": round(rs_bytes / t_rs / 1e9 / PEAK_HBM_GBS, 5), "codewords": n_cw},
        # MFMA work actually executed per image: first conv + the C -> C convs, over the whole step (all
        # kernels, launch gaps and the RS decode included in the time).  The final conv + average
        # pool is evaluated in closed form from nine channel sums of the last block (it is linear), so its
        # 2*9*C*n_bits*l^2 FLOPs are NOT credited here.
        "extractor_mfma_tflops": round(mfma_flops_per_image * value / 1e12, 2),
        "extractor_frac_of_bf16_peak": round(mfma_flops_per_image * value / 1e12 / PEAK_BF16_TFLOPS, 4),
        "extractor_nominal_tflops_incl_final_conv": round(cfg.flops_per_image() * value / 1e12, 2),
    }

    # ---- CPU oracle on a bounded sample of the same workload (reported baseline, not the target)
    cpu = None
    if args.cpu_sample > 0:
        import oracle
        ns = min(args.cpu_sample, N)
        imgs = d_img[:ns].cpu().numpy()
        t1 = time.perf_counter()
        ref = oracle.detect(wts, imgs, off[:ns], cfg.tile, cfg.m, cfg.prim_poly, cfg.n, cfg.k, cfg.fcr)
        t_cpu = time.perf_counter() - t1
        cpu = {"value": round(ns / t_cpu, 3), "unit": "images/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"first {ns} images of the same {args.config} batch, whole path (fp64 direct conv + RS)",
               "seconds": round(t_cpu, 2)}
        # cheap sanity: the timed GPU outputs for the sample agree with what the oracle just computed
        g = d_logits[:ns].cpu().numpy().astype(np.float64)
        err = float((np.abs(g - ref["logits"]) / np.maximum(1.0, np.abs(ref["logits"]))).max())
        cpu["max_scaled_logit_error_vs_gpu"] = round(err, 5)

    out = {
        "metric": "images/sec end-to-end detection on 1 MI355X",
        "value": round(value, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: {N} images 3x{cfg.H}x{cfg.W} u8, one {cfg.tile}x{cfg.tile} tile each "
                               f"({args.policy} origin), {cfg.n_blocks}x conv3x3 {cfg.channels}ch + conv->{cfg.n_bits} "
                               f"+ pool + linear, RS({cfg.n},{cfg.k}) over GF(2^{cfg.m})",
                   "images": N, "tile": cfg.tile, "inputs": "resident in HBM before the timed region",
                   "micro_batch": args.micro_batch or "default"},
        "roofline": roofline,
        "stages": stages,
        "cpu_baseline": cpu,
        "context": "paper: 2.43x over its sequential baseline; Stable Signature ~30 min per 1M 256x256 images "
                   "(~556 img/s) on 1x H100 + EPYC 9534 (context only, other hardware)",
    }
    print(json.dumps(out))
    ctx.close()
    return 0


def bench_stream(args, cfg, torch, np, synth, q) -> int:
    """Streaming configuration: images start in pinned HOST memory; upload, kernels and result download of
    different chunks overlap on the library's own streams (qrm_detect_host).  Three pre-generated chunks
    are recycled, so nothing is generated inside the timed region.  The number is bound by the host
    link, not by the GPU: the bare pinned upload rate is measured beside it."""
    chunk, n_chunks, lanes = args.chunk_images, args.chunks, args.streams
    wts = synth.config_weights(cfg)
    ctx = q.Context(weights=wts, rs=dict(m=cfg.m, prim_poly=cfg.prim_poly, n=cfg.n, k=cfg.k, fcr=cfg.fcr))
    if args.micro_batch:
        ctx.qrm_set_micro_batch(args.micro_batch)
    n_buf = min(3, n_chunks)
    bufs = [torch.empty((chunk, 3, cfg.H, cfg.W), dtype=torch.uint8, pin_memory=True) for _ in range(n_buf)]
    obufs = [torch.empty((chunk, 2), dtype=torch.int32, pin_memory=True) for _ in range(n_buf)]
    for b in range(n_buf):
        synth.images(cfg, b * chunk, chunk, out=bufs[b].numpy())
        obufs[b].copy_(torch.from_numpy(synth.offsets(cfg, b * chunk, chunk, args.policy)))
    n_total = n_chunks * chunk
    h_msg = torch.empty((n_total, cfg.k), dtype=torch.uint8, pin_memory=True)
    h_ne = torch.empty((n_total,), dtype=torch.int8, pin_memory=True)
    order = [b % n_buf for b in range(n_chunks)]

    def step():
        ctx.qrm_detect_host([bufs[b] for b in order], chunk, cfg.H, cfg.W, [obufs[b] for b in order], cfg.tile, lanes,
                            h_msg, None, h_ne)          # returns when every chunk is done

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    value = n_total * args.steps / dt
    # the link on its own: the same chunks uploaded back to back, nothing else running
    d_stage = torch.empty((chunk, 3, cfg.H, cfg.W), dtype=torch.uint8, device="cuda")
    d_stage.copy_(bufs[0], non_blocking=True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for b in order:
        d_stage.copy_(bufs[b], non_blocking=True)
    torch.cuda.synchronize()
    t_up = time.perf_counter() - t1
    chunk_bytes = chunk * 3 * cfg.H * cfg.W
    link_gbs = n_chunks * chunk_bytes / t_up / 1e9
    # the same images resident in device memory (no link): what the kernels alone sustain
    d_off = obufs[0].cuda()
    d_msg = torch.empty((chunk, cfg.k), dtype=torch.uint8, device="cuda")
    d_ne = torch.empty((chunk,), dtype=torch.int8, device="cuda")
    ctx.qrm_detect(d_stage, chunk, cfg.H, cfg.W, d_off, cfg.tile, None, None, d_msg, None, d_ne)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(3):
        ctx.qrm_detect(d_stage, chunk, cfg.H, cfg.W, d_off, cfg.tile, None, None, d_msg, None, d_ne)
    torch.cuda.synchronize()
    resident = 3 * chunk / (time.perf_counter() - t2)
    out = {
        "metric": "images/sec end-to-end detection on 1 MI355X", "value": round(value, 1), "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt * 1e3 / args.steps, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"C5 (streamed): {n_chunks} chunks x {chunk} images 3x{cfg.H}x{cfg.W} u8 per step from "
                               f"pinned host memory ({n_buf} buffers recycled), {lanes} chunks in flight; one {cfg.tile}x{cfg.tile} "
                               f"tile each, {cfg.n_blocks}x conv3x3 {cfg.channels}ch, RS({cfg.n},{cfg.k}) over GF(2^{cfg.m})",
                   "images": n_total, "inputs": "pinned HOST memory: the upload is inside the timed region"},
        "roofline": {"bound": "host link", "achieved": round(value * 3 * cfg.H * cfg.W / 1e9, 2),
                     "peak": round(link_gbs, 2), "unit": "GB/s",
                     "frac": round(value * 3 * cfg.H * cfg.W / 1e9 / link_gbs, 4), "traffic": None,
                     "note": "peak = bare pinned upload of the same chunks measured in this run (not a published figure)"},
        "stages": {"bare_upload_GBs": round(link_gbs, 2), "bare_upload_images_per_s": round(link_gbs * 1e9 / (3 * cfg.H * cfg.W), 1),
                   "resident_images_per_s": round(resident, 1)},
        "cpu_baseline": None,
    }
    print(json.dumps(out))
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
