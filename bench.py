"""Benchmark of the MAE input-pipeline hot path on one MI355X.

A step is one pass of the whole path over one batch: mae_prep_batch (crop parameters, masking
order, fused crop/resize/flip/normalise/patchify/gather) followed by mae_normpix_loss (loss and
gradient), on synthetic images already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--no-cpu-baseline]

The first consumer of the path's output, mae_patch_embed, and the finetuning-mode input pipeline
("3 Aug", "3 Aug+") are timed by themselves after the steps and reported under "patch_embed" and
"finetune_prep", and so is the input pipeline on JPEG files ("crop decode", under "jpeg_prep");
they are not part of the step or of `value`.
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

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix rate

# HBM bytes per launch of the loss kernel from rocprofv3 counters (FETCH_SIZE and WRITE_SIZE runs,
# each scaled by what the counter reads for a plain device copy of known size; the summaries are
# under profiles/).  Only valid for the kernel source they were taken on: keyed by its hash.
LOSS_KERNEL_SOURCES = ("paper_2404_00509_amd/csrc/normpix_loss.hip",
                       "paper_2404_00509_amd/csrc/mae_device.hpp")
MEASURED_TRAFFIC = {
    # workload: (sha256 of the sources above, bytes read + written per launch)
    "c4": ("f3d523a5a507f86208dbb543cf73813f2700e950d9ea3024d7e6f9bcc4926460", 6.172e9),
    "c5": ("f3d523a5a507f86208dbb543cf73813f2700e950d9ea3024d7e6f9bcc4926460", 4.415e9),
}


def measured_traffic(workload):
    import hashlib

    entry = MEASURED_TRAFFIC.get(workload)
    if entry is None:
        return None
    h = hashlib.sha256()
    for rel in LOSS_KERNEL_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return entry[1] if h.hexdigest() == entry[0] else None


def algorithmic_bytes(wl, K):
    """Bytes the method must move per launch (plain dataflow, target materialised once).

    prep : read the crop bytes is data dependent (about half of each image); counted from the
           crop boxes of the run.  write visible K*D*e + target L*D*4 + mask/ids.
    loss : read pred and target of the masked rows, write the whole gradient.
    """
    e = 2 if wl.dtype == "bf16" else 4
    prep_write = wl.B * (K * wl.D * e + wl.L * wl.D * 4 + wl.L * 5 + K * 4)
    masked = wl.L - K
    loss = wl.B * (masked * wl.D * (e + 4) + wl.L * wl.D * e + wl.L)
    return prep_write, loss


def time_scheme(args, mae, synth, torch, dev, wl, bf16):
    """Per-stage step time of a progressive pretraining scheme; one allocation for all stages."""
    stages = [mae.mae_pretrain_stage(args.scheme, s) for s in (1, 2, 3)]
    bufs = mae.ProgressiveBuffers(wl.B, wl.patch, stages, bf16=bf16)
    D = 3 * wl.patch * wl.patch
    max_l = max(sh[1] for sh in bufs.shapes)
    gen = torch.Generator(device="cuda").manual_seed(2)
    pred_store = torch.randn(wl.B * max_l * D, generator=gen, device="cuda")
    if bf16:
        pred_store = pred_store.to(torch.bfloat16)
    grad_store = torch.empty_like(pred_store)
    loss = torch.zeros(1, device="cuda")
    stream = torch.cuda.current_stream()
    rows = []
    for i, (res, m) in enumerate(stages):
        _, L, K, _ = bufs.shapes[i]
        buf = bufs.stage(i)
        pred = pred_store[:wl.B * L * D].view(wl.B, L, D)
        grad = grad_store[:wl.B * L * D].view(wl.B, L, D)
        desc = mae.make_prep_desc(*dev, out_size=res, patch=wl.patch, num_keep=K, seed=0,
                                  batch_index=0,
                                  out_dtype=mae.MAE_BF16 if bf16 else mae.MAE_F32)
        ldesc = mae.make_loss_desc(pred, buf.target, buf.mask, num_masked=wl.B * (L - K))
        lws = torch.empty(max(mae.mae_loss_workspace_bytes(ldesc), 256), dtype=torch.uint8,
                          device="cuda")

        def step(j):
            desc.batch_index = 1000 * (i + 1) + j
            mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep,
                               buf.target, buf.crop, buf.workspace, stream=stream)
            mae.mae_normpix_loss(ldesc, loss, grad, lws, stream=stream)

        for j in range(args.warmup):
            step(j)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for j in range(args.steps):
            step(args.warmup + j)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        rows.append({"stage": i + 1, "out_size": res, "mask_ratio": m, "L": L, "K": K,
                     "ms_per_step": round(dt * 1e3 / args.steps, 4),
                     "images_per_s": round(wl.B * args.steps / dt, 1)})
    return rows


def time_embed(args, mae, synth, torch, dev, wl, K, E):
    """mae_patch_embed on every visible row of the batch (bf16 in, bf16 out), timed by itself with
    events on the launch stream.  Not part of the step above."""
    import numpy as np

    desc = mae.make_prep_desc(*dev, out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0,
                              batch_index=0, out_dtype=mae.MAE_BF16)
    buf = mae.alloc_prep_buffers(desc)
    stream = torch.cuda.current_stream()
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                       buf.crop, buf.workspace, stream=stream)
    weight, bias, pos = synth.make_embed_params(0, wl.D, E, wl.L)
    w = torch.from_numpy(weight).cuda().to(torch.bfloat16)
    b, p = torch.from_numpy(bias).cuda(), torch.from_numpy(pos).cuda()
    tokens = torch.empty((wl.B, K, E), dtype=torch.bfloat16, device="cuda")
    edesc = mae.make_embed_desc(buf.visible, buf.ids_keep, w, b, p, out_dtype=mae.MAE_BF16)
    for _ in range(max(args.warmup, 1)):
        mae.mae_patch_embed(edesc, tokens, stream=stream)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for e in ev:
        e[0].record(stream)
        mae.mae_patch_embed(edesc, tokens, stream=stream)
        e[1].record(stream)
    torch.cuda.synchronize()
    ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    M = wl.B * K
    flops = 2.0 * M * wl.D * E
    nbytes = 2 * M * wl.D + 2 * M * E + 2 * E * wl.D + 4 * M + 4 * wl.L * E + 4 * E
    tflops = flops / (ms * 1e-3) / 1e12
    return {
        "kernel": "patch_embed_kernel (mae_patch_embed), bf16 x bf16 -> fp32 -> bf16",
        "M": M, "D": wl.D, "E": E, "avg_ms": round(ms, 4),
        "bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
        "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "flops": flops, "algorithmic_bytes": nbytes,
        "achieved_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
        "checksum": float(tokens.float().abs().mean().item()),
    }


def time_finetune(args, mae, torch, dev, wl):
    """mae_prep_batch in finetuning mode (Table 7, last stage: 224 px, crop side ratio 0.28..1,
    every patch kept, fp32 tokens in `visible`, no `target`) with "3 Aug" and "3 Aug+", timed by
    itself with events on the launch stream.  Not part of the step above."""
    import numpy as np

    rows = []
    res, lo, hi, _ = mae.mae_finetune_stage(1, 3)
    G = res // wl.patch
    L = G * G
    stream = torch.cuda.current_stream()
    for mode, name in ((mae.MAE_AUG_THREE, "3 Aug"), (mae.MAE_AUG_THREE_PLUS, "3 Aug+")):
        desc = mae.make_prep_desc(*dev, out_size=res, patch=wl.patch, num_keep=L, scale=(lo, hi),
                                  seed=0, batch_index=0, aug_mode=mode, jitter=0.3)
        buf = mae.alloc_prep_buffers(desc, want_target=False)

        def run(i):
            desc.batch_index = i
            mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None,
                               buf.crop, buf.workspace, stream=stream)

        for i in range(max(args.warmup, 1)):
            run(i)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
        for i, e in enumerate(ev):
            e[0].record(stream)
            run(args.warmup + i)
            e[1].record(stream)
        torch.cuda.synchronize()
        assert mae.mae_prep_status(buf.workspace) == 0
        ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
        crop = buf.crop.cpu().numpy().astype(np.int64)
        crop_bytes = int((crop[:, 2] * crop[:, 3] * 3).sum())
        # the method's bytes: the crop read once, tokens, mask and ids written.  What the
        # implementation moves on top of that is reported beside it, not counted: the 8-bit
        # resized crop of the images that drew the blur (a third of them), written once and read
        # once per pass of the blur kernel, and for "3 Aug+" the second read of the crops.
        nbytes = crop_bytes + wl.B * (L * wl.D * 4 + L * 5 + L * 4)
        u8_third = wl.B * res * res * 3 // 3
        extra = u8_third * (3 if mode == mae.MAE_AUG_THREE_PLUS else 2) \
            + (crop_bytes * 2 // 3 if mode == mae.MAE_AUG_THREE_PLUS else 0)
        rows.append({"augmentation": name, "out_size": res, "avg_ms": round(ms, 4),
                     "images_per_s": round(wl.B / (ms * 1e-3), 1),
                     "algorithmic_bytes": nbytes, "intermediate_bytes_estimate": extra,
                     "achieved_GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
        del buf
    return rows


def time_without_target(args, mae, torch, dev, wl, K, M, pred, grad, crop_bytes, want_loss):
    """The same step without a stored target: mae_prep_batch with target = NULL (visible tokens,
    mask and ids only) and mae_normpix_loss_from_images, which takes the masked patches' pixels
    from the images again.  Same outputs except `target`; timed like the step above."""
    import numpy as np

    bf16 = wl.dtype == "bf16"
    desc = mae.make_prep_desc(*dev, out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0,
                              batch_index=0, out_dtype=mae.MAE_BF16 if bf16 else mae.MAE_F32)
    buf = mae.alloc_prep_buffers(desc, want_target=False)
    ldesc = mae.make_loss_desc(pred, None, buf.mask, num_masked=M)
    lws = torch.empty(max(mae.mae_loss_from_images_workspace_bytes(desc, ldesc), 256),
                      dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, device="cuda")
    stream = torch.cuda.current_stream()

    def step(i, ev=None):
        desc.batch_index = i
        if ev is not None:
            ev[0].record(stream)
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None,
                           buf.crop, buf.workspace, stream=stream)
        if ev is not None:
            ev[1].record(stream)
        mae.mae_normpix_loss_from_images(desc, buf.workspace, ldesc, loss, grad, lws,
                                         stream=stream)
        if ev is not None:
            ev[2].record(stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert mae.mae_prep_status(buf.workspace) == 0
    got = float(loss.item())
    assert abs(got - want_loss) <= 1e-5 + 1e-5 * abs(want_loss), (got, want_loss)
    prep_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    loss_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    e = 2 if bf16 else 4
    # what this dataflow must move: the crop's bytes twice, the visible tokens, mask and ids;
    # the masked rows of the prediction, the whole gradient
    prep_bytes = crop_bytes + wl.B * (K * wl.D * e + wl.L * 5 + K * 4)
    loss_bytes = crop_bytes + wl.B * ((wl.L - K) * wl.D * e + wl.L * wl.D * e + wl.L)
    ms = elapsed * 1e3 / args.steps
    return {
        "what": "mae_prep_batch(target = NULL) + mae_normpix_loss_from_images",
        "ms_per_step": round(ms, 4), "images_per_s": round(wl.B * args.steps / elapsed, 1),
        "loss_value": got,
        "kernels": {
            "mae_prep_batch": {"avg_ms": round(prep_ms, 4), "algorithmic_bytes": prep_bytes,
                               "achieved_GBps": round(prep_bytes / (prep_ms * 1e-3) / 1e9, 1)},
            "mae_normpix_loss_from_images": {
                "avg_ms": round(loss_ms, 4), "algorithmic_bytes": loss_bytes,
                "achieved_GBps": round(loss_bytes / (loss_ms * 1e-3) / 1e9, 1),
                "frac": round(loss_bytes / (loss_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
        },
    }


def time_jpeg(args, mae, synth, torch, wl, K, kind=None, B=None):
    """mae_prep_batch fed with JPEG files ("crop decode", Sec. 4.1): the same batch written as
    baseline JPEG (quality 90, 4:2:0, one restart interval per row of MCUs), timed by itself with
    events on the launch stream.  Not part of the step above."""
    import numpy as np

    t0 = time.time()
    kind = kind or wl.kind
    B = B or wl.B
    files, offsets, sizes = synth.make_jpegs(kind, B, seed=0)
    enc_s = time.time() - t0
    dev = [torch.from_numpy(a).cuda() for a in (files, offsets, sizes)]
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, file_sizes=dev[2], out_size=wl.out_size,
                              patch=wl.patch, num_keep=K, seed=0, batch_index=0,
                              max_image_side=512 if kind == "gradient500" else 0,
                              out_dtype=mae.MAE_BF16 if wl.dtype == "bf16" else mae.MAE_F32)
    buf = mae.alloc_prep_buffers(desc)
    stream = torch.cuda.current_stream()

    def run(i):
        desc.batch_index = i
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)

    for i in range(max(args.warmup, 1)):
        run(i)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(args.steps)]
    for i, e in enumerate(ev):
        e[0].record(stream)
        run(args.warmup + i)
        e[1].record(stream)
    torch.cuda.synchronize()
    assert mae.mae_prep_status(buf.workspace) == 0
    ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    crop = buf.crop.cpu().numpy().astype(np.int64)
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle beside it: whole-file decode (its definition of the input) of a small sample
        import oracle

        n = min(256 if kind != "gradient500" else 64, B)
        t0 = time.perf_counter()
        for o, m in zip(offsets[:n], sizes[:n]):
            oracle.jpeg_decode(files[o:o + m].tobytes())
        dt = time.perf_counter() - t0
        cpu = {"images_per_s": round(n / dt, 1), "cores": 1, "kind": "oracle",
               "sample": f"whole-file decode of the first {n} files of the batch, decode only"}
    return {
        "cpu_oracle_decode": cpu,
        "input": "baseline JPEG, quality 90, 4:2:0, restart interval = one row of MCUs",
        "file_bytes": int(files.size), "encode_s_on_host": round(enc_s, 1),
        "images": kind, "B": B,
        "avg_ms": round(ms, 4), "images_per_s": round(B / (ms * 1e-3), 1),
        "compressed_GBps": round(files.size / (ms * 1e-3) / 1e9, 1),
        "mean_crop_area_px": round(float((crop[:, 2] * crop[:, 3]).mean()), 1),
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c4", choices=["c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=4096, help="images timed on the CPU oracle")
    ap.add_argument("--cpu-reps", type=int, default=4,
                    help="passes of the CPU oracle over the sample")
    ap.add_argument("--scheme", type=int, default=0,
                    help="also time the three stages of pretraining scheme 1..6 (Table 9) on "
                         "buffers allocated once; adds a 'stages' list to the JSON line")
    ap.add_argument("--embed", type=int, default=768,
                    help="embedding width E for the separately timed mae_patch_embed launch over "
                         "the batch's visible rows (adds 'patch_embed' to the JSON line); 0 = skip")
    ap.add_argument("--no-jpeg", action="store_true",
                    help="skip the separately timed calls on JPEG input ('jpeg_prep')")
    ap.add_argument("--no-finetune", action="store_true",
                    help="skip the separately timed finetuning-mode calls ('finetune_prep')")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, run one plain device copy of known size "
                         "(grad <- pred) so that a counter run has a reference kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no multi-GPU part (samples are "
              "independent, so a batch shards by sample and only the loss scalar would be "
              "exchanged). Run with --gpus 1.",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2404_00509_amd as mae
    from paper_2404_00509_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    mae.load()  # fail loudly if the HIP library is missing

    wl = synth.WORKLOADS[args.workload]
    bf16 = wl.dtype == "bf16"
    K = mae.mae_num_keep(wl.L, wl.mask_ratio)
    M = wl.B * (wl.L - K)

    t0 = time.time()
    images, offsets, heights, widths = synth.make_images(wl.kind, wl.B, seed=0)
    gen_s = time.time() - t0
    dev = [torch.from_numpy(a).cuda() for a in (images, offsets, heights, widths)]
    desc = mae.make_prep_desc(*dev, out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0,
                              batch_index=0, out_dtype=mae.MAE_BF16 if bf16 else mae.MAE_F32)
    buf = mae.alloc_prep_buffers(desc)
    gen = torch.Generator(device="cuda").manual_seed(1)
    pred = torch.randn((wl.B, wl.L, wl.D), generator=gen, device="cuda", dtype=torch.float32)
    if bf16:
        pred = pred.to(torch.bfloat16)
    grad = torch.empty_like(pred)
    loss = torch.zeros(1, device="cuda")
    ldesc = mae.make_loss_desc(pred, buf.target, buf.mask, num_masked=M)
    lws = torch.empty(max(mae.mae_loss_workspace_bytes(ldesc), 256), dtype=torch.uint8,
                      device="cuda")
    stream = torch.cuda.current_stream()  # the stream the library launches on

    def step(i, ev=None):
        desc.batch_index = i
        if ev is not None:
            ev[0].record(stream)
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)
        if ev is not None:
            ev[1].record(stream)
        mae.mae_normpix_loss(ldesc, loss, grad, lws, stream=stream)
        if ev is not None:
            ev[2].record(stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_per_step = elapsed * 1e3 / args.steps
    value = wl.B * args.steps / elapsed
    prep_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    loss_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    assert mae.mae_prep_status(buf.workspace) == 0
    final_loss = float(loss.item())
    if args.calibration_copy:
        grad.copy_(pred)  # reads and writes pred.numel() * element_size bytes each
        torch.cuda.synchronize()

    crop = buf.crop.cpu().numpy().astype(np.int64)
    crop_bytes = int((crop[:, 2] * crop[:, 3] * 3).sum())
    prep_write, loss_bytes = algorithmic_bytes(wl, K)
    prep_bytes = prep_write + crop_bytes
    loss_gbps = loss_bytes / (loss_ms * 1e-3) / 1e9
    prep_gbps = prep_bytes / (prep_ms * 1e-3) / 1e9

    out = {
        "metric": "images/sec and achieved HBM GB/s (% of peak) at 224px, B=4096, 1 MI355X",
        "value": round(value, 1),
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: B={wl.B} uint8 images (max side 256) -> {wl.out_size}px, "
                        f"patch {wl.patch}, L={wl.L}, keep {K}, prep + normpix loss + grad",
            "B": wl.B, "out_size": wl.out_size, "patch": wl.patch, "L": wl.L, "K": K, "D": wl.D,
            "input_generation_s": round(gen_s, 1),
        },
        "roofline": {
            "kernel": "normpix_loss_kernel (mae_normpix_loss; includes its 1-workgroup finish "
                      "kernel)",
            "bound": "hbm",
            "achieved": round(loss_gbps, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(loss_gbps / HBM_PEAK_GBPS, 4),
            "traffic": measured_traffic(wl.name),
            "algorithmic_bytes": loss_bytes,
            "avg_ms": round(loss_ms, 4),
        },
        "kernels": {
            "mae_prep_batch": {"avg_ms": round(prep_ms, 4), "algorithmic_bytes": prep_bytes,
                               "achieved_GBps": round(prep_gbps, 1),
                               "frac": round(prep_gbps / HBM_PEAK_GBPS, 4)},
            "mae_normpix_loss": {"avg_ms": round(loss_ms, 4), "algorithmic_bytes": loss_bytes,
                                 "achieved_GBps": round(loss_gbps, 1),
                                 "frac": round(loss_gbps / HBM_PEAK_GBPS, 4)},
        },
        "step_GBps": round((prep_bytes + loss_bytes) / (ms_per_step * 1e-3) / 1e9, 1),
        "step_frac_of_hbm_peak": round((prep_bytes + loss_bytes) / (ms_per_step * 1e-3) / 1e9
                                       / HBM_PEAK_GBPS, 4),
        "loss_value": final_loss,
    }

    if wl.patch % 2 == 0:
        out["without_target"] = time_without_target(args, mae, torch, dev, wl, K, M, pred, grad,
                                                    crop_bytes, final_loss)

    if args.embed > 0:
        out["patch_embed"] = time_embed(args, mae, synth, torch, dev, wl, K, args.embed)

    if not args.no_jpeg:
        out["jpeg_prep"] = time_jpeg(args, mae, synth, torch, wl, K)
        # the paper's crop-decode benchmark reads files of maximum side 500 (Sec. 4.1)
        out["jpeg_prep_500"] = time_jpeg(args, mae, synth, torch, wl, K, kind="gradient500")

    if not args.no_finetune and wl.patch % 4 == 0:
        out["finetune_prep"] = time_finetune(args, mae, torch, dev, wl)

    if args.scheme:
        out["stages"] = time_scheme(args, mae, synth, torch, dev, wl, bf16)

    if not args.no_cpu_baseline:
        import oracle

        n = min(args.cpu_sample, wl.B)
        pred_host = pred[:n].float().cpu().numpy()
        kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0, batch_index=0)
        reps = max(1, args.cpu_reps)
        t0 = time.perf_counter()
        for r in range(reps):
            kw["batch_index"] = r
            ref = oracle.prep_batch(images, offsets, heights, widths, b_begin=0, b_end=n, **kw)
            oracle.normpix_loss(pred_host, ref["target"], ref["mask"],
                                num_masked=n * (wl.L - K))
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(n * reps / cpu_s, 1),
            "unit": "images/s",
            "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"first {n} images of the same batch, prep + loss + grad, {reps} passes "
                      f"with different batch indices, {cpu_s:.2f} s wall on "
                      f"{oracle.threads()} threads",
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
