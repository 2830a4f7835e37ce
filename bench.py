"""Benchmark of the MAE input-pipeline hot path on one MI355X.

A step is one pass of the whole path over one batch: mae_prep_batch (crop parameters, masking
order, fused crop/resize/flip/normalise/patchify/gather) followed by mae_normpix_loss (loss and
gradient), on synthetic images already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c4] [--no-cpu-baseline]

`value` is measured on the headline workload (c4).  The other workloads with a loss (c3, c5) are
timed the same way and reported under "configs".  The first consumer of the path's output,
mae_patch_embed, the finetuning-mode input pipeline ("3 Aug", "3 Aug+"), the input pipeline on
JPEG files ("crop decode"), the stages of a progressive schedule and a patch size that takes the
element-wise kernel are timed by themselves after the steps and reported under "patch_embed",
"finetune_prep", "jpeg_prep*", "stages" and "odd_patch_prep"; they are not part of the step or of
`value`.

Every duration comes from events recorded on the stream the library launches on; mean, median and
minimum are given.  Bytes counted by hardware counters come from the summaries under profiles/
(`profiles/counters.md`) and are only quoted while the kernel sources they were taken on are
unchanged.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix rate
# Vector instruction issue: 256 compute units x 4 SIMDs, a 64-lane instruction occupies its SIMD
# for 4 cycles, 2.4 GHz -> 614.4 G wavefront instructions per second.
VALU_PEAK_GINST = 256 * 4 * 2.4 / 4.0

CSRC = "paper_2404_00509_amd/csrc/"
# Kernel sources whose change invalidates the counter figures of a row of profiles/counters.md.
COUNTER_SOURCES = {
    "loss": [CSRC + "normpix_loss.hip", CSRC + "mae_device.hpp"],
    "prep": [CSRC + "crop_patch.hip", CSRC + "mask_params.hip", CSRC + "mae_device.hpp"],
    "finetune": [CSRC + "crop_patch.hip", CSRC + "three_aug.hip", CSRC + "aug_device.hpp",
                 CSRC + "mask_params.hip", CSRC + "mae_device.hpp"],
    "jpeg": [CSRC + "jpeg_decode.hip", CSRC + "mae_device.hpp"],
    "embed": [CSRC + "patch_embed.hip", CSRC + "mae_device.hpp"],
}
COUNTERS_FILE = os.path.join(ROOT, "profiles", "counters.md")


def source_hash(key):
    """Hash of the code of the sources behind a counter row: `//` comments, indentation and empty
    lines do not count, so that rewording a comment does not retire the measurements."""
    h = hashlib.sha256()
    for rel in COUNTER_SOURCES[key]:
        with open(os.path.join(ROOT, rel), "r") as f:
            for line in f:
                code = line.split("//", 1)[0].strip()
                if code:
                    h.update(code.encode() + b"\n")
    return h.hexdigest()[:16]


def profile_counters(key, name):
    """Figures of the row `counter <key> <name> <hash> a=.. b=..` of profiles/counters.md, or None
    when there is no such row or the kernel sources have changed since it was written."""
    try:
        with open(COUNTERS_FILE) as f:
            lines = f.read().splitlines()
    except OSError:
        return None
    for line in lines:
        t = line.replace("`", "").split()
        if len(t) >= 4 and t[0] == "counter" and t[1] == key and t[2] == name:
            if t[3] != source_hash(key):
                print(f"bench.py: profiles/counters.md row '{key} {name}' was taken on other "
                      f"kernel sources; its counter figures are not quoted", file=sys.stderr)
                return None
            return {k: float(v) for k, v in (kv.split("=") for kv in t[4:])}
    return None


def traffic_of(c):
    return None if c is None else c.get("fetch_bytes", 0.0) + c.get("write_bytes", 0.0)


def stats(ms):
    import numpy as np

    a = np.asarray(ms, np.float64)
    return {"avg_ms": round(float(a.mean()), 4), "median_ms": round(float(np.median(a)), 4),
            "min_ms": round(float(a.min()), 4)}


def timed(torch, stream, fn, steps, warmup):
    """fn(i) enqueues one call; returns the per-call durations in ms (events on `stream`)."""
    for i in range(max(warmup, 1)):
        fn(i)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    for i, e in enumerate(ev):
        e[0].record(stream)
        fn(warmup + i)
        e[1].record(stream)
    torch.cuda.synchronize()
    return [e[0].elapsed_time(e[1]) for e in ev]


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


class Workload:
    """Inputs and buffers of one workload, resident on the device."""

    def __init__(self, mae, synth, torch, name):
        self.wl = wl = synth.WORKLOADS[name]
        self.bf16 = wl.dtype == "bf16"
        self.K = mae.mae_num_keep(wl.L, wl.mask_ratio)
        self.M = wl.B * (wl.L - self.K)
        t0 = time.time()
        self.host = synth.make_images(wl.kind, wl.B, seed=0)
        self.gen_s = time.time() - t0
        self.dev = [torch.from_numpy(a).cuda() for a in self.host]
        self.desc = mae.make_prep_desc(*self.dev, out_size=wl.out_size, patch=wl.patch,
                                       num_keep=self.K, seed=0, batch_index=0,
                                       out_dtype=mae.MAE_BF16 if self.bf16 else mae.MAE_F32)
        self.buf = mae.alloc_prep_buffers(self.desc)
        gen = torch.Generator(device="cuda").manual_seed(1)
        pred = torch.randn((wl.B, wl.L, wl.D), generator=gen, device="cuda", dtype=torch.float32)
        self.pred = pred.to(torch.bfloat16) if self.bf16 else pred
        self.grad = torch.empty_like(self.pred)
        self.loss = torch.zeros(1, device="cuda")
        self.ldesc = mae.make_loss_desc(self.pred, self.buf.target, self.buf.mask,
                                        num_masked=self.M)
        self.lws = torch.empty(max(mae.mae_loss_workspace_bytes(self.ldesc), 256),
                               dtype=torch.uint8, device="cuda")
        self.crop_bytes = 0


def run_steps(mae, torch, w, steps, warmup):
    """`steps` timed passes of prep + loss over the workload.  Returns the report of the step and
    of its two calls, and the wall-clock time of the timed region."""
    import numpy as np

    wl, buf, desc, stream = w.wl, w.buf, w.desc, torch.cuda.current_stream()

    def step(i, ev=None):
        desc.batch_index = i
        if ev is not None:
            ev[0].record(stream)
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)
        if ev is not None:
            ev[1].record(stream)
        mae.mae_normpix_loss(w.ldesc, w.loss, w.grad, w.lws, stream=stream)
        if ev is not None:
            ev[2].record(stream)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(warmup + i, events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert mae.mae_prep_status(buf.workspace) == 0

    prep = stats([e[0].elapsed_time(e[1]) for e in events])
    loss = stats([e[1].elapsed_time(e[2]) for e in events])
    both = stats([e[0].elapsed_time(e[2]) for e in events])
    crop = buf.crop.cpu().numpy().astype(np.int64)
    w.crop_bytes = int((crop[:, 2] * crop[:, 3] * 3).sum())
    prep_write, loss_bytes = algorithmic_bytes(wl, w.K)
    prep_bytes = prep_write + w.crop_bytes

    def rate(nbytes, st, key):
        gbps = nbytes / (st["avg_ms"] * 1e-3) / 1e9
        out = dict(st, algorithmic_bytes=nbytes, achieved_GBps=round(gbps, 1),
                   frac=round(gbps / HBM_PEAK_GBPS, 4))
        out["traffic"] = traffic_of(profile_counters(key, wl.name))
        if out["traffic"]:
            out["counter_GBps"] = round(out["traffic"] / (st["avg_ms"] * 1e-3) / 1e9, 1)
            out["counter_frac"] = round(out["counter_GBps"] / HBM_PEAK_GBPS, 4)
        return out

    ms_per_step = elapsed * 1e3 / steps
    report = {
        "ms_per_step": round(ms_per_step, 4),
        "images_per_s": round(wl.B * steps / elapsed, 1),
        "step_ms_by_events": both,
        "kernels": {"mae_prep_batch": rate(prep_bytes, prep, "prep"),
                    "mae_normpix_loss": rate(loss_bytes, loss, "loss")},
        "step_GBps": round((prep_bytes + loss_bytes) / (ms_per_step * 1e-3) / 1e9, 1),
        "step_frac_of_hbm_peak": round((prep_bytes + loss_bytes) / (ms_per_step * 1e-3) / 1e9
                                       / HBM_PEAK_GBPS, 4),
        "loss_value": float(w.loss.item()),
    }
    counted = [k["traffic"] for k in report["kernels"].values()]
    if all(counted):  # the step on the bytes the hardware counters saw
        gbps = sum(counted) / (ms_per_step * 1e-3) / 1e9
        report["step_counter_GBps"] = round(gbps, 1)
        report["step_counter_frac_of_hbm_peak"] = round(gbps / HBM_PEAK_GBPS, 4)
    return report, elapsed


def time_copy(torch, w, steps):
    """A plain device copy of the size of the loss call's tensors (grad <- pred): what this machine's
    memory system delivers to the simplest kernel there is (read + write, same size)."""
    stream = torch.cuda.current_stream()
    st = stats(timed(torch, stream, lambda i: w.grad.copy_(w.pred), steps, 2))
    nbytes = 2 * w.pred.numel() * w.pred.element_size()
    gbps = nbytes / (st["avg_ms"] * 1e-3) / 1e9
    return dict(st, bytes=nbytes, GBps=round(gbps, 1),
                frac_of_peak=round(gbps / HBM_PEAK_GBPS, 4),
                what="torch copy_ of the prediction tensor into the gradient tensor")


def time_stages(args, mae, torch, w):
    """Per-stage times of the paper's progressive schedules on buffers allocated once: pretraining
    scheme 5 (Table 9: 224 -> 192 -> 224, prep + loss per step) and finetuning scheme 1 (Table 7:
    160 / 192 / 224 with the stage's crop range and augmentation, prep only, every patch kept)."""
    wl, bf16, dev = w.wl, w.bf16, w.dev
    stream = torch.cuda.current_stream()
    steps = max(3, args.steps // 3)
    out = {}
    scheme = args.scheme or 5
    stages = [mae.mae_pretrain_stage(scheme, s) for s in (1, 2, 3)]
    bufs = mae.ProgressiveBuffers(wl.B, wl.patch, stages, bf16=bf16)
    D = 3 * wl.patch * wl.patch
    max_l = max(sh[1] for sh in bufs.shapes)
    pred_store = torch.randn(wl.B * max_l * D, device="cuda")
    if bf16:
        pred_store = pred_store.to(torch.bfloat16)
    grad_store = torch.empty_like(pred_store)
    loss = torch.zeros(1, device="cuda")
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

        def step(j, i=i, desc=desc, buf=buf, ldesc=ldesc, grad=grad, lws=lws):
            desc.batch_index = 1000 * (i + 1) + j
            mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep,
                               buf.target, buf.crop, buf.workspace, stream=stream)
            mae.mae_normpix_loss(ldesc, loss, grad, lws, stream=stream)

        st = stats(timed(torch, stream, step, steps, 2))
        rows.append(dict(st, stage=i + 1, out_size=res, mask_ratio=m, L=L, K=K,
                         images_per_s=round(wl.B / (st["avg_ms"] * 1e-3), 1)))
    out[f"pretrain_scheme{scheme}"] = rows
    del bufs, pred_store, grad_store

    if wl.patch % 4 == 0:
        plan = [mae.mae_finetune_stage(mae.MAE_FINETUNE_SCHEME_1, s) for s in (1, 2, 3)]
        bufs = mae.ProgressiveBuffers(wl.B, wl.patch, [(res, 0.0) for res, _, _, _ in plan],
                                      want_target=False, aug_mode=mae.MAE_AUG_THREE_PLUS)
        rows = []
        for i, (res, lo, hi, aug) in enumerate(plan):
            _, L, K, _ = bufs.shapes[i]
            buf = bufs.stage(i)
            desc = mae.make_prep_desc(*dev, out_size=res, patch=wl.patch, num_keep=L,
                                      scale=(lo, hi), seed=0, batch_index=0, aug_mode=aug,
                                      jitter=0.3)

            def step(j, i=i, desc=desc, buf=buf):
                desc.batch_index = 2000 * (i + 1) + j
                mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep,
                                   None, buf.crop, buf.workspace, stream=stream)

            st = stats(timed(torch, stream, step, steps, 2))
            rows.append(dict(st, stage=i + 1, out_size=res,
                             augmentation="3 Aug+" if aug == mae.MAE_AUG_THREE_PLUS else "3 Aug",
                             images_per_s=round(wl.B / (st["avg_ms"] * 1e-3), 1)))
        out["finetune_scheme1"] = rows
    return out


def time_embed(args, mae, synth, torch, w, E):
    """mae_patch_embed on every visible row of the batch (bf16 in, bf16 out), timed by itself with
    events on the launch stream.  Not part of the step above."""
    wl, K = w.wl, w.K
    desc = mae.make_prep_desc(*w.dev, out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0,
                              batch_index=0, out_dtype=mae.MAE_BF16)
    buf = mae.alloc_prep_buffers(desc, want_target=False)
    stream = torch.cuda.current_stream()
    mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None,
                       buf.crop, buf.workspace, stream=stream)
    weight, bias, pos = synth.make_embed_params(0, wl.D, E, wl.L)
    wt = torch.from_numpy(weight).cuda().to(torch.bfloat16)
    b, p = torch.from_numpy(bias).cuda(), torch.from_numpy(pos).cuda()
    tokens = torch.empty((wl.B, K, E), dtype=torch.bfloat16, device="cuda")
    edesc = mae.make_embed_desc(buf.visible, buf.ids_keep, wt, b, p, out_dtype=mae.MAE_BF16)
    st = stats(timed(torch, stream, lambda i: mae.mae_patch_embed(edesc, tokens, stream=stream),
                     args.steps, args.warmup))
    M = wl.B * K
    # for scale only: the vendor library's bare product of the same shape (no bias, no positional
    # rows, no gather), through torch.mm on the same stream
    vis2 = buf.visible.view(M, wl.D)
    ref = torch.empty((M, E), dtype=torch.bfloat16, device="cuda")
    lib = stats(timed(torch, stream, lambda i: torch.mm(vis2, wt.t(), out=ref), args.steps,
                      args.warmup))
    flops = 2.0 * M * wl.D * E
    nbytes = 2 * M * wl.D + 2 * M * E + 2 * E * wl.D + 4 * M + 4 * wl.L * E + 4 * E
    tflops = flops / (st["avg_ms"] * 1e-3) / 1e12
    return dict(st, **{
        "kernel": "patch_embed_kernel (mae_patch_embed), bf16 x bf16 -> fp32 -> bf16",
        "M": M, "D": wl.D, "E": E,
        "bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
        "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "flops": flops, "algorithmic_bytes": nbytes,
        "traffic": traffic_of(profile_counters("embed", wl.name)),
        "achieved_GBps": round(nbytes / (st["avg_ms"] * 1e-3) / 1e9, 1),
        "checksum": float(tokens.float().abs().mean().item()),
        "library_bare_product": dict(lib, what="torch.mm of the same operands: no bias, no "
                                               "positional rows; for scale"),
    })


def alu_roofline(key, name, avg_ms):
    """Vector-instruction issue rate of a call whose kernels are bound by it, from the instruction
    count of its counter run (profiles/counters.md) and the duration measured here."""
    c = profile_counters(key, name)
    if c is None or "valu_insts" not in c:
        return None
    ginst = c["valu_insts"] / (avg_ms * 1e-3) / 1e9
    return {"bound": "alu", "achieved": round(ginst, 1), "peak": VALU_PEAK_GINST,
            "unit": "G wavefront instructions/s", "frac": round(ginst / VALU_PEAK_GINST, 4),
            "valu_insts": c["valu_insts"],
            "model": "a 64-lane vector instruction occupies one of the 1024 SIMDs for 4 cycles "
                     "at 2.4 GHz; instructions counted by SQ_INSTS_VALU over the call's kernels"}


def time_finetune(args, mae, torch, w):
    """mae_prep_batch in finetuning mode (Table 7, last stage: 224 px, crop side ratio 0.28..1,
    every patch kept, fp32 tokens in `visible`, no `target`) with "3 Aug" and "3 Aug+", timed by
    itself with events on the launch stream.  Not part of the step above."""
    import numpy as np

    wl, dev = w.wl, w.dev
    rows = []
    res, lo, hi, _ = mae.mae_finetune_stage(mae.MAE_FINETUNE_SCHEME_1, 3)
    L = (res // wl.patch) ** 2
    stream = torch.cuda.current_stream()
    for mode, name in ((mae.MAE_AUG_THREE, "3 Aug"), (mae.MAE_AUG_THREE_PLUS, "3 Aug+")):
        desc = mae.make_prep_desc(*dev, out_size=res, patch=wl.patch, num_keep=L, scale=(lo, hi),
                                  seed=0, batch_index=0, aug_mode=mode, jitter=0.3)
        buf = mae.alloc_prep_buffers(desc, want_target=False)

        def run(i, desc=desc, buf=buf):
            desc.batch_index = i
            mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, None,
                               buf.crop, buf.workspace, stream=stream)

        st = stats(timed(torch, stream, run, args.steps, args.warmup))
        assert mae.mae_prep_status(buf.workspace) == 0
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
        key = "three" if mode == mae.MAE_AUG_THREE else "three_plus"
        gbps = nbytes / (st["avg_ms"] * 1e-3) / 1e9
        rows.append(dict(st, augmentation=name, out_size=res,
                         images_per_s=round(wl.B / (st["avg_ms"] * 1e-3), 1),
                         algorithmic_bytes=nbytes, intermediate_bytes_estimate=extra,
                         traffic=traffic_of(profile_counters("finetune", key)),
                         achieved_GBps=round(gbps, 1), frac=round(gbps / HBM_PEAK_GBPS, 4),
                         alu=alu_roofline("finetune", key, st["avg_ms"])))
        del buf
    return rows


def time_odd_patch(args, mae, torch, w):
    """mae_prep_batch with a patch size whose rows are not whole 16-byte groups (3 p p % 4 != 0):
    the same images to 225 px in patches of 15 (D = 675), keep a quarter.  These shapes take the
    element-wise kernel instead of the staged one; this is what that costs."""
    wl, dev = w.wl, w.dev
    S, p = 225, 15
    L = (S // p) ** 2
    K = mae.mae_num_keep(L, 0.75)
    desc = mae.make_prep_desc(*dev, out_size=S, patch=p, num_keep=K, seed=0, batch_index=0)
    buf = mae.alloc_prep_buffers(desc)
    stream = torch.cuda.current_stream()

    def run(i):
        desc.batch_index = i
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)

    st = stats(timed(torch, stream, run, max(5, args.steps // 3), 2))
    assert mae.mae_prep_status(buf.workspace) == 0
    D = 3 * p * p
    nbytes = w.crop_bytes + wl.B * (K * D * 4 + L * D * 4 + L * 5 + K * 4)
    gbps = nbytes / (st["avg_ms"] * 1e-3) / 1e9
    return dict(st, out_size=S, patch=p, D=D, algorithmic_bytes=nbytes,
                achieved_GBps=round(gbps, 1), frac=round(gbps / HBM_PEAK_GBPS, 4),
                images_per_s=round(wl.B / (st["avg_ms"] * 1e-3), 1))


def time_without_target(args, mae, torch, w, want_loss):
    """The same step without a stored target: mae_prep_batch with target = NULL (visible tokens,
    mask and ids only) and mae_normpix_loss_from_images, which takes the masked patches' pixels
    from the images again.  Same outputs except `target`; timed like the step above."""
    wl, K, M, bf16 = w.wl, w.K, w.M, w.bf16
    desc = mae.make_prep_desc(*w.dev, out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0,
                              batch_index=0, out_dtype=mae.MAE_BF16 if bf16 else mae.MAE_F32)
    buf = mae.alloc_prep_buffers(desc, want_target=False)
    ldesc = mae.make_loss_desc(w.pred, None, buf.mask, num_masked=M)
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
        mae.mae_normpix_loss_from_images(desc, buf.workspace, ldesc, loss, w.grad, lws,
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
    prep = stats([e[0].elapsed_time(e[1]) for e in events])
    lst = stats([e[1].elapsed_time(e[2]) for e in events])
    e = 2 if bf16 else 4
    # what this dataflow must move: the crop's bytes twice, the visible tokens, mask and ids;
    # the masked rows of the prediction, the whole gradient
    prep_bytes = w.crop_bytes + wl.B * (K * wl.D * e + wl.L * 5 + K * 4)
    loss_bytes = w.crop_bytes + wl.B * ((wl.L - K) * wl.D * e + wl.L * wl.D * e + wl.L)
    ms = elapsed * 1e3 / args.steps
    return {
        "what": "mae_prep_batch(target = NULL) + mae_normpix_loss_from_images",
        "ms_per_step": round(ms, 4), "images_per_s": round(wl.B * args.steps / elapsed, 1),
        "loss_value": got,
        "kernels": {
            "mae_prep_batch": dict(prep, algorithmic_bytes=prep_bytes,
                                   achieved_GBps=round(prep_bytes / (prep["avg_ms"] * 1e-3) / 1e9,
                                                       1)),
            "mae_normpix_loss_from_images": dict(
                lst, algorithmic_bytes=loss_bytes,
                achieved_GBps=round(loss_bytes / (lst["avg_ms"] * 1e-3) / 1e9, 1),
                frac=round(loss_bytes / (lst["avg_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)),
        },
    }


def time_jpeg(args, mae, synth, torch, w, kind=None, restart_rows=1, name="jpeg_prep",
              indexed=False):
    """mae_prep_batch fed with JPEG files ("crop decode", Sec. 4.1): the same batch written as
    baseline JPEG (quality 90, 4:2:0; one restart interval per row of MCUs, or no restart markers
    at all, which is what an encoder writes by default), timed by itself with events on the
    launch stream.  indexed: the call is given the files' row index, which mae_jpeg_index computes
    once (timed beside it).  Not part of the step above."""
    import numpy as np

    wl, K = w.wl, w.K
    t0 = time.time()
    kind = kind or wl.kind
    B = wl.B
    files, offsets, sizes = synth.make_jpegs(kind, B, seed=0, restart_rows=restart_rows)
    enc_s = time.time() - t0
    dev = [torch.from_numpy(a).cuda() for a in (files, offsets, sizes)]
    stream = torch.cuda.current_stream()
    kw = dict(file_sizes=dev[2], out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0,
              batch_index=0, max_image_side=512 if kind == "gradient500" else 0,
              out_dtype=mae.MAE_BF16 if wl.dtype == "bf16" else mae.MAE_F32)
    index, index_ms = None, None
    if indexed:
        # the files' row index: computed once per file (here: once, timed), reused by every call
        d0 = mae.make_prep_desc(dev[0], dev[1], None, None, **kw)
        index = torch.empty(mae.mae_jpeg_index_bytes(d0), dtype=torch.uint8, device="cuda")
        ws0 = torch.empty(mae.mae_prep_workspace_bytes(d0), dtype=torch.uint8, device="cuda")
        index_ms = stats(timed(torch, stream, lambda i: mae.mae_jpeg_index(d0, index, ws0,
                                                                           stream=stream), 3, 1))
        del ws0
    desc = mae.make_prep_desc(dev[0], dev[1], None, None, row_index=index, **kw)
    buf = mae.alloc_prep_buffers(desc)

    def run(i):
        desc.batch_index = i
        mae.mae_prep_batch(desc, buf.visible, buf.mask, buf.ids_restore, buf.ids_keep, buf.target,
                           buf.crop, buf.workspace, stream=stream)

    st = stats(timed(torch, stream, run, max(3, args.steps // 2), 2))
    assert mae.mae_prep_status(buf.workspace) == 0
    crop = buf.crop.cpu().numpy().astype(np.int64)
    out = dict(st, **{
        "input": "baseline JPEG, quality 90, 4:2:0, "
                 + ("restart interval = one row of MCUs" if restart_rows == 1
                    else "no restart markers"),
        "file_bytes": int(files.size), "encode_s_on_host": round(enc_s, 1),
        "images": kind, "B": B,
        "images_per_s": round(B / (st["avg_ms"] * 1e-3), 1),
        "compressed_GBps": round(files.size / (st["avg_ms"] * 1e-3) / 1e9, 1),
        "mean_crop_area_px": round(float((crop[:, 2] * crop[:, 3]).mean()), 1),
        "roofline": alu_roofline("jpeg", name, st["avg_ms"]),
    })
    if indexed:
        out["input"] += ", with the files' row index (mae_jpeg_index)"
        out["index_once"] = dict(index_ms, bytes=int(index.numel()),
                                 what="mae_jpeg_index over the batch's files, once per file")
    if not args.no_cpu_baseline and name == "jpeg_prep":
        # the oracle beside it: whole-file decode (its definition of the input) of a small sample
        import oracle

        n = min(256, B)
        t0 = time.perf_counter()
        for o, m in zip(offsets[:n], sizes[:n]):
            oracle.jpeg_decode(files[o:o + m].tobytes())
        dt = time.perf_counter() - t0
        out["cpu_oracle_decode"] = {
            "images_per_s": round(n / dt, 1), "cores": 1, "kind": "oracle",
            "sample": f"whole-file decode of the first {n} files of the batch, decode only"}
    return out


def cpu_baseline(args, w):
    """The oracle as it stands on the host cores: all of them on a bounded sample of the same
    batch, and one thread on a 256-image slice."""
    import oracle

    wl, K = w.wl, w.K
    images, offsets, heights, widths = w.host
    n = min(args.cpu_sample, wl.B)
    pred_host = w.pred[:n].float().cpu().numpy()
    kw = dict(out_size=wl.out_size, patch=wl.patch, num_keep=K, seed=0, batch_index=0)

    def passes(count, reps):
        t0 = time.perf_counter()
        for r in range(reps):
            kw["batch_index"] = r
            ref = oracle.prep_batch(images, offsets, heights, widths, b_begin=0, b_end=count, **kw)
            oracle.normpix_loss(pred_host[:count], ref["target"], ref["mask"],
                                num_masked=count * (wl.L - K))
        return time.perf_counter() - t0

    reps = max(1, args.cpu_reps)
    cores = oracle.threads()
    all_s = passes(n, reps)
    oracle.set_threads(1)
    one_n = min(256, wl.B)
    one_s = passes(one_n, 1)
    oracle.set_threads(0)
    return {
        "value": round(n * reps / all_s, 1), "unit": "images/s", "cores": cores, "kind": "oracle",
        "sample": f"first {n} images of the same batch, prep + loss + grad, {reps} passes with "
                  f"different batch indices, {all_s:.2f} s wall on {cores} threads",
        "single_thread": {"value": round(one_n / one_s, 1), "unit": "images/s", "cores": 1,
                          "sample": f"first {one_n} images, one pass, {one_s:.2f} s wall"},
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
                    help="pretraining scheme 1..6 (Table 9) whose stages are timed (default 5)")
    ap.add_argument("--embed", type=int, default=768,
                    help="embedding width E for the separately timed mae_patch_embed launch over "
                         "the batch's visible rows (adds 'patch_embed' to the JSON line); 0 = skip")
    ap.add_argument("--no-jpeg", action="store_true",
                    help="skip the separately timed calls on JPEG input ('jpeg_prep*')")
    ap.add_argument("--no-finetune", action="store_true",
                    help="skip the separately timed finetuning-mode calls ('finetune_prep')")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other workloads ('configs') and the schedules ('stages')")
    ap.add_argument("--only", default="",
                    help="comma-separated extras to run after the steps instead of all of them "
                         "(embed, jpeg, jpeg_no_markers, jpeg_indexed, jpeg_500, finetune, configs, stages, "
                         "without_target, odd_patch, none); for profiling runs")
    ap.add_argument("--source-hashes", action="store_true",
                    help="print the hashes that key the rows of profiles/counters.md and exit")
    args = ap.parse_args()
    if args.source_hashes:
        print(json.dumps({k: source_hash(k) for k in COUNTER_SOURCES}))
        return 0
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no multi-GPU part (samples are "
              "independent, so a batch shards by sample and only the loss scalar would be "
              "exchanged). Run with --gpus 1.",
              file=sys.stderr)
        return 2

    import torch

    import paper_2404_00509_amd as mae
    from paper_2404_00509_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    mae.load()  # fail loudly if the HIP library is missing

    only = set(filter(None, args.only.split(",")))

    def want(name):
        return name in only if only else True

    w = Workload(mae, synth, torch, args.workload)
    wl, K = w.wl, w.K
    report, _ = run_steps(mae, torch, w, args.steps, args.warmup)
    lk = report["kernels"]["mae_normpix_loss"]

    out = {
        "metric": "images/sec and achieved HBM GB/s (% of peak) at 224px, B=4096, 1 MI355X",
        "value": report["images_per_s"],
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": report["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if w.bf16 else "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{wl.name}: B={wl.B} uint8 images (max side 256) -> {wl.out_size}px, "
                        f"patch {wl.patch}, L={wl.L}, keep {K}, prep + normpix loss + grad",
            "B": wl.B, "out_size": wl.out_size, "patch": wl.patch, "L": wl.L, "K": K, "D": wl.D,
            "input_generation_s": round(w.gen_s, 1),
        },
        "roofline": {
            "kernel": "normpix_loss_kernel (mae_normpix_loss; includes its 1-workgroup finish "
                      "kernel)",
            "bound": "hbm",
            "achieved": lk["achieved_GBps"],
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": lk["frac"],
            "traffic": lk["traffic"],
            "algorithmic_bytes": lk["algorithmic_bytes"],
            "avg_ms": lk["avg_ms"], "median_ms": lk["median_ms"], "min_ms": lk["min_ms"],
        },
        "step_ms_by_events": report["step_ms_by_events"],
        "kernels": report["kernels"],
        "step_GBps": report["step_GBps"],
        "step_frac_of_hbm_peak": report["step_frac_of_hbm_peak"],
        "step_counter_GBps": report.get("step_counter_GBps"),
        "step_counter_frac_of_hbm_peak": report.get("step_counter_frac_of_hbm_peak"),
        "loss_value": report["loss_value"],
        "hbm_copy_ceiling": time_copy(torch, w, 10),
    }

    if wl.patch % 2 == 0 and want("without_target"):
        out["without_target"] = time_without_target(args, mae, torch, w, report["loss_value"])
    if args.embed > 0 and want("embed"):
        out["patch_embed"] = time_embed(args, mae, synth, torch, w, args.embed)
    if not args.no_jpeg:
        if want("jpeg"):
            out["jpeg_prep"] = time_jpeg(args, mae, synth, torch, w)
        if want("jpeg_no_markers"):
            out["jpeg_prep_no_markers"] = time_jpeg(args, mae, synth, torch, w, restart_rows=0,
                                                    name="jpeg_prep_no_markers")
        if want("jpeg_indexed"):
            out["jpeg_prep_no_markers_indexed"] = time_jpeg(
                args, mae, synth, torch, w, restart_rows=0, name="jpeg_prep_no_markers_indexed",
                indexed=True)
        if want("jpeg_500"):
            # the paper's crop-decode benchmark reads files of maximum side 500 (Sec. 4.1)
            out["jpeg_prep_500"] = time_jpeg(args, mae, synth, torch, w, kind="gradient500",
                                             name="jpeg_prep_500")
    if not args.no_finetune and wl.patch % 4 == 0 and want("finetune"):
        out["finetune_prep"] = time_finetune(args, mae, torch, w)
    if want("odd_patch"):
        out["odd_patch_prep"] = time_odd_patch(args, mae, torch, w)
    if not args.no_configs and want("stages"):
        out["stages"] = time_stages(args, mae, torch, w)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args, w)

    if not args.no_configs and want("configs"):
        # the other workloads with a loss, timed like the headline one (fewer steps)
        del w
        torch.cuda.empty_cache()
        out["configs"] = {}
        for name in ("c3", "c4", "c5"):
            if name == args.workload:
                continue
            other = Workload(mae, synth, torch, name)
            rep, _ = run_steps(mae, torch, other, max(5, args.steps // 2), 3)
            rep["dtype"] = "bf16" if other.bf16 else "f32"
            rep["B"], rep["out_size"], rep["patch"] = other.wl.B, other.wl.out_size, other.wl.patch
            if other.wl.patch % 2 == 0:
                a2 = argparse.Namespace(**vars(args))
                a2.steps, a2.warmup = max(5, args.steps // 2), 3
                rep["without_target"] = time_without_target(a2, mae, torch, other,
                                                            rep["loss_value"])
            out["configs"][name] = rep
            del other
            torch.cuda.empty_cache()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
