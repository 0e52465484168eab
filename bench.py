#!/usr/bin/env python3
"""Benchmark of the spatially partitioned 3x3x3 convolution hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic 512^3 x 32-channel bf16 volume on a
4x4x1 tile grid (the one-GPU share at the paper's largest resolution):

    partition x -> halo pack -> halo unpack -> conv3d_fwd -> unpartition y
    partition dy -> halo pack -> halo unpack -> conv3d_dgrad -> unpartition dx
    conv3d_wgrad (dw, db)

The padded arrays are zeroed once when they are allocated, so the step's halo calls carry the SP_HALO_* flags:
nothing is packed for directions in which a tile has no neighbour and the zero margins at the volume border are
not rewritten.  Their bandwidth figures count the bytes such a call moves (regions with a neighbour, read once
and written once); the same calls without the flags (every region packed, border margins zero-filled) are timed
after the step and reported beside them with their own byte counts.

Inputs are resident in HBM before the timed region.  Prints ONE JSON line.  `value` is 3 conv passes'
FLOPs divided by the whole step time, i.e. it is charged for partitioning and halo exchange too;
`roofline` rates the dominant kernel (algorithmic FLOPs of one launch / its HIP-event time) against the
dense bf16 peak, `cpu_baseline` is the fp64 oracle timed on the host cores on a corner box of the same
tensors.
"""
import argparse
import itertools
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E

# HBM traffic per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script with --calib-copy (each counter scaled by what it reads for the plain 1 GiB copy of known size:
# FETCH_SIZE x 2.0, WRITE_SIZE x 1.0); None = not measured at that size.
MEASURED_TRAFFIC_BYTES = {512: 18.53e9}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--size", type=int, default=512, help="volume edge (512 = headline workload)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default="c4", choices=["c4", "c5", "paper512", "paper2d"],
                    help="c4 = headline single-layer workload (default); c5 = the whole U-Net convolution "
                         "stack of the workload list (256^3, channels 32/64/128/256), forward + backward; "
                         "paper512 = the network the paper trains at 512^3 (six blocks of four convolutions, "
                         "32 ... 1024 filters), forward + backward, all 16 tiles in this GPU's HBM; "
                         "paper2d = the paper's 2-D U-Net (same architecture, 2-D operations) on a batch of "
                         "512 x 512 x 5 slabs, grid 1x4x4")
    ap.add_argument("--slabs", type=int, default=16, help="paper2d: slabs per step (the stack axis of the tensors)")
    ap.add_argument("--grid", default=None,
                    help="U-Net workloads: tile grid gd,gh,gw (default 4,4,1; paper2d: 1,2,2)")
    ap.add_argument("--loss", action="store_true",
                    help="U-Net workloads: compute the upstream gradient with sp_dice_ce_loss on seeded labels "
                         "instead of the N(0,1) stand-in of the workload list (adds the loss passes to the step)")
    ap.add_argument("--halo", type=int, default=1, choices=[1, 2],
                    help="U-Net workloads: margin width of the layout; 2 = two layers of a block share one exchange "
                         "(the first also computes the voxel shell the second reads)")
    ap.add_argument("--coarse-grid", default=None,
                    help="U-Net workloads: tile grid gd,gh,gw of the coarse levels (tiles merged below "
                         "--coarse-from); default: the same grid at every level")
    ap.add_argument("--coarse-from", type=int, default=3,
                    help="U-Net workloads: first level (0 = full resolution) that uses --coarse-grid")
    ap.add_argument("--gather", action="store_true",
                    help="no halo exchange where the kernels can gather (SP_HALO_GATHER: the convolutions read "
                         "their margin voxels from the neighbour tiles' interiors); in the headline workload the "
                         "step then has no halo_pack / halo_unpack launches")
    ap.add_argument("--bits", action="store_true",
                    help="U-Net workloads: ReLU masks between the layers of a block as one bit per value "
                         "(conv3d_fwd_bits / conv3d_dgrad_bits) instead of re-reading the activation")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (torch copy_) so that profiler "
                         "byte counters can be scaled against a kernel of known traffic")
    ap.add_argument("--no-calib-gemm", dest="calib_gemm", action="store_false",
                    help="skip timing the vendor library's dense bf16 GEMM (torch.matmul, 8192^3, normal data; "
                         "reported as `library_gemm_tflops`: context for what a matrix-core-bound kernel "
                         "sustains on this box, measured after the timed steps and not part of them)")
    return ap.parse_args()


def bench_unet(args):
    """Secondary workload: the U-Net convolution stack (configuration 5), one step = forward + backward."""
    import numpy as np
    import torch
    from paper_1909_03108_amd import sp3d, synth, unet

    torch.cuda.set_device(0)
    flat = args.workload == "paper2d"
    paper = args.workload == "paper512" or flat
    S = args.size if (paper or args.size != 512) else 256
    channels, in_ch, classes = ((32, 64, 128, 256, 512, 1024) if paper else (32, 64, 128, 256)), (5 if flat else 1), 3
    convs = 4 if paper else 2
    n, dhw, grid = 1, ((args.slabs, S, S) if flat else (S, S, S)), ((1, 2, 2) if flat else (4, 4, 1))
    if args.grid:
        grid = tuple(int(v) for v in args.grid.split(","))
        assert len(grid) == 3
    plan = unet.layer_plan(channels, in_ch, classes, convs, flat=flat)
    nd = 2 if flat else 3

    def dev(a):
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    if flat:     # a slab = 5 neighbouring slices as channels: five draws of the CT-like generator
        x = dev(np.concatenate([synth.ct_like_volume((n,) + dhw + (1,), synth.seed_for(5, synth.T_INPUT) + 977 * i,
                                                     "bf16") for i in range(in_ch)], axis=-1))
    else:
        x = dev(synth.ct_like_volume((n,) + dhw + (in_ch,), synth.seed_for(5, synth.T_INPUT), "bf16"))
    w = {name: dev(synth.weights(shape[nd], shape[nd + 1], synth.seed_for(5, synth.T_WEIGHT0 + k), "bf16",
                                 taps=shape[:nd])) for k, (name, shape) in enumerate(plan)}
    dl = dev(synth.normal_volume((n,) + dhw + (classes,), synth.seed_for(5, synth.T_UPSTREAM), "bf16"))
    grids = None
    if args.coarse_grid:
        cg = tuple(int(v) for v in args.coarse_grid.split(","))
        grids = [grid if i < args.coarse_from else cg for i in range(len(channels))]
    net = unet.UNet(n, dhw, grid, w, channels, in_ch, classes, convs=convs, halo=args.halo, flat=flat,
                    gather=args.gather, grids=grids, bits=args.bits)

    labels = None
    if args.loss:
        lab = np.random.default_rng(synth.seed_for(5, synth.T_UPSTREAM)).integers(0, classes, size=(n,) + dhw + (1,))
        labels = dev(synth.f32_to_bf16_bits(lab.astype(np.float32)))

    def step():
        net.forward(x)
        if labels is not None:
            net.loss(labels)
            net.backward(None, input_grad=False)
        else:
            net.backward(dl, input_grad=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    vox = n * dhw[0] * dhw[1] * dhw[2]
    flop = 0.0
    for name, shape in plan:
        lvl_vox = vox
        if name[:3] in ("enc", "dec"):
            lvl_vox = vox >> (nd * int(name[3]))
        elif name[:2] == "up":
            lvl_vox = vox >> (nd * int(name[2]))
        taps = int(np.prod(shape[:nd]))
        per = 2.0 * shape[nd] * shape[nd + 1] * lvl_vox * (taps if taps != 2 ** nd else 1)   # up-conv: 1 tap per output voxel
        flop += 3 * per
    flop -= 2.0 * 3 ** nd * in_ch * channels[0] * vox               # no image gradient
    if flat:
        name = ("paper2d_unet_%dx%dx%d: %d slabs of %d slices as channels, six blocks of four 3x3 convolutions, "
                "32/64/128/256/512/1024 filters" % (S, S, in_ch, args.slabs, in_ch))
    else:
        name = ("paper512_unet_%d^3: six blocks of four 3x3x3 convolutions, 32/64/128/256/512/1024 filters"
                if paper else "c5_unet_%d^3: channels 32/64/128/256") % S
    print(json.dumps({
        "metric": "U-Net conv stack fwd+bwd TFLOP/s (bf16), secondary workload", "value": round(flop / ms / 1e9, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name + (", grid %dx%dx%d, halo %d, forward + backward (weight and data gradients, "
                                       "no image gradient)" % (grid + (args.halo,))) + (", upstream gradient from the Dice + CE loss"
                                                              if args.loss else "")
                               + (", halos gathered by the convolutions (no exchange)" if args.gather else "")
                               + (", one-bit ReLU masks inside the blocks" if args.bits else "")
                               + (", grid %s from level %d on" % (args.coarse_grid, args.coarse_from) if grids else ""),
                   "tflop_per_step": round(flop / 1e12, 2),
                   "hbm_allocated_gb": round(torch.cuda.max_memory_allocated() / 1e9, 1)}}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all tiles of the grid live in one HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.workload in ("c5", "paper512", "paper2d"):
        return bench_unet(args)

    import numpy as np
    import torch
    from paper_1909_03108_amd import sp3d, synth

    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[4]
    S = args.size
    dhw, grid, c = (S, S, S), cfg["grid"], 32
    n = 1
    g = sp3d.Geom(n, dhw, grid)
    dt = sp3d.SP_BF16

    # ---- seeded synthetic inputs (host), then resident in HBM -------------------------------------
    t0 = time.time()
    x_h, ws_h, dy_h = synth.config_tensors(4, dhw=dhw)
    w_h = ws_h[0]
    t_gen = time.time() - t0

    def dev(a):
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)

    x_vol, dy_vol, w = dev(x_h), dev(dy_h), dev(w_h)
    vol_shape = (n,) + dhw + (c,)
    y_vol = torch.empty(vol_shape, dtype=torch.bfloat16, device="cuda")
    dx_vol = torch.empty(vol_shape, dtype=torch.bfloat16, device="cuda")
    Px, Py = sp3d.alloc_padded(g, c, dt), sp3d.alloc_padded(g, c, dt)
    Pdy, Pdx = sp3d.alloc_padded(g, c, dt), sp3d.alloc_padded(g, c, dt)
    M = sp3d.alloc_msg(g, c, dt)
    dw = torch.empty((3, 3, 3, c, c), dtype=torch.float32, device="cuda")
    db = torch.empty((c,), dtype=torch.float32, device="cuda")
    wsp = {op: sp3d.alloc_ws(sp3d.sp_workspace_bytes(op, g, c, c, dt)) for op in (0, 1, 2)}
    stream = torch.cuda.current_stream()
    gb = g.with_opts(sp3d.SP_HALO_SKIP_SEND | sp3d.SP_HALO_KEEP_ZERO)    # halo calls of the step

    gc = g.with_opts(sp3d.SP_HALO_GATHER) if args.gather else g    # convolutions of the step
    calls = [
        ("sp_partition", lambda: sp3d.sp_partition(x_vol, Px, g, c, dt, stream)),
        ("halo_pack", lambda: sp3d.halo_pack(Px, M, gb, c, dt, stream)),
        ("halo_unpack", lambda: sp3d.halo_unpack(Px, M, gb, c, dt, stream)),
        ("conv3d_fwd", lambda: sp3d.conv3d_fwd(Px, w, None, Py, gc, c, c, dt, 0, wsp[0], stream)),
        ("sp_unpartition", lambda: sp3d.sp_unpartition(Py, y_vol, g, c, dt, stream)),
        ("sp_partition", lambda: sp3d.sp_partition(dy_vol, Pdy, g, c, dt, stream)),
        ("halo_pack", lambda: sp3d.halo_pack(Pdy, M, gb, c, dt, stream)),
        ("halo_unpack", lambda: sp3d.halo_unpack(Pdy, M, gb, c, dt, stream)),
        ("conv3d_dgrad", lambda: sp3d.conv3d_dgrad(Pdy, w, Pdx, gc, c, c, dt, wsp[1], stream)),
        ("sp_unpartition", lambda: sp3d.sp_unpartition(Pdx, dx_vol, g, c, dt, stream)),
        ("conv3d_wgrad", lambda: sp3d.conv3d_wgrad(Px, Pdy, dw, db, gc, c, c, dt, wsp[2], stream)),
    ]
    if args.gather:        # the convolutions read their neighbours' voxels themselves: no pack, no unpack
        calls = [kv for kv in calls if not kv[0].startswith("halo_")]

    def step(events=None):
        for name, f in calls:
            if events is not None:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                f()
                e1.record(stream)
                events.append((name, e0, e1))
            else:
                f()

    if args.calib_copy:
        a = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda")
        b = torch.ones((1 << 30,), dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        a.copy_(b)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    gemm_tflops = None
    if args.calib_gemm:
        ma = torch.randn(8192, 8192, device="cuda").bfloat16()
        mb = torch.randn(8192, 8192, device="cuda").bfloat16()
        for _ in range(3):
            mc = ma @ mb
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(20):
            mc = ma @ mb
        e1.record()
        torch.cuda.synchronize()
        gemm_tflops = 20 * 2.0 * 8192 ** 3 / (e0.elapsed_time(e1) * 1e-3) / 1e12
        del ma, mb, mc

    # outside the timed step: the one-pass exchange (what a one-GPU caller would use instead of pack + unpack), and
    # pack / unpack / exchange without the border flags (all 26 regions packed, border margins zero-filled)
    def median_ms(f, reps=10):
        ev = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            f()
            e1.record(stream)
            ev.append((e0, e1))
        torch.cuda.synchronize()
        return sorted(a.elapsed_time(b) for a, b in ev)[len(ev) // 2]

    # an event pair around a single launch of 70 us also times the gaps between the markers and the kernel (a few
    # microseconds: the kernel trace of the same launches reads 4 - 6 % less); a run of launches between one pair
    # of events, divided by their number, is closer to the kernel's own duration
    def batch_ms(f, reps=20):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            f()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    batch = {"halo_pack": batch_ms(lambda: sp3d.halo_pack(Px, M, gb, c, dt, stream)),
             "halo_unpack": batch_ms(lambda: sp3d.halo_unpack(Px, M, gb, c, dt, stream))}
    exchange_ms = median_ms(lambda: sp3d.sp_halo_exchange(Px, gb, c, dt, stream))
    full_ms = {"halo_pack": median_ms(lambda: sp3d.halo_pack(Px, M, g, c, dt, stream)),
               "halo_unpack": median_ms(lambda: sp3d.halo_unpack(Px, M, g, c, dt, stream)),
               "sp_halo_exchange": median_ms(lambda: sp3d.sp_halo_exchange(Px, g, c, dt, stream))}

    # The same forward launch on an all-zero input: its arithmetic, memory traffic and instruction stream are
    # unchanged, only the operands' bits stop toggling.  If it runs faster, the rate of the real launch is set by
    # the chip's power management (clock under load), not by the kernel's schedule.
    Pzero = torch.zeros_like(Py)
    fwd_zero_ms = median_ms(lambda: sp3d.conv3d_fwd(Pzero, w, None, Py, g, c, c, dt, 0, wsp[0], stream), reps=5)
    del Pzero

    # The data gradient with the ReLU mask of the layer input (every inner layer of a conv + ReLU stack): mask read
    # from the activation tensor, and mask given as one bit per value (written by conv3d_fwd_bits of the layer before)
    Bx = torch.empty(sp3d.sp_relu_bits_bytes(g, c) // 2, dtype=torch.int16, device="cuda")
    sp3d.sp_relu_bits(Px, Bx, g, c, dt, stream)
    masked_ms = {
        "conv3d_dgrad": median_ms(lambda: sp3d.conv3d_dgrad(Pdy, w, Pdx, g, c, c, dt, wsp[1], stream), reps=5),
        "conv3d_dgrad_relu": median_ms(lambda: sp3d.conv3d_dgrad_relu(Pdy, w, Px, Pdx, g, c, c, dt, wsp[1], stream), reps=5),
        "conv3d_dgrad_bits": median_ms(lambda: sp3d.conv3d_dgrad_bits(Pdy, w, Bx, Pdx, g, c, c, dt, wsp[1], stream), reps=5),
        "conv3d_fwd_relu": median_ms(lambda: sp3d.conv3d_fwd(Px, w, None, Py, g, c, c, dt, sp3d.SP_FLAG_RELU, wsp[0], stream), reps=5),
        "conv3d_fwd_bits": median_ms(lambda: sp3d.conv3d_fwd_bits(Px, w, None, Py, Bx, g, c, c, dt, sp3d.SP_FLAG_RELU, wsp[0], stream), reps=5),
    }
    del Bx

    per = {}
    for name, e0, e1 in events:
        per.setdefault(name, []).append(e0.elapsed_time(e1))
    avg_ms = {k: sum(v) / len(v) for k, v in per.items()}            # per launch
    count = {k: len(v) // args.steps for k, v in per.items()}        # launches per step

    vox = n * S * S * S
    flop_pass = 2.0 * 27 * c * c * vox
    value = 3 * flop_pass / (ms_per_step * 1e-3) / 1e12
    if args.gather:        # not part of the step: timed once each for the report
        avg_ms["halo_pack"] = median_ms(lambda: sp3d.halo_pack(Px, M, gb, c, dt, stream))
        avg_ms["halo_unpack"] = median_ms(lambda: sp3d.halo_unpack(Px, M, gb, c, dt, stream))
        count["halo_pack"] = count["halo_unpack"] = 0
    halo_ms = (avg_ms["halo_pack"] * count["halo_pack"] + avg_ms["halo_unpack"] * count["halo_unpack"])
    part_ms = (avg_ms["sp_partition"] * count["sp_partition"]
               + avg_ms["sp_unpartition"] * count["sp_unpartition"])
    kernel_ms = sum(avg_ms[k] * count[k] for k in avg_ms)

    # dominant kernel: the implicit-GEMM conv kernel behind conv3d_fwd and conv3d_dgrad
    conv_ms = 0.5 * (avg_ms["conv3d_fwd"] + avg_ms["conv3d_dgrad"])
    achieved = flop_pass / (conv_ms * 1e-3) / 1e12
    roofline = {"kernel": "conv_mfma_kernel (conv3d_fwd / conv3d_dgrad)", "bound": "mfma",
                "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": MEASURED_TRAFFIC_BYTES.get(S),
                "traffic_source": ("not measured in this run: a constant taken from the rocprofv3 --pmc FETCH_SIZE / "
                                   "WRITE_SIZE runs summarised in profiles/bench_512_hbm_traffic.md"
                                   if MEASURED_TRAFFIC_BYTES.get(S) else None)}
    msg_bytes = sp3d.sp_msg_elems(g, c) * 2
    # halo_unpack writes every margin region and reads only those whose neighbour tile exists
    tile = (S // grid[0], S // grid[1], S // grid[2])
    nb_vox = 0
    for delta in itertools.product((-1, 0, 1), repeat=3):
        if delta == (0, 0, 0):
            continue
        region = 1
        tiles = 1
        for ax in range(3):
            region *= tile[ax] if delta[ax] == 0 else 1
            tiles *= grid[ax] if delta[ax] == 0 else grid[ax] - 1
        nb_vox += n * tiles * region
    nb_bytes = nb_vox * c * 2              # message bytes that have a receiving tile
    unpack_bytes = msg_bytes + nb_bytes    # without the flags: every margin written, those with a neighbour read

    def hbm(kernel, nbytes, ms, note, ms_batch=None):
        gbs = nbytes / (ms * 1e-3) / 1e9
        r = {"kernel": kernel, "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(gbs / PEAK_HBM_GBS, 4), "bytes": int(nbytes), "ms": round(ms, 4), "what": note}
        if ms_batch is not None:       # 20 launches in a row between one pair of events, per launch
            r["ms_in_a_batch"] = round(ms_batch, 4)
            r["frac_in_a_batch"] = round(nbytes / (ms_batch * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
        return r

    other = [
        {"kernel": "wgrad_mfma_kernel (conv3d_wgrad)", "bound": "mfma",
         "achieved": round(flop_pass / (avg_ms["conv3d_wgrad"] * 1e-3) / 1e12, 1),
         "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
         "frac": round(flop_pass / (avg_ms["conv3d_wgrad"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
        hbm("halo_pack", 2 * nb_bytes, avg_ms["halo_pack"],
            "in the step, SP_HALO_SKIP_SEND: the regions that have a receiver, read + written once",
            batch["halo_pack"]),
        hbm("halo_unpack", 2 * nb_bytes, avg_ms["halo_unpack"],
            "in the step, SP_HALO_KEEP_ZERO: the margins that have a neighbour, read + written once",
            batch["halo_unpack"]),
        hbm("halo_pack, all 26 regions", 2 * msg_bytes, full_ms["halo_pack"],
            "after the step, no flags: every region read + written (a third of them have no receiver on this grid)"),
        hbm("halo_unpack, border zero-filled", unpack_bytes, full_ms["halo_unpack"],
            "after the step, no flags: every margin written, those with a neighbour read"),
        {"kernel": "sp_unpartition", "bound": "hbm",
         "achieved": round(2 * vox * c * 2 / (avg_ms["sp_unpartition"] * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
         "unit": "GB/s",
         "frac": round(2 * vox * c * 2 / (avg_ms["sp_unpartition"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
        {"kernel": "sp_partition", "bound": "hbm",
         "achieved": round(2 * vox * c * 2 / (avg_ms["sp_partition"] * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
         "unit": "GB/s",
         "frac": round(2 * vox * c * 2 / (avg_ms["sp_partition"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    ]

    out = {
        "metric": "conv3d fwd+bwd TFLOP/s (bf16) at 512^3 tiles; halo overhead % of step time",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d^3 volume, Cin=Cout=32, grid %dx%dx%d, halo 1, "
                               "fwd+dgrad+wgrad with partition/halo/unpartition%s"
                               % (cfg["name"] if S == 512 else "c4 recipe at reduced size", S, *grid,
                                  " (--gather: no pack / unpack in the step, the convolutions read their "
                                  "neighbours' voxels themselves)" if args.gather else ""),
                   "input_gen_s": round(t_gen, 1)},
        "halo_overhead_pct": round(100.0 * halo_ms / kernel_ms, 2),
        "partition_halo_overhead_pct": round(100.0 * (halo_ms + part_ms) / kernel_ms, 2),
        "paper_context": "paper reports ~5% of training time for partitioning+reshaping+halo exchange "
                         "on TPU pods (its own hardware; not a target)",
        "ms_per_launch": {k: round(v, 4) for k, v in avg_ms.items()},
        "conv_stack": {"what": "conv3d_fwd + conv3d_dgrad + conv3d_wgrad launches alone",
                       "tflops": round(3 * flop_pass / ((avg_ms["conv3d_fwd"] + avg_ms["conv3d_dgrad"]
                                                          + avg_ms["conv3d_wgrad"]) * 1e-3) / 1e12, 1),
                       "frac_of_bf16_peak": round(3 * flop_pass / ((avg_ms["conv3d_fwd"] + avg_ms["conv3d_dgrad"]
                                                                   + avg_ms["conv3d_wgrad"]) * 1e-3) / 1e12
                                                  / PEAK_BF16_TFLOPS, 4)},
        "halo_exchange_fused_ms": round(exchange_ms, 4),
        "halo_exchange_fused_zero_fill_ms": round(full_ms["sp_halo_exchange"], 4),
        "library_gemm_tflops": None if gemm_tflops is None else round(gemm_tflops, 1),
        "power_probe": {"conv3d_fwd_ms": round(avg_ms["conv3d_fwd"], 4), "conv3d_fwd_zero_input_ms": round(fwd_zero_ms, 4),
                        "what": "the same launch on an all-zero input tensor (same work, operand bits do not toggle), "
                                "timed after the step: a faster run means the real one is held by the chip's power "
                                "management; library_gemm_tflops is the vendor GEMM (torch.matmul 8192^3 bf16, N(0,1) "
                                "data) on this box for comparison"},
        "relu_mask_ms": dict({k: round(v, 4) for k, v in masked_ms.items()},
                             what="after the step: the data gradient plain, masked by the activation tensor, and masked "
                                  "by the one-bit form; the forward pass with ReLU without / with writing the bits"),
        "roofline": roofline,
        "roofline_other": other,
    }

    # ---- CPU baseline: the fp64 oracle, as it stands, on a bounded sample of the same workload ----
    if not args.no_cpu_baseline:
        from oracle import conv3d as oc
        b = min(128, S)          # about 17 s of oracle work on 16 host cores
        xs = np.ascontiguousarray(x_h[:, :b, :b, :b])
        dys = np.ascontiguousarray(dy_h[:, :b, :b, :b])
        w64 = synth.bf16_bits_to_f32(w_h).astype(np.float64)
        t0 = time.perf_counter()
        oc.conv3d_fwd(xs, w64)
        oc.conv3d_dgrad(dys, w64)
        oc.conv3d_wgrad(xs, dys)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(3 * 2.0 * 27 * c * c * b ** 3 / t_cpu / 1e12, 5), "unit": "TFLOP/s",
            "cores": int(os.environ.get("OMP_NUM_THREADS", 0)) or len(os.sched_getaffinity(0)),
            "kind": "oracle",
            "sample": "fp64 direct-convolution oracle (gcc -O3 -fopenmp, untuned): fwd + dgrad + wgrad "
                      "on the %d^3 corner box of the same tensors, %.1f s" % (b, t_cpu)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
