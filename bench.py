"""Benchmark of the ternary-linear hot path on one MI355X.

One step = one pass of the decode-shape sweep (K = 4096; N = 4096 and N = 14336; M in
{1, 2, 4, 8, 16}): ten GEMMs on packed weights that are already in HBM, handed to the library
as one tl_ternary_gemm_grouped call (one kernel launch).  Every GEMM reads a different copy of
its weight matrix, taken from a ring of copies that is several times larger than the 256 MB
last-level cache, so the weights really stream from HBM as they do when a model walks through
its layers.  The same step issued as ten separate tl_ternary_gemm calls is timed as well
(`single_calls`, `per_call`).

Prints one JSON line: `value` is the sweep's algorithmic bytes per second (packed W + x + y
of all ten GEMMs / time of a step).  `roofline` is measured live for the dominant kernel (the
grouped launch), `cpu_baseline` is the CPU oracle timed on the same workload.

Timing protocol.  `steps` steps are captured into one HIP graph (a batch).  The graph is replayed
untimed until the GPU has run that workload for 80 ms -- the chip raises its clock over the first
tens of milliseconds of sustained load (measured inside the kernel: 1.7-1.9 GHz in the first
replays after idle, 2.3-2.4 GHz from about 50 ms on), and a step takes 19-24 us before that against
17-18 us after -- and then 11 batches are timed one by one with events on the launch stream.  A
figure is the median batch divided by `steps`; p10 and p90 of the batches are printed beside it.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0          # dense fp16
PAPER_CONTEXT = ("paper (arXiv 2506.23025): up to 5x end-to-end generation speed-up over PyTorch FP16 "
                 "on one NVIDIA L40S at 64 input / 64 output tokens; no absolute kernel figures published")


def algorithmic_bytes(M, N, K):
    """Bytes the method itself must move: packed W once, x once, y once."""
    return N * (K // 16) * 4 + 2 * M * K + 2 * M * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mode", choices=("sweep", "dominant", "copy", "prefill", "one_point_six", "mfma_probe"), default="sweep",
                    help="sweep: the benchmark; the others run one kernel `steps` times for rocprofv3: dominant (the "
                         "grouped sweep launch), copy (the plain copy probe), prefill (the large-M kernel at M = 2048), "
                         "one_point_six (the 1.6-bit kernel, 4096 -> 14336 at M = 1), mfma_probe (tl_probe_mfma)")
    ap.add_argument("--no-per-call", action="store_true", help="skip the ten-separate-calls measurements")
    ap.add_argument("--weights", choices=("workload", "pm1", "zero"), default="workload",
                    help="weight values: the workload's iid ternary draw (default); +-1 only (no zeros: codes 0 and 2); "
                         "all zero (constant words).  Same bytes and instructions, other data: the time of the "
                         "sweep depends on it (the chip's power management answers to the switching in the matrix pipes)")
    ap.add_argument("--eager", action="store_true",
                    help="launch every call from the host instead of replaying a captured HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the kernel has no cross-GPU part); "
                 "use --gpus 1")

    import torch

    import paper_2506_23025_amd as tl
    import synth_inputs as si

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    L = tl.raw()
    tl.tl_init()                                        # every kernel prepared before anything is captured
    stream = torch.cuda.current_stream().cuda_stream

    if args.mode == "copy":
        # calibration for the HBM counters: a plain copy of known size (256 MiB read + written)
        nbytes = 256 << 20
        src = torch.full((nbytes,), 3, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(args.steps):
            st = L.tl_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream)
            if st != tl.TL_OK:
                raise tl.TlError(st, "tl_probe_copy")
        torch.cuda.synchronize()
        print(json.dumps({"mode": "copy", "launches": args.steps, "bytes_read_per_launch": nbytes,
                          "bytes_written_per_launch": nbytes}))
        return

    # ---------------- synthetic workload (seeded), resident in HBM -------------------------
    rng = np.random.default_rng(si.SEEDS["c2"])
    K = 4096
    shapes = [(name,) + si.SHAPES[name] for name in si.DECODE_SWEEP_SHAPES]   # (name, K, N)
    Ms = si.DECODE_SWEEP_M
    RING_BYTES = 1280 << 20
    layers = {}
    for name, k, N in shapes:
        assert k == K
        W = si.ternary_weights(rng, N, K)
        if args.weights == "pm1":
            W = np.where(W == 0, np.int8(1), W).astype(np.int8)
        elif args.weights == "zero":
            W = np.zeros_like(W)
        g = si.gamma_uniform(rng)
        Wp = tl.tl_pack_2bit(W)
        copies = max(2 * len(Ms), min(96, RING_BYTES // Wp.nbytes // len(shapes)))
        ring = torch.empty((copies,) + Wp.shape, dtype=torch.int32, device=dev)
        ring[0].copy_(torch.from_numpy(Wp.view(np.int32)))
        for i in range(1, copies):
            ring[i].copy_(ring[0])
        layers[name] = dict(N=N, W=W, Wp=Wp, gamma=g, gbits=si.gamma_bits(g), ring=ring, copies=copies)
    xs = {M: si.activations(rng, M, K) for M in Ms}
    xd = {M: torch.from_numpy(xs[M].view(np.int16)).to(dev) for M in Ms}
    yd = {(name, M): torch.empty((M, layers[name]["N"]), dtype=torch.int16, device=dev)
          for name, _, _ in shapes for M in Ms}
    calls = [(name, M) for name, _, _ in shapes for M in Ms]
    cursor = {name: 0 for name, _, _ in shapes}

    def launch(name, M):
        lay = layers[name]
        i = cursor[name]
        cursor[name] = (i + 1) % lay["copies"]
        st = L.tl_ternary_gemm(xd[M].data_ptr(), lay["ring"][i].data_ptr(), lay["gbits"],
                               yd[(name, M)].data_ptr(), M, lay["N"], K, stream)
        if st != tl.TL_OK:
            raise tl.TlError(st, "tl_ternary_gemm")

    def step():
        for name, M in calls:
            launch(name, M)

    def step_grouped():
        jobs = []
        for name, M in calls:
            lay = layers[name]
            i = cursor[name]
            cursor[name] = (i + 1) % lay["copies"]
            jobs.append((xd[M], lay["ring"][i], lay["gbits"], yd[(name, M)], M, lay["N"], K))
        arr = tl.make_jobs(jobs)
        st = L.tl_ternary_gemm_grouped(arr, len(arr), stream)
        if st != tl.TL_OK:
            raise tl.TlError(st, "tl_ternary_gemm_grouped")

    step_bytes = sum(algorithmic_bytes(M, layers[name]["N"], K) for name, M in calls)
    if args.mode == "dominant":
        for _ in range(args.steps):
            step_grouped()
        torch.cuda.synchronize()
        print(json.dumps({"mode": "dominant", "launches": args.steps, "kernel": "grouped sweep launch",
                          "algorithmic_bytes_per_launch": step_bytes}))
        return

    # large-M inputs: 4096 -> 14336 at the prefill batch sizes (MFMA-bound leg of the metric)
    pre_name = "mlp_up_8b"
    pre_N = layers[pre_name]["N"]
    pre_M = si.PREFILL_M
    pre_x = torch.from_numpy(si.activations(rng, max(pre_M), K).view(np.int16)).to(dev)
    pre_y = torch.empty((max(pre_M), pre_N), dtype=torch.int16, device=dev)

    def launch_prefill(M, path=tl.TL_PATH_MFMA):
        lay = layers[pre_name]
        i = cursor[pre_name]
        cursor[pre_name] = (i + 1) % lay["copies"]
        st = L.tl_ternary_gemm_path(pre_x.data_ptr(), lay["ring"][i].data_ptr(), lay["gbits"],
                                    pre_y.data_ptr(), M, pre_N, K, stream, path)
        if st != tl.TL_OK:
            raise tl.TlError(st, "tl_ternary_gemm_path")

    if args.mode == "mfma_probe":
        fsink = torch.zeros(4, dtype=torch.float32, device=dev)
        wp0 = layers[pre_name]["ring"][0]
        for _ in range(args.steps):
            flops = tl.tl_probe_mfma(pre_x, pre_x.numel(), wp0, wp0.numel(), 4096, fsink, stream)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "mfma_probe", "launches": args.steps, "flops_per_launch": flops}))
        return

    if args.mode == "one_point_six":
        lay = layers[pre_name]
        W3 = tl.tl_pack_1p6bit(lay["W"])
        copies3 = 24
        ring3 = torch.empty((copies3,) + W3.shape, dtype=torch.uint8, device=dev)
        for i in range(copies3):
            ring3[i].copy_(torch.from_numpy(W3))
        fy = torch.empty((1, pre_N), dtype=torch.int16, device=dev)
        for i in range(args.steps):
            st = L.tl_ternary_gemm_1p6(xd[1].data_ptr(), ring3[i % copies3].data_ptr(), lay["gbits"], fy.data_ptr(), 1, pre_N, K, stream)
            if st != tl.TL_OK:
                raise tl.TlError(st, "tl_ternary_gemm_1p6")
        torch.cuda.synchronize()
        print(json.dumps({"mode": "one_point_six", "launches": args.steps, "M": 1, "N": pre_N, "K": K,
                          "algorithmic_bytes_per_launch": pre_N * W3.shape[1] + 2 * K + 2 * pre_N}))
        return

    if args.mode == "prefill":
        for _ in range(args.steps):
            launch_prefill(max(pre_M))
        torch.cuda.synchronize()
        print(json.dumps({"mode": "prefill", "launches": args.steps, "M": max(pre_M), "N": pre_N, "K": K,
                          "flops_per_launch": 2 * max(pre_M) * pre_N * K}))
        return

    # ---------------- timed region: exactly `steps` steps ---------------------------------
    # The launches are captured once into a HIP graph (as a serving loop would do for a decode
    # step) and replayed, so that the host's per-call cost is not part of the figure.
    WARM_MS = 80.0          # sustained load before timing (clock ramp)
    N_BATCH = 11            # timed batches per figure

    def timed(fn, reps):
        """Median, p10 and p90 (ms) over N_BATCH batches of `reps` executions of fn() on a side stream,
        graph-replayed unless --eager, after WARM_MS of the same load."""
        nonlocal stream
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            stream = side.cuda_stream
            fn()                                            # untimed: loads code, touches buffers
            side.synchronize()
            if args.eager:
                def batch():
                    for _ in range(reps):
                        fn()
            else:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    for _ in range(reps):
                        fn()
                batch = g.replay
            t_w = time.perf_counter()
            n_w = 0
            while n_w < 3 or (time.perf_counter() - t_w) * 1e3 < WARM_MS:
                batch()
                n_w += 1
                if n_w % 4 == 0:
                    side.synchronize()
            side.synchronize()
            # the timed batches are enqueued back to back with an event between them and waited for
            # once, so that the GPU does not idle (and clock down) between batches and the host's
            # launch of a batch overlaps the batch before it; a batch is the interval between two events
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(N_BATCH + 1)]
            evs[0].record(side)
            for i in range(N_BATCH):
                batch()
                evs[i + 1].record(side)
            side.synchronize()
            ts = [evs[i].elapsed_time(evs[i + 1]) for i in range(N_BATCH)]
        stream = torch.cuda.current_stream().cuda_stream
        ts.sort()
        return dict(ms=ts[len(ts) // 2], p10=ts[len(ts) // 10], p90=ts[-1 - len(ts) // 10], batches=len(ts))

    def per_unit(st, reps, scale=1e3):
        """(median, p10, p90) of a timed() result per execution, in us by default."""
        return tuple(st[k] * scale / reps for k in ("ms", "p10", "p90"))

    def us_row(st, reps):
        m, lo, hi = per_unit(st, reps)
        return dict(us=round(m, 3), us_p10=round(lo, 3), us_p90=round(hi, 3))

    # a read-only kernel over `nbytes` bytes (a different stretch of the largest weight ring per
    # launch): what the memory system gives a single launch of that size
    big = max(layers.values(), key=lambda l: l["ring"].numel())["ring"].view(-1)
    sink = torch.zeros(4, dtype=torch.int32, device=dev)

    def probe_us(nbytes, reps):
        nbytes = (nbytes + 15) // 16 * 16
        slots = max(1, big.numel() * 4 // nbytes)
        pc = [0]

        def probe_step():
            off = (pc[0] % slots) * nbytes
            pc[0] += 1
            st = L.tl_probe_read(big.data_ptr() + off, nbytes, sink.data_ptr(), stream)
            if st != tl.TL_OK:
                raise tl.TlError(st, "tl_probe_read")

        return per_unit(timed(probe_step, reps), reps)[0]

    for _ in range(args.warmup):
        step_grouped()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    head = timed(step_grouped, args.steps)
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = head["ms"] / args.steps
    value = step_bytes / (ms_per_step * 1e-3) / 1e9
    us_probe = probe_us(step_bytes, args.steps)

    # the same step on the same weight buffers every time (96 MB: it stays in the 256 MB last-level
    # cache), and the latency of one launch into an idle GPU
    warm_same = None
    latency = None
    if not args.no_per_call:
        def step_same():
            jobs = [(xd[M], layers[name]["ring"][0], layers[name]["gbits"], yd[(name, M)], M, layers[name]["N"], K)
                    for name, M in calls]
            arr = tl.make_jobs(jobs)
            st = L.tl_ternary_gemm_grouped(arr, len(arr), stream)
            if st != tl.TL_OK:
                raise tl.TlError(st, "tl_ternary_gemm_grouped")

        st = timed(step_same, args.steps)
        warm_same = dict(us_row(st, args.steps), GBps=round(step_bytes / per_unit(st, args.steps)[0] / 1e3, 1),
                         note="every step reads the same ten weight buffers (96 MB, resident in the last-level cache)")
        lat = []
        cur = torch.cuda.current_stream()
        for _ in range(21):
            torch.cuda.synchronize()
            time.sleep(0.002)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(cur)
            step_grouped()
            b.record(cur)
            torch.cuda.synchronize()
            lat.append(a.elapsed_time(b) * 1e3)
        lat.sort()
        latency = dict(us=round(lat[len(lat) // 2], 2), us_p10=round(lat[2], 2), us_p90=round(lat[-3], 2),
                       note="one grouped launch of the sweep into an idle GPU, event to event on the launch stream "
                            "(includes the launch itself and the idle clock)")

    # ---------------- the same step as ten separate calls; per-call figures ----------------
    per_call = []
    single = None
    if not args.no_per_call:
        st = timed(step, args.steps)
        ms_single = st["ms"] / args.steps
        single = dict(ms_per_step=round(ms_single, 5), GBps=round(step_bytes / ms_single / 1e6, 1),
                      hbm_frac=round(step_bytes / ms_single / 1e6 / HBM_PEAK_GBS, 4),
                      ms_p10=round(st["p10"] / args.steps, 5), ms_p90=round(st["p90"] / args.steps, 5),
                      note="ten tl_ternary_gemm calls per step: what a chain of dependent layers gets")
    for name, M in ([] if args.no_per_call else calls):
        st = timed(lambda: launch(name, M), args.steps)
        us = per_unit(st, args.steps)[0]
        N = layers[name]["N"]
        b = algorithmic_bytes(M, N, K)
        pus = probe_us(b, args.steps)
        per_call.append(dict(layer=name, M=M, N=N, K=K, **us_row(st, args.steps), GBps=round(b / us / 1e3, 1),
                             hbm_frac=round(b / us / 1e3 / HBM_PEAK_GBS, 4),
                             TFLOPs=round(2.0 * M * N * K / us / 1e6, 3),
                             read_only_probe_us=round(pus, 3), kernel_vs_probe=round(pus / us, 4)))

    # lone calls with long K: the down projections that close a block (11008 -> 4096, 14336 -> 4096),
    # which a decode step issues on their own; their own weights, cycled as above
    long_k_calls = []
    if not args.no_per_call:
        lrng = np.random.default_rng(si.SEEDS["c3"] + 17)
        for lk, lN in ((11008, 4096), (14336, 4096)):
            lWp = tl.tl_pack_2bit(si.ternary_weights(lrng, lN, lk))
            lcopies = max(4, min(32, (400 << 20) // lWp.nbytes))
            lring = torch.empty((lcopies,) + lWp.shape, dtype=torch.int32, device=dev)
            lring[0].copy_(torch.from_numpy(lWp.view(np.int32)))
            for i in range(1, lcopies):
                lring[i].copy_(lring[0])
            lg = si.gamma_bits(si.gamma_uniform(lrng))
            for M in (1, 16):
                lx = torch.from_numpy(si.activations(lrng, M, lk).view(np.int16)).to(dev)
                ly = torch.empty((M, lN), dtype=torch.int16, device=dev)
                lcur = [0]

                def call_long():
                    i = lcur[0]
                    lcur[0] = (i + 1) % lcopies
                    st_ = L.tl_ternary_gemm(lx.data_ptr(), lring[i].data_ptr(), lg, ly.data_ptr(), M, lN, lk, stream)
                    if st_ != tl.TL_OK:
                        raise tl.TlError(st_, "tl_ternary_gemm")

                reps = max(1, min(args.steps, 200))
                st = timed(call_long, reps)
                us = per_unit(st, reps)[0]
                b = algorithmic_bytes(M, lN, lk)
                pus = probe_us(b, reps)
                long_k_calls.append(dict(M=M, N=lN, K=lk, **us_row(st, reps), GBps=round(b / us / 1e3, 1),
                                         hbm_frac=round(b / us / 1e3 / HBM_PEAK_GBS, 4),
                                         read_only_probe_us=round(pus, 3), kernel_vs_probe=round(pus / us, 4)))
            del lring

    # large M: the LDS-tiled MFMA kernel against the dense fp16 MFMA peak, and against a kernel that
    # only issues the same matrix instruction on the same kind of operands; and the batch sizes in
    # between with whichever kernel the library picks
    prefill, mid_batch = [], []
    mfma_probe = None
    if not args.no_per_call:
        fsink = torch.zeros(4, dtype=torch.float32, device=dev)
        wp0 = layers[pre_name]["ring"][0]
        flops_box = [0.0]

        def probe_mfma_step():
            flops_box[0] = tl.tl_probe_mfma(pre_x, pre_x.numel(), wp0, wp0.numel(), 4096, fsink, stream)

        reps = max(1, min(args.steps, 20))
        st = timed(probe_mfma_step, reps)
        pus = per_unit(st, reps)[0]
        mfma_probe = dict(kernel="probe_mfma_kernel: v_mfma_f32_32x32x16_f16 only, 8 accumulators per wave, two waves per SIMD, "
                                 "activations x ternary weights as operands",
                          **us_row(st, reps), TFLOPs=round(flops_box[0] / pus / 1e6, 1),
                          frac_of_peak=round(flops_box[0] / pus / 1e6 / MFMA_PEAK_TFLOPS, 4))
    for M in ([] if args.no_per_call else pre_M):
        reps = max(1, min(args.steps, 40))
        st = timed(lambda: launch_prefill(M), reps)
        us = per_unit(st, reps)[0]
        fl = 2.0 * M * pre_N * K
        which = {tl.TL_PATH_GEMV: "small-M kernel", tl.TL_PATH_MFMA: "mfma_kernel",
                 tl.TL_PATH_GENERIC: "generic kernel"}[tl.tl_ternary_gemm_which(M, pre_N, K)]
        us_auto = us if which == "mfma_kernel" else per_unit(timed(lambda: launch_prefill(M, tl.TL_PATH_AUTO), reps), reps)[0]
        prefill.append(dict(layer=pre_name, M=M, N=pre_N, K=K, kernel="mfma_kernel", **us_row(st, reps),
                            TFLOPs=round(fl / us / 1e6, 1), mfma_frac=round(fl / us / 1e6 / MFMA_PEAK_TFLOPS, 4),
                            kernel_vs_mfma_probe=round(fl / us / 1e6 / mfma_probe["TFLOPs"], 4),
                            tl_ternary_gemm=dict(kernel=which, us=round(us_auto, 2), TFLOPs=round(fl / us_auto / 1e6, 1),
                                                 mfma_frac=round(fl / us_auto / 1e6 / MFMA_PEAK_TFLOPS, 4))))
    if prefill:
        # The same launch on operands that switch nothing in the matrix pipes (x = 0, every weight 0):
        # the instruction stream is identical, so the difference to the row above is what the chip's
        # power management takes at the workload's data, and this figure is what the kernel's own
        # structure (waits, tile rounds) allows.
        M = max(pre_M)
        zx = torch.zeros_like(pre_x)
        zw = torch.from_numpy(tl.tl_pack_2bit(np.zeros((pre_N, K), dtype=np.int8)).view(np.int32)).to(dev)
        zrings = [zw.clone() for _ in range(4)]
        zc = [0]

        def launch_zero():
            i = zc[0]
            zc[0] = (i + 1) % len(zrings)
            st_ = L.tl_ternary_gemm_path(zx.data_ptr(), zrings[i].data_ptr(), layers[pre_name]["gbits"],
                                         pre_y.data_ptr(), M, pre_N, K, stream, tl.TL_PATH_MFMA)
            if st_ != tl.TL_OK:
                raise tl.TlError(st_, "tl_ternary_gemm_path")

        reps = max(1, min(args.steps, 40))
        st = timed(launch_zero, reps)
        us = per_unit(st, reps)[0]
        fl = 2.0 * M * pre_N * K
        prefill[-1]["same_kernel_zero_operands"] = dict(**us_row(st, reps), TFLOPs=round(fl / us / 1e6, 1),
                                                        mfma_frac=round(fl / us / 1e6 / MFMA_PEAK_TFLOPS, 4))
        del zx, zw, zrings
    for M in ([] if args.no_per_call else (32, 64, 128, 256, 512)):
        reps = max(1, min(args.steps, 40))
        st = timed(lambda: launch_prefill(M, tl.TL_PATH_AUTO), reps)
        us = per_unit(st, reps)[0]
        fl = 2.0 * M * pre_N * K
        mid_batch.append(dict(layer=pre_name, M=M, N=pre_N, K=K, kernel="picked by tl_ternary_gemm", **us_row(st, reps),
                              TFLOPs=round(fl / us / 1e6, 1), GBps=round(algorithmic_bytes(M, pre_N, K) / us / 1e3, 1)))

    # the linears of a block (QKV, O, gate+up, down) as one grouped call: the unit the paper's
    # kernel benchmark is quoted on (App. G)
    block = []
    if not args.no_per_call:
        brng = np.random.default_rng(si.SEEDS["c3"])
        blay = []
        for name in si.BLOCK_SHAPES:
            k, N = si.SHAPES[name]
            Wp = tl.tl_pack_2bit(si.ternary_weights(brng, N, k))
            copies = 6
            ring = torch.empty((copies,) + Wp.shape, dtype=torch.int32, device=dev)
            ring[0].copy_(torch.from_numpy(Wp.view(np.int32)))
            for i in range(1, copies):
                ring[i].copy_(ring[0])
            blay.append(dict(name=name, K=k, N=N, ring=ring, copies=copies, gbits=si.gamma_bits(si.gamma_uniform(brng))))
        for M in si.BLOCK_M:
            bx = {k: torch.from_numpy(si.activations(brng, M, k).view(np.int16)).to(dev) for k in {l["K"] for l in blay}}
            by = [torch.empty((M, l["N"]), dtype=torch.int16, device=dev) for l in blay]
            bcur = [0]

            def block_step():
                i = bcur[0]
                bcur[0] = (i + 1) % 6
                arr = tl.make_jobs([(bx[l["K"]], l["ring"][i], l["gbits"], y, M, l["N"], l["K"]) for l, y in zip(blay, by)])
                st = L.tl_ternary_gemm_grouped(arr, len(arr), stream)
                if st != tl.TL_OK:
                    raise tl.TlError(st, "tl_ternary_gemm_grouped")

            reps = max(1, min(args.steps, 60))
            st = timed(block_step, reps)
            us = per_unit(st, reps)[0]
            bb = sum(algorithmic_bytes(M, l["N"], l["K"]) for l in blay)
            block.append(dict(M=M, layers=[l["name"] for l in blay], algorithmic_bytes=bb, **us_row(st, reps),
                              GBps=round(bb / us / 1e3, 1), hbm_frac=round(bb / us / 1e3 / HBM_PEAK_GBS, 4)))
        del blay

    # the 1.6-bit formats (plain base 3, decoded through a table; the paper's fixed-point code of
    # Sec. 3.2, same kernel with the table filled from that code) and per-group scales beside the
    # 2-bit, single-gamma kernel (one call each)
    formats = []
    grouped_formats = None
    if not args.no_per_call:
        rings3, scales256 = {}, {}
        frng = np.random.default_rng(si.SEEDS["c5"])
        for name in si.DECODE_SWEEP_SHAPES:
            lay = layers[name]
            N = lay["N"]
            W3 = tl.tl_pack_1p6bit(lay["W"])
            W3fx = tl.tl_pack_1p6bit_fx(lay["W"])
            copies3 = max(2, min(24, (512 << 20) // W3.nbytes))
            ring3 = torch.empty((copies3,) + W3.shape, dtype=torch.uint8, device=dev)
            ring3fx = torch.empty((copies3,) + W3.shape, dtype=torch.uint8, device=dev)
            ring3[0].copy_(torch.from_numpy(W3))
            ring3fx[0].copy_(torch.from_numpy(W3fx))
            for i in range(1, copies3):
                ring3[i].copy_(ring3[0])
                ring3fx[i].copy_(ring3fx[0])
            group = 256
            sc = torch.from_numpy(si.group_scales(frng, K // group, N).view(np.int16)).to(dev)
            sc128 = torch.from_numpy(si.group_scales(frng, K // 128, N).view(np.int16)).to(dev)
            for M in (1, 4, 16):
                cur = [0]
                fy = torch.empty((M, N), dtype=torch.int16, device=dev)    # the sweep's outputs stay as they are

                def call3(fn=L.tl_ternary_gemm_1p6, ring=ring3, what="tl_ternary_gemm_1p6"):
                    i = cur[0]
                    cur[0] = (i + 1) % copies3
                    st = fn(xd[M].data_ptr(), ring[i].data_ptr(), lay["gbits"], fy.data_ptr(), M, N, K, stream)
                    if st != tl.TL_OK:
                        raise tl.TlError(st, what)

                def call_gs(scales=sc, grp=group):
                    i = cursor[name]
                    cursor[name] = (i + 1) % lay["copies"]
                    st = L.tl_ternary_gemm_gs(xd[M].data_ptr(), lay["ring"][i].data_ptr(), scales.data_ptr(), grp,
                                              fy.data_ptr(), M, N, K, stream)
                    if st != tl.TL_OK:
                        raise tl.TlError(st, "tl_ternary_gemm_gs")

                reps = max(1, min(args.steps, 200))
                us2 = per_unit(timed(lambda: launch(name, M), reps), reps)[0]
                us3 = per_unit(timed(call3, reps), reps)[0]
                us3fx = per_unit(timed(lambda: call3(L.tl_ternary_gemm_1p6_fx, ring3fx, "tl_ternary_gemm_1p6_fx"), reps), reps)[0]
                usg = per_unit(timed(call_gs, reps), reps)[0]
                usg128 = per_unit(timed(lambda: call_gs(sc128, 128), reps), reps)[0]
                b2 = algorithmic_bytes(M, N, K)
                b3 = N * W3.shape[1] + 2 * M * K + 2 * M * N
                formats.append(dict(layer=name, M=M, N=N, K=K,
                                    two_bit=dict(us=round(us2, 3), GBps=round(b2 / us2 / 1e3, 1)),
                                    one_point_six_bit=dict(us=round(us3, 3), GBps=round(b3 / us3 / 1e3, 1),
                                                           time_vs_two_bit=round(us3 / us2, 3)),
                                    one_point_six_bit_fixed_point_code=dict(us=round(us3fx, 3), GBps=round(b3 / us3fx / 1e3, 1),
                                                                            time_vs_two_bit=round(us3fx / us2, 3)),
                                    two_bit_group_scales_256=dict(us=round(usg, 3), GBps=round((b2 + 2 * (K // group) * N) / usg / 1e3, 1)),
                                    two_bit_group_scales_128=dict(us=round(usg128, 3), GBps=round((b2 + 2 * (K // 128) * N) / usg128 / 1e3, 1))))
            rings3[name] = (ring3, copies3, W3.shape[1])
            scales256[name] = sc
            del ring3fx
        # the sweep as ONE grouped launch in the other weight forms (tl_ternary_gemm_1p6_grouped,
        # tl_ternary_gemm_gs_grouped), beside the 2-bit headline
        gy = {(name, M): torch.empty((M, layers[name]["N"]), dtype=torch.int16, device=dev) for name, M in calls}
        cur3 = {name: 0 for name in rings3}

        def step_grouped_1p6():
            jobs = []
            for name, M in calls:
                ring, copies3, _ = rings3[name]
                i = cur3[name]
                cur3[name] = (i + 1) % copies3
                jobs.append((xd[M], ring[i], layers[name]["gbits"], gy[(name, M)], M, layers[name]["N"], K))
            arr = tl.make_jobs(jobs)
            st = L.tl_ternary_gemm_1p6_grouped(arr, len(arr), tl.TL_FMT_1P6BIT, stream)
            if st != tl.TL_OK:
                raise tl.TlError(st, "tl_ternary_gemm_1p6_grouped")

        def step_grouped_gs():
            jobs = []
            for name, M in calls:
                lay = layers[name]
                i = cursor[name]
                cursor[name] = (i + 1) % lay["copies"]
                jobs.append((xd[M], lay["ring"][i], scales256[name], 256, gy[(name, M)], M, lay["N"], K))
            arr = tl.make_gs_jobs(jobs)
            st = L.tl_ternary_gemm_gs_grouped(arr, len(arr), stream)
            if st != tl.TL_OK:
                raise tl.TlError(st, "tl_ternary_gemm_gs_grouped")

        reps = max(1, min(args.steps, 200))
        us3g = per_unit(timed(step_grouped_1p6, reps), reps)[0]
        usgg = per_unit(timed(step_grouped_gs, reps), reps)[0]
        b3g = sum(layers[name]["N"] * rings3[name][2] + 2 * M * K + 2 * M * layers[name]["N"] for name, M in calls)
        bgg = step_bytes + sum(2 * (K // 256) * layers[name]["N"] for name, M in calls)
        grouped_formats = dict(
            note="the decode sweep as one grouped launch in the other weight forms; two_bit is the headline",
            two_bit=dict(us=round(ms_per_step * 1e3, 3), GBps=round(step_bytes / ms_per_step / 1e6, 1)),
            one_point_six_bit=dict(us=round(us3g, 3), GBps=round(b3g / us3g / 1e3, 1), algorithmic_bytes=b3g,
                                   time_vs_two_bit=round(us3g / (ms_per_step * 1e3), 3)),
            two_bit_group_scales_256=dict(us=round(usgg, 3), GBps=round(bgg / usgg / 1e3, 1), algorithmic_bytes=bgg,
                                          time_vs_two_bit=round(usgg / (ms_per_step * 1e3), 3)))
        del rings3, gy

    # dominant kernel: the small-M kernel in its grouped launch; one launch = one step.  Counter
    # figures come from the rocprofv3 runs summarised under profiles/; they are quoted only while
    # the kernel source is the one they were measured on.
    us_launch = ms_per_step * 1e3
    traffic = None
    valu_per_weight = None
    counters_note = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if os.path.exists(tpath):
        import hashlib
        kv = {}
        for line in open(tpath):
            if "=" in line and not line.startswith("#"):
                k_, v_ = line.split("=", 1)
                kv[k_.strip()] = v_.strip()
        # hash of the code alone: comments and white space do not change what was measured
        code = []
        for line in open(os.path.join(ROOT, "paper_2506_23025_amd", "csrc", "tl_gemv.hip")):
            line = "".join(line.split("//", 1)[0].split())
            if line:
                code.append(line)
        src_hash = hashlib.sha256("\n".join(code).encode()).hexdigest()
        if kv.get("kernel_code_sha256") == src_hash:
            traffic = float(kv["grouped_sweep_bytes_per_launch"])
            weights = sum(layers[name]["N"] * K for name, _ in calls)
            if "grouped_sweep_valu_insts_per_launch" in kv:
                # wave instructions x 64 lanes / weights of a step (MFMA issues not included)
                valu_per_weight = round(float(kv["grouped_sweep_valu_insts_per_launch"]) * 64 / weights, 4)
        else:
            counters_note = "profiles/hbm_traffic.txt was measured on another version of tl_gemv.hip: counter figures withheld"
    roofline = dict(bound="hbm", kernel="gemv_lean_kernel<3>, grouped launch of the ten GEMMs of a step",
                    achieved=round(step_bytes / us_launch / 1e3, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(step_bytes / us_launch / 1e3 / HBM_PEAK_GBS, 4),
                    bytes_per_launch=step_bytes, us_per_launch=round(us_launch, 3),
                    us_per_launch_p10=round(head["p10"] / args.steps * 1e3, 3), us_per_launch_p90=round(head["p90"] / args.steps * 1e3, 3),
                    timed_batches=head["batches"], traffic=traffic,
                    valu_lane_ops_per_weight=valu_per_weight, counters_note=counters_note,
                    read_only_probe=dict(kernel="probe_read_kernel: the same bytes, loads only, one launch",
                                         us_per_launch=round(us_probe, 3), GBps=round(step_bytes / us_probe / 1e3, 1),
                                         frac_of_peak=round(step_bytes / us_probe / 1e3 / HBM_PEAK_GBS, 4),
                                         kernel_vs_probe=round(us_probe / us_launch, 4)))

    # ---------------- CPU oracle on the same sweep (reported baseline, not a target) -------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from parity import REL_TOL, rel_err
        torch.cuda.synchronize()
        worst = 0.0
        t_or = 0.0
        for name, M in calls:
            lay = layers[name]
            t1 = time.perf_counter()
            ref = oracle.gemm_packed2(xs[M], lay["Wp"], lay["gamma"], K)
            t_or += time.perf_counter() - t1
            got = yd[(name, M)].cpu().numpy().view(np.float16)
            worst = max(worst, rel_err(got, ref, xs[M], lay["gamma"]))
        if worst > REL_TOL:
            sys.exit(f"bench.py: GPU result differs from the oracle: max relative error {worst:.3e}")
        cpu = dict(value=round(step_bytes / t_or / 1e9, 4), unit="GB/s", cores=oracle.num_threads(),
                   kind="oracle", seconds=round(t_or, 2),
                   sample="the whole step: all ten GEMMs of the sweep, once each (unpack + fp64 dot products)",
                   max_rel_err_gpu_vs_oracle=float(f"{worst:.3e}"))

    out = {
        "metric": "ternary GEMM decode sweep, achieved HBM GB/s on algorithmic bytes (M=1-16)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x int2 -> f32 accumulate -> f16", "data": "synthetic",
        "config": {"workload": "decode-shape sweep: K=4096, N in {4096, 14336}, M in {1,2,4,8,16}, "
                               "2-bit packed ternary W (P(-1)=P(+1)=0.3), x fp16 ~ N(0,1), one fp16 gamma per matrix",
                   "gemms_per_step": len(calls), "launches_per_step": 1, "weight_ring_copies": {n: layers[n]["copies"] for n in layers},
                   "algorithmic_bytes_per_step": step_bytes},
        "hbm_frac_of_peak": round(value / HBM_PEAK_GBS, 4),
        "ms_per_step_p10": round(head["p10"] / args.steps, 5), "ms_per_step_p90": round(head["p90"] / args.steps, 5),
        "timing": {"batches": head["batches"], "steps_per_batch": args.steps, "figure": "median batch", "untimed_load_before_timing_ms": WARM_MS},
        "roofline": roofline, "cpu_baseline": cpu, "single_calls": single, "warm_same_buffer": warm_same,
        "single_launch_latency_us": latency, "per_call": per_call, "long_k_calls": long_k_calls, "mfma_probe": mfma_probe, "prefill": prefill,
        "mid_batch": mid_batch, "block": block, "formats": formats, "grouped_formats": grouped_formats,
        "launch_mode": "eager" if args.eager else "hip_graph_replay", "weights": args.weights,
        "host_wall_ms_timed_region_incl_capture": round(wall_ms, 2), "context": PAPER_CONTEXT,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
