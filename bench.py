#!/usr/bin/env python3
"""Benchmark of the Fira optimizer step on one MI355X.

A "step" is one fira_step call over ALL weight matrices of the workload (default: the LLaMA-1B
shape set, 168 matrices, r = 512, bf16 W/G with fp32 state): projection, Adam on the low-rank
gradient, factor norms, residual norm, limiter, back-projection and weight update.  Inputs are
synthetic and resident in HBM before the timed region; three gradient sets rotate so that no step
finds its gradient in the last-level cache.  Before the warm-up steps asked for, 40 untimed settling steps
bring the optimizer state from its zero start to the steady state (the limiter acts on the first steps of a run).

Prints ONE JSON line: whole-job optimizer steps/s, plus
  "roofline":     achieved vs peak for the kernel that takes the most time (HIP events recorded by
                  the library around every kernel of every timed step), and "kernels" with the same
                  figures for all of them;
  "limiter_active": the same step timed with the limiter acting on every matrix (not part of value);
  "cpu_baseline": the CPU oracle timed on this machine's host cores on a bounded sample;
  "power" (--power-seconds): socket power of the step, of a plain copy and of the vendor library's bf16
                  matrix product against the power cap; config.socket_power_w is sampled over the timed steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, GB/s
PEAK_MFMA_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, TFLOP/s


def kernel_models(shapes, r, norm_mode):
    """Algorithmic flops and HBM bytes of each kernel for one step over `shapes` (bf16 W/G, fp32
    state), and the roofline that bounds it.  mn: elements of W; Lr: elements of each low-rank array;
    Sr: elements of P; L: number of scaling factors.  Every array is counted once per kernel that
    must touch it; operand re-reads that hit in L2 are not algorithmic traffic."""
    mn = sum(m * n for m, n in shapes)
    Lr = sum(max(m, n) * r for m, n in shapes)
    Sr = sum(min(m, n) * r for m, n in shapes)
    L = sum(max(m, n) for m, n in shapes)
    gemm = 2.0 * mn * r
    gram = norm_mode == "gram"
    proj_bytes = 2 * mn + 2 * Sr + 4 * Lr + (4 * L if gram else 0)
    # the projection is a dense contraction (MFMA roofline) unless the rank is so small that reading G
    # takes longer at the HBM peak than the multiplies at the MFMA peak (r = 32: ten times longer)
    proj_bound = "mfma" if gemm / (PEAK_MFMA_BF16_TFLOPS * 1e12) >= 0.95 * proj_bytes / (PEAK_HBM_GBS * 1e9) else "hbm"
    return {
        # R = P^T G: read G and P once, write R (fp32)
        "project": dict(flops=gemm, bytes=proj_bytes, bound=proj_bound),
        # fused form of the two kernels around it (R stays in registers): read G and P, read and write M
        # and V (fp32), write Z (bf16) and the factors.  2 mn r flops against 2 mn + 18 Lr bytes: at
        # r = 512 the HBM time is twice the MFMA time
        "project_adam": dict(flops=gemm, bytes=2 * mn + 2 * Sr + (8 + 8 + 2) * Lr + 12 * L, bound="hbm"),
        # read R, M, V (fp32); write M, V (fp32), the bf16 operand Z (for an inactive limiter), the
        # factors; R as a second bf16 operand only when the residual contraction follows
        "adam_norms": dict(flops=0.0, bytes=(4 + 8 + 8 + 2 + (0 if gram else 2)) * Lr + (12 if gram else 4) * L,
                           bound="hbm"),
        # ||k (G - P R)||: read G, R (bf16), P; dense contraction (skipped on the Gram route)
        "residual_norm": dict(flops=0.0 if gram else gemm, bytes=0.0 if gram else 2 * mn + 2 * Lr + 2 * Sr,
                              bound="mfma"),
        "limiter": dict(flops=0.0, bytes=4 * L if gram else 0.0, bound="hbm"),
        # Z += (1 - c) k R, only for matrices whose limiter factor c came out below 1: with the
        # stationary synthetic gradients none does, so the launch only reads c and exits
        "make_z": dict(flops=0.0, bytes=0.0, bound="hbm"),
        # W -= lr alpha (P Z + c k G): read G, W, Z, P; write W.  2 mn r flops against 6 mn bytes:
        # at r = 512 the HBM time (bytes / 8 TB/s) is twice the MFMA time (flops / 2.5 PFLOP/s)
        "update": dict(flops=gemm, bytes=6 * mn + 2 * Lr + 2 * Sr, bound="hbm"),
    }


def kernel_sources_hash():
    """Hash of the kernel sources (csrc/*): a traffic record in profiles/ carries the hash of the sources it
    was measured on and is dropped when they have changed since."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2410_01623_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".h", ".hip")) and "microbench" not in name:
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


class PowerSampler:
    """Socket power from the amdgpu hwmon file (microwatts), sampled by a thread while work runs.  mean() is None
    when the file is not readable."""

    def __init__(self, period=0.02):
        import glob
        import threading
        files = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        self.path = files[0] if files else None
        self.period, self.samples = period, []
        self._stop, self._thread = threading.Event(), None
        self._threading = threading

    def cap(self):
        try:
            return int(open(self.path.replace("power1_input", "power1_cap")).read()) / 1e6
        except Exception:
            return None

    def _run(self):
        while not self._stop.is_set():
            try:
                self.samples.append(int(open(self.path).read()) / 1e6)
            except Exception:
                return
            time.sleep(self.period)

    def __enter__(self):
        if self.path:
            self._thread = self._threading.Thread(target=self._run, daemon=True)
            self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        if self._thread:
            self._thread.join()

    def mean(self, skip_first_third=False):
        x = self.samples[len(self.samples) // 3:] if skip_first_third else self.samples
        return round(sum(x) / len(x), 1) if x else None


def read_traffic(workload, norm_mode):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the same
    counters on a plain 1 GiB copy), as recorded in profiles/; {} when no record matches the workload or
    the record was made on other kernel sources (line "# kernel_sources <hash>")."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}_{norm_mode}.txt")
    out, stamp = {}, None
    if os.path.exists(path):
        for line in open(path):
            p = line.split()
            if line.startswith("# kernel_sources") and len(p) >= 3:
                stamp = p[2]
            if len(p) >= 2 and not line.startswith("#"):
                try:
                    out[p[0]] = float(p[1])
                except ValueError:
                    pass
    if stamp != kernel_sources_hash():
        return {}
    return out


def cpu_baseline(wl, sample_mats, steps=1):
    """The oracle as it stands, on the host cores, on `sample_mats` of the workload."""
    import numpy as np
    from oracle import fira_oracle as orc
    from paper_2410_01623_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    hp = orc.OracleHparams()
    data = []
    for i in sample_mats:
        m, n = wl.shapes[i]
        W = synth.gen_W(wl, i).astype(np.float64)
        G = synth.gen_G(wl, i, 0).astype(np.float64)
        P = synth.store_projector(synth.random_orthonormal_projector(wl, i, min(m, n), wl.rank), wl.dtype)
        data.append((W, G, P.astype(np.float64), orc.OracleState.zeros(m, n, wl.rank)))
    t0 = time.perf_counter()
    for _ in range(steps):
        for (W, G, P, st) in data:
            orc.fira_step(W, G, P, st, hp, store_bf16=(wl.dtype == "bf16"))
    dt = (time.perf_counter() - t0) / steps
    frac = sum(m * n for m, n in (wl.shapes[i] for i in sample_mats)) / sum(m * n for m, n in wl.shapes)
    return dict(value=frac / dt, unit="steps/s", cores=int(cores),
                kind=f"oracle (numpy fp64; its matrix products run in the BLAS numpy links, {int(cores)} threads)",
                sample=f"{len(sample_mats)} of {wl.n_matrices} matrices (one block), {steps} step(s), "
                       f"{dt:.2f} s per step of the sample ({dt * steps:.1f} s in all), scaled by the sample's share "
                       f"of the elements ({frac:.4f})")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10, help="untimed steps directly before the timed ones")
    ap.add_argument("--settle-steps", type=int, default=40,
                    help="untimed steps before the warm-up that bring the optimizer state from its zero start to "
                         "the steady state: from M = V = 0 the factors move and the limiter (Eq. 12) acts on the "
                         "first 30 or so steps of a run, which belong to the limiter-active regime that is timed "
                         "separately (--limited-steps), not to the steady state that `value` reports; whatever "
                         "--warmup says, the timed region then starts with no matrix limited "
                         "(config.matrices_limited_after_settling)")
    ap.add_argument("--limited-steps", type=int, default=30,
                    help="after the timed steps, also time this many steps in which the limiter acts on every matrix "
                         "(gradients whose part outside the subspace is eight times larger; reported under "
                         "\"limiter_active\", not part of value); 0 = skip")
    ap.add_argument("--workload", default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy (for scaling HBM traffic counters)")
    ap.add_argument("--pad-ld", type=int, default=0,
                    help="round the leading dimension of W and G up to a multiple of this many elements "
                         "(0 = dense rows, ld = n: the headline configuration)")
    ap.add_argument("--refresh-iters", type=int, default=0,
                    help="also time fira_refresh_projectors over all matrices with this many rounds of subspace "
                         "iteration (after the timed steps; reported under \"refresh\", not part of value)")
    ap.add_argument("--power-seconds", type=float, default=3.0,
                    help="after the timed steps, keep stepping for this many seconds while the socket power is sampled "
                         "(reported under \"power\", together with a plain copy and a library bf16 matrix product "
                         "run the same way for comparison; not part of value; 0 = skip)")
    ap.add_argument("--no-fusion", action="store_true",
                    help="run the projection and Adam as two kernels with R in memory")
    ap.add_argument("--norm-mode", choices=["gram", "residual"], default="gram",
                    help="how the limiter norm ||S|| is obtained (both are parity-tested)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives); use --gpus 1")

    import torch
    from paper_2410_01623_amd import fira, synth

    name = args.workload or synth.HEADLINE
    wl = synth.WORKLOADS[name]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    dt_t = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    dt_f = fira.FIRA_BF16 if wl.dtype == "bf16" else fira.FIRA_F32
    shapes = wl.shapes
    gen = torch.Generator(device=dev)
    gen.manual_seed(1000 * wl.config_id)
    lds = [((n + args.pad_ld - 1) // args.pad_ld) * args.pad_ld if args.pad_ld else n for (m, n) in shapes]
    ctx = fira.FiraContext(shapes, wl.rank, dt_f, fira.make_hparams(), device=dev, lds=lds)
    ctx.fira_set_options(norm_mode=fira.FIRA_NORM_GRAM if args.norm_mode == "gram" else fira.FIRA_NORM_RESIDUAL)
    if args.no_fusion:
        ctx.fira_set_fusion(False)
    # projectors: one seeded orthonormal basis per distinct short side, installed into every matrix
    cache, Ps = {}, []
    for i, (m, n) in enumerate(shapes):
        key = (min(m, n), m <= n)
        if key not in cache:
            P = synth.store_projector(synth.random_orthonormal_projector(wl, len(cache), min(m, n), wl.rank), wl.dtype)
            cache[key] = torch.from_numpy(P).to(dt_t).to(dev)
        Ps.append(cache[key])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ctx.fira_set_projectors(range(len(shapes)), Ps)   # one launch per phase for every 16 matrices
    torch.cuda.synchronize()
    install_ms = (time.perf_counter() - t0) * 1e3
    def draw(scale, i):
        m, n = shapes[i]
        t = (scale * torch.randn((m, lds[i]), device=dev, generator=gen)).to(dt_t)
        return t[:, :n]
    W = [draw(0.02, i) for i in range(len(shapes))]
    n_sets = 3
    Gsets = [[draw(wl.grad_scale, i) for i in range(len(shapes))] for _ in range(n_sets)]
    idx = list(range(len(shapes)))
    prepared = [ctx.prepare(idx, W, G) for G in Gsets]
    torch.cuda.synchronize()

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for s in range(args.settle_steps):
        ctx.fira_step(prepared=prepared[s % n_sets])
    torch.cuda.synchronize()
    # (read here, not between the warm-up and the timed steps: 168 small copies with a synchronisation each are a
    # pause of some milliseconds, after which the chip takes a few steps to bring its clock up again)
    limited_at_start = sum(1 for i in range(len(shapes)) if ctx.fira_get_diag(i)[2] < 1.0)
    power = PowerSampler()
    for s in range(args.warmup):
        ctx.fira_step(prepared=prepared[(args.settle_steps + s) % n_sets])
    torch.cuda.synchronize()
    ctx.fira_profile_begin(args.steps)
    with power:
        t0 = time.perf_counter()
        for s in range(args.steps):
            ctx.fira_step(prepared=prepared[(args.settle_steps + args.warmup + s) % n_sets])
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    ms_sum, rec = ctx.fira_profile_end()
    fused = ctx.fira_last_step_fused()
    if fused:   # one kernel did the work of the first two slots
        ms_sum = dict([("project_adam", ms_sum["project"] + ms_sum["adam_norms"])] +
                      [(k, v) for k, v in ms_sum.items() if k not in ("project", "adam_norms")])
    finite = all(bool(torch.isfinite(w).all()) for w in W[:7])
    limited = sum(1 for i in range(len(shapes)) if ctx.fira_get_diag(i)[2] < 1.0)   # limiter active in the last step

    model = kernel_models(shapes, wl.rank, args.norm_mode)
    traffic = read_traffic(name, args.norm_mode)
    kernels = {}
    for k, tot in ms_sum.items():
        avg_ms = tot / max(rec, 1)
        mdl = model[k]
        bound = mdl["bound"]
        if bound == "mfma":
            ach, peak, unit = (mdl["flops"] / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0), PEAK_MFMA_BF16_TFLOPS, "TFLOP/s"
        else:
            ach, peak, unit = (mdl["bytes"] / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0), PEAK_HBM_GBS, "GB/s"
        kernels[k] = dict(avg_ms=round(avg_ms, 4), bound=bound, achieved=round(ach, 2), peak=peak, unit=unit,
                          frac=round(ach / peak, 4), gflop=round(mdl["flops"] / 1e9, 1),
                          gbyte=round(mdl["bytes"] / 1e9, 3), traffic=traffic.get(k))
    dom = max((k for k in kernels if k != "limiter"), key=lambda k: kernels[k]["avg_ms"])
    roof = dict(kernel=dom, bound=kernels[dom]["bound"], achieved=kernels[dom]["achieved"], peak=kernels[dom]["peak"],
                unit=kernels[dom]["unit"], frac=kernels[dom]["frac"], traffic=kernels[dom]["traffic"],
                avg_ms=kernels[dom]["avg_ms"])

    out = {
        "metric": "fira_optimizer_steps_per_s", "value": round(args.steps / dt, 3), "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(1e3 * dt / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": name, "matrices": len(shapes), "rank": wl.rank,
                   "params": sum(m * n for m, n in shapes), "state_bytes": ctx.state_bytes,
                   "gradient_sets": n_sets, "norm_mode": args.norm_mode, "fused_projection_adam": fused, "ld": "n" if not args.pad_ld else f"n rounded up to {args.pad_ld}", "finite": finite,
                   "matrices_limited_last_step": limited, "matrices_limited_after_settling": limited_at_start,
                   "projector_install_ms": round(install_ms, 3), "settle_steps": args.settle_steps,
                   "socket_power_w": power.mean(), "socket_power_cap_w": power.cap()},
        "roofline": roof, "kernels": kernels,
    }
    if args.limited_steps > 0:
        # The limiter-active regime (Algorithm 1's limiter line fires whenever ||S_t|| grows by more than gamma):
        # gradients whose out-of-subspace part is eight times larger, G + 7 (G - P P^T G).  R, M, V and the
        # factors are unchanged, ||S_t|| is eight times larger, and since the limiter lets the remembered norm
        # grow by 1 % a step, every matrix stays limited for about 200 steps.  The inputs are prepared here
        # with torch (input generation, outside the timed region).
        def spiked(i, g):
            m, n = shapes[i]
            P = cache[(min(m, n), m <= n)].float()
            gf = g.float()
            out = gf - P @ (P.t() @ gf) if m <= n else gf - (gf @ P) @ P.t()
            t = torch.empty((m, lds[i]), dtype=dt_t, device=dev)[:, :n]
            t.copy_((gf + 7.0 * out).to(dt_t))
            return t
        Gspike = [[spiked(i, g) for i, g in enumerate(G)] for G in Gsets]
        prep_spike = [ctx.prepare(idx, W, G) for G in Gspike]
        torch.cuda.synchronize()
        for s in range(5):
            ctx.fira_step(prepared=prep_spike[s % n_sets])
        torch.cuda.synchronize()
        ctx.fira_profile_begin(args.limited_steps)
        t1 = time.perf_counter()
        for s in range(args.limited_steps):
            ctx.fira_step(prepared=prep_spike[s % n_sets])
        torch.cuda.synchronize()
        dtl = time.perf_counter() - t1
        ms_l, rec_l = ctx.fira_profile_end()
        cs = [ctx.fira_get_diag(i)[2] for i in range(len(shapes))]
        out["limiter_active"] = dict(ms_per_step=round(1e3 * dtl / args.limited_steps, 4), steps=args.limited_steps,
                                     matrices_limited=sum(1 for c in cs if c < 1.0), c_mean=round(sum(cs) / len(cs), 4),
                                     make_z_ms=round(ms_l["make_z"] / max(rec_l, 1), 4),
                                     finite=all(bool(torch.isfinite(w).all()) for w in W[:7]))
        del Gspike, prep_spike
    if args.power_seconds > 0:
        try:
            # What the step draws against the socket's power cap, next to a plain copy and the vendor library's bf16
            # matrix product measured the same way: the chip lowers its clock to stay under the cap, so the energy
            # of a step, not the occupancy of one unit, is what its time follows.
            def powered(fn, work_per_call):
                fn()
                torch.cuda.synchronize()
                with PowerSampler(0.05) as ps:
                    t1, n = time.perf_counter(), 0
                    while time.perf_counter() - t1 < args.power_seconds:
                        for _ in range(10):
                            fn()
                        torch.cuda.synchronize()
                        n += 10
                    el = time.perf_counter() - t1
                return dict(ms_per_call=round(1e3 * el / n, 4), rate=round(work_per_call * n / el, 1), socket_w=ps.mean(True))
            state = {"s": 0}
            def one_step():
                ctx.fira_step(prepared=prepared[state["s"] % n_sets])
                state["s"] += 1
            pw = {"cap_w": PowerSampler().cap(), "seconds_each": args.power_seconds}
            pw["fira_step"] = powered(one_step, 1.0)                                   # rate: steps/s
            src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
            dst = torch.empty_like(src)
            pw["copy_1GiB"] = powered(lambda: dst.copy_(src), 2.0 * (1 << 30) / 1e9)   # rate: GB/s read + written
            del src, dst
            A = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
            B = torch.randn(8192, 8192, device=dev).to(torch.bfloat16)
            pw["library_matmul_bf16_8192"] = powered(lambda: torch.matmul(A, B), 2.0 * 8192 ** 3 / 1e12)   # rate: TFLOP/s
            del A, B
            torch.cuda.synchronize()
            with PowerSampler(0.05) as ps:      # nothing running (the clocks have not yet dropped to the low-power state)
                time.sleep(2.0)
            pw["idle_w"] = ps.mean(True)
            out["power"] = pw
        except Exception as e:   # a reported comparison, never a reason to lose the line
            out["power"] = {"error": repr(e)}
    if args.refresh_iters > 0:
        # projector refresh (Algorithm 1's "if t mod T = 0" branch) over every matrix, from the first gradient set
        idx_all = list(range(len(shapes)))
        ws = torch.empty(ctx.fira_refresh_workspace_bytes(idx_all), dtype=torch.uint8, device=dev)
        ctx.fira_refresh_projectors(idx_all, Gsets[0], iters=args.refresh_iters, seed=1, workspace=ws)   # warm-up
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ctx.fira_refresh_projectors(idx_all, Gsets[0], iters=args.refresh_iters, seed=2, workspace=ws)
        torch.cuda.synchronize()
        rms = 1e3 * (time.perf_counter() - t1)
        # what was timed must be a usable projector: finite, orthonormal to the bf16 rounding of its entries
        defect = 0.0
        for i in sorted(set([0, len(wl.block_shapes) - 1, len(shapes) - 1])):
            Pi = ctx.fira_get_projector(i).double()
            assert bool(torch.isfinite(Pi).all()), f"refresh left a non-finite projector for matrix {i}"
            defect = max(defect, float((Pi.t() @ Pi - torch.eye(wl.rank, dtype=torch.float64)).abs().max()))
        assert defect < 2e-2, f"refreshed projector is not orthonormal: max |P^T P - I| = {defect:.3g}"
        # the subspace iteration multiplies by G four times per round (two contractions of 2 mn r flops each way)
        out["refresh"] = dict(ms=round(rms, 2), iters=args.refresh_iters, workspace_bytes=int(ws.numel()),
                              max_orthonormality_defect=round(defect, 6),
                              ms_per_step_at_T200=round(rms / 200.0, 4),
                              contraction_tflops=round(args.refresh_iters * 2 * 2.0 * sum(m * n for m, n in shapes) * wl.rank / (rms * 1e-3) / 1e12, 1))
        del ws
    if not args.no_cpu_baseline:
        nb = len(wl.block_shapes)
        out["cpu_baseline"] = cpu_baseline(wl, list(range(nb)), steps=10)   # about 10 s of host work
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
