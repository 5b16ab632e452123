"""Benchmark of the per-block Shampoo step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload transformer|resnet50|uniform|rootstress]
                    [--block-size 2048|4096|8192]

Workload (default): the transformer-shaped parameter set -- 24 layers at d = 2048
(QKV 2048x6144, attention out 2048x2048, MLP up 2048x8192, MLP down 8192x2048,
LayerNorm vectors), block size 1024 -> 1152 blocks of 1024x1024, 1.21e9 parameters,
bf16 gradients N(0, 1e-3^2), float32 factors / roots / state, beta2 = 0.999,
epsilon = 1e-12, root exponent 1/4, precondition_frequency = 100, AdaGrad grafting
(eps 1e-10), momentum 0.9, lr 0.01.  Everything is synthetic and seeded; gradients are
resident in HBM before the timed region (a pool of two pre-generated sets is cycled).

A "step" is one whole shampoo_step: factor updates, grafting pass, two-sided
preconditioning, rescale + momentum + parameter update, 1-D parameters.  Step 0 holds
the root-inverse refresh; it runs in the warm-up and its time is reported separately
(`refresh_ms`).  The K timed steps are non-refresh steps.

One JSON line is printed:
  metric/value        milliseconds per (non-refresh) step, whole job, one GPU; next to it
                      `refresh_ms` (one root-inverse refresh of every factor, taken at the first
                      timed refresh) and `amortized_ms_per_step` = value + refresh_ms / f
  later_refresh       after the timed steps the run goes on, untimed and with a fresh gradient set
                      per step, to the next refresh (step f later) and times that one too: its
                      factors are moving averages over many independent gradients, as at every
                      refresh of a training run but the first (--no-later-refresh skips this)
  roofline            the dominant kernel: for blocks above 128 the second GEMM of the two-sided
                      preconditioning, P = T Rbar.  `achieved` is its ALGORITHMIC rate: 2 m n^2 flops
                      per block x blocks per launch / average launch duration, against the dense
                      peak of the matrix-core type it runs on.  With bf16 gradients that is the fp16
                      matrix cores (2.5 PFLOP/s): the float32 operands are split into two scaled
                      fp16 planes and three exact fp16 products make one float32 product, so the
                      matrix cores execute three times the algorithmic flops: `executed_tflops` /
                      `executed_frac` give that utilisation separately.  With --fp32-matrix-cores
                      or float32 gradients it is the float32-MFMA kernel against 157.3 TFLOP/s
                      (the default run carries that variant's step and roofline in
                      `fp32_matrix_cores`, from a short second run without refresh).  For workloads
                      whose blocks are at most 128 x 128 the dominant kernel is the
                      single-workgroup block-step kernel, which is bound by HBM (algorithmic
                      bytes per launch / average launch duration).  Durations come from HIP
                      events recorded by the library on the step's stream
  cpu_baseline        the fp64 numpy oracle timed on the host, stage by stage, on a sample of
                      blocks (48 of the largest bucket for a non-refresh step, 16 factors for
                      the refresh), scaled linearly to the whole block set

--workload rootstress times the root-inverse stress case instead (256 matrices of 2048 x 2048,
rank 64 + 1e-6 I): one JSON line with metric root_inverse_ms.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_F16_MFMA_TFLOPS = 2500.0
# HBM bytes per launch of the dominant kernel (P = T Rbar) on the transformer workload, from
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a 1 GiB copy (x2.0 / x1.0):
# profiles/transformer_b1024_hbm_traffic_pmc.md
TRAFFIC_BYTES = {"transformer": 14.43e9 + 4.83e9}
# the same for the single-workgroup block-step kernel on the ResNet-50 shapes:
# profiles/resnet50_b128_hbm_traffic_pmc.md
FUSED_TRAFFIC_BYTES = {"resnet50": 0.849e9 + 0.631e9}
# and for P = T Rbar on the fp16 matrix cores (two-plane operands) of the transformer workload:
# profiles/transformer_b1024_hbm_traffic_pmc.md
X2_TRAFFIC_BYTES = {"transformer": 9.66e9 + 4.83e9}
PEAK_HBM_GBS = 8000.0
TILE = 128


def workload(name, block_size=None):
    from paper_2309_06497_amd import workloads as wl
    from paper_2309_06497_amd import binding as B
    if name == "transformer":
        b = block_size or 1024
        return dict(shapes=wl.transformer_shapes(), block=b, sigma=1e-3, f=100, bf16=True,
                    label=f"transformer 24 x d2048, block {b}, bf16 gradients")
    if name == "resnet50":
        return dict(shapes=wl.resnet50_shapes(), block=128, sigma=1e-3, f=50, bf16=False,
                    label="ResNet-50 shapes, block 128, 1576 blocks, fp32 gradients")
    if name == "uniform":
        return dict(shapes=wl.uniform_shapes(), block=128, sigma=1e-3, f=100, bf16=False,
                    label="512 blocks of 128x128, fp32 gradients")
    raise SystemExit(f"unknown workload {name}")


def flop_counts(table):
    """Algorithmic flops per step (symmetric updates at triangular cost) and the flops the
    128 x 128-tiled kernels execute (whole diagonal tiles)."""
    alg_factor = alg_precond = exe_factor = exe_precond = 0.0
    for row in table:
        m, n = float(row[3]), float(row[4])
        alg_factor += m * n * (m + n)
        alg_precond += 2 * m * n * (m + n)
        tm, tn = -(-int(m) // TILE), -(-int(n) // TILE)
        exe_factor += 2.0 * TILE * TILE * (tm * (tm + 1) / 2 * n + tn * (tn + 1) / 2 * m)
        exe_precond += 2.0 * TILE * TILE * tm * tn * (m + n)
    return alg_factor, alg_precond, exe_factor, exe_precond


def fused_bytes(table, gsz):
    """Algorithmic HBM bytes per step of the blocks that take the single-workgroup kernel
    (m, n <= 128): G once, L and R read + written, Lbar and Rbar read, A, M, W read + written."""
    total = 0.0
    for row in table:
        m, n = float(row[3]), float(row[4])
        if m <= 128 and n <= 128:
            total += (gsz + 24.0) * m * n + 12.0 * (m * m + n * n)
    return total


def cpu_baseline(wk, table, rng_seed=0):
    """The oracle, untuned, on the host cores, stage by stage: a bounded sample of blocks of
    the largest bucket for one non-refresh step, and a few factors for the refresh; scaled
    linearly to the whole block set (blocks are independent)."""
    from oracle import shampoo_oracle as so
    rng = np.random.default_rng(rng_seed)
    sizes = {}
    for row in table:
        sizes[(int(row[3]), int(row[4]))] = sizes.get((int(row[3]), int(row[4])), 0) + 1
    (m, n), _ = max(sizes.items(), key=lambda kv: kv[1] * kv[0][0] * kv[0][1])
    elems_total = sum(float(r[3]) * float(r[4]) for r in table)
    n_step = 48 if m * n >= 512 * 512 else 256
    if m * n >= 4096 * 2048:
        n_step = 4
    n_root = 8 if m >= 512 else 64
    if m >= 4096:
        n_root = 1
    f32 = lambda v: float(np.float32(v))
    state = []
    for _ in range(n_step):
        G = (rng.standard_normal((m, n)) * wk["sigma"]).astype(np.float32)
        L, R = so.factor_update(np.zeros((m, m)), np.zeros((n, n)), G, f32(0.999))
        state.append([L, R, np.eye(m), np.eye(n), np.zeros((m, n)), np.zeros((m, n)), np.zeros((m, n))])
    stage = {"factor": 0.0, "graft": 0.0, "precond": 0.0, "update": 0.0}
    clk = time.perf_counter
    for st in state:
        G = (rng.standard_normal((m, n)) * wk["sigma"]).astype(np.float32)
        t0 = clk()
        st[0], st[1] = so.factor_update(st[0], st[1], G, f32(0.999))
        t1 = clk()
        st[4] = so.graft_state_update(st[4], G)
        Pg = so.graft_direction(G, st[4], f32(1e-10))
        t2 = clk()
        Psh = so.shampoo_direction(st[2], G, st[3])
        t3 = clk()
        P = so.grafted_direction(Psh, Pg)
        st[5] = f32(0.9) * st[5] + P
        st[6] += f32(0.01) * st[5]
        t4 = clk()
        stage["factor"] += t1 - t0; stage["graft"] += t2 - t1; stage["precond"] += t3 - t2; stage["update"] += t4 - t3
    scale = elems_total / (n_step * m * n)
    stage_ms = {k: v * scale * 1e3 for k, v in stage.items()}
    t0 = clk()
    for st in state[:n_root]:
        so.root_inverse(st[0], f32(1e-12), 0.25)
        so.root_inverse(st[1], f32(1e-12), 0.25)
    t_root = (clk() - t0) / (n_root * (m * m + n * n)) * sum(
        float(r[3]) ** 2 + float(r[4]) ** 2 for r in table)
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": sum(stage_ms.values()), "unit": "ms/step", "cores": cores, "kind": "oracle",
            "stage_ms_per_step": stage_ms, "refresh_ms": t_root * 1e3,
            "sample": f"{n_step} of {len(table)} blocks ({m}x{n}) for one non-refresh step, timed stage by "
                      f"stage, and {2 * n_root} factors for the refresh, numpy float64 (LAPACK eigh), "
                      f"scaled linearly to the whole block set (extrapolated)"}


def rootstress(args):
    """The root-inverse stress case: 256 matrices of 2048 x 2048, rank 64 + 1e-6 I."""
    import torch
    from paper_2309_06497_amd import binding as B
    from oracle import shampoo_oracle as so
    n, rank, batch = 2048, 64, 256
    dev = torch.device("cuda", 0)
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    a = torch.empty((batch, n, n), dtype=torch.float32, device=dev)
    for i in range(0, batch, 16):     # formed in float64, rounded once to float32
        g = torch.randn((16, n, rank), generator=gen, device=dev, dtype=torch.float64)
        a[i:i + 16] = (g @ g.transpose(1, 2) + 1e-6 * torch.eye(n, dtype=torch.float64, device=dev)).to(torch.float32)
    times = []
    for rep in range(max(args.warmup, 1) + max(args.steps // 5, 1)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        x, failed = B.shampoo_root_inverse(a, 1e-12, 0.25, False, True)
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3)
    timed = times[max(args.warmup, 1):]
    ms = sum(timed) / len(timed)
    out = {"metric": "root_inverse_ms", "value": ms, "unit": "ms", "n_gpus": 1, "steps": len(timed),
           "warmup": max(args.warmup, 1), "ms_per_step": ms, "higher_is_better": False, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32 in / out, f32 + f64 sweeps", "data": "synthetic",
           "config": {"workload": "root-inverse stress: 256 matrices of 2048 x 2048, rank 64 + 1e-6 I, eps 1e-12, exponent 1/4"},
           "ms_per_matrix": ms / batch, "failed_roots": int(failed.sum())}
    if not args.no_cpu_baseline:
        a_host = a[:2].cpu().numpy()
        t0 = time.perf_counter()
        for k in range(2):
            so.root_inverse(a_host[k], float(np.float32(1e-12)), 0.25)
        t_cpu = (time.perf_counter() - t0) / 2 * batch
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": t_cpu * 1e3, "unit": "ms", "cores": cores, "kind": "oracle",
                               "sample": "2 of the 256 matrices, numpy float64 (LAPACK eigh), scaled linearly (extrapolated)"}
    print(json.dumps(out))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="transformer")
    ap.add_argument("--block-size", type=int, default=None,
                    help="block size of the transformer workload (default 1024; 2048, 4096 and 8192 are the "
                         "larger preconditioner sizes of Sec. 4.2.1 / Table 5)")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the short second run of the default workload on the float32 matrix cores")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-later-refresh", action="store_true",
                    help="stop after the timed steps instead of going on to the next refresh and timing it")
    ap.add_argument("--skip-refresh", action="store_true",
                    help="number the steps from 4 so that no root refresh runs (roots stay the identity); "
                         "for counter runs of the per-step kernels only")
    ap.add_argument("--root-method", default="eigh", choices=["eigh", "newton"],
                    help="root-inverse routine of the refresh: eigendecomposition (default) or the coupled "
                         "inverse Newton iteration (float32; meant for well-conditioned factors)")
    ap.add_argument("--first-refresh-at", type=int, default=0,
                    help="run this many untimed grafting-only steps first (start_preconditioning_step), so that "
                         "the timed refresh sees factors accumulated over that many gradients; must be a "
                         "multiple of the workload's precondition_frequency")
    ap.add_argument("--fp32-matrix-cores", action="store_true",
                    help="keep the preconditioning products on the float32 matrix cores (default: bf16 matrix "
                         "cores with the two-plane split when the gradients are bf16)")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also run one 1 GiB device-to-device copy, the reference for scaling HBM counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the multi-GPU distribution of the "
              "paper is out of scope); rerun with --gpus 1", file=sys.stderr)
        return 2
    if args.workload == "rootstress":
        return rootstress(args)
    import torch
    from paper_2309_06497_amd import binding as B

    wk = workload(args.workload, args.block_size)
    shapes = wk["shapes"]
    f = wk["f"]
    warm = max(args.warmup, 1)
    t_first = args.first_refresh_at
    if t_first % f != 0 or t_first < 0 or (t_first and args.skip_refresh):
        print(f"bench.py: --first-refresh-at must be a non-negative multiple of {f}", file=sys.stderr)
        return 2
    if warm + args.steps > f:
        print(f"bench.py: warmup + steps must stay below precondition_frequency = {f}", file=sys.stderr)
        return 2
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    gdt = torch.bfloat16 if wk["bf16"] else torch.float32
    params = [torch.randn(s, generator=gen, device=dev, dtype=torch.float32) * 0.02 for s in shapes]
    pool = [[(torch.randn(s, generator=gen, device=dev, dtype=torch.float32) * wk["sigma"]).to(gdt)
             for s in shapes] for _ in range(2)]
    opt = B.Shampoo(shapes, wk["block"], 0.999, 1e-12, 0.25, f, t_first, 1e-10, 0.9,
                    B.GRAD_BF16 if wk["bf16"] else B.GRAD_F32,
                    root_method=B.ROOT_NEWTON if args.root_method == "newton" else B.ROOT_EIGH,
                    precond_matrix_cores=B.MATRIX_CORES_FP32 if args.fp32_matrix_cores else B.MATRIX_CORES_AUTO)
    table, n_buckets = opt.plan()
    n_elems = sum(int(np.prod(s)) for s in shapes)

    # warm-up: step 0 carries the root-inverse refresh
    opt.set_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    # --skip-refresh: steps are numbered from 4 (no refresh before step f, and the bf16 factor
    # update has left its float64-accumulating variant for young factors behind by then)
    base = 4 if args.skip_refresh else t_first
    for t in range(t_first):          # untimed: factors accumulate, the step is the grafted one
        if t >= 2:                    # a fresh gradient set per step, so that the factors at the refresh are those of
            for g in pool[t % 2]:     # t_first + 1 independent gradients (cycling two sets would leave them at rank 2 n)
                g.copy_(torch.randn(g.shape, generator=gen, device=dev, dtype=torch.float32) * wk["sigma"])
        opt.step(params, pool[t % 2], 0.01, t)
    torch.cuda.synchronize()
    opt.get_timing()
    if args.copy_ref:
        ref_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_(generator=gen)
        ref_dst = torch.empty_like(ref_src)
        ref_dst.copy_(ref_src)
    opt.step(params, pool[0], 0.01, base)
    torch.cuda.synchronize()
    first_step_ms = (time.perf_counter() - t0) * 1e3
    refresh_ms = opt.get_timing()["root"][0]
    for t in range(1, warm):
        opt.step(params, pool[t % 2], 0.01, base + t)
    torch.cuda.synchronize()
    opt.get_timing()

    t0 = time.perf_counter()
    for t in range(warm, warm + args.steps):
        opt.step(params, pool[t % 2], 0.01, base + t)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    stages = opt.get_timing()
    status = opt.status()

    # on to the next refresh: the factors it sees are moving averages over many independent gradient sets
    later = None
    if not args.skip_refresh and not args.no_later_refresh:
        t_next = base + f
        for t in range(base + warm + args.steps, t_next + 1):
            for g in pool[t % 2]:
                g.copy_(torch.randn(g.shape, generator=gen, device=dev, dtype=torch.float32) * wk["sigma"])
            if t == t_next:
                torch.cuda.synchronize()
                opt.get_timing()
            opt.step(params, pool[t % 2], 0.01, t)
        torch.cuda.synchronize()
        later_ms = opt.get_timing()["root"][0]
        later = {"at_step": t_next, "refresh_ms": later_ms, "amortized_ms_per_step": ms_per_step + later_ms / f,
                 "status": opt.status()}

    alg_f, alg_p, exe_f, exe_p = flop_counts(table)
    st_ms = {k: v[0] / args.steps for k, v in stages.items()}
    # the dominant kernel is the second product of the preconditioning stage, P = T Rbar
    # (2 m n^2 flops per block; one launch per bucket and step)
    alg_p2 = sum(2.0 * float(r[3]) * float(r[4]) ** 2 for r in table)
    n_launch = stages["precond2"][1]
    launch_ms = stages["precond2"][0] / max(n_launch, 1)
    gemm_flops_per_launch = alg_p2 * args.steps / max(n_launch, 1)
    achieved = gemm_flops_per_launch / (launch_ms * 1e-3) / 1e12 if launch_ms > 0 else 0.0
    st_ms["precond"] += st_ms.pop("precond2")
    first_ms = stages["precond"][0] / max(stages["precond"][1], 1)
    gsz = 2 if wk["bf16"] else 4
    ew_bytes = {"graft": (gsz + 8.0) * n_elems, "update": 20.0 * n_elems}
    x2 = wk["bf16"] and not args.fp32_matrix_cores and wk["block"] % 8 == 0
    default_shape = args.workload == "transformer" and wk["block"] == 1024
    if x2:
        # P = T Rbar executes 3 fp16 products per float32 product (T = Lbar G: 2, the gradient is one plane)
        executed = achieved * 3.0
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_F16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_F16_MFMA_TFLOPS,
                    "traffic": X2_TRAFFIC_BYTES.get(args.workload) if default_shape else None,
                    "kernel": "gemm_f16x2_kernel<256, 128, 2, 0> (P = T Rbar, fp16 MFMA on two-plane float32 operands)",
                    "matrix_core_dtype": "f16", "products_per_float32_product": 3,
                    "launch_ms": launch_ms, "flops_per_launch": gemm_flops_per_launch,
                    "executed_flops_per_launch": gemm_flops_per_launch * 3.0,
                    "executed_tflops": executed, "executed_frac": executed / PEAK_F16_MFMA_TFLOPS,
                    "first_product_launch_ms": first_ms,
                    "frac_of_fp32_mfma_peak": achieved / PEAK_FP32_MFMA_TFLOPS}
    else:
        roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS,
                    "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                    "traffic": TRAFFIC_BYTES.get(args.workload) if default_shape else None,
                    "kernel": "gemm_mfma_kernel<0, 1, float, float, 1, false, 0> (P = T Rbar, fp32 MFMA)",
                    "matrix_core_dtype": "f32", "first_product_launch_ms": first_ms,
                    "launch_ms": launch_ms, "flops_per_launch": gemm_flops_per_launch}
    fused_ms, fused_launches = stages["fused"]
    if fused_launches > 0 and fused_ms >= stages["precond"][0] + stages["precond2"][0]:
        bytes_per_launch = fused_bytes(table, gsz) * args.steps / fused_launches
        f_launch_ms = fused_ms / fused_launches
        gbs = bytes_per_launch / (f_launch_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": gbs / PEAK_HBM_GBS, "traffic": FUSED_TRAFFIC_BYTES.get(args.workload),
                    "kernel": "block_step_small_kernel (whole step of a block <= 128 x 128 in one workgroup)",
                    "launch_ms": f_launch_ms, "bytes_per_launch": bytes_per_launch}
    out = {
        "metric": "shampoo_step_ms",
        "value": ms_per_step,
        "unit": "ms/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": warm,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 state and accumulation, operands of the preconditioning products as two fp16 planes" if x2 else "f32",
        "data": "synthetic",
        "config": {"workload": wk["label"], "params": n_elems, "blocks": int(len(table)),
                   "buckets": int(n_buckets), "block_size": wk["block"], "precondition_frequency": f,
                   "grad_dtype": "bf16" if wk["bf16"] else "f32", "root_method": args.root_method,
                   "precond_matrix_cores": "f32" if (args.fp32_matrix_cores or not wk["bf16"]) else "f16x2",
                   "first_refresh_at_step": t_first},
        "refresh_ms": refresh_ms,
        "first_step_ms": first_step_ms,
        "amortized_ms_per_step": ms_per_step + refresh_ms / f,
        "tflops_algorithmic": (alg_f + alg_p) / (ms_per_step * 1e-3) / 1e12,
        "tflops_executed": (exe_f + exe_p) / (ms_per_step * 1e-3) / 1e12,
        "stage_ms_per_step": st_ms,
        "roofline": roofline,
        "stage_roofline": {
            # bf16 gradients: G G^T runs on the bf16 matrix cores (exact products, float32 / float64
            # accumulation); the figure is algorithmic flops per second, comparable to the float32 peak
            "factor": {"bound": "mfma", "matrix_core_dtype": "bf16" if wk["bf16"] else "f32",
                       "tflops_algorithmic": alg_f / (st_ms["factor"] * 1e-3) / 1e12 if st_ms["factor"] else 0,
                       "tflops_executed": exe_f / (st_ms["factor"] * 1e-3) / 1e12 if st_ms["factor"] else 0},
            "precond": {"bound": "mfma", "tflops": alg_p / (st_ms["precond"] * 1e-3) / 1e12 if st_ms["precond"] else 0},
            "graft": {"bound": "hbm", "GBps": ew_bytes["graft"] / (st_ms["graft"] * 1e-3) / 1e9 if st_ms["graft"] else 0},
            "update": {"bound": "hbm", "GBps": ew_bytes["update"] / (st_ms["update"] * 1e-3) / 1e9 if st_ms["update"] else 0},
        },
        "status": status,
    }
    if later is not None:
        out["later_refresh"] = later
    if x2 and default_shape and not args.no_secondary and not args.skip_refresh:
        out["fp32_matrix_cores"] = secondary_fp32(B, torch, wk, shapes, params, pool, alg_p2, args.steps)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wk, table)
    print(json.dumps(out))
    return 0


def secondary_fp32(B, torch, wk, shapes, params, pool, alg_p2, steps):
    """The same workload with the preconditioning products kept on the float32 matrix cores
    (bench.py --fp32-matrix-cores runs it in full): a short second run without refresh (the
    roots stay the identity, which changes no kernel's work), for the step time and the
    roofline of the float32 MFMA kernel."""
    opt = B.Shampoo(shapes, wk["block"], 0.999, 1e-12, 0.25, wk["f"], 0, 1e-10, 0.9, B.GRAD_BF16,
                    precond_matrix_cores=B.MATRIX_CORES_FP32)
    opt.set_timing(True)
    w = [p.clone() for p in params]
    for t in range(4, 6):
        opt.step(w, pool[t % 2], 0.01, t)
    torch.cuda.synchronize()
    opt.get_timing()
    n = max(3, steps // 2)
    t0 = time.perf_counter()
    for t in range(6, 6 + n):
        opt.step(w, pool[t % 2], 0.01, t)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    st = opt.get_timing()
    launch_ms = st["precond2"][0] / max(st["precond2"][1], 1)
    tf = alg_p2 * n / max(st["precond2"][1], 1) / (launch_ms * 1e-3) / 1e12
    return {"ms_per_step": ms, "steps": n, "roots": "identity (no refresh in this second run)",
            "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                         "frac": tf / PEAK_FP32_MFMA_TFLOPS, "launch_ms": launch_ms,
                         "kernel": "gemm_mfma_kernel<0, 1, float, float, 1, false, 0> (P = T Rbar, fp32 MFMA)"},
            "command": "python bench.py --fp32-matrix-cores"}


if __name__ == "__main__":
    sys.exit(main())
