#!/usr/bin/env python3
"""Benchmark of the 4-bit GEMM path on one MI355X.

Workload: the large GEMM of the benchmark configuration (M = N = K = 8192, uint4 codes
packed two per byte, B given as K x N, za = 7, zb = 8, int32 output), seeded synthetic data
already resident in HBM.  One step = one q4_gemm call = the whole path: transposing re-pack of
B, depth sums of A and B, int8-MFMA product, zero-point epilogue.  Prints ONE JSON line.

  value      effective TOPS = 2*M*N*K / step time
  roofline   the product kernel alone (q4_gemm_presummed launches exactly that kernel), timed
             with HIP events on the launch stream, against the int8 dense MFMA peak
  cpu_baseline  the plain-loop CPU oracle on a slab of rows of the same product
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X published dense int8 rate, 5.0 POP/s
HBM_PEAK_GBS = 8000.0


def _traffic_from_profile():
    """HBM bytes per launch of the product kernel from the committed counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "q4_gemm_cfg5_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--size", type=int, default=8192, help="M = N = K (default: the benchmark's 8192)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a 256 MiB fill and a 256 MiB read-modify-write (calibrates FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2009_06488_amd import q4, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    S = args.size
    c = wl.config5(S, S, S)
    M, N, K = c.M, c.N, c.K
    ops = 2.0 * M * N * K

    A = torch.from_numpy(c.a_packed).to(dev)
    Bkn = torch.from_numpy(c.b_packed_kn).to(dev)
    C = torch.empty((M, N), dtype=torch.int32, device=dev)
    ws = torch.empty(q4.gemm_workspace_bytes(M, N, K, q4.B_KN), dtype=torch.uint8, device=dev)

    if args.copy_probe:
        probe = torch.ones(64 * 1024 * 1024, dtype=torch.int32, device=dev)   # fill: writes 256 MiB
        probe.add_(1)                                                           # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del probe

    def step():
        q4.q4_gemm(A, c.za, Bkn, c.zb, M, N, K, q4.B_KN, out=C, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tops = ops / (ms_per_step * 1e-3) / 1e12

    # ---- the dominant kernel alone, HIP events on the stream it is launched on
    Bnk = q4.q4_repack_kn_to_nk(Bkn, K, N)
    rs = q4.q4_rowsum(A, K)
    cs = q4.q4_rowsum(Bnk, K)
    C2 = torch.empty_like(C)
    for _ in range(max(2, args.warmup)):
        q4.q4_gemm_presummed(A, c.za, rs, Bnk, c.zb, cs, M, N, K, out=C2)
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        q4.q4_gemm_presummed(A, c.za, rs, Bnk, c.zb, cs, M, N, K, out=C2)
        e1.record()
    torch.cuda.synchronize()
    kern_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    kern_avg_ms = sum(kern_ms) / len(kern_ms)
    kern_tops = ops / (kern_avg_ms * 1e-3) / 1e12
    same = bool(torch.equal(C, C2))

    # ---- whole call with B already in N x K form (weights packed once)
    ws_nk = torch.empty(q4.gemm_workspace_bytes(M, N, K, q4.B_NK), dtype=torch.uint8, device=dev)
    for _ in range(2):
        q4.q4_gemm(A, c.za, Bnk, c.zb, M, N, K, q4.B_NK, out=C2, workspace=ws_nk)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        q4.q4_gemm(A, c.za, Bnk, c.zb, M, N, K, q4.B_NK, out=C2, workspace=ws_nk)
    torch.cuda.synchronize()
    nk_ms = (time.perf_counter() - t2) * 1e3 / args.steps

    out = {
        "metric": "4-bit GEMM effective TOPS and % of int8 MFMA peak (1 MI355X)",
        "value": round(tops, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "dtype_note": "uint4 codes widened to int8 MFMA operands, exact int32 accumulation",
        "data": "synthetic",
        "config": {"workload": f"config 5: uint4 GEMM M=N=K={S}, B given K x N packed, za=7 zb=8, int32 out",
                   "M": M, "N": N, "K": K, "step": "q4_gemm(Q4_B_KN): repack B + depth sums + MFMA product + epilogue"},
        "pct_of_int8_mfma_peak": round(100.0 * tops / INT8_MFMA_PEAK_TOPS, 2),
        "roofline": {
            "kernel": "q4_gemm_direct_kernel<256,256,4,2,4,4>",
            "bound": "mfma",
            "achieved": round(kern_tops, 2),
            "peak": INT8_MFMA_PEAK_TOPS,
            "unit": "TOP/s",
            "frac": round(kern_tops / INT8_MFMA_PEAK_TOPS, 4),
            "kernel_avg_ms": round(kern_avg_ms, 4),
            "kernel_min_ms": round(min(kern_ms), 4),
            "algorithmic_ops_per_launch": ops,
            "algorithmic_bytes_per_launch": M * K // 2 + N * K // 2 + 4 * M * N + 4 * (M + N),
            "traffic": _traffic_from_profile(),
        },
        "extras": {
            "ms_per_step_b_prepacked_nk": round(nk_ms, 4),
            "tops_b_prepacked_nk": round(ops / (nk_ms * 1e-3) / 1e12, 2),
            "presummed_equals_full_call": same,
        },
    }

    # ---- the paper's comparison: the same product with 8-bit codes (one per byte), same kernel minus the split
    if not args.no_extras:
        g8 = torch.Generator(device=dev)
        g8.manual_seed(5008)
        A8 = torch.randint(0, 256, (M, K), dtype=torch.uint8, device=dev, generator=g8)
        B8 = torch.randint(0, 256, (N, K), dtype=torch.uint8, device=dev, generator=g8)
        ws8 = torch.empty(int(q4.lib.q8_gemm_workspace_bytes(M, N)), dtype=torch.uint8, device=dev)
        ms8 = _time_ms(lambda: q4.q8_gemm(A8, 128, B8, 128, M, N, K, out=C2, workspace=ws8), torch, reps=50, warm=10)
        out["extras"]["q8_gemm_ms"] = round(ms8, 4)
        out["extras"]["q8_gemm_tops"] = round(ops / (ms8 * 1e-3) / 1e12, 2)
        out["extras"]["speedup_4bit_over_8bit_nk_calls"] = round(ms8 / nk_ms, 3)
        del A8, B8, ws8

    if not args.no_cpu_baseline:
        from oracle import q4_oracle as o
        rng = np.random.default_rng(7)
        probe = np.sort(rng.choice(M, size=min(16, M), replace=False))
        tp = time.perf_counter()
        want = o.gemm_rows(c.a_packed, c.za, c.b_packed_kn, c.zb, probe, N, K, o.B_KN)
        tp = time.perf_counter() - tp
        rows = int(min(max(16, 16 * 15.0 / max(tp, 1e-3)), min(M, 2048)))
        sample = np.sort(rng.choice(M, size=rows, replace=False))
        tb = time.perf_counter()
        want = o.gemm_rows(c.a_packed, c.za, c.b_packed_kn, c.zb, sample, N, K, o.B_KN)
        tb = time.perf_counter() - tb
        got = C[torch.from_numpy(sample).to(dev)].cpu().numpy()
        out["cpu_baseline"] = {
            "value": round(2.0 * rows * N * K / tb / 1e12, 6),
            "unit": "TOPS",
            "cores": o.threads(),
            "kind": "oracle",
            "sample": f"{rows} of {M} rows of A (all {N} columns, full depth {K}) through the plain-loop C oracle, "
                      f"{tb:.1f} s; host reports {os.cpu_count()} CPUs",
        }
        out["bit_exact_on_sample"] = bool(np.array_equal(got, want))

    if not args.no_extras:
        out["extras"].update(_extras(q4, wl, torch, np, dev))

    print(json.dumps(out))


def _time_ms(fn, torch, reps=20, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t) * 1e3 / reps


def _extras(q4, wl, torch, np, dev):
    """Secondary workloads (conv layer + re-quantization; the OCR-style CNN), GPU time only.
    Inputs are packed with q4_pack; parity of all of these is covered by tests/."""
    ex = {}

    # memory-bound helpers at the size of the large GEMM: algorithmic bytes / time
    S = 8192
    codes = torch.randint(0, 16, (S, S), dtype=torch.uint8, device=dev)
    packed = torch.empty((S, S // 2), dtype=torch.uint8, device=dev)
    ms = _time_ms(lambda: q4.q4_pack(codes, out=packed), torch)
    ex["pack_8192x8192_GBps"] = round(1.5 * S * S / (ms * 1e-3) / 1e9, 1)
    sums = torch.empty(S, dtype=torch.int32, device=dev)
    ms = _time_ms(lambda: q4.q4_rowsum(packed, S, out=sums), torch)
    ex["rowsum_8192x8192_GBps"] = round(0.5 * S * S / (ms * 1e-3) / 1e9, 1)
    tr = torch.empty_like(packed)
    ms = _time_ms(lambda: q4.q4_repack_kn_to_nk(packed, S, S, out=tr), torch)
    ex["repack_8192x8192_GBps"] = round(1.0 * S * S / (ms * 1e-3) / 1e9, 1)
    acc = torch.randint(-400000, 400000, (S, S), dtype=torch.int32, device=dev)
    ms = _time_ms(lambda: q4.q4_requant(acc, 24576, 20, 8, out=packed), torch)
    ex["requant_8192x8192_GBps"] = round(4.5 * S * S / (ms * 1e-3) / 1e9, 1)
    pooled = torch.empty(S * S // 8, dtype=torch.uint8, device=dev)
    # the 32 MiB of `packed` seen as an NHWC tensor of 64 x 64 x 32 x 512 codes (= 8192 * 8192)
    ms = _time_ms(lambda: q4.q4_maxpool2x2(packed.reshape(-1), 64, 64, 32, 512, out=pooled), torch)
    ex["maxpool_64x64x32x512_GBps"] = round(0.625 * S * S / (ms * 1e-3) / 1e9, 1)
    xf = torch.randn(S * S, dtype=torch.float32, device=dev)
    ms = _time_ms(lambda: q4.q4_quantize_f32(xf), torch)
    ex["quantize_f32_64M_GBps"] = round(4.5 * S * S / (ms * 1e-3) / 1e9, 1)
    ms = _time_ms(lambda: q4.q4_dequant_f32(acc.reshape(-1), 0.01, out=xf), torch)
    ex["dequant_f32_64M_GBps"] = round(8.0 * S * S / (ms * 1e-3) / 1e9, 1)
    del codes, packed, sums, tr, acc, pooled, xf

    def flat_pack(codes):
        t = torch.from_numpy(np.ascontiguousarray(codes).reshape(1, -1)).to(dev)
        return q4.q4_pack(t).reshape(-1)

    # configs 1 and 2: small GEMMs (launch / latency bound), whole q4_gemm call with B given K x N
    for (M_, N_, K_) in ((64, 32, 72), (64, 64, 72), (256, 256, 288), (1024, 1024, 1152), (1024, 64, 1152)):
        a_ = torch.randint(0, 256, (M_, K_ // 2), dtype=torch.uint8, device=dev)
        b_ = torch.randint(0, 256, (K_, N_ // 2), dtype=torch.uint8, device=dev)
        c_ = torch.empty((M_, N_), dtype=torch.int32, device=dev)
        w_ = torch.empty(q4.gemm_workspace_bytes(M_, N_, K_, q4.B_KN), dtype=torch.uint8, device=dev)
        ms = _time_ms(lambda: q4.q4_gemm(a_, 7, b_, 8, M_, N_, K_, q4.B_KN, out=c_, workspace=w_), torch, reps=50, warm=5)
        ex[f"gemm_{M_}x{N_}x{K_}_us"] = round(ms * 1e3, 2)

    # config 3: one conv layer + requant
    c = wl.config3()
    x = flat_pack(c.x_codes)
    w = q4.q4_pack(torch.from_numpy(c.w_codes.reshape(c.OC, -1)).to(dev))
    d = q4.conv_desc(c.N, c.H, c.W, c.C, c.KH, c.KW, c.stride, c.pad, c.OC)
    y = torch.empty((c.N * c.OH * c.OW, c.OC), dtype=torch.int32, device=dev)
    qo = torch.empty((y.shape[0], c.OC // 2), dtype=torch.uint8, device=dev)
    wsc = torch.empty(q4.conv2d_workspace_bytes(d), dtype=torch.uint8, device=dev)

    def conv_step():
        q4.q4_conv2d_im2col(d, x, c.zx, w, c.zw, out=y, workspace=wsc)
        q4.q4_requant(y, c.mult, c.shift, c.zo, out=qo)

    ms = _time_ms(conv_step, torch)
    ex["cfg3_conv_requant_us"] = round(ms * 1e3, 2)
    ms_f = _time_ms(lambda: q4.q4_conv2d_requant(d, x, c.zx, w, c.zw, c.mult, c.shift, c.zo, out=qo, workspace=wsc), torch)
    ex["cfg3_conv_requant_fused_us"] = round(ms_f * 1e3, 2)
    ex["cfg3_tops"] = round(2.0 * y.shape[0] * c.OC * c.depth / (ms * 1e-3) / 1e12, 3)

    # config 4: OCR-style CNN, batch 64
    case = wl.config4()
    act0 = flat_pack(case.x_codes)
    weights = [q4.q4_pack(torch.from_numpy(L.w_codes.reshape(L.cout, -1)).to(dev)) for L in case.layers]
    # per-layer weight sums are part of the stored layer (computed once, Sec. 3.2 of the paper)
    wsums = [q4.q4_rowsum(wt, 9 * L.cin) for L, wt in zip(case.layers, weights)]

    def cnn_step(fused=False):
        act, zx, cin, H, W = act0, case.zx, 1, case.H, case.W
        for L, wt, ws_ in zip(case.layers, weights, wsums):
            dd = q4.conv_desc(case.batch, H, W, cin, 3, 3, (1, 1), (case.pad, case.pad), L.cout)
            H, W = q4.conv_out_hw(dd)
            if fused and L.pool_after:
                act = q4.q4_conv2d_requant_pool2x2(dd, act, zx, wt, L.zw, L.mult, L.shift, L.zo, w_colsum=ws_)
                zx, cin = L.zo, L.cout
                H, W = H // 2, W // 2
                continue
            if fused:
                act = q4.q4_conv2d_requant(dd, act, zx, wt, L.zw, L.mult, L.shift, L.zo, w_colsum=ws_).reshape(-1)
            else:
                yy = q4.q4_conv2d_im2col(dd, act, zx, wt, L.zw, w_colsum=ws_)
                act = q4.q4_requant(yy, L.mult, L.shift, L.zo).reshape(-1)
            zx, cin = L.zo, L.cout
            if L.pool_after:
                act = q4.q4_maxpool2x2(act, case.batch, H, W, cin)
                H, W = H // 2, W // 2
        return act

    ms = _time_ms(cnn_step, torch, reps=10)
    ex["cfg4_cnn_forward_ms"] = round(ms, 4)
    ex["cfg4_images_per_s"] = round(case.batch / (ms * 1e-3), 1)
    ms = _time_ms(lambda: cnn_step(fused=True), torch, reps=10)
    ex["cfg4_cnn_forward_fused_requant_ms"] = round(ms, 4)
    ex["cfg4_images_per_s_fused_requant"] = round(case.batch / (ms * 1e-3), 1)
    return ex


if __name__ == "__main__":
    main()
