#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One "step" = one adaptation step of Algorithm 1 over one synthetic batch of the WideResNet-28-10 workload
(batch 200, fp32, 28 convolutions): the extra importance pass at the static ratio 0.9 (select + pack, dW from
packed, Gradient Importance for every layer), the ratio rule of Eq. 5-7 on the host, then the adaptation pass
(select + pack at the per-layer ratios, dW from packed).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is dense activation bytes pushed through the whole step per second;
`roofline` is for the dominant kernel (the MFMA weight-gradient kernel, which serves every layer with more than
17 - 22 % of its elements kept), timed with HIP events inside the library on the launching stream; `stages` gives the same
figures for the two HBM-bound kernel classes and for the weight-gradient kernel that works from the kept elements alone
(fp32 3x3 stride-1 layers with at most 17 - 22 % kept: the importance pass and the last stage of the adaptation pass);
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0       # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PEAK_VALU_F32_TFLOPS = 78.6  # non-packed fp32 FMA on the vector ALU
METRIC = "pruned-activation GB/s (select+pack) + packed-dW TFLOP/s, % of MI355X roofline"
WORKLOAD_NAMES = {
    0: "cfg0 single linear 512->256, 64 tokens, fp32, r=0.5",
    1: "cfg1 WideResNet-28-10 conv stack, batch 200, 32x32, fp32, 28 convs, group_len 4096, "
       "importance pass r=0.9 + adaptation pass r_l in [0.3,0.9]",
    2: "cfg2 ResNet-50 conv stack, batch 64, 224x224, bf16, 53 convs, group_len 4096, r_l in [0.5,0.95]",
    3: "cfg3 ViT-B/16 encoder linears, batch 64 x 197 tokens, bf16, 48 linears, group_len = in_features",
    4: "cfg4 segmentation transformer linears, batch 2, 1024x512, bf16, 266 linears, r_l in [0.6,0.95]",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=1, help="workload (default 1 = the configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (used under rocprofv3)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "dw_conv_wrn28_hbm_traffic.txt"),
                    help="text file whose line starting with '{' holds the HBM bytes per launch of the dominant kernel "
                    "(from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs); reported as roofline.traffic")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain elementwise kernel reading and writing 1 GiB, as the known-size reference "
                    "for scaling FETCH_SIZE / WRITE_SIZE under rocprofv3 --pmc")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2503_20354_amd as surgeon
    import surgeon_workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    surgeon.load_library()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = args.cfg
    layers = wl.config_layers(cfg)
    dtype = layers[0].dtype
    dt = surgeon.F32 if dtype == "f32" else surgeon.BF16
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    r_lo, r_hi = wl.RATIO_RANGE[cfg]
    r_imp = wl.IMPORTANCE_PASS_RATIO if cfg else 0.5

    # ---- resident inputs and pre-sized outputs (nothing is allocated inside the timed region)
    st = []
    ws_bytes = 16
    for li, L in enumerate(layers):
        A, dY = wl.layer_tensors(cfg, li, L, device=dev)
        e = {"L": L, "A": A, "dY": dY,
             "vals": torch.empty(L.n, dtype=tdt, device=dev),
             "mask": torch.empty((L.n + 63) // 64, dtype=torch.int64, device=dev),
             "dW": torch.empty(L.dw_shape, dtype=torch.float32, device=dev)}
        if L.kind == "linear":
            e["desc"] = surgeon.linear_desc(L.M, L.K, L.N, dt, 0)
        else:
            e["desc"] = surgeon.conv2d_desc(L.Nb, L.Ci, L.H, L.W, L.Co, L.kh, L.kw, L.stride, L.pad, dt, 0)
        ws_bytes = max(ws_bytes, surgeon.surgeon_dw_ws_bytes(e["desc"]), surgeon.surgeon_grad_importance_ws_bytes(L.n_w),
                       surgeon.surgeon_packed_sizes(L.n, L.group_len, 0.5, dt)[3])
        st.append(e)
    ws_bytes = max(ws_bytes, surgeon.surgeon_grad_importance_batched_ws_bytes([e["dW"] for e in st]))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    G_dev = torch.zeros(len(layers), dtype=torch.float32, device=dev)
    G_host = torch.zeros(len(layers), dtype=torch.float32).pin_memory()
    m_bytes = [L.n * L.elem_bytes for L in layers]
    acct = {"sp_bytes": 0.0, "dw_flops": 0.0, "imp_bytes": 0.0, "nnz_flops": 0.0,
            "sparse_dense_flops": 0.0, "sparse_nnz_flops": 0.0}

    def forward_half(ratios, count):
        for e, r in zip(st, ratios):
            L = e["L"]
            k = surgeon.surgeon_packed_sizes(L.n, L.group_len, r, dt)[0]
            e["desc"].k_total = k
            e["desc"].group_len, e["desc"].r = L.group_len, r
            surgeon.surgeon_prune_pack(e["A"], L.group_len, r, e["vals"], e["mask"], None, ws)
            if count:
                acct["sp_bytes"] += L.n * L.elem_bytes + k * L.elem_bytes + 8 * ((L.n + 63) // 64)
                # flops go to the kernel class the library will use for this (shape, kept count); asked once per pair
                cls = e.setdefault("cls", {})
                if k not in cls:
                    cls[k] = surgeon.surgeon_dw_kernel_class(e["desc"])
                if cls[k] == "dw_sparse":
                    acct["sparse_dense_flops"] += L.dense_flops
                    acct["sparse_nnz_flops"] += L.dense_flops * (k / L.n)
                else:
                    acct["dw_flops"] += L.dense_flops
                    acct["nnz_flops"] += L.dense_flops * (k / L.n)

    dW_list = [e["dW"] for e in st]

    def backward_half(with_importance, count):
        for li in range(len(st) - 1, -1, -1):
            e = st[li]
            surgeon.surgeon_dw_from_packed(e["desc"], e["vals"], e["mask"], e["dY"], e["dW"], ws)
        if with_importance:  # Eq. 4 for every layer in one call, once all weight gradients of the pass exist
            surgeon.surgeon_grad_importance_batched(dW_list, G_dev, ws)
            if count:
                acct["imp_bytes"] += 4 * sum(e["L"].n_w for e in st)

    def step(count=False):
        # extra forward-backward at a static ratio to obtain the layer importances (Alg. 1 line 2)
        forward_half([r_imp] * len(st), count)
        backward_half(True, count)
        G_host.copy_(G_dev, non_blocking=False)  # the only device->host transfer of the step: l floats
        if cfg == 0:
            ratios = [0.5]
        else:
            ratios = surgeon.surgeon_layer_ratios(G_host, m_bytes, r_lo, r_hi).tolist()
        # adaptation pass (Alg. 1 lines 3-13) at the per-layer ratios
        forward_half(ratios, count)
        backward_half(False, count)
        return ratios

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB read + 1 GiB written by one add kernel
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    surgeon.surgeon_profile_begin()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ratios = step(count=True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = surgeon.surgeon_profile_end()
    sec = t1 - t0
    ms_per_step = 1e3 * sec / args.steps
    act_bytes_per_step = float(sum(m_bytes))

    def rate(work, ms):
        return work / (ms * 1e-3) if ms > 0 else 0.0

    dw_ms, dw_n = prof["dw"]
    sp_ms, sp_n = prof["select_pack"]
    imp_ms, imp_n = prof["importance"]
    dws_ms, dws_n = prof["dw_sparse"]
    dw_tflops = rate(acct["dw_flops"], dw_ms) / 1e12
    sp_gbps = rate(acct["sp_bytes"], sp_ms) / 1e9
    imp_gbps = rate(acct["imp_bytes"], imp_ms) / 1e9
    traffic = None
    if cfg == 1 and args.traffic_file and os.path.exists(args.traffic_file):
        for line in open(args.traffic_file):
            if line.startswith("{"):
                traffic = json.loads(line).get("dw_hbm_bytes_per_launch")
    peak = PEAK_MFMA_TFLOPS[dtype]
    out = {
        "metric": METRIC, "value": round(act_bytes_per_step * args.steps / sec / 1e9, 3), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": WORKLOAD_NAMES[cfg], "layers": len(layers),
                   "activation_bytes_per_step": int(act_bytes_per_step),
                   "ratios_min_max": [round(min(ratios), 4), round(max(ratios), 4)]},
        "roofline": {"kernel": "dw_conv_kernel" if layers[0].kind == "conv2d" else "dw_linear_kernel",
                     "bound": "mfma", "achieved": round(dw_tflops, 3), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(dw_tflops / peak, 4), "traffic": traffic,
                     "launches": int(dw_n), "avg_launch_ms": round(dw_ms / max(dw_n, 1), 5),
                     "flops_per_launch": acct["dw_flops"] / max(dw_n, 1),
                     "nonzero_tflops": round(rate(acct["nnz_flops"], dw_ms) / 1e12, 3)},
        "stages": {
            "select_pack": {"bound": "hbm", "achieved": round(sp_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": round(sp_gbps / PEAK_HBM_GBPS, 4), "launches": int(sp_n),
                            "avg_launch_ms": round(sp_ms / max(sp_n, 1), 5), "ms_per_step": round(sp_ms / args.steps, 4)},
            "importance": {"bound": "hbm", "achieved": round(imp_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                           "frac": round(imp_gbps / PEAK_HBM_GBPS, 4), "launches": int(imp_n),
                           "avg_launch_ms": round(imp_ms / max(imp_n, 1), 5), "ms_per_step": round(imp_ms / args.steps, 4)},
            "dw": {"ms_per_step": round(dw_ms / args.steps, 4), "tflops_dense_equiv": round(dw_tflops, 3)},
            # layers with few kept elements (fp32 3x3 stride 1, <= 17 - 22 % kept): the sum of Eq. 2 over the kept elements
            # only, on the vector ALU; achieved = multiply-adds actually done, peak = fp32 vector FMA rate (256 CUs x
            # 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz; packed fp32 is disabled in this build)
            "dw_sparse": {"bound": "alu", "achieved": round(rate(acct["sparse_nnz_flops"], dws_ms) / 1e12, 3),
                          "peak": PEAK_VALU_F32_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(rate(acct["sparse_nnz_flops"], dws_ms) / 1e12 / PEAK_VALU_F32_TFLOPS, 4),
                          "launches": int(dws_n), "avg_launch_ms": round(dws_ms / max(dws_n, 1), 5),
                          "ms_per_step": round(dws_ms / args.steps, 4),
                          "tflops_dense_equiv": round(rate(acct["sparse_dense_flops"], dws_ms) / 1e12, 3)},
            "dw_aux": {"ms_per_step": round(prof["dw_aux"][0] / args.steps, 4), "launches": int(prof["dw_aux"][1])},
            "select_other": {"ms_per_step": round(prof["select_other"][0] / args.steps, 4)},
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl)
    print(json.dumps(out))


def cpu_baseline(cfg, wl):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: every layer of the config at a
    reduced batch, one full step (importance pass, ratio rule, adaptation pass)."""
    import numpy as np

    import oracle

    layers = wl.config_layers(cfg)
    div = {0: 1, 1: 8, 2: 64, 3: 197, 4: 64}[cfg]  # sized for roughly 10-30 s of CPU work on a 16-core host
    sample = [wl.shrink(L, div) for L in layers]
    tensors = [tuple(wl.to_numpy_bits(t) for t in wl.layer_tensors(cfg, li, L)) for li, L in enumerate(sample)]
    r_lo, r_hi = wl.RATIO_RANGE[cfg]
    r_imp = wl.IMPORTANCE_PASS_RATIO if cfg else 0.5

    def dw(L, vals, mask, dY):
        if L.kind == "linear":
            return oracle.dw_linear(vals, mask, dY, L.M, L.K, L.N)
        return oracle.dw_conv2d(vals, mask, dY, L.Nb, L.Ci, L.H, L.W, L.Co, L.kh, L.kw, L.stride, L.pad)

    oracle.lib()
    t0 = time.perf_counter()
    G = []
    for L, (A, dY) in zip(sample, tensors):
        vals, mask, _, _ = oracle.prune_pack(A.reshape(-1), L.group_len, r_imp)
        G.append(oracle.grad_importance(dw(L, vals, mask, dY)))
    m = np.array([L.n * L.elem_bytes for L in sample], np.uint64)
    ratios = oracle.layer_ratios(np.array(G, np.float32), m, r_lo, r_hi) if cfg else [0.5]
    for L, (A, dY), r in zip(sample, tensors, ratios):
        vals, mask, _, _ = oracle.prune_pack(A.reshape(-1), L.group_len, float(r))
        dw(L, vals, mask, dY)
    sec = time.perf_counter() - t0
    act_bytes = float(sum(L.n * L.elem_bytes for L in sample))
    return {"value": round(act_bytes / sec / 1e9, 6), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
            "seconds": round(sec, 2),
            "sample": "one full step of all %d layers at 1/%d of the batch (%.1f MB of activations)" %
                      (len(sample), div, act_bytes / 1e6)}


if __name__ == "__main__":
    main()
