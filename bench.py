#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One "step" = one adaptation step of Algorithm 1 over one synthetic batch of a workload: the extra importance pass
at the static ratio 0.9 (select + pack, then dW from packed with Gradient Importance taken inside the same call, for
every layer), the ratio rule of Eq. 5-7 on the host, then the adaptation pass (select + pack at the per-layer ratios,
dW from packed).  Inputs are resident in HBM before the timed region.

The headline line is the WideResNet-28-10 workload (batch 200, fp32, 28 convolutions).  Prints ONE JSON line:
  value        dense activation bytes pushed through the whole step per second
  roofline     the dominant kernel class (the MFMA weight-gradient kernels): achieved = dense-equivalent flops / the
               time of those kernels PLUS their rank pre-pass, dense copy and split reduction (Alg. 1 lines 11-12 are
               one stage); the matrix kernels alone are given as `kernel_only`
  stages       select+pack and Gradient Importance against 8 TB/s, the kept-elements kernel against the fp32 vector peak
  configs      the same per-stage figures for the other four workloads at full size, timed the same way
  next         the rows built beyond the hot path: activation gradient, gradient step, normalisation-layer gradients,
               grouped convolution, whole-tensor selection
  cpu_baseline the CPU oracle on a bounded sample of the headline workload, all cores and one core
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0       # MI355X HBM3E
PEAK_MFMA_TFLOPS = {"f32": 157.3, "bf16": 2500.0}
PEAK_VALU_F32_TFLOPS = 78.6  # non-packed fp32 FMA on the vector ALU: 256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz
PEAK_LDS_TBPS = 78.6         # LDS data path: 256 compute units x 128 bytes per clock x 2.4 GHz
METRIC = "pruned-activation GB/s (select+pack) + packed-dW TFLOP/s, % of MI355X roofline"
WORKLOAD_NAMES = {
    0: "cfg0 single linear 512->256, 64 tokens, fp32, r=0.5",
    1: "cfg1 WideResNet-28-10 conv stack, batch 200, 32x32, fp32, 28 convs, group_len 4096, "
       "importance pass r=0.9 + adaptation pass r_l in [0.3,0.9]",
    2: "cfg2 ResNet-50 conv stack, batch 64, 224x224, bf16, 53 convs, group_len 4096, r_l in [0.5,0.95]",
    3: "cfg3 ViT-B/16 encoder linears, batch 64 x 197 tokens, bf16, 48 linears, group_len = in_features",
    4: "cfg4 segmentation transformer linears, batch 2, 1024x512, bf16, 266 linears, r_l in [0.6,0.95]",
}


def _rate(work, ms):
    return work / (ms * 1e-3) if ms > 0 else 0.0


def run_config(cfg, steps, warmup, torch, surgeon, wl, dev, plain_steps=0):
    """One workload at full size: resident tensors, `warmup` untimed steps, `steps` timed ones.  Returns the figures."""
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
             "dW": torch.empty(L.dw_shape, dtype=torch.float32, device=dev), "cls": {}}
        if L.kind == "linear":
            e["desc"] = surgeon.linear_desc(L.M, L.K, L.N, dt, 0)
        else:
            e["desc"] = surgeon.conv2d_desc(L.Nb, L.Ci, L.H, L.W, L.Co, L.kh, L.kw, L.stride, L.pad, dt, 0)
        ws_bytes = max(ws_bytes, surgeon.surgeon_dw_gi_ws_bytes(e["desc"]),
                       surgeon.surgeon_packed_sizes(L.n, L.group_len, 0.5, dt)[3])
        st.append(e)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    G_dev = torch.zeros(len(layers), dtype=torch.float32, device=dev)
    G_host = torch.zeros(len(layers), dtype=torch.float32).pin_memory()
    G_slot = [G_dev[i:i + 1] for i in range(len(layers))]
    m_bytes = [L.n * L.elem_bytes for L in layers]
    acct = {"sp_bytes": 0.0, "imp_bytes": 0.0, "dw": 0.0, "dw_nnz": 0.0, "dw_sparse": 0.0, "dw_sparse_nnz": 0.0}

    all_A, all_vals, all_mask = [e["A"] for e in st], [e["vals"] for e in st], [e["mask"] for e in st]
    all_g = [e["L"].group_len for e in st]

    def forward_half(ratios, count):
        # Alg. 1 lines 6-7 for every layer of the pass in one call (all layers select in groups of at most 4096)
        surgeon.surgeon_prune_pack_batched(all_A, all_g, ratios, all_vals, all_mask)
        for e, r in zip(st, ratios):
            L = e["L"]
            k = surgeon.surgeon_packed_sizes(L.n, L.group_len, r, dt)[0]
            e["desc"].k_total = k
            e["desc"].group_len, e["desc"].r = L.group_len, r
            if count:
                acct["sp_bytes"] += L.n * L.elem_bytes + k * L.elem_bytes + 8 * ((L.n + 63) // 64)
                # flops go to the kernel class the library will use for this (shape, kept count); asked once per pair
                if k not in e["cls"]:
                    e["cls"][k] = surgeon.surgeon_dw_kernel_class(e["desc"])
                c = "dw_sparse" if e["cls"][k] == "dw_sparse" else "dw"
                acct[c] += L.dense_flops
                acct[c + "_nnz"] += L.dense_flops * (k / L.n)

    def backward_half(with_importance, count):
        for li in range(len(st) - 1, -1, -1):
            e = st[li]
            if with_importance:  # Eq. 4 inside the weight-gradient call: dW is not read again
                surgeon.surgeon_dw_from_packed_gi(e["desc"], e["vals"], e["mask"], e["dY"], e["dW"], G_slot[li], ws)
            else:
                surgeon.surgeon_dw_from_packed(e["desc"], e["vals"], e["mask"], e["dY"], e["dW"], ws)
        if with_importance and count:
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

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # the same steps without the per-kernel events of the timing aid (each kernel then goes out as a plain launch):
    # what a caller who does not profile sees; matters for workloads of many small kernels
    plain = [torch.cuda.Event(enable_timing=True) for _ in range(plain_steps + 1)]
    if plain_steps:
        plain[0].record()
        for i in range(plain_steps):
            step()
            plain[i + 1].record()
        torch.cuda.synchronize()
    plain_ms = [plain[i].elapsed_time(plain[i + 1]) for i in range(plain_steps)]
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    surgeon.surgeon_profile_begin()
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(steps):
        ratios = step(count=True)
        marks[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = surgeon.surgeon_profile_end()
    sec = t1 - t0
    per_step = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]
    act_bytes = float(sum(m_bytes))
    ms = {k: v[0] for k, v in prof.items()}
    n_launch = {k: int(v[1]) for k, v in prof.items()}
    peak = PEAK_MFMA_TFLOPS[dtype]
    dw_stage_ms = ms["dw"] + ms["dw_aux"] + ms["dw_grouped"]
    dw_tf_kernel = _rate(acct["dw"], ms["dw"]) / 1e12
    dw_tf_stage = _rate(acct["dw"], dw_stage_ms) / 1e12
    sp_gbps = _rate(acct["sp_bytes"], ms["select_pack"] + ms["select_other"]) / 1e9
    imp_gbps = _rate(acct["imp_bytes"], ms["importance"]) / 1e9
    sparse_ms = ms["dw_sparse"] + ms["dw_sparse_aux"]
    res = {
        "workload": WORKLOAD_NAMES[cfg], "dtype": dtype, "layers": len(layers), "steps": steps,
        "ms_per_step": round(1e3 * sec / steps, 4), "ms_per_step_median": round(statistics.median(per_step), 4),
        "ms_per_step_min": round(min(per_step), 4),
        "ms_per_step_without_kernel_events": round(statistics.median(plain_ms), 4) if plain_ms else None,
        "value_GBps": round(act_bytes * steps / sec / 1e9, 3), "activation_bytes_per_step": int(act_bytes),
        "ratios_min_max": [round(min(ratios), 4), round(max(ratios), 4)],
        "roofline": {"kernel": "dw_conv_kernel" if layers[0].kind == "conv2d" else "dw_linear_bf16_big_kernel / dw_linear_kernel",
                     "bound": "mfma", "achieved": round(dw_tf_stage, 3), "peak": peak, "unit": "TFLOP/s",
                     "frac": round(dw_tf_stage / peak, 4),
                     "what": "dense-equivalent flops / (matrix kernels + rank pre-pass + dense copy + split reduction)",
                     "kernel_only": {"achieved": round(dw_tf_kernel, 3), "frac": round(dw_tf_kernel / peak, 4),
                                     "launches": n_launch["dw"], "avg_launch_ms": round(ms["dw"] / max(n_launch["dw"], 1), 5),
                                     "flops_per_launch": acct["dw"] / max(n_launch["dw"], 1)},
                     "aux_ms_per_step": round(ms["dw_aux"] / steps, 4), "aux_launches": n_launch["dw_aux"],
                     "nonzero_tflops": round(_rate(acct["dw_nnz"], dw_stage_ms) / 1e12, 3)},
        "stages": {
            "select_pack": {"bound": "hbm", "achieved": round(sp_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": round(sp_gbps / PEAK_HBM_GBPS, 4), "launches": n_launch["select_pack"] + n_launch["select_other"],
                            "ms_per_step": round((ms["select_pack"] + ms["select_other"]) / steps, 4)},
            # Eq. 4 rides on the split reduction of the weight gradient; what is left as its own kernels is the finishing
            # launch per layer (and a read of dW for the few layers whose contraction is not split)
            "importance": {"bound": "hbm", "achieved": round(imp_gbps, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                           "frac": round(imp_gbps / PEAK_HBM_GBPS, 4), "launches": n_launch["importance"],
                           "ms_per_step": round(ms["importance"] / steps, 4), "fused_into": "dw split reduction",
                           "note": "no read of dW is left: the time is one finishing launch per layer; achieved = 4*N_w over "
                                   "that time (the stand-alone kernel's HBM rate is next.grad_importance_batched)"},
            "dw": {"ms_per_step": round(dw_stage_ms / steps, 4), "tflops_dense_equiv": round(dw_tf_stage, 3)},
            # layers with few kept elements (fp32 3x3 stride 1, <= 17 - 22 % kept): the sum of Eq. 2 over the kept elements
            # only, on the vector ALU; achieved = multiply-adds actually done (with the kernel's own pre-pass and reduction)
            "dw_sparse": {"bound": "alu", "achieved": round(_rate(acct["dw_sparse_nnz"], sparse_ms) / 1e12, 3),
                          "peak": PEAK_VALU_F32_TFLOPS, "unit": "TFLOP/s",
                          "frac": round(_rate(acct["dw_sparse_nnz"], sparse_ms) / 1e12 / PEAK_VALU_F32_TFLOPS, 4),
                          "launches": n_launch["dw_sparse"], "ms_per_step": round(sparse_ms / steps, 4),
                          "kernel_only_ms_per_step": round(ms["dw_sparse"] / steps, 4),
                          "tflops_dense_equiv": round(_rate(acct["dw_sparse"], sparse_ms) / 1e12, 3),
                          # every multiply-add of this kernel takes its dY operand from LDS (4 bytes per lane): the LDS
                          # data path (128 bytes per clock and compute unit) is the unit it fills first
                          "lds": {"achieved": round(_rate(acct["dw_sparse_nnz"] / 2 * 4, ms["dw_sparse"]) / 1e12, 2),
                                  "peak": PEAK_LDS_TBPS, "unit": "TB/s",
                                  "frac": round(_rate(acct["dw_sparse_nnz"] / 2 * 4, ms["dw_sparse"]) / 1e12 / PEAK_LDS_TBPS, 4)}},
        },
    }
    extras = {"st": st, "ws": ws, "layers": layers, "dt": dt, "tdt": tdt}
    return res, extras


def next_rows(extras, torch, surgeon, wl, dev, cfg):
    """The rows built beyond the hot path, on the headline workload's shapes: each timed by the library's own events."""
    st, layers, dt, tdt = extras["st"], extras["layers"], extras["dt"], extras["tdt"]
    out = {}
    es = layers[0].elem_bytes
    reps = 3

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        surgeon.surgeon_profile_begin()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return {k: (v[0] / reps, v[1] // reps) for k, v in surgeon.surgeon_profile_end().items()}

    # activation gradient dA = dY . W for every layer (Eq. 2, first line)
    Ws = [(wl.draw(e["L"].dw_shape, "normal", e["L"].dtype, 4242 + i, device=dev) * 0.05).to(tdt) for i, e in enumerate(st)]
    dA = torch.empty(max(e["L"].n for e in st), dtype=tdt, device=dev)

    def run_da():
        for e, W in zip(st, Ws):
            surgeon.surgeon_da(e["desc"], e["dY"], W, dA[:e["L"].n])
    p = timed(run_da)
    flops = float(sum(e["L"].dense_flops for e in st))
    tf = _rate(flops, p["da"][0]) / 1e12
    out["da"] = {"bound": "mfma", "achieved": round(tf, 3), "peak": PEAK_MFMA_TFLOPS["f32"], "unit": "TFLOP/s",
                 "frac": round(tf / PEAK_MFMA_TFLOPS["f32"], 4), "ms": round(p["da"][0], 4), "launches": p["da"][1],
                 "note": "fp32 matrix cores for both dtypes (bf16 widened while staging): band kernel for 3x3 stride 1, "
                         "cell kernel for 3x3 stride 2, gathering kernel for the rest"}

    # the same gradient for bf16 1x1 convolutions on the bf16 matrix cores, on four ResNet-50 layer shapes at batch 64
    rows, t_ms, fl = [], 0.0, 0.0
    for name, (Ci, HWm, Co, stride) in {"c256_14_c1024": (256, 14, 1024, 1), "c64_56_c256": (64, 56, 256, 1),
                                        "c512_7_c2048": (512, 7, 2048, 1), "c1024_14_c2048_s2": (1024, 14, 2048, 2)}.items():
        OHm = (HWm - 1) // stride + 1
        dYb = wl.draw((64, Co, OHm, OHm), "normal", "bf16", 87, device=dev)
        Wb = (wl.draw((Co, Ci, 1, 1), "normal", "bf16", 88, device=dev) * 0.05).to(torch.bfloat16)
        dAb = torch.empty((64, Ci, HWm, HWm), dtype=torch.bfloat16, device=dev)
        d = surgeon.conv2d_desc(64, Ci, HWm, HWm, Co, 1, 1, stride, 0, surgeon.BF16, 0)
        p = timed(lambda: surgeon.surgeon_da(d, dYb, Wb, dAb))
        t_ms += p["da"][0]
        fl += 2.0 * 64 * OHm * OHm * Ci * Co
        rows.append((name, round(p["da"][0] * 1e3, 1)))
        del dYb, Wb, dAb
    tf = _rate(fl, t_ms) / 1e12
    out["da_bf16_conv1x1"] = {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_MFMA_TFLOPS["bf16"], "unit": "TFLOP/s",
                              "frac": round(tf / PEAK_MFMA_TFLOPS["bf16"], 4), "ms": round(t_ms, 4),
                              "us_per_layer": dict(rows), "what": "one launch per layer, bf16 results stored by the kernel"}

    # the same gradient for bf16 linear layers on the bf16 matrix cores (workspace entry), on the four layer shapes of a
    # ViT-B/16 block at 12 608 tokens
    rows, t_ms, fl = [], 0.0, 0.0
    rows_plain, t_plain = [], 0.0
    for name, (M, K, N) in {"qkv": (12608, 768, 2304), "proj": (12608, 768, 768), "fc1": (12608, 768, 3072),
                            "fc2": (12608, 3072, 768)}.items():
        dYb = wl.draw((M, N), "normal", "bf16", 77, device=dev)
        Wb = (wl.draw((N, K), "normal", "bf16", 78, device=dev) * 0.05).to(torch.bfloat16)
        dAb = torch.empty((M, K), dtype=torch.bfloat16, device=dev)
        d = surgeon.linear_desc(M, K, N, surgeon.BF16, 0)
        wsb = torch.empty(surgeon.surgeon_da_ws_bytes(d), dtype=torch.uint8, device=dev)
        p = timed(lambda: surgeon.surgeon_da_ws(d, dYb, Wb, dAb, wsb))
        t_ms += p["da"][0]
        fl += 2.0 * M * K * N
        rows.append((name, round(p["da"][0] * 1e3, 1)))
        p = timed(lambda: surgeon.surgeon_da(d, dYb, Wb, dAb))  # no workspace: dY read in place
        t_plain += p["da"][0]
        rows_plain.append((name, round(p["da"][0] * 1e3, 1)))
        del dYb, Wb, dAb, wsb
    tf = _rate(fl, t_ms) / 1e12
    out["da_bf16_linear"] = {"bound": "mfma", "achieved": round(tf, 1), "peak": PEAK_MFMA_TFLOPS["bf16"], "unit": "TFLOP/s",
                             "frac": round(tf / PEAK_MFMA_TFLOPS["bf16"], 4), "ms": round(t_ms, 4),
                             "us_per_layer": dict(rows), "what": "transpose of dY + contraction; the kernel stores bf16 itself when one split suffices",
                             "without_workspace": {"achieved": round(_rate(fl, t_plain) / 1e12, 1), "ms": round(t_plain, 4),
                                                   "us_per_layer": dict(rows_plain), "what": "surgeon_da: dY read in place"}}

    # Eq. 4 as a call of its own over every layer's dW (the path above computes it inside the weight-gradient call and
    # never reads dW again; this is the stand-alone, HBM-bound kernel for callers that have dW from elsewhere)
    dWs = [e["dW"].reshape(-1) for e in st]
    G_all = torch.empty(len(st), device=dev)
    ws_gi = torch.empty(max(surgeon.surgeon_grad_importance_batched_ws_bytes(dWs), 16), dtype=torch.uint8, device=dev)
    p = timed(lambda: surgeon.surgeon_grad_importance_batched(dWs, G_all, ws_gi))
    gb = _rate(4.0 * sum(e["L"].n_w for e in st), p["importance"][0]) / 1e9
    out["grad_importance_batched"] = {"bound": "hbm", "achieved": round(gb, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                      "frac": round(gb / PEAK_HBM_GBPS, 4), "ms": round(p["importance"][0], 4),
                                      "launches": p["importance"][1]}

    # gradient step W <- W - lr dW (Alg. 1 line 14)
    def run_update():  # all layers in one call (at most 64 tensors per launch)
        surgeon.surgeon_weight_update_batched(Ws, [e["dW"].reshape(-1) for e in st], 1e-4)
    p = timed(run_update)
    nbytes = float(sum(e["L"].n_w * (2 * es + 4) for e in st))
    gb = _rate(nbytes, p["update"][0]) / 1e9
    out["weight_update"] = {"bound": "hbm", "achieved": round(gb, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                            "frac": round(gb / PEAK_HBM_GBPS, 4), "ms": round(p["update"][0], 4), "launches": p["update"][1]}

    # scale / shift gradients of normalisation layers on the distinct activation shapes (batch norm for conv stacks,
    # layer norm for token matrices), from the packed activation of the importance pass
    seen, tot_ms, tot_bytes, n_l, n_shapes = set(), 0.0, 0.0, 0, 0
    r = wl.IMPORTANCE_PASS_RATIO if cfg else 0.5
    for e in st:
        L = e["L"]
        if L.a_shape in seen:
            continue
        seen.add(L.a_shape)
        outer, C, inner = (L.M, L.K, 1) if L.kind == "linear" else (L.Nb, L.Ci, L.H * L.W)
        k = surgeon.surgeon_packed_sizes(L.n, L.group_len, r, dt)[0]
        surgeon.surgeon_prune_pack(e["A"], L.group_len, r, e["vals"], e["mask"], None, extras["ws"])
        dYn = wl.draw(L.a_shape, "normal", L.dtype, 99, device=dev)
        dg, db = torch.empty(C, device=dev), torch.empty(C, device=dev)
        wsa = torch.empty(surgeon.surgeon_affine_grad_ws_bytes(outer, C, inner), dtype=torch.uint8, device=dev)
        p = timed(lambda: surgeon.surgeon_affine_grad(e["vals"], e["mask"], dYn, outer, C, inner, k, dg, db, wsa))
        tot_ms += p["affine"][0]
        n_l += p["affine"][1]
        n_shapes += 1
        tot_bytes += k * es + 8 * ((L.n + 63) // 64) + L.n * es
        del dYn, wsa
    gb = _rate(tot_bytes, tot_ms) / 1e9
    out["affine_grad"] = {"bound": "hbm", "achieved": round(gb, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                          "frac": round(gb / PEAK_HBM_GBPS, 4), "ms": round(tot_ms, 4), "launches": n_l,
                          "shapes": n_shapes, "bytes": "k*s + n/8 + n*s (dY) per layer; time includes the rank pre-pass"}

    # grouped 3x3 convolution of a ResNeXt-29-shaped stage (32 groups) and a depthwise 3x3, batch 200 / 2
    g_out = {}
    for name, (Nb, C, HW, Co, groups) in {"resnext_3x3_g32": (200, 256, 16, 256, 32), "depthwise_3x3": (2, 1280, 64, 1280, 1280)}.items():
        A = wl.draw((Nb, C, HW, HW), "relu", layers[0].dtype, 7, device=dev)
        dYg = wl.draw((Nb, Co, HW, HW), "normal", layers[0].dtype, 8, device=dev)
        pk = surgeon.prune_pack(A, 4096, 0.7)
        d = surgeon.conv2d_desc(Nb, C, HW, HW, Co, 3, 3, 1, 1, dt, pk.k_total, 4096, 0.7, groups=groups)
        dWg = torch.empty((Co, C // groups, 3, 3), device=dev)
        wsg = torch.empty(surgeon.surgeon_dw_ws_bytes(d), dtype=torch.uint8, device=dev)
        p = timed(lambda: surgeon.surgeon_dw_from_packed(d, pk.vals, pk.mask, dYg, dWg, wsg))
        fl = 2.0 * Nb * HW * HW * Co * (C // groups) * 9
        t_ms = p["dw_grouped"][0] + p["dw_aux"][0]
        g_out[name] = {"ms": round(t_ms, 4), "tflops_dense_equiv": round(_rate(fl, t_ms) / 1e12, 3),
                       "frac_of_fp32_vector_peak": round(_rate(fl, t_ms) / 1e12 / PEAK_VALU_F32_TFLOPS, 4)}
        if groups == C:
            # nine multiply-adds per pixel: bound by the bytes of the packed activation and dY, not by the vector ALU
            nb = pk.k_total * es + 8 * ((A.numel() + 63) // 64) + dYg.numel() * es
            g_out[name].update({"hbm_gbps": round(_rate(nb, t_ms) / 1e9, 1), "frac_of_hbm": round(_rate(nb, t_ms) / 1e9 / PEAK_HBM_GBPS, 4)})
    out["dw_grouped"] = dict(bound="alu", peak=PEAK_VALU_F32_TFLOPS, unit="TFLOP/s", **g_out)

    # what the memory pattern of the fused select+pack kernel reaches without the selection (a fixed threshold instead of
    # the search): every layer of the workload that is packed in 4096-element groups, the same bytes counted
    thr_bits = int(torch.tensor(0.35, dtype=tdt).view(torch.int32 if es == 4 else torch.int16).item())
    probe = [e for e in st if e["L"].n % 4096 == 0]
    if probe:
        kcap = 4096
        big = torch.cat([e["A"].reshape(-1) for e in probe])  # one launch, as the batched call packs a pass in one or two
        pv = torch.empty(big.numel(), dtype=tdt, device=dev)
        pm = torch.empty(big.numel() // 64, dtype=torch.int64, device=dev)
        p = timed(lambda: surgeon.surgeon_select_pack_pattern_probe(big, thr_bits, kcap, pv, pm))
        kept = int((big.abs() >= 0.35).sum().item())
        nb = big.numel() * (es + 1.0 / 8.0) + kept * es
        gb = _rate(nb, p["select_other"][0]) / 1e9
        out["select_pack_pattern_probe"] = {"bound": "hbm", "achieved": round(gb, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                            "frac": round(gb / PEAK_HBM_GBPS, 4), "ms": round(p["select_other"][0], 4),
                                            "launches": p["select_other"][1], "kept_fraction": round(kept / big.numel(), 3),
                                            "what": "loads, ballot / prefix-rank compaction, stores and mask words of select+pack with a "
                                                    "fixed threshold: the rate the memory system gives this access pattern"}
        del pv, pm, big

    # selection over the whole tensor (group_len = n), the paper-literal scope: reported against 2*n*s + outputs
    e = max(st, key=lambda x: x["L"].n)
    L = e["L"]
    r = 0.5
    k, _, _, wsb = surgeon.surgeon_packed_sizes(L.n, L.n, r, dt)
    wsg = torch.empty(max(wsb, 16), dtype=torch.uint8, device=dev)
    p = timed(lambda: surgeon.surgeon_prune_pack(e["A"], L.n, r, e["vals"], e["mask"], None, wsg))
    t_ms = p["select_other"][0] + p["select_pack"][0]
    nbytes = 2.0 * L.n * es + k * es + 8 * ((L.n + 63) // 64)
    gb = _rate(nbytes, t_ms) / 1e9
    out["whole_tensor_select"] = {"bound": "hbm", "achieved": round(gb, 1), "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                  "frac": round(gb / PEAK_HBM_GBPS, 4), "ms": round(t_ms, 4), "n": L.n, "r": r,
                                  "bytes": "2*n*s + k*s + n/8", "launches": p["select_other"][1] + p["select_pack"][1]}
    return out


def stored_traffic():
    """HBM bytes per launch of the dominant kernel from the stored rocprofv3 counter summary, with the library commit
    the summary was taken on (written by profile_summary.py; compare with `library` to see whether it is stale)."""
    path = os.path.join(ROOT, "profiles", "dw_conv_wrn28_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        if line.startswith("{"):
            d = json.loads(line)
            return d.get("dw_hbm_bytes_per_launch"), d.get("library_commit")
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=1, help="headline workload (default 1 = the configuration the metric is quoted on)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (used under rocprofv3)")
    ap.add_argument("--only-headline", action="store_true", help="skip the other workloads and the extra rows")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the other workloads, keep the extra rows")
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
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB read + 1 GiB written by one add kernel
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    head, extras = run_config(args.cfg, args.steps, args.warmup, torch, surgeon, wl, dev, plain_steps=3)
    traffic, traffic_commit = stored_traffic() if args.cfg == 1 else (None, None)
    build_info = {}
    try:
        build_info = json.load(open(os.path.join(ROOT, "paper_2503_20354_amd", "build_info.json")))
    except Exception:
        pass
    head["roofline"]["traffic"] = traffic
    head["roofline"]["traffic_from_library_commit"] = traffic_commit
    out = {
        "metric": METRIC, "value": head["value_GBps"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "ms_per_step_median": head["ms_per_step_median"],
        "ms_per_step_min": head["ms_per_step_min"],
        "ms_per_step_without_kernel_events": head["ms_per_step_without_kernel_events"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic", "library": build_info,
        "config": {"workload": head["workload"], "layers": head["layers"],
                   "activation_bytes_per_step": head["activation_bytes_per_step"], "ratios_min_max": head["ratios_min_max"]},
        "roofline": head["roofline"], "stages": head["stages"],
    }
    if not args.only_headline:
        out["next"] = next_rows(extras, torch, surgeon, wl, dev, args.cfg)
    del extras
    torch.cuda.empty_cache()
    if not args.only_headline and not args.no_other_configs:
        out["configs"] = {}
        for cfg in (0, 2, 3, 4):
            if cfg == args.cfg:
                continue
            res, ex = run_config(cfg, 3, 1, torch, surgeon, wl, dev, plain_steps=3)
            del ex
            torch.cuda.empty_cache()
            out["configs"]["cfg%d" % cfg] = res
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.cfg, wl)
    print(json.dumps(out))


def cpu_baseline(cfg, wl):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: every layer of the config at a
    reduced batch, one full step (importance pass, ratio rule, adaptation pass); once on all cores, once on one."""
    import ctypes

    import numpy as np

    import oracle

    layers = wl.config_layers(cfg)
    r_lo, r_hi = wl.RATIO_RANGE[cfg]
    r_imp = wl.IMPORTANCE_PASS_RATIO if cfg else 0.5

    def dw(L, vals, mask, dY):
        if L.kind == "linear":
            return oracle.dw_linear(vals, mask, dY, L.M, L.K, L.N)
        return oracle.dw_conv2d(vals, mask, dY, L.Nb, L.Ci, L.H, L.W, L.Co, L.kh, L.kw, L.stride, L.pad)

    def one_step(div):
        sample = [wl.shrink(L, div) for L in layers]
        tensors = [tuple(wl.to_numpy_bits(t) for t in wl.layer_tensors(cfg, li, L)) for li, L in enumerate(sample)]
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
        return float(sum(L.n * L.elem_bytes for L in sample)), sec

    oracle.lib()
    div_all = {0: 1, 1: 8, 2: 64, 3: 197, 4: 64}[cfg]   # sized for roughly 10-20 s of CPU work on a 16-core host
    div_one = {0: 1, 1: 100, 2: 64, 3: 197, 4: 64}[cfg]  # and a smaller one for the single-thread run
    cores = oracle.threads()
    act_bytes, sec = one_step(div_all)
    res = {"value": round(act_bytes / sec / 1e9, 6), "unit": "GB/s", "cores": cores, "kind": "oracle", "seconds": round(sec, 2),
           "sample": "one full step of all %d layers at 1/%d of the batch (%.1f MB of activations)" %
                     (len(layers), div_all, act_bytes / 1e6)}
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        act1, sec1 = one_step(div_one)
        gomp.omp_set_num_threads(cores)
        res["single_thread"] = {"value": round(act1 / sec1 / 1e9, 6), "unit": "GB/s", "cores": 1, "seconds": round(sec1, 2),
                                "sample": "the same step at 1/%d of the batch (%.1f MB of activations)" % (div_one, act1 / 1e6)}
    except OSError:
        pass
    return res


if __name__ == "__main__":
    main()
