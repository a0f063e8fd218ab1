#!/usr/bin/env python3
"""Benchmark of the HAP per-device hot path on one MI355X.

One step = one pass of the path over one batch of synthetic input:
  host   LP sharding ratios + integer rounding for the workload's device speeds,
  device fwd + bwd of the largest and the smallest shard of the GPT-style MLP block
         (hidden 4096, ffn 16384 sharded over 3 virtual devices with speeds 1 / 0.6 / 0.35, 8192 tokens, bf16),
         and the sufficient-factor rebuild of dW1[4096 x 16384] from 8 devices' gathered factors
         (token counts 512,512,384,384,256,256,128,128).
Value = algorithmic TFLOP/s of the whole step (2*M*N*K per GEMM over valid rows / columns only).
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--moe-only", action="store_true", help="only run the MoE expert rows (profiling aid)")
    ap.add_argument("--main-only", action="store_true",
                    help="timed step and roofline only: no ceilings, other_rows, cost_model or cpu_baseline (profiling aid)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy 10 times (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (each virtual device's shard runs in turn on it); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import hapgen
    from hapgen import TensorId as T
    import paper_2401_05965_amd as hap
    from paper_2401_05965_amd.programs import EncoderLayerProgram, MlpShard, MoeExpertShard, SfbRebuild

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        src = torch.ones((1 << 26,), dtype=torch.float32, device=dev); dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_each_way": src.numel() * 4, "launches": 10}))
        return

    def dev_bf16(seed, tid, shape, sigma):
        _, bits = hapgen.normal_bf16(seed, tid, shape, sigma)
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev)

    w2 = hapgen.WORKLOADS["cfg2_mlp_bf16"]; w3 = hapgen.WORKLOADS["cfg3_sfb_bf16"]
    Tn, h, F = w2.dims["tokens"], w2.dims["hidden"], w2.dims["ffn"]
    t_setup = time.time()
    X = dev_bf16(0, T.X, (Tn, h), 1.0)
    W1 = dev_bf16(0, T.W, (h, F), 0.02); b1 = dev_bf16(0, T.BIAS, (F,), 0.02)
    W2 = dev_bf16(0, T.W2, (F, h), 0.02)
    dOut = dev_bf16(0, T.DY, (Tn, h), 1.0)
    cap, rows = w3.dims["capacity"], w3.dims["rows"]
    sX = [dev_bf16(0, T.SFB_X + i, (cap, w3.dims["in_features"]), 1.0) for i in range(len(rows))]
    sdY = [dev_bf16(0, T.SFB_DY + i, (cap, w3.dims["out_features"]), 1.0) for i in range(len(rows))]
    t_setup = time.time() - t_setup

    stages = [(1.0, 0.0, 0.0, 0.0)]        # compute-only single stage: the ratios the workload's shard sizes come from

    def host_part():
        ratios, _ = hap.hap_shard_ratios(w2.speeds, stages)
        return hap.hap_round_shards(ratios, F)

    sizes, offsets = host_part()
    assert sizes == [8402, 5041, 2941], sizes
    shards = [MlpShard(Tn, h, F, offsets, j, X, W1, b1, W2, dOut) for j in (0, 2)]
    sfb = SfbRebuild(sX, sdY, rows, w3.dims["in_features"], w3.dims["out_features"])
    del W1, W2
    step_flops = sum(sum(s.flops()) for s in shards) + sfb.flops()

    stream = torch.cuda.current_stream()
    marks = {}
    held = {}      # device results of the untimed rows, kept for the parity leg

    def steady_time(fn, n=10):
        """Seconds per call of fn in steady state.  The GPU drops its clocks while the host prepares inputs and needs tens of
        milliseconds of work to raise them again (the first 20 ms after an idle phase run ~15 % slow), so fn is repeated for
        about 50 ms before the timed repetitions, which cover at least 20 ms."""
        fn(); fn()
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record(stream); fn(); b.record(stream); b.synchronize()
        est = max(a.elapsed_time(b), 0.005)                      # ms
        for _ in range(min(2000, int(50.0 / est) + 1)):
            fn()
        n = max(n, min(2000, int(20.0 / est) + 1))
        a.record(stream)
        for _ in range(n):
            fn()
        b.record(stream); b.synchronize()
        return a.elapsed_time(b) / n * 1e-3

    def timer(label, fn):
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record(stream); fn(); b.record(stream)
        marks.setdefault(label, []).append((a, b))

    def step(tm=None):
        host_part()
        for s in shards:
            s.forward(None if tm is None else (lambda l, f, s=s: tm(f"{l}[f={s.f}]", f)))
            s.backward(None if tm is None else (lambda l, f, s=s: tm(f"{l}[f={s.f}]", f)))
        sfb.run(tm)

    def ceilings():
        """Achievable ceilings measured in this run: MFMA issue rate on register operands, plain copy bandwidth."""
        scratch = torch.empty((256 * 512,), dtype=torch.float32, device=dev)
        res = {}
        # where the roofline's peak comes from: compute units x clock x 4096 bf16 flop per clock and unit (4 SIMDs, each one
        # 32x32x16 MFMA = 32768 flop per 32 clocks), with the unit count and clock this device reports
        units, khz = hap.hap_device_info()
        res["peak_derivation"] = {"compute_units": units, "clock_ghz": round(khz / 1e6, 3), "bf16_flop_per_clock_per_unit": 4096,
                                  "tflops": round(units * khz * 1e3 * 4096 / 1e12, 1)}
        for name, rnd in (("mfma_bf16_constant_operands_tflops", False), ("mfma_bf16_random_operands_tflops", True)):
            for _ in range(20):
                fl = hap.hap_probe_mfma_bf16(rnd, 2000, scratch)
            a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(100):
                fl = hap.hap_probe_mfma_bf16(rnd, 2000, scratch)
            b.record(stream); b.synchronize()
            res[name] = round(fl * 100 / (a.elapsed_time(b) * 1e-3) / 1e12, 1)
        src = torch.ones((1 << 26,), dtype=torch.float32, device=dev); dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(20):
            dst.copy_(src)
        b.record(stream); b.synchronize()
        res["copy_read_plus_write_gbs"] = round(2 * src.numel() * 4 * 20 / (a.elapsed_time(b) * 1e-3) / 1e9, 1)
        del src, dst
        # context only: the vendor library's GEMM (torch.matmul -> hipBLASLt) on the roofline launch's shape and on its
        # bwd-weight counterpart, same box, same run; the product path never calls it
        big = shards[0]
        A = torch.randn((big.T, big.f), device=dev).to(torch.bfloat16); Bm = (torch.randn((big.f, big.h), device=dev) * 0.02).to(torch.bfloat16)
        G = torch.randn((big.T, big.h), device=dev).to(torch.bfloat16)
        for name, fn in (("vendor_gemm_roofline_shape_tflops", lambda: torch.matmul(A, Bm)), ("vendor_gemm_bwd_weight_shape_tflops", lambda: torch.matmul(A.t(), G))):
            for _ in range(3):
                fn()
            a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(10):
                fn()
            b.record(stream); b.synchronize()
            res[name] = round(2.0 * big.T * big.f * big.h * 10 / (a.elapsed_time(b) * 1e-3) / 1e12, 1)
        return res

    def moe_rows(res, timeit):
        """Rows for the unevenly placed MoE experts (Sec. 7.6); also run alone by --moe-only (profiling aid)."""
        # MoE feed-forward layer with 30 experts on 4 devices of speeds (1, 1, .5, .5): the LP + rounding places (10, 10, 5, 5);
        # an even split has to pad to 32 experts, 8 per device.  One device's forward + backward, all expert buffers full.
        wm = hapgen.WORKLOADS["moe_experts_bf16"]
        Em, Cm, Hm, Fm = (wm.dims[k] for k in ("experts", "capacity", "hidden", "ffn"))
        rm, _ = hap.hap_shard_ratios(list(wm.speeds), [(1.0, 0.0, 0.0, 0.0)])
        msizes, moffs = hap.hap_round_shards(rm, Em, 1)
        genm = torch.Generator(device=dev); genm.manual_seed(5)
        rnd = lambda shp, sg: (torch.randn(shp, generator=genm, device=dev) * sg).to(torch.bfloat16)
        nmax = max(max(msizes), (Em + len(msizes) - 1) // len(msizes))
        mX, mdO = rnd((nmax, Cm, Hm), 1.0), rnd((nmax, Cm, Hm), 1.0)
        mW1, mb1, mW2, mb2 = rnd((nmax, Hm, Fm), 0.02), rnd((nmax, Fm), 0.02), rnd((nmax, Fm, Hm), 0.02), rnd((nmax, Hm), 0.02)

        def moe_row(n, rows):
            sh = MoeExpertShard(n, Cm, Hm, Fm, [0, n], 0, mX, mW1, mb1, mW2, mb2, rows, mdO)
            t = timeit(lambda: (sh.forward(), sh.backward()), n=10)
            f, b = sh.flops(None if rows is None else rows[:n].tolist())
            return {"experts": n, "ms": round(t * 1e3, 3), "gflop": round((f + b) / 1e9, 1), "tflops": round((f + b) / t / 1e12, 1)}
        res["moe_expert_placement"] = msizes
        res["moe_ffn_fwd_bwd_device0"] = moe_row(msizes[0], None)
        res["moe_ffn_fwd_bwd_device2"] = moe_row(msizes[2], None)
        res["moe_ffn_fwd_bwd_even_split_padded_to_32"] = moe_row((Em + len(msizes) - 1) // len(msizes), None)
        ragged = torch.randint(Cm // 2, Cm + 1, (nmax,), generator=genm, device=dev, dtype=torch.int32)
        res["moe_ffn_fwd_bwd_device0_ragged_tokens"] = moe_row(msizes[0], ragged)
        del mX, mdO, mW1, mW2

    def cost_model_rows():
        """Cost model of Sec. 3.2 fed with MEASURED kernel times (Sec. 7.7 checks the model's accuracy): the MLP block's
        forward + backward time is fitted as alpha * B + beta through shards 0 and 2 and compared with the measured middle
        shard; the fitted stage then goes through the LP for a range of All-Gather bandwidths next to the proportional (CP)
        and even (EV) splits of Sec. 2.3 (predictions of the model, not measurements: one GPU, no exchange)."""
        def t_block(sh, n=10):
            return steady_time(lambda: (sh.forward(), sh.backward()), n)
        gen7 = torch.Generator(device=dev); gen7.manual_seed(7)
        W1r = (torch.randn((h, F), generator=gen7, device=dev) * 0.02).to(torch.bfloat16)
        W2r = (torch.randn((F, h), generator=gen7, device=dev) * 0.02).to(torch.bfloat16)
        b1r = torch.zeros((F,), dtype=torch.bfloat16, device=dev)
        mid = MlpShard(Tn, h, F, offsets, 1, X, W1r, b1r, W2r, dOut)
        t0, t2, t1 = t_block(shards[0]), t_block(shards[1]), t_block(mid)
        # the same shard with whole tensors handed over (operands_are_full = 1): its columns start at byte 16804 of a row, so every view
        # is skewed and the epilogues store through chunks aligned in the destination's own address space
        whole = MlpShard(Tn, h, F, offsets, 1, X, W1r, b1r, W2r, dOut, whole_tensors=True)
        t1_whole = t_block(whole)
        del W1r, W2r, whole
        B0, B1, B2 = (sizes[j] / F for j in range(3))
        alpha = (t0 - t2) / (B0 - B2); beta = t0 - alpha * B0
        pred1 = alpha * B1 + beta
        out = {"block_fwd_bwd_ms_by_shard": {str(sizes[0]): round(t0 * 1e3, 3), str(sizes[1]): round(t1 * 1e3, 3), str(sizes[2]): round(t2 * 1e3, 3)},
               "fit_seconds": {"per_unit_ratio": round(alpha, 6), "fixed": round(beta, 6)},
               "middle_shard_predicted_ms": round(pred1 * 1e3, 3), "middle_shard_error_pct": round(100 * (pred1 - t1) / t1, 2),
               "middle_shard_whole_tensor_operands_ms": round(t1_whole * 1e3, 3), "whole_vs_compact_pct": round(100 * (t1_whole - t1) / t1, 2)}
        # one stage: compute = (alpha * B_j + beta) / relative speed_j; communication = one All-Gather forward and one
        # Reduce-Scatter backward of the block's [tokens x hidden] bf16 activations, time = bytes / bandwidth * max_j B_j
        act_bytes = 2.0 * Tn * h * 2
        speeds = list(w2.speeds)
        cp = [v / sum(speeds) for v in speeds]; ev = [1.0 / len(speeds)] * len(speeds)
        table = []
        for bw in (1.25e9, 2.5e9, 5e9, 12.5e9, 50e9, 200e9, 900e9):      # 10 GbE ... xGMI-class
            st = [(alpha, beta, 0.0, act_bytes / bw)]
            Blp, tlp = hap.hap_shard_ratios(speeds, st)
            table.append({"allgather_GBps": bw / 1e9, "t_cp_ms": round(hap.hap_iteration_time(speeds, st, cp) * 1e3, 3),
                          "t_ev_ms": round(hap.hap_iteration_time(speeds, st, ev) * 1e3, 3), "t_lp_ms": round(tlp * 1e3, 3),
                          "B_lp": [round(v, 4) for v in Blp]})
        out["cp_ev_lp_predictions"] = table
        return out

    def other_rows():
        """Throughput of the path's remaining kernels, measured in this run; not part of `value`: attention slice and
        row / element ops at config 4's shard-0 shapes (16 x 5 heads x 1024 x 128; 16384 x 2048 rows), config 5's
        attention slice and deep-K SFB rebuild, and config 3 done the naive way (local dW_i + sum) next to the rebuild."""
        B, S, nh, dh, hid = 16, 1024, 5, 128, 2048
        N = B * S
        res = {}

        timeit = steady_time

        qkv = dev_bf16(1, T.Q, (N, 3 * nh * dh), 1.0); dqkv = torch.zeros_like(qkv)
        o = torch.zeros((N, nh * dh), dtype=torch.bfloat16, device=dev); do = dev_bf16(1, T.DO, (N, nh * dh), 1.0)
        lse = torch.zeros((B, nh, S), dtype=torch.float32, device=dev)
        ad = hap.AttnDesc(B, nh, S, dh, True, [0, nh], stride_b=S * 3 * nh * dh, stride_s=3 * nh * dh, stride_h=dh, o_strides=(S * nh * dh, nh * dh, dh))
        aws = torch.empty((hap.hap_attn_bwd_workspace(ad, 0),), dtype=torch.uint8, device=dev)
        q = qkv.data_ptr(); dq = dqkv.data_ptr(); hd2 = nh * dh * 2
        fl = 4.0 * B * nh * S * S * dh
        t = timeit(lambda: hap.hap_sharded_attn_fwd(ad, 0, q, q + hd2, q + 2 * hd2, o, lse))
        res["attn_fwd_tflops"] = round(fl / t / 1e12, 1)
        t = timeit(lambda: hap.hap_sharded_attn_bwd(ad, 0, q, q + hd2, q + 2 * hd2, o, lse, do, dq, dq + hd2, dq + 2 * hd2, aws))
        res["attn_bwd_tflops_2.5x_fwd_flops"] = round(2.5 * fl / t / 1e12, 1)
        x = dev_bf16(1, T.X, (N, hid), 1.0); y = torch.zeros_like(x); dy = dev_bf16(1, T.DY, (N, hid), 1.0)
        g = torch.ones((hid,), dtype=torch.bfloat16, device=dev); be = torch.zeros_like(g)
        mean = torch.zeros((N,), dtype=torch.float32, device=dev); rstd = torch.zeros_like(mean)
        dg = torch.zeros((hid,), dtype=torch.float32, device=dev); dbe = torch.zeros_like(dg)
        lws = torch.empty((max(hap.hap_layernorm_bwd_workspace(N, hid), hap.hap_colsum_workspace(N, hid)),), dtype=torch.uint8, device=dev)
        nb = N * hid * 2
        t = timeit(lambda: hap.hap_layernorm_fwd(N, hid, hap.BF16, x, g, be, y, mean, rstd)); res["layernorm_fwd_gbs"] = round(2 * nb / t / 1e9)
        t = timeit(lambda: hap.hap_layernorm_bwd(N, hid, hap.BF16, x, g, mean, rstd, dy, y, dg, dbe, lws)); res["layernorm_bwd_gbs"] = round(3 * nb / t / 1e9)
        t = timeit(lambda: hap.hap_gelu_bwd(N, hid, hap.BF16, x, hid, dy, hid, y, hid)); res["gelu_bwd_gbs"] = round(3 * nb / t / 1e9)
        t = timeit(lambda: hap.hap_add(N, hid, hap.BF16, x, hid, dy, hid, g, y, hid)); res["add_bias_gbs"] = round(3 * nb / t / 1e9)
        t = timeit(lambda: hap.hap_colsum(N, hid, hap.BF16, dy, hid, dg, lws)); res["colsum_gbs"] = round(nb / t / 1e9)
        del qkv, dqkv, o, do, x, y, dy
        # config 5, shard 0: attention over a batch slice (79 x 16 heads x 197 x 64), SFB rebuilds with K = 50432 (split-K)
        B5, S5, H5, D5 = 79, 197, 16, 64
        q5 = dev_bf16(2, T.Q, (B5 * S5, 3 * H5 * D5), 1.0); dq5 = torch.zeros_like(q5)
        o5 = torch.zeros((B5 * S5, H5 * D5), dtype=torch.bfloat16, device=dev); do5 = dev_bf16(2, T.DO, (B5 * S5, H5 * D5), 1.0)
        lse5 = torch.zeros((B5, H5, S5), dtype=torch.float32, device=dev)
        ad5 = hap.AttnDesc(B5, H5, S5, D5, False, [0, B5], stride_b=S5 * 3 * H5 * D5, stride_s=3 * H5 * D5, stride_h=D5, o_strides=(S5 * H5 * D5, H5 * D5, D5))
        aws5 = torch.empty((hap.hap_attn_bwd_workspace(ad5, 0),), dtype=torch.uint8, device=dev)
        p5 = q5.data_ptr(); g5 = dq5.data_ptr(); w5 = H5 * D5 * 2
        fl5 = 4.0 * B5 * H5 * S5 * S5 * D5
        t = timeit(lambda: hap.hap_sharded_attn_fwd(ad5, 0, p5, p5 + w5, p5 + 2 * w5, o5, lse5)); res["cfg5_attn_fwd_tflops"] = round(fl5 / t / 1e12, 1)
        t = timeit(lambda: hap.hap_sharded_attn_bwd(ad5, 0, p5, p5 + w5, p5 + 2 * w5, o5, lse5, do5, g5, g5 + w5, g5 + 2 * w5, aws5))
        res["cfg5_attn_bwd_tflops_2.5x_fwd_flops"] = round(2.5 * fl5 / t / 1e12, 1)
        del q5, dq5, o5, do5
        # ---- configs 5, 4 and 1 below run on hapgen's seeded inputs and keep their device results in `held`: the parity leg compares them
        # with the oracle, tensor by tensor, after the timed part (max |gpu - oracle| / max |oracle| over all elements).
        w5 = hapgen.WORKLOADS["cfg5_vit_bf16"]; d5 = w5.dims
        r5, _ = hap.hap_shard_ratios(list(w5.speeds), [(1.0, 0.0, 0.0, 0.0)])
        b5sizes, b5offs = hap.hap_round_shards(r5, d5["batch"])
        s5, o5f = hap.hap_round_shards(r5, d5["ffn"])
        assert b5sizes == [79, 63, 63, 31, 20] and s5 == [1261, 1008, 1008, 504, 315], (b5sizes, s5)
        T5, h5, F5 = d5["batch"] * d5["seq"], d5["hidden"], d5["ffn"]
        # SFB rebuild of both MLP weight gradients from five devices' gathered factors: K = 50432 in ragged segments 197 * b_j (split-K)
        rows5 = [d5["seq"] * b for b in b5sizes]
        X5 = [dev_bf16(5, T.SFB_X + i, (r, h5), 1.0) for i, r in enumerate(rows5)]
        dY5 = [dev_bf16(5, T.SFB_DY + i, (r, F5), 1.0) for i, r in enumerate(rows5)]
        dW5 = torch.zeros((h5, F5), dtype=torch.float32, device=dev)
        ws5 = torch.empty((max(16, hap.hap_sfb_workspace(len(rows5), rows5, h5, F5)),), dtype=torch.uint8, device=dev)
        t = timeit(lambda: hap.hap_sfb_grad(X5, dY5, rows5, h5, F5, h5, F5, hap.BF16, dW5, F5, ws=ws5))
        res["cfg5_sfb_dW1_tflops"] = round(2.0 * h5 * F5 * sum(rows5) / t / 1e12, 1)
        # dW2 [4096 x 1024]: the factors swap roles (hidden activations [rows x 4096], output gradients [rows x 1024])
        dW5b = torch.zeros((F5, h5), dtype=torch.float32, device=dev)
        t = timeit(lambda: hap.hap_sfb_grad(dY5, X5, rows5, F5, h5, F5, h5, hap.BF16, dW5b, h5, ws=ws5))
        res["cfg5_sfb_dW2_tflops"] = round(2.0 * h5 * F5 * sum(rows5) / t / 1e12, 1)
        held["cfg5_sfb"] = dict(rows=rows5, dW1=dW5, dW2=dW5b)
        del X5, dY5, ws5
        # config 5's MLP with the ffn axis sharded (1261 | 1008 | 1008 | 504 | 315 of 4096) over all 50432 tokens: devices 0 and 4
        Xm, dOm = dev_bf16(5, T.X, (T5, h5), 1.0), dev_bf16(5, T.DY, (T5, h5), 1.0)
        W1m, b1m, W2m = dev_bf16(5, T.W, (h5, F5), 0.02), dev_bf16(5, T.BIAS, (F5,), 0.02), dev_bf16(5, T.W2, (F5, h5), 0.02)
        held["cfg5_mlp"] = dict(offs=o5f, shards={})
        for j5 in (0, 4):
            sh5 = MlpShard(T5, h5, F5, o5f, j5, Xm, W1m, b1m, W2m, dOm)
            t = timeit(lambda: (sh5.forward(), sh5.backward()), n=5)
            f5, b5 = sh5.flops()
            res[f"cfg5_mlp_fwd_bwd_device{j5}_ffn{s5[j5]}"] = {"ms": round(t * 1e3, 3), "gflop": round((f5 + b5) / 1e9, 1), "tflops": round((f5 + b5) / t / 1e12, 1)}
            held["cfg5_mlp"]["shards"][j5] = sh5
        del Xm, dOm, W1m, W2m
        # Whole layers, forward + backward.  Every virtual device's shard is built from the same seeded parameters; the rows time ONE device's
        # instruction list (every GEMM, attention and row kernel in order, its own partial products standing in for what the All-Reduce would
        # deliver); afterwards the whole program (all devices in turn, partial tensors summed) runs once for the parity leg.
        def layer_params(seed, hid, ffn):
            prm = {"Wq": dev_bf16(seed, T.WQ, (hid, hid), 0.02), "Wk": dev_bf16(seed, T.WK, (hid, hid), 0.02), "Wv": dev_bf16(seed, T.WV, (hid, hid), 0.02),
                   "Wo": dev_bf16(seed, T.WO, (hid, hid), 0.02), "W1": dev_bf16(seed, T.W, (hid, ffn), 0.02), "W2": dev_bf16(seed, T.W2, (ffn, hid), 0.02)}
            for i, (n, sz) in enumerate((("bq", hid), ("bk", hid), ("bv", hid), ("bo", hid), ("b1", ffn), ("b2", hid), ("be1", hid), ("be2", hid))):
                prm[n] = dev_bf16(seed, T.MISC + i, (sz,), 0.1)
            for i, n in enumerate(("g1", "g2")):      # gamma = 1 + small, snapped to bf16
                g = 1.0 + hapgen.normal_bf16(seed, T.MISC + 20 + i, (hid,), 0.1)[0]
                prm[n] = torch.from_numpy(hapgen.to_bf16_bits(g.astype(np.float32)).view(np.int16)).view(torch.bfloat16).to(dev)
            return prm

        def layer_rows(tag, style, seed, w, hoffs, foffs, boffs, which, names):
            d = w.dims
            B, S, hid, heads, dh, ffn = d["batch"], d["seq"], d["hidden"], d["heads"], d["head_dim"], d["ffn"]
            prm = layer_params(seed, hid, ffn)
            x = dev_bf16(seed, T.X, (B * S, hid), 1.0); dy = dev_bf16(seed, T.DY, (B * S, hid), 1.0)
            prog = EncoderLayerProgram(style, B, S, hid, heads, dh, ffn, hoffs, foffs, boffs, prm, x, dy)
            for j, name in zip(which, names):
                sh = prog.shards[j]
                xs, dys = (x, dy) if style == "tensor" else (sh.rows(x), sh.rows(dy))
                buf = {n: torch.zeros_like(xs) for n in ("x1", "y", "dx1", "dx")}
                buf["dbo"] = torch.zeros((hid,), dtype=torch.float32, device=dev); buf["db2"] = torch.zeros_like(buf["dbo"])
                t = timeit(lambda: sh.device_step(xs, dys, buf, prm["bo"], prm["b2"]), n=5)
                f, b = sh.flops()
                res[name] = {"ms": round(t * 1e3, 3), "gflop": round((f + b) / 1e9, 1), "tflops": round((f + b) / t / 1e12, 1)}
                del buf
            prog.forward(); prog.backward()
            torch.cuda.synchronize()
            held[tag] = dict(prog=prog, seed=seed, style=style, w=w, hoffs=hoffs, foffs=foffs, boffs=boffs)
        w4 = hapgen.WORKLOADS["cfg4_encoder_bf16"]; d4 = w4.dims
        r4, _ = hap.hap_shard_ratios(list(w4.speeds), [(1.0, 0.0, 0.0, 0.0)])
        h4sizes, h4offs = hap.hap_round_shards(r4, d4["heads"]); f4sizes, f4offs = hap.hap_round_shards(r4, d4["ffn"])
        assert h4sizes == [5, 5, 3, 3] and f4sizes == [2731, 2731, 1365, 1365], (h4sizes, f4sizes)
        layer_rows("cfg4", "tensor", 4, w4, h4offs, f4offs, [0, d4["batch"]], (0, 2),
                   ("cfg4_layer_fwd_bwd_device0_5heads_ffn2731", "cfg4_layer_fwd_bwd_device2_3heads_ffn1365"))
        layer_rows("cfg5_layer", "data", 5, w5, [0, d5["heads"]], [0, d5["ffn"]], b5offs, (0, 4),
                   ("cfg5_layer_fwd_bwd_device0_79samples", "cfg5_layer_fwd_bwd_device4_20samples"))
        # config 1: one fp32 fully-connected layer, 64 x 1024 x 1024, rows split (38, 26): latency-bound, reported in microseconds (warm)
        w1 = hapgen.WORKLOADS["cfg1_fc_f32"]
        r1, _ = hap.hap_shard_ratios(list(w1.speeds), [(1.0, 0.0, 0.0, 0.0)])
        s1, o1 = hap.hap_round_shards(r1, w1.dims["tokens"])
        assert s1 == [38, 26], s1
        dev_f32 = lambda tid, shape, sigma: torch.from_numpy(hapgen.normal(1, tid, shape, sigma, dtype=np.float32)).to(dev)
        X1 = dev_f32(T.X, (64, 1024), 1.0); W1c = dev_f32(T.W, (1024, 1024), 0.02); dY1 = dev_f32(T.DY, (64, 1024), 1.0)
        Y1 = torch.zeros_like(dY1); dX1 = torch.zeros_like(X1); dW1c = torch.zeros_like(W1c)
        d1 = hap.LinearDesc(64, 1024, 1024, hap.SHARD_BATCH, o1, hap.F32)
        ws1 = torch.empty((hap.hap_linear_bwd_workspace(d1, 0),), dtype=torch.uint8, device=dev)
        c1 = {"rows": s1}
        for j1 in range(2):
            c1[f"fwd_dev{j1}_us"] = round(timeit(lambda: hap.hap_sharded_linear_fwd(d1, j1, X1, W1c, None, Y1, None, ws1), n=50) * 1e6, 1)
            c1[f"bwd_dev{j1}_us"] = round(timeit(lambda: hap.hap_sharded_linear_bwd(d1, j1, X1, W1c, None, dY1, dX1, dW1c, hap.F32, None, ws1), n=50) * 1e6, 1)
        # cold: the caches (4 MB L2 per XCD, 256 MB last-level) are flushed by overwriting a 1 GiB buffer before every single
        # timed call; median of 15.  Every other figure of this report is warm (nothing flushed between repetitions).
        flush = torch.empty((1 << 30,), dtype=torch.uint8, device=dev)
        def cold(fn, n=15):
            ts = []
            for _ in range(n):
                flush.fill_(1)
                a = torch.cuda.Event(enable_timing=True); b = torch.cuda.Event(enable_timing=True)
                a.record(stream); fn(); b.record(stream); b.synchronize()
                ts.append(a.elapsed_time(b) * 1e3)
            return round(sorted(ts)[n // 2], 1)
        c1["fwd_dev0_cold_us"] = cold(lambda: hap.hap_sharded_linear_fwd(d1, 0, X1, W1c, None, Y1, None, ws1))
        c1["bwd_dev0_cold_us"] = cold(lambda: hap.hap_sharded_linear_bwd(d1, 0, X1, W1c, None, dY1, dX1, dW1c, hap.F32, None, ws1))
        del flush
        c1["sfb_rebuild_us"] = round(timeit(lambda: hap.hap_sfb_grad([X1[:s1[0]], X1[s1[0]:]], [dY1[:s1[0]], dY1[s1[0]:]], s1, 1024, 1024, 1024, 1024,
                                                                   hap.F32, dW1c, 1024, ws=ws1), n=50) * 1e6, 1)
        # the whole config-1 step (forward + backward of both devices, SFB rebuild: 11 small kernels), eager and replayed from a HIP graph
        def step1():
            for j1 in range(2):
                hap.hap_sharded_linear_fwd(d1, j1, X1, W1c, None, Y1, None, ws1)
                hap.hap_sharded_linear_bwd(d1, j1, X1, W1c, None, dY1, dX1, dW1c, hap.F32, None, ws1)
            hap.hap_sfb_grad([X1[:s1[0]], X1[s1[0]:]], [dY1[:s1[0]], dY1[s1[0]:]], s1, 1024, 1024, 1024, 1024, hap.F32, dW1c, 1024, ws=ws1)
        c1["step_eager_us"] = round(timeit(step1, n=50) * 1e6, 1)
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            step1()
        side.synchronize()
        graph1 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph1, stream=side):
            step1()
        c1["step_hip_graph_us"] = round(timeit(graph1.replay, n=50) * 1e6, 1)
        res["cfg1_fc_f32_latency"] = c1
        # one more pass of config 1 with every device's results kept apart (for the parity leg): rows of Y and dX, the devices' partial dW, the rebuild
        dWp = [torch.zeros_like(W1c) for _ in range(2)]; dWs = torch.zeros_like(W1c)
        Y1.zero_(); dX1.zero_()
        for j1 in range(2):
            hap.hap_sharded_linear_fwd(d1, j1, X1, W1c, None, Y1, None, ws1)
            hap.hap_sharded_linear_bwd(d1, j1, X1, W1c, None, dY1, dX1, dWp[j1], hap.F32, None, ws1)
        hap.hap_sfb_grad([X1[:s1[0]], X1[s1[0]:]], [dY1[:s1[0]], dY1[s1[0]:]], s1, 1024, 1024, 1024, 1024, hap.F32, dWs, 1024, ws=ws1)
        torch.cuda.synchronize()
        held["cfg1"] = dict(Y=Y1, dX=dX1, dW_partials=dWp, dW_sfb=dWs, rows=s1)
        # uneven All-Gather data movement (Sec. 2.3.1): the padded slots of config 2's hidden activations (8402 | 5041 | 2941 of 16384
        # columns: byte offsets 16804 and 26886, nothing 16-byte aligned) and of config 5's token rows (batch 79 | 63 | 63 | 31 | 20 x 197)
        def gather_row(rows_, cols_, dim_, offs_):
            gd = hap.GatherDesc(rows_, cols_, dim_, offs_, 2)
            cap = hap.hap_allgather_capacity(gd)
            m_ = len(offs_) - 1
            shp = (cap, cols_) if dim_ == 0 else (rows_, cap)
            slots = torch.empty((m_,) + shp, dtype=torch.bfloat16, device=dev).normal_()
            outg = torch.empty((rows_, cols_), dtype=torch.bfloat16, device=dev)
            ptrs = [slots[j_].data_ptr() for j_ in range(m_)]
            t_ = timeit(lambda: hap.hap_allgather_assemble(gd, ptrs, [shp[1]] * m_, outg, cols_))
            # the reverse before a padded Reduce-Scatter: the full tensor read once, m capacity-sized slots (zeros included) written
            t2_ = timeit(lambda: hap.hap_reducescatter_split(gd, outg, cols_, ptrs, [shp[1]] * m_))
            return round(2.0 * rows_ * cols_ * 2 / t_ / 1e9), round((rows_ * cols_ + m_ * shp[0] * shp[1]) * 2 / t2_ / 1e9)
        res["allgather_trim_cfg2_hidden_dim1_gbs"], res["reducescatter_split_cfg2_hidden_dim1_gbs"] = gather_row(Tn, F, 1, offsets)
        res["allgather_trim_cfg5_tokens_dim0_gbs"], res["reducescatter_split_cfg5_tokens_dim0_gbs"] = gather_row(256 * 197, 1024, 0, [197 * b for b in (0, 79, 142, 205, 236, 256)])
        moe_rows(res, timeit)
        # config 3 the naive way (Fig. "sfb"(b)): every device's own fp32 dW_i, then their sum (what the All-Reduce delivers)
        inf, outf = w3.dims["in_features"], w3.dims["out_features"]
        parts = [torch.zeros((inf, outf), dtype=torch.float32, device=dev) for _ in rows]

        def naive():
            for i, r in enumerate(rows):
                hap.hap_sfb_grad([sX[i]], [sdY[i]], [r], inf, outf, inf, outf, hap.BF16, parts[i], outf)
            for i in range(1, len(rows)):
                hap.hap_add(inf, outf, hap.F32, parts[0], outf, parts[i], outf, None, parts[0], outf)
        t = timeit(naive, n=3); res["cfg3_naive_local_dW_plus_sum_ms"] = round(t * 1e3, 3)
        t = timeit(lambda: sfb.run(None), n=5); res["cfg3_sfb_rebuild_ms"] = round(t * 1e3, 3)
        return res

    if args.moe_only:
        timeit = steady_time
        res = {}
        moe_rows(res, timeit)
        print(json.dumps(res))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    step_marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    step_marks[0].record(stream)
    for i in range(args.steps):
        step(timer)
        step_marks[i + 1].record(stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(step_marks[i].elapsed_time(step_marks[i + 1]) for i in range(args.steps))
    ms = dt / args.steps * 1e3
    value = step_flops / (dt / args.steps) / 1e12

    # per-call durations measured with events on the launch stream inside the timed region
    per = {k: sum(a.elapsed_time(b) for a, b in v) / len(v) for k, v in marks.items()}
    big = shards[0]
    gemm = 2.0 * big.T * big.h * big.f
    call_flops = {f"fc1_fwd[f={big.f}]": gemm, f"fc2_fwd[f={big.f}]": gemm, "sfb_grad": sfb.flops()}
    # Dominant kernel: the 256x256x64 bf16 MFMA GEMM.  fc2_fwd of the largest shard is ONE launch of it
    # (M = 8192 tokens, N = 4096, K = 8402: 512 output tiles, no remainder strip), bracketed by events above.
    dom = f"fc2_fwd[f={big.f}]"
    achieved = call_flops[dom] / (per[dom] * 1e-3) / 1e12
    # HBM-side bytes of that launch: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (KiB per dispatch) scaled by the factors a plain
    # 256 MiB copy gives.  Counters cannot be read from inside this process, so the figure comes from the committed summary of the
    # profiler runs (profiles/roofline_traffic.json: counter values, factors, the commands and the library commit they were taken
    # on) and is reported with that source; null when the file is not there.
    traffic_bytes, traffic_source = None, None
    tj = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "roofline_traffic.json")
    if os.path.exists(tj):
        with open(tj) as fh:
            t = json.load(fh)
        traffic_bytes = int((t["fetch_size_kib_per_dispatch"] * t["copy_calibration_factor_fetch"] +
                             t["write_size_kib_per_dispatch"] * t["copy_calibration_factor_write"]) * 1024)
        traffic_source = {"file": "profiles/roofline_traffic.json", "summary": t["source"], "library_commit": t["library_commit"]}
    out = {
        "metric": "TFLOP/s of sharded fwd+bwd + SFB dW at uneven ratios; % of MFMA peak",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 3), "ms_per_step_median": round(per_step[len(per_step) // 2], 3), "ms_per_step_min": round(per_step[0], 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2_mlp_bf16 shards 0 and 2 fwd+bwd + cfg3_sfb_bf16 rebuild", "tokens": Tn, "hidden": h, "ffn": F,
                   "speeds": list(w2.speeds), "shard_sizes": sizes, "sfb_rows": list(rows), "step_gflop": round(step_flops / 1e9, 1),
                   "pct_of_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2)},
        "roofline": {"bound": "mfma", "kernel": "gemm_pp_kernel<bf16,256x256x32,4 stages> (" + dom + ": M=8192 N=4096 K=8402)",
                     "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic_bytes, "traffic_source": traffic_source,
                     "algorithmic_bytes": int(2 * (big.T * big.f + big.f * big.h + big.T * big.h)),
                     "launch_ms": round(per[dom], 4)},
        "calls_ms": {k: round(v, 4) for k, v in sorted(per.items())},
        "calls_tflops": {k: round(call_flops[k] / (per[k] * 1e-3) / 1e12, 1) for k in call_flops},
        "setup_s": round(t_setup, 1),
    }
    if not args.main_only:
        out["achievable"] = ceilings()
        out["other_rows"] = other_rows()
        out["cost_model"] = cost_model_rows()
    if not args.no_cpu_baseline and not args.main_only:
        # The oracle's sample IS the timed workload (same seeded arrays, both shards and the SFB rebuild): what the timed step
        # left in the device buffers is compared with it tensor by tensor, max |gpu - oracle| / max |oracle| over ALL elements.
        step()
        torch.cuda.synchronize()
        errs = {}

        def compare(tag, ref):
            if tag == "sfb":
                got = {"sfb_dW": sfb.dW}
                want = {"sfb_dW": ref}
            else:
                sj = shards[0] if tag == sizes[0] else shards[1]
                assert sj.f == tag
                got = {"H": sj.H[:, :sj.f], "P": sj.P, sj.dH_holds: sj.dH[:, :sj.f], "dX": sj.dX, "dW1": sj.dW1[:, :sj.f], "db1": sj.db1, "dW2": sj.dW2}
                want = {"H": ref["H"], "P": ref["out"], sj.dH_holds: ref[sj.dH_holds], "dX": ref["dX"], "dW1": ref["dW1"], "db1": ref["db1"], "dW2": ref["dW2"]}
            for k in got:
                g = got[k].float().cpu().numpy().astype(np.float64)
                errs[f"{k}[f={tag}]" if tag != "sfb" else k] = float(np.abs(g - want[k]).max() / np.abs(want[k]).max())

        out["cpu_baseline"] = cpu_baseline(np, hapgen, T, w2, offsets, compare)
        tol = 2e-2
        fmt = lambda e: {k: float(f"{v:.3g}") for k, v in e.items()}
        out["parity"] = {"against": "oracle, all elements of both timed shards' tensors and of the SFB gradient", "tolerance": tol,
                         "max_rel_err": fmt(errs), "pass": bool(max(errs.values()) <= tol)}
        # every configuration at its stated size: what the untimed rows left on the device against the oracle (same seeded inputs), per tensor
        per_cfg = {"cfg2_mlp_bf16 + cfg3_sfb_bf16 (the timed step)": {"tolerance": tol, "max_rel_err": fmt(errs), "pass": out["parity"]["pass"]}}
        for name, (e, t_) in config_parity(np, hapgen, T, held).items():
            per_cfg[name] = {"tolerance": t_, "max_rel_err": fmt(e), "pass": bool(max(e.values()) <= t_)}
        out["parity"]["configs"] = per_cfg
        out["parity"]["all_configs_pass"] = bool(all(v["pass"] for v in per_cfg.values()))
    print(json.dumps(out))


def config_parity(np, hapgen, T, held):
    """Configs 1, 4 and 5 at their stated sizes: the device results the untimed rows kept (`held`) against the float64 oracle on the same
    seeded inputs, max |gpu - oracle| / max |oracle| per tensor over all elements.  Returns {config: (errors, tolerance)}."""
    from oracle import layers, sfb
    res = {}

    def host(t):
        return t.detach().float().cpu().numpy().astype(np.float64)

    def rel(got, ref):
        ref = np.asarray(ref, dtype=np.float64)
        return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30)) if np.isfinite(got).all() else float("inf")

    if "cfg1" in held:
        h = held["cfg1"]
        X = hapgen.normal(1, T.X, (64, 1024), 1.0, dtype=np.float32).astype(np.float64)
        W = hapgen.normal(1, T.W, (1024, 1024), 0.02, dtype=np.float32).astype(np.float64)
        dY = hapgen.normal(1, T.DY, (64, 1024), 1.0, dtype=np.float32).astype(np.float64)
        dWo = X.T @ dY
        res["cfg1_fc_f32"] = ({"Y": rel(host(h["Y"]), X @ W), "dX": rel(host(h["dX"]), dY @ W.T),
                               "dW (sum of the devices' partials)": rel(sum(host(t) for t in h["dW_partials"]), dWo),
                               "dW (SFB rebuild)": rel(host(h["dW_sfb"]), dWo)}, 1e-5)
    if "cfg5_sfb" in held:
        h = held["cfg5_sfb"]
        Xs = [hapgen.normal_bf16(5, T.SFB_X + i, (r, 1024), 1.0)[0] for i, r in enumerate(h["rows"])]
        Ys = [hapgen.normal_bf16(5, T.SFB_DY + i, (r, 4096), 1.0)[0] for i, r in enumerate(h["rows"])]
        res["cfg5_vit_bf16: SFB rebuild of dW1, dW2 (K = 50432)"] = ({"dW1": rel(host(h["dW1"]), sfb.sfb_grad(Xs, Ys, h["rows"])),
                                                                      "dW2": rel(host(h["dW2"]), sfb.sfb_grad(Ys, Xs, h["rows"]))}, 2e-2)
        del Xs, Ys
    if "cfg5_mlp" in held:
        h = held["cfg5_mlp"]
        any_shard = next(iter(h["shards"].values()))
        tok, hid, F = any_shard.T, any_shard.h, any_shard.F
        X = hapgen.normal_bf16(5, T.X, (tok, hid), 1.0)[0]; dO = hapgen.normal_bf16(5, T.DY, (tok, hid), 1.0)[0]
        W1 = hapgen.normal_bf16(5, T.W, (hid, F), 0.02)[0]; b1 = hapgen.normal_bf16(5, T.BIAS, (F,), 0.02)[0]; W2 = hapgen.normal_bf16(5, T.W2, (F, hid), 0.02)[0]
        e = {}
        for j, sh in h["shards"].items():     # the block restricted to the device's ffn columns IS the device's program: its out / dX are the partial sums
            lo, hi = h["offs"][j], h["offs"][j + 1]
            ref = layers.mlp_block(X, np.ascontiguousarray(W1[:, lo:hi]), b1[lo:hi], np.ascontiguousarray(W2[lo:hi]), np.zeros(hid), dO)
            f = sh.f
            for n, got, want in (("H", sh.H[:, :f], "H"), ("P", sh.P, "out"), (sh.dH_holds, sh.dH[:, :f], sh.dH_holds), ("dX", sh.dX, "dX"),
                                 ("dW1", sh.dW1[:, :f], "dW1"), ("db1", sh.db1[:f], "db1"), ("dW2", sh.dW2[:f], "dW2")):
                e[f"{n}[device {j}, ffn {f}]"] = rel(host(got), ref[want])
            del ref
        res["cfg5_vit_bf16: ffn-sharded MLP over 50432 tokens"] = (e, 2e-2)
        del X, dO, W1, W2
    for tag, title in (("cfg4", "cfg4_encoder_bf16: whole layer, 4 devices (heads 5|5|3|3, ffn 2731|2731|1365|1365)"),
                       ("cfg5_layer", "cfg5_vit_bf16: whole layer, 5 devices (batch 79|63|63|31|20)")):
        if tag not in held:
            continue
        h = held[tag]; prog = h["prog"]; d = h["w"].dims; seed = h["seed"]
        B, S, hid, heads, dh, ffn = d["batch"], d["seq"], d["hidden"], d["heads"], d["head_dim"], d["ffn"]
        nb = hapgen.normal_bf16
        ph = {"Wq": nb(seed, T.WQ, (hid, hid), 0.02)[0], "Wk": nb(seed, T.WK, (hid, hid), 0.02)[0], "Wv": nb(seed, T.WV, (hid, hid), 0.02)[0],
              "Wo": nb(seed, T.WO, (hid, hid), 0.02)[0], "W1": nb(seed, T.W, (hid, ffn), 0.02)[0], "W2": nb(seed, T.W2, (ffn, hid), 0.02)[0]}
        for i, (n, sz) in enumerate((("bq", hid), ("bk", hid), ("bv", hid), ("bo", hid), ("b1", ffn), ("b2", hid), ("be1", hid), ("be2", hid))):
            ph[n] = nb(seed, T.MISC + i, (sz,), 0.1)[0]
        for i, n in enumerate(("g1", "g2")):
            g = 1.0 + nb(seed, T.MISC + 20 + i, (hid,), 0.1)[0]
            ph[n] = hapgen.from_bf16_bits(hapgen.to_bf16_bits(g.astype(np.float32)))
        ref = layers.encoder_layer(nb(seed, T.X, (B * S, hid), 1.0)[0], ph, nb(seed, T.DY, (B * S, hid), 1.0)[0], B, S, heads, dh)
        e = {n: rel(host(t), ref[n]) for n, t in (("x1", prog.x1), ("y", prog.y), ("dx1", prog.dx1), ("dx", prog.dx), ("db2", prog.db2), ("dbo", prog.dbo))}
        if h["style"] == "tensor":      # every device's exact slices of the weight gradients; the worst device is reported per tensor
            worst = {}
            for j, sh in enumerate(prog.shards):
                c = slice(h["hoffs"][j] * dh, h["hoffs"][j + 1] * dh); fc = slice(h["foffs"][j], h["foffs"][j + 1]); hd, f = sh.hd, sh.f
                got = host(sh.dWqkv)
                pairs = [("dWq", got[:, :hd], ref["dWq"][:, c]), ("dWk", got[:, hd:2 * hd], ref["dWk"][:, c]), ("dWv", got[:, 2 * hd:3 * hd], ref["dWv"][:, c]),
                         ("dWo", host(sh.dWo)[:hd], ref["dWo"][c]), ("o", host(sh.o)[:, :hd], ref["o"][:, c]),
                         ("dW1", host(sh.dW1)[:, :f], ref["dW1"][:, fc]), ("db1", host(sh.db1)[:f], ref["db1"][fc]), ("dW2", host(sh.dW2)[:f], ref["dW2"][fc])]
                for n, g_, r_ in pairs:
                    worst[n] = max(worst.get(n, 0.0), rel(g_, r_))
            e.update({f"{n} (worst device)": v for n, v in worst.items()})
            s0 = prog.shards[0]
            e.update({n: rel(host(t), ref[n]) for n, t in (("dg1", s0.dg1), ("dbe1", s0.dbe1), ("dg2", s0.dg2), ("dbe2", s0.dbe2))})
        else:                           # batch shards: the devices' partial weight gradients summed = the all-reduced gradient
            acc = {}
            for sh in prog.shards:
                got = host(sh.dWqkv)
                parts = {"dWq": got[:, :hid], "dWk": got[:, hid:2 * hid], "dWv": got[:, 2 * hid:3 * hid], "dWo": host(sh.dWo), "dW1": host(sh.dW1)[:, :ffn],
                         "dW2": host(sh.dW2), "db1": host(sh.db1), "dg1": host(sh.dg1), "dbe1": host(sh.dbe1), "dg2": host(sh.dg2), "dbe2": host(sh.dbe2)}
                for n, v in parts.items():
                    acc[n] = acc.get(n, 0) + v
            e.update({f"{n} (sum over devices)": rel(v, ref[n]) for n, v in acc.items()})
        res[title] = (e, 2e-2)
        del ref, ph
    return res


def cpu_baseline(np, hapgen, T, w2, offsets, compare=None):
    """The oracle as it stands, timed on this host's cores on the timed workload itself: MLP fwd+bwd of both timed shards
    (the smallest and the largest) over all tokens plus the SFB rebuild - one whole step, 10-20 s of float64 numpy.  Only the
    oracle's own calls are timed; compare(tag, reference) hands each result to the caller's parity check and drops it."""
    from oracle import layers, sfb
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    w3 = hapgen.WORKLOADS["cfg3_sfb_bf16"]
    h, tok, F = w2.dims["hidden"], w2.dims["tokens"], w2.dims["ffn"]
    X = hapgen.normal_bf16(0, T.X, (tok, h), 1.0)[0]
    W1f = hapgen.normal_bf16(0, T.W, (h, F), 0.02)[0]; b1f = hapgen.normal_bf16(0, T.BIAS, (F,), 0.02)[0]
    W2f = hapgen.normal_bf16(0, T.W2, (F, h), 0.02)[0]; dOut = hapgen.normal_bf16(0, T.DY, (tok, h), 1.0)[0]
    dt, flops = 0.0, 0.0
    for j in (2, 0):
        lo, hi = offsets[j], offsets[j + 1]
        W1 = np.ascontiguousarray(W1f[:, lo:hi]); W2 = np.ascontiguousarray(W2f[lo:hi])
        t0 = time.perf_counter()
        ref = layers.mlp_block(X, W1, b1f[lo:hi], W2, np.zeros(h), dOut)
        dt += time.perf_counter() - t0
        flops += 12.0 * tok * h * (hi - lo)
        if compare:
            compare(hi - lo, ref)
        del ref, W1, W2
    rows, cap = w3.dims["rows"], w3.dims["capacity"]
    sX = [hapgen.normal_bf16(0, T.SFB_X + i, (cap, w3.dims["in_features"]), 1.0)[0] for i in range(len(rows))]
    sdY = [hapgen.normal_bf16(0, T.SFB_DY + i, (cap, w3.dims["out_features"]), 1.0)[0] for i in range(len(rows))]
    t0 = time.perf_counter()
    ref = sfb.sfb_grad(sX, sdY, rows)
    dt += time.perf_counter() - t0
    flops += 2.0 * w3.dims["in_features"] * w3.dims["out_features"] * sum(rows)
    if compare:
        compare("sfb", ref)
    return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle (float64 numpy): one whole step - MLP fwd+bwd of shards 2 and 0 over all {tok} tokens + SFB rebuild, "
                      f"{flops / 1e9:.0f} GFLOP in {dt:.1f} s"}


if __name__ == "__main__":
    main()
