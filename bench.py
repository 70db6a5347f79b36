#!/usr/bin/env python3
"""Benchmark of one GPU's share of Ulysses sequence parallelism on MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
    pack_qkv(x_q, x_k, x_v)        3 x [N/P, H, d]      -> P send chunks each, one launch
    unpack_qkv(r_q, r_k, r_v)      3 x P received chunks -> [N, H/P, d] each, one launch   (the exchange itself
                                                           is not part of this library)
    attention forward, attention backward over the unpacked q, k, v (causal, batch 1)
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config gpt7b] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
# HBM-side bytes per launch of the dK/dV kernel, from the committed rocprofv3 counter runs of this
# same command (profiles/bench_gpt7b_kernels.md): FETCH_SIZE 2.755e6 KiB x 2.0 + WRITE_SIZE 2.63e5 KiB
# (the fetch figure varies between runs, 5 - 20 GiB: it depends on how well the workgroups stay in step).
# Counters cannot be read from inside this script, so the figure is only reported for that workload.
DKV_TRAFFIC_BYTES = {"gpt7b": (2.755e6 * 2.0 + 2.63e5) * 1024}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="gpt7b", help="workload name from synth_inputs.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-rows", type=int, default=640, help="query rows the CPU oracle is timed on")
    ap.add_argument("--sparse-window", type=int, default=0,
                    help="also time block-sparse attention: local window of this many 256-token blocks plus the "
                         "first block column (0 = off; extra 'sparse' object in the output)")
    ap.add_argument("--d", type=int, default=0,
                    help="head dimension to use instead of the workload's (64, 128 or 256; N, P and the head count stay)")
    ap.add_argument("--layouts", action="store_true",
                    help="also time every layout transform (forward and reverse direction, both layouts, one and "
                         "three tensors per launch) at this workload's shapes (extra 'layout_transforms' object)")
    ap.add_argument("--xattn", default="",
                    help="also time attention without a mask for these (queries, keys) counts, e.g. "
                         "'131072x131072,16384x131072': rows of the same tensors (extra 'xattn' list in the output)")
    ap.add_argument("--sparse-pattern", choices=["window_global", "fixed", "global_rows"], default="window_global",
                    help="with --sparse-window W: 'window_global' = blocks r - c < W plus the first block column; "
                         "'fixed' = windows of W blocks, a block row sees its own window and the last block of every "
                         "earlier window; 'global_rows' = blocks r - c < W, and every 64th block row sees everything "
                         "before it")
    ap.add_argument("--elem", choices=["bf16", "fp16"], default="bf16",
                    help="element type of the tensors (the headline metric is bf16)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU's share only (no collectives, no second GPU); "
              "run it with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2309_14509_amd as uly
    import synth_inputs as synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    uly.load()     # raises if libulysses.so is not built: there is no fallback path
    torch.cuda.set_device(0)

    c = synth.CONFIGS[args.config]
    N, P, H, d = c["N"], c["P"], c["H"], args.d or c["d"]
    nl, Hl = N // P, H // P
    scale = 1.0 / math.sqrt(d)
    seed = synth.config_seed(args.config)

    etype = torch.float16 if args.elem == "fp16" else torch.bfloat16
    lay = uly.LAYOUT_SEQ_HEAD | (uly.ELEM_F16 if args.elem == "fp16" else 0)      # attention entry points only

    def dev_bf16(bits):      # bf16 bit patterns -> device tensor of the chosen element type
        return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16).to(etype)

    # ---- synthetic inputs, resident in HBM ---------------------------------------------------
    # sequence-sharded activations this rank would send (3 tensors: q, k, v projections)
    xs = [dev_bf16(synth.normal_bf16((nl, H, d), seed, synth.TID_X + 10 * i)) for i in range(3)]
    # chunks this rank would have received: they ARE q, k, v of the local heads for the full sequence
    q_bits, k_bits, v_bits, do_bits = synth.attention_inputs(N, Hl, d, seed, c["qk_mult"])
    recvs = [dev_bf16(b.reshape(P, nl, Hl, d)) for b in (q_bits, k_bits, v_bits)]
    dout = dev_bf16(do_bits)
    sends = [torch.empty((P, nl, Hl, d), dtype=etype, device="cuda") for _ in range(3)]
    qkv = [torch.empty((N, Hl, d), dtype=etype, device="cuda") for _ in range(3)]
    o = torch.empty((N, Hl, d), dtype=etype, device="cuda")
    lse = torch.empty((Hl, N), dtype=torch.float32, device="cuda")
    grads = tuple(torch.empty((N, Hl, d), dtype=etype, device="cuda") for _ in range(3))
    ws = torch.empty(max(uly.ulysses_attn_bwd_workspace_bytes(N, Hl, d), 16), dtype=torch.uint8, device="cuda")
    # forward workspace: empty at the headline shape; short sequences cut long rows into work items with it
    fws_bytes = uly.ulysses_attn_fwd_workspace_bytes(N, Hl, d, True)
    fws = torch.empty(max(fws_bytes, 16), dtype=torch.uint8, device="cuda")

    lib = uly.load()
    stream = torch.cuda.current_stream()
    sp = uly._stream()

    def ptr(t):
        return t.data_ptr()

    import ctypes
    ptr3 = lambda ts: (ctypes.c_void_p * 3)(*[t.data_ptr() for t in ts])
    x_ptrs, send_ptrs, recv_ptrs, qkv_ptrs = ptr3(xs), ptr3(sends), ptr3(recvs), ptr3(qkv)

    # Events bracket each kernel on the stream the kernels run on (torch's current stream is the one
    # handed to the library).
    names = ["pack", "unpack", "attn_fwd", "attn_bwd_delta", "attn_bwd_dkv", "attn_bwd_dq"]

    def step(record=None):
        def mark():
            if record is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record(stream)
                record.append(e)
        mark()
        uly._check(lib.ulysses_pack_qkv(x_ptrs, send_ptrs, nl, H, d, P, 2, sp), "pack_qkv")
        mark()
        uly._check(lib.ulysses_unpack_qkv(recv_ptrs, qkv_ptrs, nl, H, d, P, 2, uly.LAYOUT_SEQ_HEAD, sp), "unpack_qkv")
        mark()
        uly._check(lib.ulysses_attn_fwd_ws(ptr(qkv[0]), ptr(qkv[1]), ptr(qkv[2]), ptr(o), ptr(lse), ptr(fws), fws_bytes, N,
                                           Hl, d, scale, 1, lay, sp), "attn_fwd")
        mark()
        for stage in (uly.BWD_STAGE_DELTA, uly.BWD_STAGE_DKV, uly.BWD_STAGE_DQ):
            uly._check(lib.ulysses_attn_bwd_stage(stage, ptr(qkv[0]), ptr(qkv[1]), ptr(qkv[2]), ptr(o), ptr(dout),
                                                  ptr(lse), ptr(grads[0]), ptr(grads[1]), ptr(grads[2]), ptr(ws),
                                                  ws.numel(), N, Hl, d, scale, 1, lay, sp), "attn_bwd")
            mark()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    per_step_events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ev = []
        step(ev)
        per_step_events.append(ev)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / args.steps

    seg_ms = {n: 0.0 for n in names}
    for ev in per_step_events:
        for i, n in enumerate(names):
            seg_ms[n] += ev[i].elapsed_time(ev[i + 1])
    seg_ms = {n: v / args.steps for n, v in seg_ms.items()}

    # ---- algorithmic work -----------------------------------------------------------------------
    unit = float(N) * N * d * Hl                     # one causal contraction (2 * N^2/2 * d * Hl)
    flop_fwd, flop_bwd = 2 * unit, 5 * unit          # recomputed contractions do not count
    attn_ms = seg_ms["attn_fwd"] + seg_ms["attn_bwd_delta"] + seg_ms["attn_bwd_dkv"] + seg_ms["attn_bwd_dq"]
    tensor_bytes = nl * H * d * 2
    pack_gbs = 3 * 2 * tensor_bytes / (seg_ms["pack"] * 1e-3) / 1e9
    unpack_gbs = 3 * 2 * tensor_bytes / (seg_ms["unpack"] * 1e-3) / 1e9
    # the dominant kernel: dK/dV.  It owns 4 of the backward's 5 algorithmic contractions (S, dP, dV, dK);
    # the dQ kernel owns 1 (its S and dP are the recomputed ones).
    dkv_tflops = 4 * unit / (seg_ms["attn_bwd_dkv"] * 1e-3) / 1e12
    result = {
        "metric": "attn fwd+bwd TFLOP/s and % bf16 MFMA peak at N=128K shard; pack/unpack GB/s",
        "value": (flop_fwd + flop_bwd) / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if args.elem == "fp16" else "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}{' with another head dimension' if d != c['d'] else ''}: one GPU's share, "
                               f"N={N} tokens, P={P}, H={H} ({Hl} local heads), "
                               f"d={d}, batch 1, causal; per step pack and unpack of 3 x [{nl},{H},{d}] {args.elem} (one launch each) and "
                               "attention fwd+bwd",
                   "N": N, "P": P, "H": H, "local_heads": Hl, "d": d},
        "attn_fwd_bwd_tflops": (flop_fwd + flop_bwd) / (attn_ms * 1e-3) / 1e12,
        "attn_frac_of_mfma_peak": (flop_fwd + flop_bwd) / (attn_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "attn_fwd_tflops": flop_fwd / (seg_ms["attn_fwd"] * 1e-3) / 1e12,
        "attn_bwd_tflops": flop_bwd / ((attn_ms - seg_ms["attn_fwd"]) * 1e-3) / 1e12,
        "pack_gbs": pack_gbs, "pack_frac_of_hbm_peak": pack_gbs / HBM_PEAK_GBS,
        "unpack_gbs": unpack_gbs, "unpack_frac_of_hbm_peak": unpack_gbs / HBM_PEAK_GBS,
        "kernel_ms": seg_ms,
        "roofline": {"kernel": "attn_bwd_dkv_kernel", "bound": "mfma", "achieved": dkv_tflops,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": dkv_tflops / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": DKV_TRAFFIC_BYTES.get(args.config) if d == c["d"] else None},
    }

    # ---- the matrix rate the device sustains with nothing but MFMAs on the same kind of data -----
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    probe_iters = 20000
    sink = torch.empty(n_cu * 256, dtype=torch.float32, device="cuda")
    probe_args = (ptr(qkv[0]), 65536, ptr(sink), sink.numel() * 4, n_cu, probe_iters, sp)
    uly._check(lib.ulysses_probe_mfma(*probe_args), "probe_mfma")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(3):
        uly._check(lib.ulysses_probe_mfma(*probe_args), "probe_mfma")
    e1.record(stream)
    torch.cuda.synchronize()
    probe_tflops = 3 * n_cu * 4 * probe_iters * 8 * 2.0 * 32 * 32 * 16 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    result["mfma_only_tflops"] = probe_tflops
    result["roofline"]["frac_of_mfma_only_loop"] = dkv_tflops / probe_tflops
    result["attn_frac_of_mfma_only_loop"] = result["attn_fwd_bwd_tflops"] / probe_tflops
    # ... and with one operand of every MFMA read from LDS, which is how the attention kernels feed the matrix pipe
    uly._check(lib.ulysses_probe_mfma_lds(*probe_args), "probe_mfma_lds")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(3):
        uly._check(lib.ulysses_probe_mfma_lds(*probe_args), "probe_mfma_lds")
    e1.record(stream)
    torch.cuda.synchronize()
    lds_probe_tflops = 3 * n_cu * 4 * probe_iters * 8 * 2.0 * 32 * 32 * 16 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    result["mfma_lds_fed_tflops"] = lds_probe_tflops
    result["roofline"]["frac_of_lds_fed_mfma_loop"] = dkv_tflops / lds_probe_tflops

    # ---- optional: every layout transform at this workload's shapes --------------------------------
    if args.layouts:
        tb = float(nl) * H * d * 2                                   # bytes of one tensor
        hm = [torch.empty((Hl, N, d), dtype=etype, device="cuda") for _ in range(3)]       # head-major tensors
        ys = [torch.empty((nl, H, d), dtype=etype, device="cuda") for _ in range(3)]
        hm_ptrs, ys_ptrs = ptr3(hm), ptr3(ys)
        SH, HS = uly.LAYOUT_SEQ_HEAD, uly.LAYOUT_HEAD_SEQ
        cases = {
            "pack": (1, lambda: lib.ulysses_pack(ptr(xs[0]), ptr(sends[0]), nl, H, d, P, 2, sp)),
            "unpack_token_major": (1, lambda: lib.ulysses_unpack(ptr(recvs[0]), ptr(qkv[0]), nl, H, d, P, 2, SH, sp)),
            "unpack_head_major": (1, lambda: lib.ulysses_unpack(ptr(recvs[0]), ptr(hm[0]), nl, H, d, P, 2, HS, sp)),
            "pack_rev_token_major": (1, lambda: lib.ulysses_pack_rev(ptr(qkv[0]), ptr(sends[0]), nl, H, d, P, 2, SH, sp)),
            "pack_rev_head_major": (1, lambda: lib.ulysses_pack_rev(ptr(hm[0]), ptr(sends[0]), nl, H, d, P, 2, HS, sp)),
            "unpack_rev": (1, lambda: lib.ulysses_unpack_rev(ptr(recvs[0]), ptr(ys[0]), nl, H, d, P, 2, sp)),
            "pack_qkv": (3, lambda: lib.ulysses_pack_qkv(x_ptrs, send_ptrs, nl, H, d, P, 2, sp)),
            "unpack_qkv_token_major": (3, lambda: lib.ulysses_unpack_qkv(recv_ptrs, qkv_ptrs, nl, H, d, P, 2, SH, sp)),
            "unpack_qkv_head_major": (3, lambda: lib.ulysses_unpack_qkv(recv_ptrs, hm_ptrs, nl, H, d, P, 2, HS, sp)),
            "pack_rev_qkv_token_major": (3, lambda: lib.ulysses_pack_rev_qkv(qkv_ptrs, send_ptrs, nl, H, d, P, 2, SH, sp)),
            "pack_rev_qkv_head_major": (3, lambda: lib.ulysses_pack_rev_qkv(hm_ptrs, send_ptrs, nl, H, d, P, 2, HS, sp)),
            "unpack_rev_qkv": (3, lambda: lib.ulysses_unpack_rev_qkv(recv_ptrs, ys_ptrs, nl, H, d, P, 2, sp)),
        }
        # Every launch is timed on its own, after copies of other tensors (512 MiB of traffic) have pushed its
        # input out of the 256 MB last-level cache: back-to-back repeats would partly read from that cache.
        reps = 10
        result["layout_transforms"] = {"unit": "GB/s (bytes read + written)", "tensor_bytes": tb, "launches_timed": reps}
        for name, (count, call) in cases.items():
            uly._check(call(), name)
            pairs = []
            for _ in range(reps):
                grads[0].copy_(o)
                grads[1].copy_(dout)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                uly._check(call(), name)
                e1.record(stream)
                pairs.append((e0, e1))
            torch.cuda.synchronize()
            ms = sum(a.elapsed_time(b) for a, b in pairs) / reps
            result["layout_transforms"][name] = 2 * count * tb / (ms * 1e-3) / 1e9

    # ---- optional: unmasked attention of Nq queries over Nk keys (cross-attention shapes) --------
    if args.xattn:
        result["xattn"] = []
        for spec in args.xattn.split(","):
            Nq, Nk = (int(x) for x in spec.lower().split("x"))
            if not (0 < Nq <= N and 0 < Nk <= N):
                print(f"bench.py: --xattn sizes must be between 1 and N = {N}", file=sys.stderr)
                return 2
            xws = torch.empty(int(lib.ulysses_xattn_bwd_workspace_bytes(Nq, Nk, Hl, d)), dtype=torch.uint8, device="cuda")
            xfw = torch.empty(max(int(lib.ulysses_xattn_fwd_workspace_bytes(Nq, Nk, Hl, d)), 16), dtype=torch.uint8,
                              device="cuda")
            xev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

            def xattn_step():
                # the first Nq (Nk) token rows of the token-major tensors are tensors of that many tokens
                xev[0].record(stream)
                uly._check(lib.ulysses_xattn_fwd(ptr(qkv[0]), ptr(qkv[1]), ptr(qkv[2]), ptr(o), ptr(lse), ptr(xfw),
                                                 xfw.numel(), Nq, Nk, Hl, d, scale, lay, sp), "xattn_fwd")
                xev[1].record(stream)
                uly._check(lib.ulysses_xattn_bwd(ptr(qkv[0]), ptr(qkv[1]), ptr(qkv[2]), ptr(o), ptr(dout), ptr(lse),
                                                 ptr(grads[0]), ptr(grads[1]), ptr(grads[2]), ptr(xws), xws.numel(),
                                                 Nq, Nk, Hl, d, scale, lay, sp), "xattn_bwd")
                xev[2].record(stream)
            xattn_step()
            torch.cuda.synchronize()
            fwd_ms = bwd_ms = 0.0
            for _ in range(args.steps):
                xattn_step()
                torch.cuda.synchronize()
                fwd_ms += xev[0].elapsed_time(xev[1]) / args.steps
                bwd_ms += xev[1].elapsed_time(xev[2]) / args.steps
            pairs = float(Nq) * Nk * d * Hl
            result["xattn"].append({"queries": Nq, "keys": Nk, "ms_fwd": fwd_ms, "ms_bwd": bwd_ms,
                                    "fwd_tflops": 4 * pairs / (fwd_ms * 1e-3) / 1e12,
                                    "bwd_tflops": 10 * pairs / (bwd_ms * 1e-3) / 1e12,
                                    "tflops": 14 * pairs / ((fwd_ms + bwd_ms) * 1e-3) / 1e12})

    # ---- optional: block-sparse causal attention on the same tensors ---------------------------
    if args.sparse_window > 0:
        nb = (N + uly.SPARSE_BLOCK - 1) // uly.SPARSE_BLOCK
        bi, bj = np.indices((nb, nb))
        W = args.sparse_window
        if args.sparse_pattern == "fixed":
            mask = (bi // W == bj // W) | ((bj % W == W - 1) & (bj < (bi // W) * W))
            pat_name = f"windows of {W} blocks; a block row sees its own window and the last block of every earlier window"
        elif args.sparse_pattern == "global_rows":
            mask = (bi - bj < W) | (bi % 64 == 63)
            pat_name = f"window of {W} blocks; every 64th block row sees everything before it"
        else:
            mask = (bi - bj < W) | (bj == 0)
            pat_name = f"window of {W} blocks + first block column"
        pat = uly.SparsePattern(mask)
        pd = pat.dev
        sws = torch.empty(int(lib.ulysses_sparse_attn_bwd_workspace_bytes(N, Hl, d)), dtype=torch.uint8, device="cuda")
        sfw = torch.empty(int(lib.ulysses_sparse_attn_fwd_workspace_bytes(N, Hl, d)), dtype=torch.uint8, device="cuda")
        sp_ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

        def sparse_step():
            sp_ev[0].record(stream)
            uly._check(lib.ulysses_sparse_attn_fwd(ptr(qkv[0]), ptr(qkv[1]), ptr(qkv[2]), ptr(o), ptr(lse),
                                                   ptr(pd["row_ptr"]), ptr(pd["col_idx"]), ptr(sfw), sfw.numel(), N, Hl,
                                                   d, scale, lay, sp), "sparse_attn_fwd")
            sp_ev[1].record(stream)
            uly._check(lib.ulysses_sparse_attn_bwd(ptr(qkv[0]), ptr(qkv[1]), ptr(qkv[2]), ptr(o), ptr(dout), ptr(lse),
                                                   ptr(grads[0]), ptr(grads[1]), ptr(grads[2]), ptr(pd["row_ptr"]),
                                                   ptr(pd["col_idx"]), ptr(pd["col_ptr"]), ptr(pd["row_idx"]), ptr(sws),
                                                   sws.numel(), N, Hl, d, scale, lay, sp),
                       "sparse_attn_bwd")
            sp_ev[2].record(stream)
        sparse_step()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            sparse_step()
        e1.record(stream)
        torch.cuda.synchronize()
        sp_ms = e0.elapsed_time(e1) / args.steps
        # visible (query, key) pairs: full blocks count 256*256, diagonal blocks 256*257/2 (N a multiple of 256 here)
        Bk = uly.SPARSE_BLOCK
        pairs = (pat.nnz - nb) * Bk * Bk + nb * Bk * (Bk + 1) // 2
        result["sparse"] = {"pattern": f"{pat_name} (blocks of {Bk} tokens)",
                            "blocks": pat.nnz, "of_lower_triangle": pat.nnz / (nb * (nb + 1) / 2),
                            "ms_fwd_bwd": sp_ms, "ms_fwd_last_step": sp_ev[0].elapsed_time(sp_ev[1]),
                            "ms_bwd_last_step": sp_ev[1].elapsed_time(sp_ev[2]), "tflops": 14.0 * pairs * d * Hl / (sp_ms * 1e-3) / 1e12}

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    if not args.no_cpu_baseline:
        import oracle
        rows = np.unique(np.linspace(0, N - 1, args.cpu_rows).astype(np.int64))
        fq, fk, fv, fdo = (oracle.bf16_to_f64(b) for b in (q_bits, k_bits, v_bits, do_bits))
        t0 = time.perf_counter()
        oracle.attn_fwd_rows(fq, fk, fv, rows, scale, True)
        oracle.attn_bwd_rows(fq, fk, fv, fdo, rows, scale, True)
        cpu_s = time.perf_counter() - t0
        cpu_flop = 14.0 * float((rows + 1).sum()) * d * Hl       # 7 contractions x 2 flop per row/key/channel
        # layout transform of the oracle on the same [nl, H, d] tensor (bytes read + written per second)
        x_host = xs[0].view(torch.int16).cpu().numpy().view(np.uint16)
        t0 = time.perf_counter()
        oracle.pack(x_host, P)
        pack_s = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": cpu_flop / cpu_s / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"fp64 oracle forward+backward on {rows.size} evenly spaced query rows of the same tensors "
                      f"({cpu_s:.1f} s); flops counted as 14*(i+1)*d*Hl per row i",
            "pack_gbs": 2 * tensor_bytes / pack_s / 1e9,
        }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
