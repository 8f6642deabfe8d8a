#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: unpad -> ALiBi varlen attention fwd+bwd -> pad.

One "step" is one pass of the whole path over one synthetic batch that is already resident in HBM:
  mb_unpad_index(mask) -> mb_unpad(fused QKV) -> mb_alibi_attn_fwd -> mb_unpad(dO) -> mb_alibi_attn_bwd ->
  mb_pad(O), mb_pad(dQKV)    (no host synchronisation inside a step).
Prints ONE JSON line.  `value` = attention flops on real tokens (14*H*D*sum(len^2): forward QK^T and PV,
backward's five products including the recomputation of the scores) divided by the whole step time.

Beside the headline (bert_base) the line carries, per call of the path, median / p10 / p90 times and the achieved
HBM rate of the gathers and scatters (`calls`), and the attention forward / backward of the other workloads
(`configs`: bert_large, long512, ragged2048 with five draws), each warm (same buffers) and cold (buffer sets in
rotation), as TFLOP/s, % of the matrix-core peak and fraction of the roof that binds.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 matrix peak (2.5 PFLOP/s)
PEAK_HBM_GBS = 8000.0
MEASURED_COPY_GBS = 6000.0    # what a plain row copy of 1 GiB each way reaches on these boxes (bench.py --ceilings)

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this
# file (KiB per dispatch), each scaled by what the same counter reads for a plain row copy of known size
# (--copy-calibration: FETCH_SIZE reads 66060.8 KiB for 131072 KiB copied -> factor 1.984; WRITE_SIZE reads
# 131072.0 KiB -> factor 1.0).  Summaries: profiles/bert_base_attn_hbm_traffic.md.
COPY_FACTOR_FETCH = 131072.0 / 66060.8
COPY_FACTOR_WRITE = 1.0
# The counted dispatches are the token_rows variants of the two kernels (same bytes per token, and the only ones that run
# on exactly this batch's tokens in that command; the packed variants' averages mix in the padded comparison).
MEASURED_TRAFFIC_KIB = {     # workload -> kernel -> (FETCH_SIZE, WRITE_SIZE) KiB per dispatch
    "bert_base": {"attn_bwd_fused128_kernel": (102251.6, 121334.6), "attn_fwd_short_kernel": (60901.2, 41788.2)},
}
TRAFFIC_SOURCE = ("profiles/bert_base_attn_hbm_traffic.md: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                  "not measured in the run that prints this line")


def measured_traffic_bytes(workload, kernel):
    kib = MEASURED_TRAFFIC_KIB.get(workload, {}).get(kernel)
    if kib is None:
        return None
    return int(round((kib[0] * COPY_FACTOR_FETCH + kib[1] * COPY_FACTOR_WRITE) * 1024))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="bert_base")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="also time each call of the path separately")
    ap.add_argument("--batch", type=int, default=None,
                    help="override the number of sequences (same recipe); not the benchmark configuration")
    ap.add_argument("--full-length", action="store_true",
                    help="every sequence gets max_len tokens (no padding): shows what the attention kernels reach "
                         "without ragged tiles; not the benchmark configuration")
    ap.add_argument("--length-sweep", action="store_true",
                    help="also time attention forward + backward, packed against padded, at max_len 128 .. 2048 with the "
                         "same number of positions (32768) and the bert_base length recipe scaled to each max_len")
    ap.add_argument("--seeds", type=int, default=1,
                    help="also time the attention calls on this many draws of the workload's length recipe (seed offsets "
                         "0..N-1) and report the mean: the ragged workloads have few, very unequal sequences")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure this machine's ceilings with probe kernels (bf16 MFMA, fp32 FMA, fp32 exp, row copy) "
                         "and print them beside the published peaks")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="after the timed steps, run a plain row copy of known size (128 MiB in, 128 MiB out, 5 launches of "
                         "gather_rows_kernel with 65536 rows) so that HBM counters of a profiler run can be scaled")
    ap.add_argument("--no-configs", action="store_true", help="skip the other workloads (bert_large, long512, ragged2048)")
    ap.add_argument("--cpu-baseline-child", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.cpu_baseline_child:      # the oracle leg, in a process of its own that never touches the GPU
        print(json.dumps(cpu_baseline_child(args.workload, args.batch)))
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path needs no communication; every box has "
              "one GPU). --gpus %d is not supported." % args.gpus, file=sys.stderr)
        sys.exit(2)

    # The oracle is timed first, in a child process started before this one initialises the GPU: it gets the
    # host cores to itself (BLAS threads set before numpy is imported there) and cannot disturb the GPU timing.
    cpu_line = None if args.no_cpu_baseline else run_cpu_baseline(args)

    import numpy as np
    import torch
    from paper_2312_17482_amd import binding as mb      # raises if the HIP library is missing
    from paper_2312_17482_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    batch = wl.make_batch(args.workload, batch=args.batch, full_length=args.full_length)
    w = batch["workload"]
    B, L, H, D = w.B, w.L, w.H, w.D
    bf16 = w.dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    lengths = batch["lengths"]
    T_host = int(lengths.sum())
    f_fwd, f_bwd = wl.attention_flops(lengths, H, D)

    def dev_t(x):
        return torch.from_numpy(np.ascontiguousarray(x)).to(tdt).to(dev)

    mask = torch.from_numpy(batch["mask"]).to(dev)
    qkv_padded = dev_t(np.concatenate([batch[x].reshape(B * L, H * D) for x in ("q", "k", "v")], axis=1))
    do_padded = dev_t(batch["do"].reshape(B * L, H * D))
    slopes = mb.mb_alibi_slopes(H).to(dev)
    scale = batch["scale"]

    # every buffer of the step is allocated once, at capacity B*L
    cap = B * L
    qkv = torch.empty((cap, 3, H, D), dtype=tdt, device=dev)
    dout = torch.empty((cap, H, D), dtype=tdt, device=dev)
    o = torch.empty((cap, H, D), dtype=tdt, device=dev)
    dqkv = torch.empty((cap, 3, H, D), dtype=tdt, device=dev)
    o_padded = torch.empty((cap, H * D), dtype=tdt, device=dev)
    dqkv_padded = torch.empty((cap, 3 * H * D), dtype=tdt, device=dev)
    ws_bytes = mb.mb_alibi_attn_bwd_workspace_bytes(B, cap, L, H, D, mb.MB_BF16 if bf16 else mb.MB_F32)
    workspace = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)
    ws_fwd = torch.empty(max(mb.mb_alibi_attn_fwd_workspace_bytes(B, cap, L, H, D, mb.MB_BF16 if bf16 else mb.MB_F32), 16),
                         dtype=torch.uint8, device=dev)
    # the any-length kernels (max_len > 128) follow a work plan: built once per step, used by forward and backward
    use_plan = bf16 and D == 64 and L > 128
    plan = torch.empty(max(mb.mb_attn_plan_bytes(B, L, H), 16), dtype=torch.uint8, device=dev) if use_plan else None
    lse_buf = torch.empty(H * cap, dtype=torch.float32, device=dev)
    seqlens = torch.empty(B, dtype=torch.int32, device=dev)
    cu = torch.empty(B + 1, dtype=torch.int32, device=dev)
    indices = torch.empty(cap, dtype=torch.int32, device=dev)
    meta = torch.empty(2, dtype=torch.int32, device=dev)
    lib = mb.raw()
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream

    q_, k_, v_ = qkv[:, 0], qkv[:, 1], qkv[:, 2]
    lse = lse_buf.view(H, cap)

    def step(record=None, traffic_probe=False):
        def mark(i):
            if record is not None:
                record[i].record(stream)
        mark(0)
        st = lib.mb_unpad_index(mask.data_ptr(), B, L, seqlens.data_ptr(), cu.data_ptr(), indices.data_ptr(),
                                meta.data_ptr(), sp)
        assert st == 0, mb.mb_last_error()
        if use_plan:
            mb.mb_attn_plan(cu, L, H, plan=plan)
        mark(1)
        # No host round trip: the token count stays on the device (meta); the attention calls get the
        # capacity B*L as their row count and L as the bound of the sequence length.
        # (the upstream gradient is unpadded right before the backward needs it, so that the packed Q/K/V
        # just written are still in cache when the forward reads them)
        mb.mb_unpad(qkv_padded, indices, cap, meta, out=qkv.view(cap, 3 * H * D))
        mark(2)
        mb.mb_alibi_attn_fwd(q_, k_, v_, cu, L, slopes, scale, out=o, lse=lse, workspace=ws_fwd, plan=plan)
        mark(3)
        mb.mb_unpad(do_padded, indices, cap, meta, out=dout.view(cap, H * D))
        mark(4)
        if traffic_probe:   # the backward's bytes in its access pattern, no arithmetic (dqkv becomes meaningless)
            mb.mb_probe_bwd_traffic(qkv, dout, o, dqkv, cu)
        else:
            mb.mb_alibi_attn_bwd(dout, q_, k_, v_, o, lse, cu, L, slopes, scale,
                                 dq=dqkv[:, 0], dk=dqkv[:, 1], dv=dqkv[:, 2], workspace=workspace, plan=plan)
        mark(5)
        mb.mb_pad(o.view(cap, H * D), indices, cap, meta, B, L, out=o_padded)
        mark(6)
        mb.mb_pad(dqkv.view(cap, 3 * H * D), indices, cap, meta, B, L, out=dqkv_padded)
        mark(7)

    # The other workloads are measured here, right before the step (they share nothing with its buffers): the GPU
    # then goes into the step's warm-up from a second or two of work instead of from the idle start-up, with its
    # clocks where a training job has them.  (Measured: from idle, the first 20 steps of 0.2 ms run 4 % slower than
    # the steps after 200.)
    configs_out = None
    if not args.no_configs and w.name == "bert_base" and args.batch is None and not args.full_length:
        configs_out = {name: time_config(mb, wl, name, dev, seeds=5 if name == "ragged2048" else 1)
                       for name in ("bert_large", "long512", "ragged2048")}

    # `value`: exactly `steps` passes between two host synchronisations, nothing else on the stream
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev_first, ev_last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev_first.record(stream)
    for i in range(args.steps):
        step()
    ev_last.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step_on_the_stream = ev_first.elapsed_time(ev_last) / args.steps
    T, max_seqlen = mb.mb_read_meta(meta)
    assert T == T_host and max_seqlen == int(lengths.max())
    mb.mb_device_status()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    # per call: the same passes again with an event on the launch stream before and after every call
    # (the events cost a little, so these passes do not count towards `value`); median, p10, p90 over the steps
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(args.steps)]
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    # ... and once more with the traffic-only twin of the single-tile backward in its place: the same bytes in the
    # same access pattern and cache state, no arithmetic -- the ceiling of that pattern on this machine
    pattern_us = None
    if bf16 and D == 64 and L <= 128:
        ev2 = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(args.steps)]
        for i in range(args.steps):
            step(ev2[i], traffic_probe=True)
        torch.cuda.synchronize()
        pattern_us = np.array([e[4].elapsed_time(e[5]) * 1e3 for e in ev2])
        step()          # leaves real gradients in the buffers again
        torch.cuda.synchronize()
    call_names = ("unpad_index", "unpad_qkv", "attn_fwd", "unpad_do", "attn_bwd", "pad_o", "pad_dqkv")
    call_us = {name: np.array([e[i].elapsed_time(e[i + 1]) * 1e3 for e in events]) for i, name in enumerate(call_names)}

    def stats(t):
        return {"median": round(float(np.median(t)), 2), "p10": round(float(np.percentile(t, 10)), 2),
                "p90": round(float(np.percentile(t, 90)), 2)}
    fwd_ms = float(np.median(call_us["attn_fwd"])) * 1e-3
    bwd_ms = float(np.median(call_us["attn_bwd"])) * 1e-3
    esize = 2 if bf16 else 4
    W1, W3 = H * D * esize, 3 * H * D * esize
    call_bytes = {"unpad_qkv": 2 * T_host * W3, "unpad_do": 2 * T_host * W1, "pad_o": (T_host + cap) * W1,
                  "pad_dqkv": (T_host + cap) * W3}
    if use_plan:
        call_names = ("unpad_index_and_plan",) + call_names[1:]
        call_us["unpad_index_and_plan"] = call_us.pop("unpad_index")
    calls = {}
    for name in call_names:
        calls[name] = dict(stats(call_us[name]), unit="us")
        if name in call_bytes:
            gbs = call_bytes[name] / (float(np.median(call_us[name])) * 1e-6) * 1e-9
            calls[name].update(algorithmic_bytes=call_bytes[name], GBs=round(gbs, 1),
                               frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 4))
    calls["note"] = ("inside the step (cold: a step touches 1.2 GB between two uses of a buffer); gather bytes = 2*T*W*e, "
                     "scatter bytes = (T + B*L)*W*e")

    # The same path with the gather and the scatter done inside the attention kernels' own row loads and
    # stores (token_rows = indices): no packed copies at all; padding rows of the outputs are zeroed.
    qp_, kp_, vp_ = (qkv_padded.view(cap, 3, H, D)[:, i] for i in range(3))
    dop_ = do_padded.view(cap, H, D)
    op_ = o_padded.view(cap, H, D)
    dqkvp_ = dqkv_padded.view(cap, 3, H, D)

    def fused_step():
        st = lib.mb_unpad_index(mask.data_ptr(), B, L, seqlens.data_ptr(), cu.data_ptr(), indices.data_ptr(),
                                meta.data_ptr(), sp)
        assert st == 0, mb.mb_last_error()
        if use_plan:
            mb.mb_attn_plan(cu, L, H, plan=plan)
        mb.mb_alibi_attn_fwd(qp_, kp_, vp_, cu, L, slopes, scale, out=op_, lse=lse, token_rows=indices, T=cap,
                             workspace=ws_fwd, plan=plan)
        mb.mb_zero_padding(o_padded, indices, cap, meta, B, L)
        mb.mb_alibi_attn_bwd(dop_, qp_, kp_, vp_, op_, lse, cu, L, slopes, scale, dq=dqkvp_[:, 0], dk=dqkvp_[:, 1],
                             dv=dqkvp_[:, 2], workspace=workspace, token_rows=indices, T=cap, plan=plan)
        mb.mb_zero_padding(dqkv_padded, indices, cap, meta, B, L)

    ref_o, ref_g = o_padded.clone(), dqkv_padded.clone()
    for _ in range(args.warmup):
        fused_step()
    torch.cuda.synchronize()
    assert torch.equal(ref_o, o_padded) and torch.equal(ref_g, dqkv_padded), "fused path differs from explicit path"
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fused_step()
    torch.cuda.synchronize()
    ms_fused = (time.perf_counter() - t0) * 1e3 / args.steps

    value = (f_fwd + f_bwd) / (ms_per_step * 1e-3) * 1e-12
    # algorithmic HBM bytes of one backward launch: dO, Q, K, V, O read and dQ, dK, dV written once each
    # ([T,H,D] elements) plus the row log-sum-exp read ([H,T] float)
    bwd_bytes = 8 * T_host * H * D * esize + 4 * H * T_host
    if bf16 and D == 64:
        bwd_kernel = "attn_bwd_fused128_kernel" if L <= 128 else "attn_bwd_dkv_kernel + attn_bwd_dq_kernel + attn_bwd_delta_kernel"
    else:
        bwd_kernel = "bwd_generic_row_kernel + bwd_generic_col_kernel"
    roof_hbm = {
        "kernel": bwd_kernel, "bound": "hbm",
        "achieved": round(bwd_bytes / (bwd_ms * 1e-3) * 1e-9, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": round(bwd_bytes / (bwd_ms * 1e-3) * 1e-9 / PEAK_HBM_GBS, 5),
        "algorithmic_bytes": bwd_bytes, "traffic": measured_traffic_bytes(w.name, bwd_kernel),
        "traffic_source": TRAFFIC_SOURCE if measured_traffic_bytes(w.name, bwd_kernel) is not None else None,
        "launch_us": stats(call_us["attn_bwd"]),
        "frac_of_measured_copy_rate": round(bwd_bytes / (bwd_ms * 1e-3) * 1e-9 / MEASURED_COPY_GBS, 4),
    }
    if pattern_us is not None:
        pat = float(np.median(pattern_us))
        roof_hbm["traffic_only_twin"] = {
            "what": "mb_probe_bwd_traffic in the backward's place inside the step: same bytes, same 8 row streams, no arithmetic",
            "launch_us": stats(pattern_us), "GBs": round(bwd_bytes / (pat * 1e-6) * 1e-9, 1),
            "kernel_frac_of_it": round(pat * 1e-3 / bwd_ms, 4)}
    roof_mfma = {
        "kernel": bwd_kernel, "bound": "mfma",
        "achieved": round(f_bwd / (bwd_ms * 1e-3) * 1e-12, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
        "frac": round(f_bwd / (bwd_ms * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 5),
        "algorithmic_flops": f_bwd, "flop_per_byte": round(f_bwd / bwd_bytes, 1), "traffic": None,
    }
    hbm_binds = f_bwd / bwd_bytes < PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    roof_primary, roof_other = (roof_hbm, roof_mfma) if hbm_binds else (roof_mfma, roof_hbm)

    out = {
        "metric": "ALiBi varlen attention fwd+bwd TFLOP/s (whole unpad->attention->pad step)",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s%s: B=%d L=%d H=%d D=%d, T=%d real tokens, sum(len^2)=%d" % (
            w.name, " (all sequences full length)" if args.full_length else "", B, L, H, D, T_host,
            int((lengths.astype(np.int64) ** 2).sum()))},
        "tokens_per_s": round(T_host / (ms_per_step * 1e-3), 1),
        # the same K steps between two events on the launch stream: without the host's share of the bracket
        # (the first launch after a synchronisation, the return of the last one), which a short run does not amortise
        "ms_per_step_between_stream_events": round(ms_per_step_on_the_stream, 5),
        "pct_of_bf16_mfma_peak": round(100.0 * value / PEAK_BF16_TFLOPS, 3),
        "attention_only": {
            "timing": "median over the steps of the event-bracketed calls inside the step (cold)",
            "fwd_ms": round(fwd_ms, 5), "bwd_ms": round(bwd_ms, 5),
            "fwd_tflops": round(f_fwd / (fwd_ms * 1e-3) * 1e-12, 2),
            "bwd_tflops": round(f_bwd / (bwd_ms * 1e-3) * 1e-12, 2),
            "fwd_bwd_tflops": round((f_fwd + f_bwd) / ((fwd_ms + bwd_ms) * 1e-3) * 1e-12, 2),
            "fwd_bwd_tflops_no_recompute_convention": round((f_fwd + f_bwd) * 12.0 / 14.0 / ((fwd_ms + bwd_ms) * 1e-3) * 1e-12, 2),
            "pct_of_bf16_mfma_peak": round(100.0 * (f_fwd + f_bwd) / ((fwd_ms + bwd_ms) * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS, 3),
        },
        # Dominant kernel: the backward attention.  `roofline` prices it against the roof that binds at this
        # workload's arithmetic intensity (flops per algorithmic byte against the machine balance of
        # 2500 TFLOP/s : 8 TB/s = 312 flop/byte); `roofline_other` gives the other roof.
        "roofline": roof_primary, "roofline_other": roof_other,
        "calls": calls,
        "gather_scatter_fused_into_attention": {
            "ms_per_step": round(ms_fused, 5), "value": round((f_fwd + f_bwd) / (ms_fused * 1e-3) * 1e-12, 3),
            "unit": "TFLOP/s", "tokens_per_s": round(T_host / (ms_fused * 1e-3), 1),
            "note": "same inputs and bit-identical padded outputs; mb_unpad/mb_pad replaced by token_rows + mb_zero_padding",
        },
        "paper_context": "MosaicBERT-Base: 79.6 GLUE in 1.13 h on 8xA100-80GB (end-to-end pretraining; not comparable)",
    }

    out["next_rows"] = {"add_layernorm_bf16": time_layernorm(mb, T_host, H * D, tdt, dev, indices, B, L),
                        "padded_attention_comparison": time_padded_vs_varlen(mb, locals())}
    if bf16 and (H * D) % 256 == 0:
        out["next_rows"]["geglu_ffn_bf16"] = time_geglu(mb, T_host, H * D, 4 * H * D, dev)
        out["next_rows"]["mlm_head_on_masked_rows"] = time_mlm_head(mb, T_host, H * D, dev)
    if args.detail:
        out["detail_us"] = time_each_call(mb, lib, locals())
    if args.length_sweep or (not args.no_configs and w.name == "bert_base" and args.batch is None):
        out["next_rows"]["length_sweep_padded_vs_varlen"] = time_length_sweep(mb, wl, dev)
    if args.seeds > 1:
        out["attention_over_seeds"] = time_attention_over_seeds(mb, wl, args, dev)
    if args.ceilings:
        out["measured_ceilings"] = measure_ceilings(mb, dev)
    if args.copy_calibration:
        rows, width = 65536, 1024                      # 65536 rows x 2048 bytes = 128 MiB each way
        src = torch.ones((rows, width), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        ident = torch.arange(rows, dtype=torch.int32, device=dev)
        for _ in range(5):
            mb.mb_unpad(src, ident, rows, None, out=dst)
        torch.cuda.synchronize()
        out["copy_calibration"] = "5 x gather_rows_kernel grid=%d: reads 131072 KiB, writes 131072 KiB per launch" % (rows // 8)

    if configs_out is not None:
        out["configs"] = configs_out
    if cpu_line is not None:
        out["cpu_baseline"] = cpu_line
    print(json.dumps(out))


def time_layernorm(mb, T, W, tdt, dev, indices, B, L):
    """Add & LayerNorm on the packed tokens of the same batch ([T, H*D]), outside the timed step: 50 launches
    between two events.  Algorithmic bytes: forward reads x, r and writes s, y (4 T W e); backward reads dy, s
    and writes ds (3 T W e).  Also the last operation of an encoder stack writing the padded batch itself
    (y_rows = indices, then mb_zero_padding) against LayerNorm followed by mb_pad."""
    import torch
    e = 2 if tdt == torch.bfloat16 else 4
    x = torch.randn(T, W, device=dev).to(tdt)
    r = torch.randn(T, W, device=dev).to(tdt)
    gamma = torch.ones(W, device=dev).to(tdt)
    beta = torch.zeros(W, device=dev).to(tdt)
    dy = torch.randn(T, W, device=dev).to(tdt)
    y, s, ds = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    mean = torch.empty(T, dtype=torch.float32, device=dev)
    rstd = torch.empty(T, dtype=torch.float32, device=dev)
    dg = torch.empty(W, dtype=torch.float32, device=dev)
    db = torch.empty(W, dtype=torch.float32, device=dev)
    ws = torch.empty(mb.mb_add_layernorm_bwd_workspace_bytes(W), dtype=torch.uint8, device=dev)
    fwd = lambda: mb.mb_add_layernorm_fwd(x, r, gamma, beta, 1e-5, y=y, s=s, mean=mean, rstd=rstd)
    bwd = lambda: mb.mb_add_layernorm_bwd(dy, s, gamma, mean, rstd, ds=ds, dgamma=dg, dbeta=db, workspace=ws)
    res = {}
    for name, fn, nbytes in (("fwd", fwd, 4 * T * W * e + 8 * T), ("bwd", bwd, 3 * T * W * e + 8 * T)):
        for _ in range(5):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(50):
            fn()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / 50
        res[name + "_us"] = round(us, 2)
        res[name + "_GBs"] = round(nbytes / (us * 1e-6) * 1e-9, 1)
        res[name + "_frac_of_hbm_peak"] = round(nbytes / (us * 1e-6) * 1e-9 / PEAK_HBM_GBS, 4)
    y_padded = torch.empty((B * L, W), dtype=tdt, device=dev)
    then_pad = lambda: (fwd(), mb.mb_pad(y, indices, T, None, B, L, out=y_padded))
    scattering = lambda: (mb.mb_add_layernorm_fwd(x, r, gamma, beta, 1e-5, y=y_padded, s=s, mean=mean, rstd=rstd,
                                                  y_rows=indices),
                          mb.mb_zero_padding(y_padded, indices, T, None, B, L))
    for name, fn in (("fwd_then_pad_us", then_pad), ("fwd_writing_the_padded_batch_us", scattering)):
        for _ in range(5):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(50):
            fn()
        b.record()
        torch.cuda.synchronize()
        res[name] = round(a.elapsed_time(b) * 1e3 / 50, 2)
    res["shape"] = "T=%d W=%d" % (T, W)
    return res


def time_mlm_head(mb, T, hidden, dev, vocab=30528, mask_ratio=0.30):
    """The output projection to the vocabulary on the masked token rows only ("Vocab Size as a Multiple of
    64" paragraph: 30528; the training recipe masks 30 % of the tokens): mb_unpad gathers the masked rows of
    the packed activations, mb_linear_fwd projects them; against projecting every token.  20 launches each
    between two events after a warm-up; the logits buffers are scratch."""
    import torch
    bf = torch.bfloat16
    x = torch.randn(T, hidden, device=dev).to(bf)
    wv = (torch.randn(vocab, hidden, device=dev) * 0.02).to(bf)
    n_masked = int(round(T * mask_ratio))
    rows = torch.sort(torch.randperm(T, device=dev)[:n_masked]).values.to(torch.int32)
    xm = torch.empty((n_masked, hidden), dtype=bf, device=dev)
    logits_m = torch.empty((n_masked, vocab), dtype=bf, device=dev)
    logits_all = torch.empty((T, vocab), dtype=bf, device=dev)

    def masked():
        mb.mb_unpad(x, rows, n_masked, None, out=xm)
        mb.mb_linear_fwd(xm, wv, y=logits_m)

    def every():
        mb.mb_linear_fwd(x, wv, y=logits_all)

    res = {"shape": "T=%d hidden=%d vocab=%d masked_rows=%d" % (T, hidden, vocab, n_masked)}
    for name, fn, nrows in (("masked_rows", masked, n_masked), ("all_rows", every, T)):
        for _ in range(20):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(20):
            fn()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / 20
        res[name + "_us"] = round(us, 1)
        res[name + "_tflops"] = round(2.0 * nrows * hidden * vocab / us * 1e-6, 1)
    res["speedup_from_masked_rows_only"] = round(res["all_rows_us"] / res["masked_rows_us"], 2)
    return res


def time_length_sweep(mb, wl, dev, H=12, D=64, positions=32768):
    """What removing padding saves in attention as max_len grows (the paper's own code ran attention over the
    padded batch; its appendix on sequence length trains at 128 .. 2048).  For each max_len L: B = 32768 / L
    sequences, lengths by the bert_base recipe scaled to L (L with probability 0.6, else uniform in
    [L/8, L-1]; NumPy default_rng(20231217 + L)), Q, K, V ~ N(0,1)/8; forward + backward on the packed tokens
    (`varlen`) and on the padded batch with a key-padding mask (`padded`: all B*L positions are queries, key_lens =
    the lengths), 10 launches each between two events."""
    import numpy as np
    import torch
    bf = torch.bfloat16
    rows = []
    for L in (128, 256, 512, 1024, 2048):
        B = positions // L
        rng = np.random.default_rng(20231217 + L)
        full = rng.random(B) < 0.6
        lengths = np.where(full, L, rng.integers(L // 8, L, size=B)).astype(np.int32)
        T = int(lengths.sum())
        f_fwd, f_bwd = wl.attention_flops(lengths, H, D)
        slopes = mb.mb_alibi_slopes(H).to(dev)
        res = {"max_len": L, "B": B, "T": T, "fraction_real": round(T / positions, 4)}
        for name, lens, klens in (("varlen", lengths, None), ("padded", np.full(B, L, dtype=np.int32), lengths)):
            n_tok = int(lens.sum())
            cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).to(dev)
            kl = None if klens is None else torch.from_numpy(klens).to(dev)
            qkv = (torch.randn(n_tok, 3, H, D, device=dev) * 0.125).to(bf)
            do = torch.randn(n_tok, H, D, device=dev).to(bf)
            o = torch.empty(n_tok, H, D, dtype=bf, device=dev)
            lse = torch.empty(H, n_tok, dtype=torch.float32, device=dev)
            dqkv = torch.empty_like(qkv)
            ws = torch.empty(max(mb.mb_alibi_attn_bwd_workspace_bytes(B, n_tok, L, H, D, mb.MB_BF16), 16), dtype=torch.uint8,
                             device=dev)
            ws_f = torch.empty(max(mb.mb_alibi_attn_fwd_workspace_bytes(B, n_tok, L, H, D, mb.MB_BF16), 16), dtype=torch.uint8,
                               device=dev)

            def run():
                mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, L, slopes, 0.125, out=o, lse=lse, workspace=ws_f,
                                     key_lens=kl)
                mb.mb_alibi_attn_bwd(do, qkv[:, 0], qkv[:, 1], qkv[:, 2], o, lse, cu, L, slopes, 0.125, dq=dqkv[:, 0],
                                     dk=dqkv[:, 1], dv=dqkv[:, 2], workspace=ws, key_lens=kl)
            for _ in range(3):
                run()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(10):
                run()
            b.record()
            torch.cuda.synchronize()
            res[name + "_fwd_bwd_us"] = round(a.elapsed_time(b) * 1e3 / 10, 1)
        res["varlen_tflops"] = round((f_fwd + f_bwd) / res["varlen_fwd_bwd_us"] * 1e-6, 1)
        res["speedup_from_unpadding"] = round(res["padded_fwd_bwd_us"] / res["varlen_fwd_bwd_us"], 3)
        rows.append(res)
    return rows


def time_config(mb, wl, name, dev, seeds=1, launches=60):
    """Attention forward and backward of another workload, called the way the step calls them (packed buffers of
    capacity B*L, max_seqlen = L, nothing read back from the device).  Per draw of the workload's recipe:
    `launches` launches each bracketed by its own pair of events on the launch stream, median / p10 / p90;
    warm = the same buffers every launch, cold = four independent buffer sets in rotation (for the small
    ragged batch what a launch reads may still sit in the 256 MB Infinity Cache either way: both are given).
    TFLOP/s by the 4*H*D*sum(len^2) / 10*H*D*sum(len^2) conventions; `roof` = min(matrix-core peak, flops per
    algorithmic byte x 8 TB/s) for forward + backward together."""
    import numpy as np
    import torch
    draws = []
    for s_off in range(seeds):
        batch = wl.make_batch(name, seed_offset=s_off)
        w = batch["workload"]
        B, L, H, D = w.B, w.L, w.H, w.D
        cap = B * L
        bf = torch.bfloat16
        lengths = batch["lengths"]
        T = int(lengths.sum())
        f_fwd, f_bwd = wl.attention_flops(lengths, H, D)
        mask = torch.from_numpy(batch["mask"]).to(dev)
        seqlens, cu, indices, meta = mb.mb_unpad_index(mask)
        slopes = mb.mb_alibi_slopes(H).to(dev)
        qkv_padded = torch.from_numpy(np.concatenate([batch[x].reshape(cap, H * D) for x in ("q", "k", "v")], axis=1)).to(bf).to(dev)
        do_padded = torch.from_numpy(np.ascontiguousarray(batch["do"].reshape(cap, H * D))).to(bf).to(dev)
        sets = []
        for _ in range(4):
            qkv = mb.mb_unpad(qkv_padded, indices, cap, meta).view(cap, 3, H, D)
            dout = mb.mb_unpad(do_padded, indices, cap, meta).view(cap, H, D)
            sets.append((qkv, dout, torch.empty((cap, H, D), dtype=bf, device=dev), torch.empty_like(qkv)))
        del qkv_padded, do_padded
        lse = torch.empty((H, cap), dtype=torch.float32, device=dev)
        ws_f = torch.empty(max(16, mb.mb_alibi_attn_fwd_workspace_bytes(B, cap, L, H, D, mb.MB_BF16)), dtype=torch.uint8, device=dev)
        ws_b = torch.empty(max(16, mb.mb_alibi_attn_bwd_workspace_bytes(B, cap, L, H, D, mb.MB_BF16)), dtype=torch.uint8, device=dev)

        # the any-length kernels' work plan is built once per batch (it serves every attention call on the batch:
        # all layers, forward and backward); its own time is reported beside the calls
        plan = mb.mb_attn_plan(cu, L, H) if L > 128 else None

        def fwd(x, do_, o_, dx):
            mb.mb_alibi_attn_fwd(x[:, 0], x[:, 1], x[:, 2], cu, L, slopes, batch["scale"], out=o_, lse=lse, workspace=ws_f,
                                 plan=plan)

        def bwd(x, do_, o_, dx):
            mb.mb_alibi_attn_bwd(do_, x[:, 0], x[:, 1], x[:, 2], o_, lse, cu, L, slopes, batch["scale"], dq=dx[:, 0],
                                 dk=dx[:, 1], dv=dx[:, 2], workspace=ws_b, plan=plan)

        def measure(fn, rotate):
            for i in range(6):
                fn(*sets[i % 4 if rotate else 0])
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(launches)]
            for i, (a, b) in enumerate(evs):
                a.record()
                fn(*sets[i % 4 if rotate else 0])
                b.record()
            torch.cuda.synchronize()
            t = np.array([a.elapsed_time(b) * 1e3 for a, b in evs])
            return {"median": round(float(np.median(t)), 2), "p10": round(float(np.percentile(t, 10)), 2),
                    "p90": round(float(np.percentile(t, 90)), 2)}
        for st in sets:                      # every set holds its own forward results before any backward is timed
            fwd(*st)
        row = {"seed_offset": s_off, "T": T, "sum_len2": int((lengths.astype(np.int64) ** 2).sum()), "max_len": int(lengths.max())}
        if plan is not None:
            row["plan_once_per_batch_us"] = measure(lambda *a: mb.mb_attn_plan(cu, L, H, plan=plan), False)
        for temp, rotate in (("warm", False), ("cold", True)):
            tf, tb = measure(fwd, rotate), measure(bwd, rotate)
            row[temp] = {"fwd_us": tf, "bwd_us": tb,
                         "fwd_tflops": round(f_fwd / tf["median"] * 1e-6, 1), "bwd_tflops": round(f_bwd / tb["median"] * 1e-6, 1),
                         "fwd_bwd_tflops": round((f_fwd + f_bwd) / (tf["median"] + tb["median"]) * 1e-6, 1)}
        mb.mb_device_status()
        nbytes = 12 * T * H * D * 2 + 2 * T * H * 4
        row["flop_per_byte"] = round((f_fwd + f_bwd) / nbytes, 1)
        roof = min(PEAK_BF16_TFLOPS, (f_fwd + f_bwd) / nbytes * PEAK_HBM_GBS * 1e-3)
        row["roof_tflops"] = round(roof, 1)
        row["roof"] = "mfma" if roof >= PEAK_BF16_TFLOPS else "hbm"
        for temp in ("warm", "cold"):
            row[temp]["pct_of_bf16_mfma_peak"] = round(100.0 * row[temp]["fwd_bwd_tflops"] / PEAK_BF16_TFLOPS, 2)
            row[temp]["frac_of_roof"] = round(row[temp]["fwd_bwd_tflops"] / roof, 4)
        draws.append(row)
        del sets
    res = {"shape": "B=%d L=%d H=%d D=%d" % (B, L, H, D), "draws": draws}
    if seeds > 1:
        for temp in ("warm", "cold"):
            res["mean_over_draws_" + temp] = {k: round(float(np.mean([d[temp][k] for d in draws])), 1)
                                              for k in ("fwd_tflops", "bwd_tflops", "fwd_bwd_tflops", "pct_of_bf16_mfma_peak")}
    return res


def time_attention_over_seeds(mb, wl, args, dev):
    """Attention forward and backward on several draws of the workload (packed inputs prepared outside the timed
    region; 20 launches of each between two events per draw)."""
    import numpy as np
    import torch
    rows = []
    for s in range(args.seeds):
        batch = wl.make_batch(args.workload, seed_offset=s, batch=args.batch, full_length=args.full_length)
        w = batch["workload"]
        B, L, H, D = w.B, w.L, w.H, w.D
        tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        lengths = batch["lengths"]
        f_fwd, f_bwd = wl.attention_flops(lengths, H, D)
        mask = torch.from_numpy(batch["mask"]).to(dev)
        seqlens, cu, indices, meta = mb.mb_unpad_index(mask)
        T, _ = mb.mb_read_meta(meta)
        cap = B * L
        packed = {}
        for key in ("q", "k", "v", "do"):
            t = torch.from_numpy(np.ascontiguousarray(batch[key].reshape(cap, H * D))).to(tdt).to(dev)
            packed[key] = mb.mb_unpad(t, indices, cap, meta)[:T].view(T, H, D)
        slopes = mb.mb_alibi_slopes(H).to(dev)
        o, lse = mb.mb_alibi_attn_fwd(packed["q"], packed["k"], packed["v"], cu, L, slopes, batch["scale"])
        dq, dk, dv = (torch.empty_like(packed["q"]) for _ in range(3))
        ws = torch.empty(max(mb.mb_alibi_attn_bwd_workspace_bytes(B, T, L, H, D, mb.MB_BF16 if w.dtype == "bf16" else mb.MB_F32), 16),
                         dtype=torch.uint8, device=dev)
        ws_f = torch.empty(max(mb.mb_alibi_attn_fwd_workspace_bytes(B, T, L, H, D, mb.MB_BF16 if w.dtype == "bf16" else mb.MB_F32), 16),
                           dtype=torch.uint8, device=dev)
        fwd = lambda: mb.mb_alibi_attn_fwd(packed["q"], packed["k"], packed["v"], cu, L, slopes, batch["scale"], out=o, lse=lse,
                                           workspace=ws_f)
        bwd = lambda: mb.mb_alibi_attn_bwd(packed["do"], packed["q"], packed["k"], packed["v"], o, lse, cu, L, slopes,
                                           batch["scale"], dq=dq, dk=dk, dv=dv, workspace=ws)
        t_us = []
        for fn in (fwd, bwd):
            for _ in range(3):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(20):
                fn()
            b.record()
            torch.cuda.synchronize()
            t_us.append(a.elapsed_time(b) * 1e3 / 20)
        rows.append({"seed_offset": s, "T": int(T), "sum_len2": int((lengths.astype(np.int64) ** 2).sum()),
                     "fwd_us": round(t_us[0], 1), "bwd_us": round(t_us[1], 1),
                     "fwd_tflops": round(f_fwd / t_us[0] * 1e-6, 1), "bwd_tflops": round(f_bwd / t_us[1] * 1e-6, 1)})
    return {"draws": rows, "mean_fwd_tflops": round(float(np.mean([r["fwd_tflops"] for r in rows])), 1),
            "mean_bwd_tflops": round(float(np.mean([r["bwd_tflops"] for r in rows])), 1)}


def measure_ceilings(mb, dev):
    """Probe kernels that saturate one unit each (3 warm-up + 10 timed launches between two events), and a plain
    row copy through the gather kernel, once with 128 MiB each way (as large as the 256 MB Infinity Cache) and once
    with 1 GiB each way (far beyond it)."""
    import torch
    scratch = torch.zeros(4, dtype=torch.float32, device=dev)
    res = {}
    for name, kind, iters, unit, scale in (("mfma_bf16_32x32x16", 0, 2000, "TFLOP/s", 1e-12),
                                           ("valu_fp32_fma", 1, 20000, "TFLOP/s", 1e-12),
                                           ("valu_fp32_exp", 2, 5000, "Texp/s", 1e-12)):
        for _ in range(3):
            work = mb.mb_probe_ceiling(kind, iters, scratch)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            mb.mb_probe_ceiling(kind, iters, scratch)
        b.record()
        torch.cuda.synchronize()
        res[name] = {"value": round(work * 10 / (a.elapsed_time(b) * 1e-3) * scale, 2), "unit": unit}
    for label, rows in (("hbm_copy_128MiB_each_way", 65536), ("hbm_copy_1GiB_each_way", 524288)):
        width = 1024                                    # 2048-byte rows
        src = torch.ones((rows, width), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        ident = torch.arange(rows, dtype=torch.int32, device=dev)
        for _ in range(3):
            mb.mb_unpad(src, ident, rows, None, out=dst)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            mb.mb_unpad(src, ident, rows, None, out=dst)
        b.record()
        torch.cuda.synchronize()
        res[label] = {"value": round(2 * rows * width * 2 * 10 / (a.elapsed_time(b) * 1e-3) * 1e-9, 1),
                      "unit": "GB/s (read + write)"}
        del src, dst
    res["published_peaks"] = {"mfma_bf16": "2500 TFLOP/s", "valu_fp32": "157.3 TFLOP/s (with packed instructions; "
                              "this build disables them: 78.6)", "hbm": "8000 GB/s"}
    return res


def time_geglu(mb, T, hidden, inter, dev):
    """GeGLU feed-forward, forward, on the packed tokens of the same batch ([T, hidden] -> [T, inter] ->
    [T, hidden]), outside the timed step: 20 launches of each arrangement between two events, after a warm-up.
    fused = mb_geglu_fwd (the activation runs on the accumulators of the first projection); the two
    unfused arrangements of the paper's appendix on GLU implementations are built from the same GEMM
    kernel: `sliced` = one double-width projection stored and sliced, `separate` = two projections; both
    then run the activation as a pass of its own.  Flops: 2 T hidden 2 inter + 2 T inter hidden."""
    import torch
    bf = torch.bfloat16
    x = torch.randn(T, hidden, device=dev).to(bf)
    w1v = (torch.randn(2 * inter, hidden, device=dev) * 0.02).to(bf)
    w1, v = w1v[:inter].contiguous(), w1v[inter:].contiguous()
    w2 = (torch.randn(hidden, inter, device=dev) * 0.02).to(bf)
    act = torch.empty((T, inter), dtype=bf, device=dev)
    y = torch.empty((T, hidden), dtype=bf, device=dev)
    hg = torch.empty((T, 2 * inter), dtype=bf, device=dev)
    h, g = torch.empty((T, inter), dtype=bf, device=dev), torch.empty((T, inter), dtype=bf, device=dev)

    def fused():
        mb.mb_geglu_fwd(x, w1v, w2, act=act, y=y)

    def sliced():
        mb.mb_linear_fwd(x, w1v, y=hg)
        mb.mb_gelu_gate(hg[:, :inter], hg[:, inter:], act=act)
        mb.mb_linear_fwd(act, w2, y=y)

    def separate():
        mb.mb_linear_fwd(x, w1, y=h)
        mb.mb_linear_fwd(x, v, y=g)
        mb.mb_gelu_gate(h, g, act=act)
        mb.mb_linear_fwd(act, w2, y=y)

    flops = 2.0 * T * hidden * 2 * inter + 2.0 * T * inter * hidden
    res = {"shape": "T=%d hidden=%d inter=%d" % (T, hidden, inter)}
    # Steady state: the clocks of this part take some 50 to 100 ms of matrix-core load to settle (the first
    # launches after the memory-bound attention step run about 15 % slower), so 200 untimed launches go first.
    for _ in range(200):
        fused()
    for name, fn in (("fused", fused), ("sliced", sliced), ("separate", separate)):
        for _ in range(10):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(20):
            fn()
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / 20
        res[name + "_us"] = round(us, 1)
        res[name + "_tflops"] = round(flops / us * 1e-6, 1)
    # backward: data gradient and fp32 weight gradients; flops 2 T hidden inter x (dA 1 + dx 2 + dW2 1 + dW1V 2),
    # plus 2 more units when x W1 | x V are computed again (fused forward) instead of handed over (sliced forward)
    dyt = torch.randn(T, hidden, device=dev).to(bf)
    dx = torch.empty_like(x)
    dw1v = torch.empty((2 * inter, hidden), dtype=torch.float32, device=dev)
    dw2 = torch.empty((hidden, inter), dtype=torch.float32, device=dev)
    ws = torch.empty(mb.mb_geglu_bwd_workspace_bytes(T, hidden, inter), dtype=torch.uint8, device=dev)
    mb.mb_linear_fwd(x, w1v, y=hg)
    unit = 2.0 * T * hidden * inter
    for name, saved, units in (("bwd_recompute", None, 8.0), ("bwd_stored_projections", hg, 6.0)):
        for _ in range(10):
            mb.mb_geglu_bwd(dyt, x, w1v, w2, act, hg=saved, dx=dx, dw1v=dw1v, dw2=dw2, workspace=ws)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            mb.mb_geglu_bwd(dyt, x, w1v, w2, act, hg=saved, dx=dx, dw1v=dw1v, dw2=dw2, workspace=ws)
        b.record()
        torch.cuda.synchronize()
        us = a.elapsed_time(b) * 1e3 / 10
        res[name + "_us"] = round(us, 1)
        res[name + "_tflops"] = round(units * unit / us * 1e-6, 1)
    res["frac_of_bf16_mfma_peak"] = round(res["fused_tflops"] / PEAK_BF16_TFLOPS, 4)
    res["unfused_slowdown"] = {"sliced": round(res["sliced_us"] / res["fused_us"], 3),
                               "separate": round(res["separate_us"] / res["fused_us"], 3)}
    return res


def time_padded_vs_varlen(mb, g):
    """What removing padding saves in attention itself: the same kernels on the same batch, once over the
    packed real tokens (cu_seqlens from the mask) and once over the padded [B, L] batch with a key-padding mask
    as the paper's own code ran attention (every position a query, key_lens = the real lengths; parity of that
    mode is a GPU test).  Forward + backward, 30 launches each between two events; outputs of the padded run are
    scratch."""
    import torch
    B, L, H, D, cap = g["B"], g["L"], g["H"], g["D"], g["cap"]
    dev = g["dev"]
    qkv_packed, dout_packed = g["qkv"], g["dout"]
    qkv_full = g["qkv_padded"].view(cap, 3, H, D)
    do_full = g["do_padded"].view(cap, H, D)
    cu_full = torch.arange(0, cap + 1, L, dtype=torch.int32, device=dev)
    o, lse, dqkv, ws = g["o"], g["lse"], g["dqkv"], g["workspace"]
    slopes, scale = g["slopes"], g["scale"]
    res = {}
    for name, x, do_, cu_, kl in (("varlen", qkv_packed, dout_packed, g["cu"], None),
                                  ("padded", qkv_full, do_full, cu_full, g["seqlens"])):
        def run():
            mb.mb_alibi_attn_fwd(x[:, 0], x[:, 1], x[:, 2], cu_, L, slopes, scale, out=o, lse=lse, workspace=g["ws_fwd"],
                                 key_lens=kl)
            mb.mb_alibi_attn_bwd(do_, x[:, 0], x[:, 1], x[:, 2], o, lse, cu_, L, slopes, scale,
                                 dq=dqkv[:, 0], dk=dqkv[:, 1], dv=dqkv[:, 2], workspace=ws, key_lens=kl)
        for _ in range(3):
            run()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(30):
            run()
        b.record()
        torch.cuda.synchronize()
        res[name + "_fwd_bwd_us"] = round(a.elapsed_time(b) * 1e3 / 30, 2)
    res["speedup_from_unpadding"] = round(res["padded_fwd_bwd_us"] / res["varlen_fwd_bwd_us"], 3)
    res["fraction_of_positions_that_are_real"] = round(g["T_host"] / cap, 4)
    return res


def time_each_call(mb, lib, env):
    """Each call of the path alone.  Per call: 100 launches each bracketed by its own pair of events (median,
    p10, p90) and 50 back-to-back launches between one pair (`loop`, amortises the event overhead).  These
    are WARM figures (the same buffers every launch; the 256 MB Infinity Cache helps).  `cold` repeats the
    attention calls over 4 independent buffer sets (1.3 GB in total) used in rotation, so that nothing a
    launch reads is left in any cache by the previous use: that is the situation inside a training step, and
    what the timed step of the main line measures."""
    import numpy as np
    import torch
    g = env
    T, _ = mb.mb_read_meta(g["meta"])
    B, L, H, D, cap = g["B"], g["L"], g["H"], g["D"], g["cap"]
    qkv, dout, o, dqkv = g["qkv"], g["dout"], g["o"], g["dqkv"]
    q_, k_, v_, lse, max_seqlen = g["q_"], g["k_"], g["v_"], g["lse"], L

    def fwd(x=qkv, o_=o):
        mb.mb_alibi_attn_fwd(x[:, 0], x[:, 1], x[:, 2], g["cu"], max_seqlen, g["slopes"], g["scale"], out=o_, lse=lse)

    def bwd(x=qkv, do_=dout, o_=o, dx=dqkv):
        mb.mb_alibi_attn_bwd(do_, x[:, 0], x[:, 1], x[:, 2], o_, lse, g["cu"], max_seqlen, g["slopes"], g["scale"],
                             dq=dx[:, 0], dk=dx[:, 1], dv=dx[:, 2], workspace=g["workspace"])

    calls = {
        "unpad_index": lambda: lib.mb_unpad_index(g["mask"].data_ptr(), B, L, g["seqlens"].data_ptr(), g["cu"].data_ptr(),
                                                  g["indices"].data_ptr(), g["meta"].data_ptr(), g["sp"]),
        "unpad_qkv": lambda: mb.mb_unpad(g["qkv_padded"], g["indices"], cap, g["meta"], out=qkv.view(cap, 3 * H * D)),
        "unpad_do": lambda: mb.mb_unpad(g["do_padded"], g["indices"], cap, g["meta"], out=dout.view(cap, H * D)),
        "attn_fwd": fwd,
        "attn_bwd": bwd,
        "attn_fwd_bwd": lambda: (fwd(), bwd()),
        "pad_o": lambda: mb.mb_pad(o.view(cap, H * D), g["indices"], cap, g["meta"], B, L, out=g["o_padded"]),
        "pad_dqkv": lambda: mb.mb_pad(dqkv.view(cap, 3 * H * D), g["indices"], cap, g["meta"], B, L, out=g["dqkv_padded"]),
        "whole_step": g["step"],
    }

    def measure(fn, rotate=None):
        for i in range(5):
            fn() if rotate is None else fn(*rotate[i % len(rotate)])
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(100)]
        for i, (a, b) in enumerate(evs):
            a.record()
            fn() if rotate is None else fn(*rotate[i % len(rotate)])
            b.record()
        torch.cuda.synchronize()
        t = np.array([a.elapsed_time(b) * 1e3 for a, b in evs])
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(50):
            fn() if rotate is None else fn(*rotate[i % len(rotate)])
        b.record()
        torch.cuda.synchronize()
        return {"median": round(float(np.median(t)), 2), "p10": round(float(np.percentile(t, 10)), 2),
                "p90": round(float(np.percentile(t, 90)), 2), "loop": round(a.elapsed_time(b) * 1e3 / 50, 2)}

    res = {"warm": {name: measure(fn) for name, fn in calls.items()}}
    sets = [(qkv.clone(), dout.clone(), o.clone(), torch.empty_like(dqkv)) for _ in range(4)]
    res["cold"] = {
        "attn_fwd": measure(lambda x, do_, o_, dx: fwd(x, o_), sets),
        "attn_bwd": measure(lambda x, do_, o_, dx: bwd(x, do_, o_, dx), sets),
        "attn_fwd_bwd": measure(lambda x, do_, o_, dx: (fwd(x, o_), bwd(x, do_, o_, dx)), sets),
        "buffer_sets": 4, "bytes_per_set": int(sum(t.numel() * t.element_size() for t in sets[0])),
    }
    esize = 2 if g["bf16"] else 4
    W1, W3 = H * D * esize, 3 * H * D * esize
    w = res["warm"]
    res["GBs_warm"] = {"unpad_qkv": round(2 * T * W3 / (w["unpad_qkv"]["loop"] * 1e-6) * 1e-9, 1),
                       "pad_dqkv": round((T + cap) * W3 / (w["pad_dqkv"]["loop"] * 1e-6) * 1e-9, 1),
                       "pad_o": round((T + cap) * W1 / (w["pad_o"]["loop"] * 1e-6) * 1e-9, 1)}
    f = g["f_fwd"] + g["f_bwd"]
    res["attn_fwd_bwd_tflops"] = {"warm": round(f / (w["attn_fwd_bwd"]["loop"] * 1e-6) * 1e-12, 1),
                                  "cold": round(f / (res["cold"]["attn_fwd_bwd"]["loop"] * 1e-6) * 1e-12, 1)}
    return res


def host_threads():
    """Threads the oracle's BLAS may use: what the environment prescribes (the GPU machines export OMP_NUM_THREADS for
    their CPU share), else every host core."""
    try:
        return max(1, int(os.environ.get("OMP_NUM_THREADS", "")))
    except ValueError:
        return os.cpu_count() or 1


def run_cpu_baseline(args):
    """Starts the oracle leg as a child process (this file with --cpu-baseline-child) and returns its JSON object."""
    import subprocess
    n = str(host_threads())
    env = dict(os.environ, OMP_NUM_THREADS=n, OPENBLAS_NUM_THREADS=n, MKL_NUM_THREADS=n)
    cmd = [sys.executable, os.path.abspath(__file__), "--cpu-baseline-child", "--workload", args.workload]
    if args.batch is not None:
        cmd += ["--batch", str(args.batch)]
    out = subprocess.run(cmd, env=env, stdout=subprocess.PIPE, text=True, check=True).stdout
    return json.loads(out.strip().splitlines()[-1])


def cpu_baseline_child(workload, batch_override):
    """The CPU oracle, as it stands, on the benchmark batch (the whole path: index maps, gather, attention
    forward + backward, scatter), timed on this host with the BLAS thread count set by the parent before numpy
    was imported: the first 256 sequences of the batch (all of bert_base), 1 warm-up on a quarter of them, then
    3 repetitions, median.  `cores` = cpu time / wall time of the median run, i.e. the cores it really kept busy
    (the oracle multiplies many small matrices, one (sequence, head) at a time, which BLAS does not spread)."""
    import numpy as np
    from oracle import mosaic_oracle as orc
    from paper_2312_17482_amd import workloads as wl
    batch = wl.make_batch(workload, batch=batch_override)
    w = batch["workload"]
    f_fwd, f_bwd = wl.attention_flops(batch["lengths"], w.H, w.D)
    flops = f_fwd + f_bwd
    sub = min(w.B, 256)            # bounded sample: the first `sub` sequences of the batch
    slopes = orc.alibi_slopes(w.H)

    def run(n):
        q, k, v, do, mask = (batch[x][:n] for x in ("q", "k", "v", "do", "mask"))
        _, cu, idx, T, mx = orc.unpad_index(mask)
        orc.unpad(q, idx)
        O, LSE = orc.attention_fwd(q, k, v, mask, slopes, batch["scale"])
        orc.attention_bwd(do, q, k, v, mask, slopes, batch["scale"])
        orc.pad(orc.unpad(O, idx), idx, n, w.L)

    run(max(1, sub // 4))
    walls, cpus = [], []
    for _ in range(3):
        c0, t0 = time.process_time(), time.perf_counter()
        run(sub)
        walls.append(time.perf_counter() - t0)
        cpus.append(time.process_time() - c0)
    order = int(np.argsort(walls)[1])
    wall, cpu = walls[order], cpus[order]
    lengths = batch["lengths"][:sub].astype(np.float64)
    frac = float((lengths ** 2).sum()) * 14.0 * w.H * w.D / flops
    cores = max(1, int(round(cpu / wall)))
    return {"value": round(flops * frac / wall * 1e-12, 6), "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "blas_threads_allowed": host_threads(), "host_cpus": os.cpu_count(),
            "sample": "first %d of %d sequences of %s, whole path (fp64 numpy), median of 3 runs: %.1f s wall, %.1f s of "
                      "cpu time each; BLAS allowed %d threads on a host of %d cpus" % (
                          sub, w.B, w.name, wall, cpu, host_threads(), os.cpu_count()),
            "tokens_per_s": round(float(lengths.sum()) / wall, 1)}


if __name__ == "__main__":
    main()
