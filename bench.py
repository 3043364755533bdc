#!/usr/bin/env python3
"""Benchmark of the mixed paged-attention pass on one MI355X.

A step is one whole pass (KV append, decode split-K, combine, prefill tiles) over one synthetic
batch that is already resident in HBM.  The default workload is the largest mixed batch (70B-like
layer, 64/8/128, e4m3 KV cache: 512 decode rows next to 16 prefill chunks of 4096 tokens, 66 048 query tokens);
the burst and the decode-only configurations are measured in the same run and reported under "extra";
`--workload` selects another main workload.
Prints one JSON line with tokens/s, the roofline of the dominant kernel (duration from HIP
events recorded on the launch stream around every launch of the timed region) and the fp64 CPU
oracle timed on a bounded sample of the same batch.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_workload(name: str, device: str):
    import workloads as W
    if name == "cfg2":
        return W.config2(device=device)
    if name == "cfg4":
        return W.config4(device=device)
    if name == "cfg5":
        return W.config5(device=device)
    if name == "cfg3":
        return W.config3_step(0, device=device)
    if name == "cfg1":
        return W.config1(device=device)
    raise SystemExit(f"unknown workload {name}")


def algorithmic_work(batch):
    """Bytes / flops the method must move or do, per kernel, from the drawn lengths."""
    import numpy as np
    sh = batch.shape
    Hq, Hkv, D = sh.num_q_heads, sh.num_kv_heads, sh.head_dim
    s_kv = {"f32": 4, "bf16": 2, "fp8": 1}[sh.kv_dtype]
    s_q = {"f32": 4, "bf16": 2}[sh.q_dtype]
    ql = batch.q_lens.astype(np.int64)
    cl = batch.ctx_lens.astype(np.int64)
    pre = cl - ql
    dec = ql == 1
    pf = ql > 1
    pages = (cl + 15) // 16
    dec_bytes = int((cl[dec] * 2 * Hkv * D * s_kv + Hq * D * 2 * s_q + pages[dec] * 4).sum())
    dec_flops = int((4 * Hq * D * cl[dec]).sum())
    pf_flops = int((4 * Hq * D * (ql[pf] * pre[pf] + ql[pf] * (ql[pf] + 1) // 2)).sum())
    pf_bytes = int((cl[pf] * 2 * Hkv * D * s_kv + 2 * ql[pf] * Hq * D * s_q).sum())
    app_bytes = int(ql.sum() * 2 * Hkv * D * (s_q + s_kv))
    return dict(decode_bytes=dec_bytes, decode_flops=dec_flops, prefill_flops=pf_flops,
                prefill_bytes=pf_bytes, append_bytes=app_bytes)


def _oracle_rows(sub, row_stride: int):
    """Oracle on a sub-batch: KV append of its new tokens and attention for every row_stride-th row.
    Returns (seconds, reference rows [T,Hq,D] with NaN where not computed)."""
    import oracle
    sh = sub.shape
    args = (sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype, sh.kv_dtype)
    kc = oracle.new_cache(sub.num_pages, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
    vc = oracle.new_cache(sub.num_pages, sh.num_kv_heads, sh.head_dim, sh.kv_dtype)
    ks = None if sub.k_scale is None else oracle.raw(sub.k_scale)
    vs = None if sub.v_scale is None else oracle.raw(sub.v_scale)
    pre = sub.prefix_lens
    if pre.sum():
        oracle.kv_append(*args, oracle.raw(sub.k_prefix), oracle.raw(sub.v_prefix), kc, vc, ks, vs,
                         sub.block_table, pre, pre, sub.num_pages)
    q_raw = oracle.raw(sub.q)
    kn, vn = oracle.raw(sub.k_new), oracle.raw(sub.v_new)
    t0 = time.perf_counter()
    oracle.kv_append(*args, kn, vn, kc, vc, ks, vs, sub.block_table, sub.q_lens, sub.ctx_lens, sub.num_pages)
    ref = oracle.mixed_paged_attention(*args, q_raw, kc, vc, ks, vs, sub.block_table, sub.q_lens,
                                       sub.ctx_lens, sub.sm_scale, sub.num_pages, row_stride=row_stride)
    return time.perf_counter() - t0, ref


def cpu_baseline(batch, out_gpu, max_decode: int, max_chunks: int, chunk_stride: int):
    """Times the oracle (as it stands) on a bounded sample of the batch -- every row of up to max_decode
    decode sequences, and every chunk_stride-th row of up to max_chunks prefill chunks -- and checks the GPU
    rows against it."""
    import numpy as np
    import oracle
    import workloads as W
    ql = batch.q_lens
    q_off = np.concatenate([[0], np.cumsum(ql)])

    def pick(idx, n):
        idx = list(idx)
        return idx[:: max(1, len(idx) // n)][:n] if n > 0 else []

    legs = [(pick(np.nonzero(ql == 1)[0], max_decode), 1), (pick(np.nonzero(ql > 1)[0], max_chunks), chunk_stride)]
    n_rows, dt, err, parts = 0, 0.0, 0.0, []
    for sample, stride in legs:
        if not sample:
            continue
        sub = W.to_cpu(W.select_sequences(batch, sample))
        t, ref = _oracle_rows(sub, stride)
        done = ~np.isnan(ref[:, 0, 0])
        got = np.concatenate([out_gpu[q_off[s]:q_off[s + 1]] for s in sample])
        if done.any():
            err = max(err, float(np.max(np.abs(got[done] - ref[done]))))
        n_rows += int(done.sum())
        dt += t
        kind = "decode sequences, every row" if stride == 1 and ql[sample[0]] == 1 else f"prefill chunks, every {stride}. row"
        parts.append(f"{int(done.sum())} rows of {len(sample)} {kind}")
    return dict(value=n_rows / dt if dt > 0 else 0.0, unit="tokens/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"{n_rows} query rows ({'; '.join(parts)}) of {batch.name}: {dt:.1f} s of fp64 CPU work "
                       f"incl. their KV append", max_abs_err_vs_gpu=err)


def recorded_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, or None when there is none
    for this kernel and workload or the kernel sources changed since it was taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload.split('_')[0]}_traffic.txt")
    if not os.path.exists(path):
        return None
    kv = dict(l.strip().split("=", 1) for l in open(path) if "=" in l and not l.startswith("#"))
    if kv.get("workload") != workload:
        return None
    h = hashlib.sha256()
    for f in kv.get("sources", "").split(","):
        fp = os.path.join(ROOT, "paper_2512_03416_amd", "csrc", f)
        if not os.path.exists(fp):
            return None
        h.update(open(fp, "rb").read())
    if h.hexdigest() != kv.get("digest"):
        return None
    return int(kv["fetch_bytes"]) + int(kv["write_bytes"])


def calibrate(nbytes: int = 2 << 30):
    import torch
    import paper_2512_03416_amd as ts
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    res = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = {}
    for name, fn, moved in (("copy", lambda: ts.calib_copy(src, dst, nbytes), 2 * nbytes),
                            ("read", lambda: ts.calib_read(src, res, nbytes), nbytes)):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            fn()
        b.record()
        torch.cuda.synchronize()
        out[name + "_GBps"] = moved * 10 / (a.elapsed_time(b) * 1e-3) / 1e9
    del src, dst
    # what the matrix cores sustain on data like the workload's (normally distributed bf16) and on
    # constant operands: the clock the chip holds under a full MFMA stream depends on the data
    g = torch.Generator(device="cuda").manual_seed(7)
    normal = torch.randn(65536, device="cuda", generator=g).to(torch.bfloat16)
    const = torch.full((65536,), 0.0078125, device="cuda", dtype=torch.bfloat16)
    for name, ops, softmax in (("mfma_normal_TFLOPs", normal, False), ("mfma_softmax_normal_TFLOPs", normal, True),
                               ("mfma_constant_TFLOPs", const, False)):
        for _ in range(2):
            ts.calib_mfma(ops, res, 4000, softmax)
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        flops = 0
        for _ in range(3):
            flops += ts.calib_mfma(ops, res, 20000, softmax)
        b.record()
        torch.cuda.synchronize()
        out[name] = flops / (a.elapsed_time(b) * 1e-3) / 1e12
    return out


CPU_SAMPLE = {   # workload -> (decode sequences, prefill chunks, chunk row stride) of the oracle's bounded sample
    "cfg1": (8, 8, 1), "cfg2": (256, 0, 1), "cfg3": (0, 8, 8), "cfg4": (64, 4, 16), "cfg5": (48, 16, 64),
}


def roofline_of(work, ktimes, batch_name, mixed_mode=1):
    """Roofline block of the kernel that takes the most time, from the algorithmic work of the batch and
    the kernel's mean duration (HIP events on the launch stream)."""
    tot = {k: v[0] * v[1] for k, v in ktimes.items()}
    dominant = max(("decode", "prefill", "rows", "mixed"), key=lambda k: tot.get(k, 0.0))
    n, ms = ktimes[dominant]
    sec = ms * 1e-3
    all_bytes = work["decode_bytes"] + work["prefill_bytes"]
    name = dominant + "_kernel"
    if dominant == "mixed" and mixed_mode == 2:
        # co-resident launch: two kernels run side by side; the duration is the span from the start of the first to
        # the end of the last (events on the caller's stream around the fork and the join)
        name = "prefill_resident_kernel || decode_kernel_lean"
    common = dict(kernel=name, kernel_ms=ms, kernel_launches_timed=n)
    if dominant == "decode":
        ach = work["decode_bytes"] / sec / 1e9
        return dict(bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS,
                    traffic=recorded_traffic("decode_kernel", batch_name), algorithmic_bytes=work["decode_bytes"], **common)
    if dominant == "prefill":
        ach = work["prefill_flops"] / sec / 1e12
        return dict(bound="mfma", achieved=ach, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=ach / PEAK_BF16_TFLOPS,
                    traffic=recorded_traffic("prefill_kernel", batch_name), algorithmic_flops=work["prefill_flops"],
                    algorithmic_bytes=work["prefill_bytes"], **common)
    if dominant == "mixed":
        # the persistent kernel runs both kinds at once: its floor is the higher of the two, and it is priced
        # against the peak of that bound (frac = floor time / kernel time)
        t_hbm = all_bytes / (PEAK_HBM_GBS * 1e9)
        t_mfma = work["prefill_flops"] / (PEAK_BF16_TFLOPS * 1e12)
        extra = dict(algorithmic_flops=work["prefill_flops"], algorithmic_bytes=all_bytes,
                     floor_ms=max(t_hbm, t_mfma) * 1e3, floor_hbm_ms=t_hbm * 1e3, floor_mfma_ms=t_mfma * 1e3,
                     traffic=recorded_traffic("mixed_kernel", batch_name), **common)
        if t_mfma >= t_hbm:
            ach = work["prefill_flops"] / sec / 1e12
            return dict(bound="mfma", achieved=ach, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=ach / PEAK_BF16_TFLOPS, **extra)
        ach = all_bytes / sec / 1e9
        return dict(bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS, **extra)
    ach = all_bytes / sec / 1e9
    return dict(bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS, traffic=None,
                algorithmic_bytes=all_bytes, **common)


def per_class_of(work, ktimes):
    """The two classes of a mixed batch priced separately, from a run with one launch per class."""
    out = {}
    if ktimes.get("decode", (0, 0))[0]:
        ach = work["decode_bytes"] / (ktimes["decode"][1] * 1e-3) / 1e9
        out["decode"] = dict(kernel="decode_kernel", bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s",
                             frac=ach / PEAK_HBM_GBS, kernel_ms=ktimes["decode"][1], algorithmic_bytes=work["decode_bytes"])
    if ktimes.get("prefill", (0, 0))[0]:
        ach = work["prefill_flops"] / (ktimes["prefill"][1] * 1e-3) / 1e12
        out["prefill"] = dict(kernel="prefill_kernel", bound="mfma", achieved=ach, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                              frac=ach / PEAK_BF16_TFLOPS, kernel_ms=ktimes["prefill"][1],
                              algorithmic_flops=work["prefill_flops"])
    return out


def run_workload(name, args, with_cpu: bool):
    """All legs of one workload: the timed region (whole pass, kernels bracketed by HIP events), for a mixed
    batch a second region with one launch per class, and the oracle on a bounded sample."""
    import numpy as np
    import torch
    import paper_2512_03416_amd as ts
    t_setup = time.perf_counter()
    batch = build_workload(name, "cuda")
    sh = batch.shape
    desc = ts.Desc.make(sh.num_q_heads, sh.num_kv_heads, sh.head_dim, sh.q_dtype, sh.kv_dtype,
                        batch.num_pages, batch.max_pages_per_seq)
    ctx = ts.Context(desc)
    if args.split_pages:
        ctx.set_option("decode_split_pages", args.split_pages)
    if args.prefetch_tiles:
        ctx.set_option("decode_prefetch_tiles", args.prefetch_tiles)
    if args.xcd_count:
        ctx.set_option("xcd_count", args.xcd_count)
    if args.no_persistent:
        ctx.set_option("mixed_mode", 0)
    nbytes = ts.cache_bytes(desc)
    kc = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    vc = torch.full((nbytes,), 0xFF, dtype=torch.uint8, device="cuda")
    bt = torch.from_numpy(batch.block_table).cuda()
    pre = batch.prefix_lens
    info = ts.plan_describe(desc, batch.q_lens, batch.ctx_lens, args.split_pages)
    ctx.reserve(batch.total_q, batch.num_seqs, int(info.ctx_pages))
    if int(pre.sum()):
        ctx.kv_append(batch.k_prefix, batch.v_prefix, kc, vc, batch.k_scale, batch.v_scale, bt, pre, pre)
    out = torch.zeros((batch.total_q, sh.num_q_heads, sh.head_dim), dtype=batch.q.dtype, device="cuda")
    torch.cuda.synchronize()
    log(f"[bench] workload {batch.name}: S={batch.num_seqs} T={batch.total_q} ctx_pages={info.ctx_pages} "
        f"pool={batch.num_pages} pages, cache 2 x {nbytes / 1e9:.2f} GB, decode items {info.n_decode_items} "
        f"(split {info.split_pages} pages), prefill tiles {info.n_prefill_tiles}, generic rows "
        f"{info.n_generic_rows}; setup {time.perf_counter() - t_setup:.1f} s")

    def step():
        ctx.mixed_paged_attention(batch.q, batch.k_new, batch.v_new, kc, vc, batch.k_scale, batch.v_scale, bt,
                                  batch.q_lens, batch.ctx_lens, batch.sm_scale, out)

    def region(steps, timing):
        """`steps` passes bracketed by synchronisations; returns (seconds, kernel times)."""
        ctx.set_option("kernel_timing", timing)
        ctx.kernel_times(reset=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kt = ctx.kernel_times()
        ctx.set_option("kernel_timing", 0)
        return dt, kt

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # reference loop without per-kernel events
    ms_plain = region(args.steps, 0)[0] * 1e3 / args.steps
    # timed region: HIP events on the launch stream around the kernel launches of every N-th step
    ctx.token_velocity(reset=True)
    elapsed, ktimes = region(args.steps, args.time_every)
    vel = ctx.token_velocity(sync=True)
    ms_step = elapsed * 1e3 / args.steps
    T = batch.total_q
    # spread of single passes: events on the caller's stream around each pass (a pass begins and ends there, the
    # co-resident launch included), outside the timed region
    n_spread = min(args.steps, 50)
    marks = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_spread)]
    for a, b in marks:
        a.record()
        step()
        b.record()
    torch.cuda.synchronize()
    per_pass = sorted(a.elapsed_time(b) for a, b in marks)
    spread = {f"p{q}": round(per_pass[min(len(per_pass) - 1, int(q / 100 * len(per_pass)))], 5) for q in (10, 50, 90)}
    log(f"[bench] {batch.name}: {ms_step:.4f} ms/step with kernel events on every {args.time_every}. step, "
        f"{ms_plain:.4f} ms/step without; kernels: " +
        ", ".join(f"{k} {v[1] * 1e3:.1f} us x{v[0]}" for k, v in ktimes.items() if v[0]))
    log(f"[bench] token velocity counters: prefill {vel.prefill_tok_per_s:.0f} tok/s, decode "
        f"{vel.decode_tok_per_s:.0f} tok/s over {vel.window_s:.3f} s ({vel.passes} passes)")
    work = algorithmic_work(batch)
    roof = roofline_of(work, ktimes, batch.name, int(info.mixed_mode))
    res = {
        "value": T * args.steps / elapsed, "ms_per_step": ms_step,
        "dtype": ("bf16" if sh.q_dtype == "bf16" else "f32") + (" (e4m3 KV cache)" if sh.kv_dtype == "fp8" else ""),
        "config": {"workload": batch.name, "num_seqs": batch.num_seqs, "query_tokens": T,
                   "decode_rows": int((batch.q_lens == 1).sum()), "prefill_tokens": int(batch.q_lens[batch.q_lens > 1].sum()),
                   "heads": f"{sh.num_q_heads}q/{sh.num_kv_heads}kv/d{sh.head_dim}", "kv_dtype": sh.kv_dtype,
                   "page_size": 16, "ctx_tokens": int(batch.ctx_lens.sum()), "pool_pages": batch.num_pages,
                   "decode_split_pages": int(info.split_pages)},
        "roofline": roof,
        "ms_per_step_without_kernel_events": ms_plain,
        "ms_per_pass_events": spread,
        "kernels_us": {k: round(v[1] * 1e3, 2) for k, v in ktimes.items() if v[0]},
    }
    if "mixed" in ktimes and ktimes["mixed"][0] and not args.no_persistent:
        # the same batch with one launch per class: what each class reaches on its own
        ctx.set_option("mixed_mode", 0)
        for _ in range(max(2, args.warmup // 3)):
            step()
        n_sep = max(4, args.steps // 2)
        dt_sep, kt_sep = region(n_sep, max(1, args.time_every // 2))
        ctx.set_option("mixed_mode", 2)
        roof["mixed_mode"] = int(info.mixed_mode)
        roof["per_class"] = per_class_of(work, kt_sep)
        roof["ms_per_step_separate_launches"] = dt_sep * 1e3 / n_sep
        log(f"[bench] {batch.name}, one launch per class: {dt_sep * 1e3 / n_sep:.4f} ms/step; kernels: " +
            ", ".join(f"{k} {v[1] * 1e3:.1f} us x{v[0]}" for k, v in kt_sep.items() if v[0]))
        step()                                               # `out` as the default launch form writes it
        torch.cuda.synchronize()
    if with_cpu:
        out_host = out.double().cpu().numpy()
        n_dec, n_chunks, stride = CPU_SAMPLE[name]
        if args.cpu_seqs:
            n_dec = min(n_dec, args.cpu_seqs)
        res["cpu_baseline"] = cpu_baseline(batch, out_host, n_dec, n_chunks, stride)
        log(f"[bench] oracle: {res['cpu_baseline']}")
    ctx.close()
    del kc, vc, out, batch
    torch.cuda.empty_cache()
    return res


def summarise_trace(path):
    """Markdown summary of a rocprofv3 --kernel-trace output folder: per kernel the calls and the mean / min / max
    duration, and for the co-resident launch the span of each pair (start of the resident prefill kernel to the
    end of whichever of the two kernels ends last)."""
    import csv
    import glob
    rows = []
    for f in glob.glob(os.path.join(path, "**", "*kernel_trace.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]), r["Kernel_Name"].split("(")[0]))
    rows.sort()
    per = {}
    for s, e, n in rows:
        if "ts::" in n or "calib" in n:
            per.setdefault(n, []).append(e - s)
    print("| kernel | calls | mean us | min us | max us |\n|---|---|---|---|---|")
    for n, d in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        print(f"| `{n}` | {len(d)} | {sum(d) / len(d) / 1e3:.1f} | {min(d) / 1e3:.1f} | {max(d) / 1e3:.1f} |")
    spans = {}
    for i, (s, e, n) in enumerate(rows):
        if "prefill_resident_kernel" not in n:
            continue
        end, partner = e, None
        for s2, e2, n2 in rows[i + 1:i + 8]:
            if "decode_kernel" in n2 and s2 < e:
                end, partner = max(end, e2), (s2 - s, e2 - s2)
                break
        if partner:
            spans.setdefault(n, []).append((end - s, e - s, partner[1], partner[0]))
    for n, v in spans.items():
        k = len(v)
        print(f"\nco-resident pairs of `{n}` ({k}): span mean {sum(x[0] for x in v) / k / 1e3:.1f} us "
              f"(min {min(x[0] for x in v) / 1e3:.1f}, max {max(x[0] for x in v) / 1e3:.1f}); the prefill kernel itself "
              f"{sum(x[1] for x in v) / k / 1e3:.1f} us, the decode kernel next to it {sum(x[2] for x in v) / k / 1e3:.1f} us, "
              f"started {sum(x[3] for x in v) / k / 1e3:.1f} us after it")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--summarise-trace", default="", metavar="DIR",
                    help="print a summary of a rocprofv3 --kernel-trace output folder and exit (no GPU needed)")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"],
                    help="the workload the line's value is measured on (default: the largest mixed batch)")
    ap.add_argument("--no-extra", action="store_true", help="skip the extra workloads reported next to the main one")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seqs", type=int, default=0, help="cap on the decode sequences in the oracle sample")
    ap.add_argument("--calibrate", action="store_true", help="also time the plain copy/read kernels")
    ap.add_argument("--split-pages", type=int, default=0)
    ap.add_argument("--prefetch-tiles", type=int, default=0)
    ap.add_argument("--xcd-count", type=int, default=0)
    ap.add_argument("--no-persistent", action="store_true",
                    help="mixed batches: one launch per class instead of the co-resident launch")
    ap.add_argument("--time-every", type=int, default=4,
                    help="record HIP events around the kernels of every N-th step of the timed region")
    args = ap.parse_args()
    if args.summarise_trace:
        summarise_trace(args.summarise_trace)
        return
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_03416_amd as ts
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    ts.load_library()
    torch.cuda.set_device(0)

    main_res = run_workload(args.workload, args, with_cpu=not args.no_cpu_baseline)
    result = {
        "metric": "mixed-batch tokens/s (decode+prefill) on 1 MI355X",
        "value": main_res.pop("value"), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res.pop("dtype"), "data": "synthetic",
    }
    result.update(main_res)
    if args.workload == "cfg5" and not args.no_extra:
        # the burst configuration and the decode-only configuration, same procedure, for context
        result["extra"] = {}
        for w in ("cfg4", "cfg2"):
            r = run_workload(w, args, with_cpu=False)
            result["extra"][r["config"]["workload"]] = dict(
                tokens_per_s=r["value"], ms_per_step=r["ms_per_step"], query_tokens=r["config"]["query_tokens"],
                ms_per_pass_events=r["ms_per_pass_events"], kernels_us=r["kernels_us"], roofline=r["roofline"])
    if args.calibrate:
        result["calibration"] = calibrate()
        log(f"[bench] calibration: {result['calibration']}")
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
