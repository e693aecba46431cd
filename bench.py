#!/usr/bin/env python3
"""Benchmark of the AnTKV online path on one MI355X.

Headline (the metric's 128K-context configuration, "cfg2"): decode attention over a VQ-coded KV cache with
1 % FP16 anchors, batch 4 x 8 KV heads x 131072 tokens, 1-bit VQ.  One step = one antkv_decode_attn call
(one decode token per sequence, one layer).  The cache is built by the library itself from seeded synthetic
K/V: encode -> Anchor Score over a 32-query window -> top-1 % -> gather.  Timed steps rotate over several
distinct copies of the cache so that no buffer is re-read out of the 256 MB last-level cache; the warm
(single-copy) rate is reported beside it.  Encode and anchor-selection rates on the 32768-token prefill
shape ("cfg3") are reported as extras.

Prints one JSON line: metric, value, unit, timing and workload fields, a `roofline` object for the decode kernel and a
`cpu_baseline` object for the CPU oracle timed on the host.
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

HBM_PEAK_GBS = 8000.0


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def algorithmic_bytes(w, k_k, k_v):
    """Bytes one decode step must read/write: codes + anchor rows + anchor indices + codebooks + q/out."""
    per_bg = w.N * w.M * 2 + (k_k + k_v) * (w.D * 2 + 4)
    return w.B * w.Hkv * per_bg + 2 * w.Hkv * w.M * w.C * w.d_sub * 2 + 2 * w.B * w.Hq * w.D * 2


def kernel_source_digest():
    """SHA-256 of the decode kernel's source file: the hardware-counter summaries record it, so that a figure measured on
    an older kernel is not attached to a newer one."""
    import hashlib
    path = os.path.join(ROOT, "paper_2506_19505_amd", "csrc", "decode_attn.hip")
    return hashlib.sha256(open(path, "rb").read()).hexdigest()


def summary_fields(name):
    """`key: value` lines of a text summary under profiles/ (empty when the file is missing)."""
    fields = {}
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if ":" in line and not line.startswith((" ", "#", "\t")):
                key, val = line.split(":", 1)
                fields[key.strip()] = val.strip()
    except OSError:
        pass
    return fields


def measured_traffic(workload):
    """HBM bytes per launch of the decode kernel from the committed hardware-counter summary (FETCH_SIZE + WRITE_SIZE,
    scaled by the copy-kernel calibration).  None when no summary covers this workload, or when the summary was taken
    on another version of the kernel source (the reason is returned beside it)."""
    f = summary_fields(f"decode_attn_{workload}_hbm_traffic.txt")
    if "traffic_bytes_per_launch" not in f:
        return None, "no hardware-counter summary for this workload"
    if f.get("kernel_source_sha256") != kernel_source_digest():
        return None, "the hardware-counter summary under profiles/ was taken on another version of decode_attn.hip"
    return float(f["traffic_bytes_per_launch"]), None


def lds_ceiling():
    """Measured LDS read rate of the chip (conflict-free 8-byte reads, all CUs), GB/s, from profiles/lds_ceiling.txt."""
    f = summary_fields("lds_ceiling.txt")
    return float(f["lds_read_GBs_all_CUs"]) if "lds_read_GBs_all_CUs" in f else None


def lds_bytes(w):
    """LDS bytes one decode step moves by the kernel's design, per token and KV head: one 8-byte table entry per
    sub-space (K side), the 256-byte V centroid row (V side), and the V codes written to and read back from the wave's
    staging area."""
    return w.B * w.Hkv * w.N * (8 * w.M + 2 * w.D + 2 * w.M)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="cfg2", help="decode workload: cfg0 | cfg1 | cfg2 | cfg4")
    ap.add_argument("--copies", type=int, default=8, help="distinct cache copies the timed steps rotate over")
    ap.add_argument("--no-extras", action="store_true", help="skip encode / anchor-select rates and the CPU baseline")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch one row-copy kernel of known size (gather_rows with identity indices), so that a "
                         "hardware-counter run can scale its byte counters against it")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="CPU time to spend on the oracle baseline")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path is a single-GPU kernel path; nothing here uses a "
              "second GPU); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2506_19505_amd as antkv
    from workloads import (CONFIGS, make_codebooks, make_decode_query, make_qkv, normal_fp16, random_anchor_sets,
                           random_codes)

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    antkv.load_library()
    devc = torch.device("cuda:0")
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(devc)
    w = CONFIGS[args.workload]
    geom = antkv.Geometry(w.B, w.Hq, w.Hkv, w.d_sub)

    # ------------------------------------------------------------------ build the cache with the library
    t_setup = time.time()
    qwin, k, v = make_qkv(w.seed, w.B, w.Hq, w.Hkv, w.N, min(w.Nq_select, 32), w.D)
    log(f"generated K/V {k.shape} in {time.time() - t_setup:.1f}s")
    cbk, cbv = make_codebooks(w.seed, k, w.d_sub, w.C, "k"), make_codebooks(w.seed, v, w.d_sub, w.C, "v")
    log(f"codebooks done at {time.time() - t_setup:.1f}s")
    kd, vd, cbk_d, cbv_d = dev(k), dev(v), dev(cbk), dev(cbv)
    del k, v
    codes_k, codes_v = antkv.encode(geom, kd, cbk_d), antkv.encode(geom, vd, cbv_d)
    idx_k, idx_v, _, _ = antkv.anchor_select(geom, dev(qwin), kd, w.scale, w.k, want_scores=False)
    rows_k, rows_v = antkv.gather_rows(geom, kd, idx_k), antkv.gather_rows(geom, vd, idx_v)
    torch.cuda.synchronize()
    del kd, vd
    torch.cuda.empty_cache()
    copy_gbs = None
    if not args.no_extras or args.calibrate:
        # 8 heads x 131072 rows x 256 B read and written once each, plus 4 B of index per row
        cal_geom = antkv.Geometry(1, w.Hq, w.Hkv, w.d_sub)
        cal_src = torch.zeros((1, w.Hkv, 131072, w.D), dtype=torch.float16, device=devc)
        cal_idx = torch.arange(131072, dtype=torch.int32, device=devc).repeat(1, w.Hkv, 1).contiguous()
        cal_dst = antkv.gather_rows(cal_geom, cal_src, cal_idx)
        torch.cuda.synchronize()
        log(f"calibration copy: gather_rows_kernel read {cal_src.numel() * 2 + cal_idx.numel() * 4} B, "
            f"wrote {cal_src.numel() * 2} B")
        # the same copy, timed: the box's plain streaming rate, for comparison with the decode kernel's
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            antkv.gather_rows(cal_geom, cal_src, cal_idx, out=cal_dst)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = (cal_src.numel() * 4 + cal_idx.numel() * 4) / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9
        log(f"row copy (read + write) {copy_gbs:.0f} GB/s")
        del cal_src, cal_idx, cal_dst
    q = dev(make_decode_query(w.seed, w.B, w.Hq, w.D))
    out = torch.empty((w.B, w.Hq, w.D), dtype=torch.float16, device=devc)
    caches = [(codes_k, codes_v, idx_k, rows_k, idx_v, rows_v)]
    for _ in range(max(args.copies, 1) - 1):
        caches.append(tuple(t.clone() for t in caches[0]))
    ws = antkv.DecodeWorkspace(geom, w.N, w.k, w.k, 0, devc)
    log(f"cache ready at {time.time() - t_setup:.1f}s ({len(caches)} copies)")

    def step(i):
        ck, cv, ik, rk, iv, rv = caches[i % len(caches)]
        antkv.decode_attn(geom, q, w.scale, ck, cv, cbk_d, cbv_d, ik, rk, iv, rv, out=out, workspace=ws)

    def timed(n, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n   # ms per call

    def settle(fn, seconds=0.25):
        """Keep the GPU busy with `fn` until it has left its idle power state: after an idle spell (input
        generation on the host) the first ~30 ms of any kernel stream run at a lower clock, 10-15 % slower than
        the sustained rate that a decode loop or a prefill sees.  Not part of the timed region or of --warmup;
        returns the number of launches it made."""
        t_end = time.time() + seconds
        i = 0
        while time.time() < t_end:
            for _ in range(20):
                fn(i)
                i += 1
            torch.cuda.synchronize()
        return i

    settle_launches = settle(step)
    for i in range(args.warmup):
        step(i)
    ms_step = timed(args.steps, step)                          # headline: rotating over the cache copies
    ms_warm = timed(args.steps, lambda i: step(0))             # same buffers every step (cache-warm)

    # A step is exactly one launch of the dominant kernel (the library launches on torch's current stream, which is
    # the stream the two events are recorded on), so the kernel's average launch duration over the timed region is
    # the region's length between its two HIP events divided by the launches in it.
    ms_kernel = ms_step

    abytes = algorithmic_bytes(w, w.k, w.k)
    traffic, traffic_note = measured_traffic(w.name)
    achieved = abytes / (ms_kernel * 1e-3) / 1e9
    lds_peak = lds_ceiling()
    lds_achieved = lds_bytes(w) / (ms_kernel * 1e-3) / 1e9
    result = {
        "metric": "decode-attn tokens/s at 128K ctx + achieved HBM GB/s (% peak); encode Mvec/s",
        "value": w.B * w.N / (ms_step * 1e-3),
        "unit": "context tokens/s (one layer, all KV heads)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "settle_launches": settle_launches,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "i16-lut/f16-pv/f32-acc",
        "data": "synthetic (seeded N(0,1) K/V with channel outliers, k-means++ codebooks; stands in for LLaMA-3-8B / "
                "Mistral-7B KV caches)",
        "config": {"workload": f"{w.name}: {w.description}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "N": w.N,
                   "d_sub": w.d_sub, "bits_per_element": w.bits_per_element, "anchors_per_head": w.k,
                   "cache_copies_rotated": len(caches)},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_note": traffic_note,
                     "kernel": "decode_attn_kernel", "kernel_ms": ms_kernel, "algorithmic_bytes": abytes},
        # the same launch against the LDS: bytes the kernel's design moves through LDS per step over the chip's measured
        # conflict-free LDS read rate (the published HBM peak above stays the headline bound)
        "roofline_lds": {"bound": "lds", "achieved": lds_achieved, "peak": lds_peak, "unit": "GB/s",
                         "frac": (lds_achieved / lds_peak) if lds_peak else None, "lds_bytes": lds_bytes(w),
                         "peak_source": "profiles/lds_ceiling.txt (measured on this chip; no published figure)"},
        "extra": {"arithmetic": "u8 codes; int16 fixed-point q.centroid table; f16 softmax weights and V centroids into "
                                "f32 MFMA accumulators; f32 online softmax; f16 output",
                  "decode_steps_per_s": w.B / (ms_step * 1e-3), "ms_per_step_warm": ms_warm,
                  "tokens_per_s_warm": w.B * w.N / (ms_warm * 1e-3),
                  "measured_copy_GBs": copy_gbs,
                  "step_GBs": abytes / (ms_step * 1e-3) / 1e9, "step_frac_of_peak": abytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
    }
    log(f"decode: {ms_step * 1e3:.1f} us/step rotating, {ms_warm * 1e3:.1f} us warm -> {achieved:.0f} GB/s "
        f"({100 * achieved / HBM_PEAK_GBS:.1f}% of peak); LDS {lds_achieved:.0f} GB/s")

    if not args.no_extras:
        # ------------------------------------------------------------ encode + anchor selection on the prefill shape
        del caches, codes_k, codes_v, rows_k, rows_v
        torch.cuda.empty_cache()
        p = CONFIGS["cfg3"]
        pg = antkv.Geometry(p.B, p.Hq, p.Hkv, p.d_sub)
        pq, pk, pv = make_qkv(p.seed, p.B, p.Hq, p.Hkv, p.N, p.N, p.D)
        pcbk, pcbv = make_codebooks(p.seed, pk, p.d_sub, p.C, "k", max_sample=4096), make_codebooks(p.seed, pv, p.d_sub, p.C, "v", max_sample=4096)
        pkd, pvd, pqd, pcbk_d, pcbv_d = dev(pk), dev(pv), dev(pq), dev(pcbk), dev(pcbv)
        ck = torch.empty((p.B, p.Hkv, p.N, p.M), dtype=torch.uint8, device=devc)
        cv = torch.empty_like(ck)

        def enc(i):
            antkv.encode(pg, pkd, pcbk_d, codes=ck)
            antkv.encode(pg, pvd, pcbv_d, codes=cv)
        settle(enc)
        ms_enc = timed(100, enc)
        n_vec = 2 * p.B * p.Hkv * p.N
        antkv.anchor_select(pg, pqd, pkd, p.scale, p.k, want_scores=False)
        ms_sel = timed(3, lambda i: antkv.anchor_select(pg, pqd, pkd, p.scale, p.k, want_scores=False))
        result["extra"].update({
            "encode_Mvec_per_s": n_vec / (ms_enc * 1e-3) / 1e6, "encode_ms": ms_enc,
            "encode_input_GBs": n_vec * 256 / (ms_enc * 1e-3) / 1e9,
            "encode_workload": f"cfg3: K and V of {p.N} tokens x {p.Hkv} KV heads, d_sub {p.d_sub} ({n_vec} vectors)",
            "anchor_select_ms": ms_sel,
            "anchor_select_TFLOPs": 2 * 2.0 * p.B * p.Hq * (p.N * (p.N + 1) / 2) * p.D / (ms_sel * 1e-3) / 1e12,
            "anchor_select_workload": f"cfg3: Nq = N = {p.N}, {p.Hq} query heads, top-{p.k} for K and V (two QK^T passes)",
        })
        # one iteration of the offline token-weighted k-means on the same K rows (assignment + weighted update)
        km_w = torch.rand((p.B, p.Hkv, p.N), dtype=torch.float32, device=devc)
        km = lambda i: antkv.kmeans_step(pg, pkd, km_w, pcbk_d)
        settle(km, 0.1)
        ms_km = timed(50, km)
        result["extra"].update({"kmeans_step_us": ms_km * 1e3,
                                "kmeans_step_Mvec_per_s": p.B * p.Hkv * p.N / (ms_km * 1e-3) / 1e6})
        del km_w
        # prompt attention that hands its row statistics to the Anchor Score pass (Alg. 1)
        p_out, p_rm, p_rs = antkv.prefill_attn(pg, pqd, pkd, pvd, p.scale)
        ms_pa = timed(3, lambda i: antkv.prefill_attn(pg, pqd, pkd, pvd, p.scale))
        antkv.anchor_select(pg, pqd, pkd, p.scale, p.k, row_max=p_rm, row_sum=p_rs, want_scores=False)
        ms_sel2 = timed(3, lambda i: antkv.anchor_select(pg, pqd, pkd, p.scale, p.k, row_max=p_rm, row_sum=p_rs,
                                                         want_scores=False))
        result["extra"].update({
            "prefill_attn_ms": ms_pa,
            "prefill_attn_TFLOPs": 2 * 2.0 * p.B * p.Hq * (p.N * (p.N + 1) / 2) * p.D / (ms_pa * 1e-3) / 1e12,
            "anchor_select_given_row_stats_ms": ms_sel2,
        })
        del p_out, p_rm, p_rs
        log(f"encode {result['extra']['encode_Mvec_per_s']:.0f} Mvec/s ({ms_enc * 1e3:.0f} us); anchor select {ms_sel:.2f} ms; "
            f"prefill attention {ms_pa:.2f} ms, anchor select after it {ms_sel2:.2f} ms; k-means iteration {ms_km * 1e3:.0f} us")
        del pkd, pvd, pqd
        torch.cuda.empty_cache()

        # ------------------------------------------------------------ decode step + anchor re-selection (cfg4)
        r = CONFIGS["cfg4"]
        rg = antkv.Geometry(r.B, r.Hq, r.Hkv, r.d_sub)
        _, rks, rvs = make_qkv(r.seed, 1, r.Hq, r.Hkv, 2048, 1, r.D)
        rcbk, rcbv = dev(make_codebooks(r.seed, rks, r.d_sub, r.C, "k")), dev(make_codebooks(r.seed, rvs, r.d_sub, r.C, "v"))
        rt = dict(q=dev(make_decode_query(r.seed, r.B, r.Hq, r.D)),
                  ck=dev(random_codes(r.seed, "k", r.B, r.Hkv, r.N, r.M)), cv=dev(random_codes(r.seed, "v", r.B, r.Hkv, r.N, r.M)),
                  ik=dev(random_anchor_sets(r.seed, "k", r.B, r.Hkv, r.N, r.k)), iv=dev(random_anchor_sets(r.seed, "v", r.B, r.Hkv, r.N, r.k)),
                  rk=dev(normal_fp16(r.seed, "rows_k", (r.B, r.Hkv, r.k, r.D))), rv=dev(normal_fp16(r.seed, "rows_v", (r.B, r.Hkv, r.k, r.D))))
        ms_r = {}
        for resel in (0, r.k):
            rws = antkv.DecodeWorkspace(rg, r.N, r.k, r.k, resel, devc)
            f = lambda i: antkv.decode_attn(rg, rt["q"], r.scale, rt["ck"], rt["cv"], rcbk, rcbv, rt["ik"], rt["rk"], rt["iv"],
                                            rt["rv"], k_resel=resel, workspace=rws)
            settle(f)
            ms_r[resel] = timed(200, f)
        result["extra"].update({
            "cfg4_decode_ms": ms_r[0], "cfg4_decode_plus_reselection_ms": ms_r[r.k],
            "cfg4_workload": f"cfg4: B1, N={r.N}, d_sub {r.d_sub}, {r.k} anchors per head (cache-shaped random codes, warm); "
                             f"re-selection = decode-time Anchor Score over all tokens + top-{r.k} for K and V",
        })
        log(f"cfg4 decode {ms_r[0] * 1e3:.0f} us; with re-selection {ms_r[r.k] * 1e3:.0f} us")
        del rt
        torch.cuda.empty_cache()

        # ------------------------------------------------------------ keys stored before RoPE, on the headline shape
        prt = dict(q=dev(make_decode_query(w.seed, w.B, w.Hq, w.D)),
                   ck=dev(random_codes(w.seed, "k", w.B, w.Hkv, w.N, w.M)), cv=dev(random_codes(w.seed, "v", w.B, w.Hkv, w.N, w.M)),
                   ik=dev(random_anchor_sets(w.seed, "k", w.B, w.Hkv, w.N, w.k)), iv=dev(random_anchor_sets(w.seed, "v", w.B, w.Hkv, w.N, w.k)),
                   rk=dev(normal_fp16(w.seed, "rows_k", (w.B, w.Hkv, w.k, w.D))), rv=dev(normal_fp16(w.seed, "rows_v", (w.B, w.Hkv, w.k, w.D))))
        pr_ws = antkv.decode_attn_prerope_workspace(geom, w.N, w.k, devc)
        fpr = lambda i: antkv.decode_attn_prerope(geom, prt["q"], w.scale, prt["ck"], prt["cv"], cbk_d, cbv_d, prt["ik"], prt["rk"],
                                                  prt["iv"], prt["rv"], rope_base=500000.0, rope_style=1, pos0=0, out=out, workspace=pr_ws)
        settle(fpr, 0.1)
        ms_pr = timed(20, fpr)
        result["extra"].update({"prerope_decode_ms": ms_pr,
                                "prerope_workload": f"{w.name}'s shape with keys stored before RoPE (a pass that de-quantises and rotates every "
                                                    f"key and leaves q.k per head, then decode on those scores); workspace {pr_ws.numel() / 1e9:.2f} GB"})
        log(f"pre-RoPE decode on {w.name}'s shape: {ms_pr:.2f} ms")
        del prt, pr_ws
        torch.cuda.empty_cache()

        # ------------------------------------------------------------ the two small decode shapes (parity-test cases, not
        # bench lines): their whole cache fits the last-level cache, so these are cache-resident times, launch-bound
        for name in ("cfg0", "cfg1"):
            sconf = CONFIGS[name]
            sg = antkv.Geometry(sconf.B, sconf.Hq, sconf.Hkv, sconf.d_sub)
            _, sks, svs = make_qkv(sconf.seed, 1, sconf.Hq, sconf.Hkv, 2048, 1, sconf.D)
            scbk, scbv = dev(make_codebooks(sconf.seed, sks, sconf.d_sub, sconf.C, "k")), dev(make_codebooks(sconf.seed, svs, sconf.d_sub, sconf.C, "v"))
            st = dict(q=dev(make_decode_query(sconf.seed, sconf.B, sconf.Hq, sconf.D)),
                      ck=dev(random_codes(sconf.seed, "k", sconf.B, sconf.Hkv, sconf.N, sconf.M)),
                      cv=dev(random_codes(sconf.seed, "v", sconf.B, sconf.Hkv, sconf.N, sconf.M)),
                      ik=dev(random_anchor_sets(sconf.seed, "k", sconf.B, sconf.Hkv, sconf.N, sconf.k)),
                      iv=dev(random_anchor_sets(sconf.seed, "v", sconf.B, sconf.Hkv, sconf.N, sconf.k)),
                      rk=dev(normal_fp16(sconf.seed, "rows_k", (sconf.B, sconf.Hkv, sconf.k, sconf.D))),
                      rv=dev(normal_fp16(sconf.seed, "rows_v", (sconf.B, sconf.Hkv, sconf.k, sconf.D))))
            sws = antkv.DecodeWorkspace(sg, sconf.N, sconf.k, sconf.k, 0, devc)
            fs = lambda i: antkv.decode_attn(sg, st["q"], sconf.scale, st["ck"], st["cv"], scbk, scbv, st["ik"], st["rk"], st["iv"],
                                             st["rv"], workspace=sws)
            settle(fs, 0.1)
            ms_s = timed(500, fs)
            result["extra"].update({f"{name}_decode_us_cache_resident": ms_s * 1e3,
                                    f"{name}_workload": f"{name}: B{sconf.B}, N={sconf.N}, d_sub {sconf.d_sub}, {sconf.k} anchors per head "
                                                        f"(random codes; {sconf.B * sconf.Hkv * sconf.N * sconf.M * 2 / 1e6:.1f} MB of codes, cache-resident)"})
            log(f"{name} decode {ms_s * 1e3:.1f} us (cache-resident)")
            del st, sws

        # ------------------------------------------------------------ 12-bit codebooks (4096 centroids): d32 = 0.375 bit, d16 = 0.75 bit
        w_ik = dev(random_anchor_sets(r.seed, "k", r.B, r.Hkv, r.N, r.k))
        w_iv = dev(random_anchor_sets(r.seed, "v", r.B, r.Hkv, r.N, r.k))
        w_rk = dev(normal_fp16(r.seed, "rows_k", (r.B, r.Hkv, r.k, r.D)))
        w_rv = dev(normal_fp16(r.seed, "rows_v", (r.B, r.Hkv, r.k, r.D)))
        w_q = dev(make_decode_query(r.seed, r.B, r.Hq, r.D))
        pkd12 = dev(pk)
        for wd in (32, 16):
            wm = r.D // wd
            wb = wm * 3 // 2                                        # code bytes per token row
            tagw = f"d{wd}m4096"
            wg = antkv.Geometry(r.B, r.Hq, r.Hkv, wd, n_centroids=4096)
            w_cbk = dev(normal_fp16(r.seed, "cb12_k", (r.Hkv, wm, 4096, wd)))
            w_cbv = dev(normal_fp16(r.seed, "cb12_v", (r.Hkv, wm, 4096, wd)))
            gen = torch.Generator(device=devc)
            gen.manual_seed(r.seed)
            w_ck = torch.randint(0, 256, (r.B, r.Hkv, r.N, wb), dtype=torch.uint8, device=devc, generator=gen)
            w_cv = torch.randint(0, 256, (r.B, r.Hkv, r.N, wb), dtype=torch.uint8, device=devc, generator=gen)
            w_ws = antkv.DecodeWorkspace(wg, r.N, r.k, r.k, 0, devc)
            fw = lambda i: antkv.decode_attn(wg, w_q, r.scale, w_ck, w_cv, w_cbk, w_cbv, w_ik, w_rk, w_iv, w_rv, workspace=w_ws)
            settle(fw)
            ms_w = timed(100, fw)
            w_ws2 = antkv.DecodeWorkspace(wg, r.N, r.k, r.k, r.k, devc)
            fw2 = lambda i: antkv.decode_attn(wg, w_q, r.scale, w_ck, w_cv, w_cbk, w_cbv, w_ik, w_rk, w_iv, w_rv, k_resel=r.k,
                                              workspace=w_ws2)
            settle(fw2)
            ms_w2 = timed(50, fw2)
            del w_ws2
            w_ws3 = antkv.decode_attn_prerope_workspace(wg, r.N, r.k, devc)
            fw3 = lambda i: antkv.decode_attn_prerope(wg, w_q, r.scale, w_ck, w_cv, w_cbk, w_cbv, w_ik, w_rk, w_iv, w_rv,
                                                      rope_base=500000.0, rope_style=1, pos0=0, workspace=w_ws3)
            settle(fw3, 0.1)
            ms_w3 = timed(30, fw3)
            del w_ck, w_cv, w_ws3
            w_codes = torch.empty((p.B, p.Hkv, p.N, wb), dtype=torch.uint8, device=devc)
            pg12 = antkv.Geometry(p.B, p.Hq, p.Hkv, wd, n_centroids=4096)
            fe = lambda i: antkv.encode(pg12, pkd12, w_cbk, codes=w_codes)
            settle(fe)
            ms_e12 = timed(20, fe)
            km_w12 = torch.rand((p.B, p.Hkv, p.N), dtype=torch.float32, device=devc)
            km12 = lambda i: antkv.kmeans_step(pg12, pkd12, km_w12, w_cbk)
            settle(km12, 0.1)
            ms_km12 = timed(20, km12)
            del km_w12
            result["extra"].update({
                f"{tagw}_decode_ms": ms_w,
                f"{tagw}_decode_plus_reselection_ms": ms_w2,
                f"{tagw}_prerope_decode_ms": ms_w3,
                f"{tagw}_decode_tokens_per_s": r.B * r.N / (ms_w * 1e-3),
                f"{tagw}_decode_L2_gather_GBs": r.B * r.Hkv * r.N * 256 / (ms_w * 1e-3) / 1e9,
                f"{tagw}_encode_ms": ms_e12,
                f"{tagw}_encode_TFLOPs": 2.0 * p.B * p.Hkv * p.N * p.D * 4096 / (ms_e12 * 1e-3) / 1e12,
                f"{tagw}_kmeans_step_ms": ms_km12,
                f"{tagw}_workload": f"12-bit codes (d_sub {wd}, 4096 centroids, {wb} bytes per token row): decode on cfg4's shape "
                                    f"(B1, N={r.N}, {r.k} anchors per head, random codebooks and codes); encode of cfg3's K rows "
                                    f"({p.B * p.Hkv * p.N} rows)",
            })
            log(f"{tagw}: decode {ms_w * 1e3:.0f} us, with re-selection {ms_w2 * 1e3:.0f} us, on keys stored before RoPE {ms_w3 * 1e3:.0f} us, encode of {p.B * p.Hkv * p.N} rows "
                f"{ms_e12:.2f} ms, k-means iteration on them {ms_km12:.2f} ms")
            del w_codes, w_cbk, w_cbv, w_ws
            torch.cuda.empty_cache()
        del pkd12

        # ------------------------------------------------------------ decode append with a 32-token FP16 window
        a_W, a_k, a_N0, a_steps = 32, 64 + 32, 1024, 200
        a_cap = a_N0 + a_steps + 20
        a_codes_k = torch.zeros((w.B, w.Hkv, a_cap, w.M), dtype=torch.uint8, device=devc)
        a_codes_v = torch.zeros_like(a_codes_k)
        a_idx = torch.cat([torch.arange(0, a_k - a_W, dtype=torch.int32), torch.arange(a_N0 - a_W, a_N0, dtype=torch.int32)])
        a_idx_k = a_idx.repeat(w.B, w.Hkv, 1).contiguous().to(devc)
        a_idx_v = a_idx_k.clone()
        a_rows_k = dev(normal_fp16(w.seed, "win_rows_k", (w.B, w.Hkv, a_k, w.D)))
        a_rows_v = dev(normal_fp16(w.seed, "win_rows_v", (w.B, w.Hkv, a_k, w.D)))
        a_new_k = dev(normal_fp16(w.seed, "new_k", (w.B, w.Hkv, w.D)))
        a_new_v = dev(normal_fp16(w.seed, "new_v", (w.B, w.Hkv, w.D)))
        a_n = [a_N0]

        def app(i):
            a_n[0] = antkv.append_token(geom, a_new_k, a_new_v, a_n[0], a_W, cbk_d, cbv_d, a_codes_k, a_codes_v,
                                        a_idx_k, a_rows_k, a_idx_v, a_rows_v)
        for i in range(10):
            app(i)
        ms_app = timed(a_steps, app)
        result["extra"].update({"append_token_us": ms_app * 1e3,
                                "append_workload": f"B={w.B}, {w.Hkv} KV heads, d_sub {w.d_sub}, window {a_W}: retire one token "
                                                   f"(encode K and V rows), shift the window, insert the new rows"})
        log(f"append_token {ms_app * 1e3:.1f} us per step")

        # ------------------------------------------------------------ CPU baseline: the oracle, as it stands
        import oracle
        oracle.build()
        sB = w.B                                                # bounded sample: whole decode steps, repeated
        c = dict(q=make_decode_query(w.seed, sB, w.Hq, w.D),
                 ck=random_codes(w.seed, "k", sB, w.Hkv, w.N, w.M), cv=random_codes(w.seed, "v", sB, w.Hkv, w.N, w.M),
                 ik=random_anchor_sets(w.seed, "k", sB, w.Hkv, w.N, w.k), iv=random_anchor_sets(w.seed, "v", sB, w.Hkv, w.N, w.k),
                 rk=normal_fp16(w.seed, "rows_k", (sB, w.Hkv, w.k, w.D)), rv=normal_fp16(w.seed, "rows_v", (sB, w.Hkv, w.k, w.D)))
        reps, t0 = 0, time.time()
        while reps < 1 or (time.time() - t0 < args.cpu_seconds and reps < 1000):
            oracle.decode_attn(c["q"], c["ck"], c["cv"], cbk, cbv, c["ik"], c["rk"], c["iv"], c["rv"], w.scale)
            reps += 1
        t_cpu = time.time() - t0
        result["cpu_baseline"] = {"value": reps * sB * w.N / t_cpu, "unit": "context tokens/s (one layer, all KV heads)",
                                  "cores": oracle.num_threads(), "kind": "oracle",
                                  "sample": f"{reps} decode steps of {w.name} (B={sB}, N={w.N}, {w.Hkv} KV heads, "
                                            f"{w.k} anchors/head, cache-shaped random codes) in {t_cpu:.1f} s wall, "
                                            f"fp16->fp64 widening included"}
        log(f"cpu oracle: {reps} steps in {t_cpu:.2f}s on {oracle.num_threads()} threads")
        # the oracle's encode on a bounded sample of cfg3's K rows (the metric's "encode Mvec/s" leg)
        e_tok = 4096
        e_x = np.ascontiguousarray(pk[:, :, :e_tok])
        e_reps, t0 = 0, time.time()
        while e_reps < 1 or (time.time() - t0 < args.cpu_seconds / 2 and e_reps < 1000):
            oracle.encode(e_x, pcbk)
            e_reps += 1
        t_enc = time.time() - t0
        result["cpu_baseline"].update({
            "encode_Mvec_per_s": e_reps * p.B * p.Hkv * e_tok / t_enc / 1e6,
            "encode_sample": f"{e_reps} encodes of the first {e_tok} tokens of cfg3's K ({p.B * p.Hkv * e_tok} rows of 128 channels, "
                             f"d_sub {p.d_sub}, 256 centroids) in {t_enc:.1f} s wall"})
        log(f"cpu oracle encode: {result['cpu_baseline']['encode_Mvec_per_s']:.2f} Mvec/s")
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
