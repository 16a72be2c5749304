#!/usr/bin/env python3
"""Turns the rocprofv3 output of a fixed set of bench.py runs into the summaries under profiles/.

It runs nothing on the GPU.  The runs it reads (each in its own rocprofv3 process; one MI355X;
`B` = `python3 bench.py --no-cpu --no-extras --gather-probe`):

  kt   rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof/kt  -- B --steps 3 --warmup 1
  rd   rocprofv3 --pmc TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_64B_sum TCC_EA0_RDREQ_128B_sum TCC_EA0_RDREQ_sum
                 --output-format csv -d gpurun_out/prof/rd -- B --steps 1 --warmup 0 --calib-copy
  wr   rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/prof/wr -- B --steps 1 --warmup 0 --calib-copy
  sq1  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_WAVE_CYCLES
                 SQ_WAIT_INST_ANY SQ_LDS_BANK_CONFLICT SQ_INSTS_LDS GRBM_GUI_ACTIVE --output-format csv
                 -d gpurun_out/prof/sq1 -- B --steps 1 --warmup 0
  sq2  rocprofv3 --pmc SQ_ACTIVE_INST_LDS SQ_INSTS_LDS_LOAD_BANDWIDTH SQ_ACTIVE_INST_VALU SQ_INSTS_VALU_TRANS_F32
                 SQ_ACTIVE_INST_VMEM SQ_WAIT_INST_LDS SQ_INSTS_VMEM GRBM_GUI_ACTIVE --output-format csv
                 -d gpurun_out/prof/sq2 -- B --steps 1 --warmup 0
  sq3  rocprofv3 --pmc SQ_LDS_IDX_ACTIVE SQ_LDS_DATA_FIFO_FULL SQ_LDS_CMD_FIFO_FULL SQ_WAIT_ANY SQ_INSTS_SALU
                 SQ_ACTIVE_INST_ANY SQ_ACTIVE_INST_SCA GRBM_GUI_ACTIVE --output-format csv
                 -d gpurun_out/prof/sq3 -- B --steps 1 --warmup 0

In every run the launches of k_attention<128, 2, false, false, false> come in this order: the sparse
launch(es) of the timed steps, three dense launches, four launches of the gather probe.

Bytes fetched over the fabric are counted directly, 32 n32 + 64 n64 + 128 n128 with n64 the
requests that are neither 32 nor 128 bytes long (the FETCH_SIZE expression of rocprofv3 counts a
128-byte request as 64 bytes on this chip, so it is not used); the 1 GiB device copy of the same
run checks the expression.  WRITE_SIZE is in KiB and matches the copy one to one.

    python3 bench_counters.py [gpurun_out/prof]     writes profiles/vs_kernels_7b_1m_last_chunk.txt
                                                     and profiles/traffic_k_attention_7b_1m.json
    python3 bench_counters.py --others [gpurun_out/prof]   writes profiles/vs_kernels_other_workloads.txt (see others())
"""
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
ATT = "k_attention<128, 2, false, false, false>"


def one(pattern):
    f = glob.glob(pattern, recursive=True)
    if not f:
        raise SystemExit(f"missing rocprofv3 output: {pattern}")
    return f[0]


def bench_line(log):
    return json.loads([l for l in open(log) if l.startswith('{"metric')][0])


def dispatches(d, base):
    """per kernel dispatch, in dispatch order: (kernel name, {counter: value summed over instances})"""
    per = collections.OrderedDict()
    for r in csv.DictReader(open(one(f"{base}/{d}/**/*counter_collection.csv"))):
        k = (int(r["Dispatch_Id"]), r["Kernel_Name"])
        per.setdefault(k, collections.defaultdict(float))[r["Counter_Name"]] += float(r["Counter_Value"])
    return [(k[1], v) for k, v in sorted(per.items())]


def pick(disp, name):
    return [c for n, c in disp if name in n]


def rd_bytes(c):
    n32, n128, n = c["TCC_EA0_RDREQ_32B_sum"], c["TCC_EA0_RDREQ_128B_sum"], c["TCC_EA0_RDREQ_sum"]
    return 32 * n32 + 128 * n128 + 64 * (n - n32 - n128)


OTHERS = [("dense_7b_64k", "--workload dense_7b_64k"), ("7b_128k", "--workload 7b_128k"), ("14b_1m", "--workload 14b_1m"),
          ("7b_1m_local", "--workload 7b_1m_local"), ("7b_1m_dca", "--workload 7b_1m_dca"),
          ("rows64", "--chunk-rows 64"), ("rows1024", "--chunk-rows 1024")]


def others(base):
    """profiles/vs_kernels_other_workloads.txt from the kernel traces kt_<name> of the other workloads:
         rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof/kt_<name>
                   -- python3 bench.py <switches> --steps 3 --warmup 1 --no-cpu --no-extras"""
    out = ["# rocprofv3 kernel traces of the other workloads (one MI355X; raw outputs stay under gpurun_out/; written by",
           "# bench_counters.py --others).  Each block: the command, the kernels of the library with their launch times over the",
           "# run, and the bench.py line of the same run.  A run is 1 warm-up + 3 timed chunk steps (+ 3 dense-kernel launches",
           "# where the workload is sparse), so the k_attention rows mix sparse and dense launches: min / max separate them.", ""]
    for name, sw in OTHERS:
        if not glob.glob(f"{base}/kt_{name}/**/*_kernel_trace.csv", recursive=True):
            continue
        out += [f"## {name}",
                f"command: rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof/kt_{name} -- python3 bench.py "
                f"{sw} --steps 3 --warmup 1 --no-cpu --no-extras"]
        per = collections.OrderedDict()
        for r in csv.DictReader(open(one(f"{base}/kt_{name}/**/*_kernel_trace.csv"))):
            if "vs::" in r["Kernel_Name"]:
                per.setdefault(r["Kernel_Name"], []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
        out.append(f"{'kernel':62s} {'calls':>5s} {'avg ms':>10s} {'min ms':>10s} {'max ms':>10s}")
        for n, v in sorted(per.items(), key=lambda x: -sum(x[1])):
            out.append(f"{n[:62]:62s} {len(v):5d} {sum(v) / len(v):10.3f} {min(v):10.3f} {max(v):10.3f}")
        d = bench_line(f"{base}/kt_{name}.log")
        ph = d["phases_ms"]
        line = (f"bench.py line: {d['value']:.2f} ms per chunk = estimate {ph['estimate']:.2f} + select {ph['select']:.2f} + sparse "
                f"attention {ph['sparse_attention']:.2f}; {d['config']['workload']}; issued tiles {d['tiles']['slash'] + d['tiles']['vertical'] or d['tiles']['dense_equivalent']}"
                f" (computed fraction {d['tiles']['computed_fraction']:.3f}), {d['effective_tflops']:.0f} TFLOP/s on issued tiles")
        if d.get("dense_ms"):
            line += f"; dense kernel {d['dense_ms']:.2f} ms = {d['dense_tflops']:.0f} TFLOP/s, speed-up {d['speedup_vs_dense']:.2f}"
        out += [line, ""]
    open(os.path.join(ROOT, "profiles", "vs_kernels_other_workloads.txt"), "w").write("\n".join(out) + "\n")
    print("\n".join(out))


def main():
    if len(sys.argv) > 1 and sys.argv[1] == "--others":
        return others(sys.argv[2] if len(sys.argv) > 2 else os.path.join(ROOT, "gpurun_out", "prof"))
    base = sys.argv[1] if len(sys.argv) > 1 else os.path.join(ROOT, "gpurun_out", "prof")
    sys.path.insert(0, ROOT)
    import bench
    out = []
    out += ["# rocprofv3 summaries: vertical-slash sparse prefill, workload 7b_1m (last 32,768-token chunk of a 1,048,576-token",
            "# context, Hq 28 / Hkv 4 / D 128, W 64, Bv 1000, Bs 6096), one MI355X.  Written by bench_counters.py from the runs",
            "# its header lists (B = python3 bench.py --no-cpu --no-extras --gather-probe); raw outputs stay under gpurun_out/.",
            f"# kernel sources: sha256[:16] of csrc/vs_attn.hip + csrc/vs_common.h = {bench.kernel_source_hash()}", ""]
    # ---- 1. kernel trace
    out += ["## 1. kernel trace",
            "command: rocprofv3 --kernel-trace --stats --output-format csv -d gpurun_out/prof/kt -- B --steps 3 --warmup 1", ""]
    per = collections.OrderedDict()
    rows = list(csv.DictReader(open(one(f"{base}/kt/**/*_kernel_trace.csv"))))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    for r in rows:
        if "vs::" in r["Kernel_Name"]:
            per.setdefault(r["Kernel_Name"], []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
    out.append(f"{'kernel':58s} {'calls':>5s} {'avg ms':>10s} {'min ms':>10s} {'max ms':>10s}")
    for n, v in sorted(per.items(), key=lambda x: -sum(x[1])):
        out.append(f"{n[:58]:58s} {len(v):5d} {sum(v) / len(v):10.3f} {min(v):10.3f} {max(v):10.3f}")
    d = bench_line(f"{base}/kt.log")
    att = [v for n, v in per.items() if ATT in n][0]
    n_sp = d["steps"] + d["warmup"]
    sp, de, ga = att[:n_sp], att[n_sp:n_sp + 3], att[n_sp + 3:]
    out += ["",
            f"k_attention, sparse launches (block list of the selected lines): n={len(sp)} avg {sum(sp) / len(sp):.3f} ms",
            f"k_attention, dense launches (every block diagonal):              n={len(de)} avg {sum(de) / len(de):.3f} ms",
            f"k_attention, gather probe (forced band + the vertical set):      n={len(ga)} avg {sum(ga) / len(ga):.3f} ms",
            f"bench.py line of the same run: sparse_attention {d['phases_ms']['sparse_attention']:.3f} ms (events; block list + "
            f"schedule + counter fill + k_attention), estimate {d['phases_ms']['estimate']:.3f} ms, select "
            f"{d['phases_ms']['select']:.3f} ms, dense {d['dense_ms']:.3f} ms",
            f"issued 64x64 tiles: slash {d['tiles']['slash']}, vertical {d['tiles']['vertical']} (dense equivalent "
            f"{d['tiles']['dense_equivalent']}); effective {d['effective_tflops']:.1f} TFLOP/s = {d['pct_bf16_mfma_peak']:.1f}% of "
            f"2500; dense {d['dense_tflops']:.1f} TFLOP/s", ""]
    kt_sparse_ms, kt_dense_ms, kt_gather_ms = sum(sp) / len(sp), sum(de) / len(de), sum(ga) / len(ga)
    # ---- 2. traffic
    rd, wr = dispatches("rd", base), dispatches("wr", base)
    copy = max(pick(rd, "copyBuffer"), key=lambda c: c["TCC_EA0_RDREQ_sum"])
    copy_w = max(c["WRITE_SIZE"] for c in pick(wr, "copyBuffer"))
    out += ["## 2. bytes between the L2 and the fabric (HBM side), per dispatch",
            "commands: rocprofv3 --pmc TCC_EA0_RDREQ_32B_sum TCC_EA0_RDREQ_64B_sum TCC_EA0_RDREQ_128B_sum TCC_EA0_RDREQ_sum "
            "--output-format csv -d gpurun_out/prof/rd -- B --steps 1 --warmup 0 --calib-copy",
            "          rocprofv3 --pmc WRITE_SIZE --output-format csv -d gpurun_out/prof/wr -- B --steps 1 --warmup 0 --calib-copy",
            "read bytes = 32 n32 + 128 n128 + 64 (n - n32 - n128)",
            f"check: the 1 GiB device copy reads {rd_bytes(copy) / 2**30:.4f} GiB by this expression "
            f"(n128 = {copy['TCC_EA0_RDREQ_128B_sum']:.0f}, n32 = {copy['TCC_EA0_RDREQ_32B_sum']:.0f}, n = "
            f"{copy['TCC_EA0_RDREQ_sum']:.0f}) and writes WRITE_SIZE = {copy_w:,.0f} KiB", ""]
    a_rd, a_wr = pick(rd, ATT), pick(wr, ATT)
    sparse_rd, dense_rd, gather_rd = rd_bytes(a_rd[0]), rd_bytes(a_rd[1]), rd_bytes(a_rd[-1])
    sparse_wr, gather_wr = a_wr[0]["WRITE_SIZE"] * 1024, a_wr[-1]["WRITE_SIZE"] * 1024
    out += [f"  k_attention sparse launch   read {sparse_rd / 1e9:9.2f} GB   written {sparse_wr / 1e9:7.3f} GB",
            f"  k_attention dense launch    read {dense_rd / 1e9:9.2f} GB",
            f"  k_attention gather probe    read {gather_rd / 1e9:9.2f} GB   written {gather_wr / 1e9:7.3f} GB"]
    for nm in ("k_estimate<128, 4, 0, false>", "k_estimate<128, 4, 1, false>", "k_sel_hist", "k_sel_count", "k_sel_write",
               "k_fill_zero(", "k_estimate_combine", "k_build_blocklist"):
        r_, w_ = pick(rd, nm), pick(wr, nm)
        out.append(f"  {nm:27s} read {(rd_bytes(r_[0]) if r_ else 0) / 1e9:9.3f} GB   written "
                   f"{(w_[0]['WRITE_SIZE'] * 1024 if w_ else 0) / 1e9:7.3f} GB")
    hbm = sparse_rd + sparse_wr
    out += [f"k_attention (sparse): {hbm / 1e9:.1f} GB per launch = {hbm / 1e9 / kt_sparse_ms:.2f} TB/s over {kt_sparse_ms:.1f} ms; "
            "touch-once minimum (Q, O, K, V) 2.62 GB; bytes copied into LDS 32 KiB per workgroup step",
            f"gather probe: {(gather_rd + gather_wr) / 1e9:.2f} GB per launch over {kt_gather_ms:.3f} ms = "
            f"{(gather_rd + gather_wr) / 1e9 / kt_gather_ms:.2f} TB/s on the HBM side"]
    e0, e1 = pick(rd, "k_estimate<128, 4, 0, false>")[0], pick(rd, "k_estimate<128, 4, 1, false>")[0]
    w1 = pick(wr, "k_estimate<128, 4, 1, false>")[0]["WRITE_SIZE"] * 1024
    ta = [v for n, v in per.items() if "k_estimate<128, 4, 0, false>" in n][0]
    tb = [v for n, v in per.items() if "k_estimate<128, 4, 1, false>" in n][0]
    ta, tb = sum(ta) / len(ta), sum(tb) / len(tb)
    out += [f"k_estimate sweep A: {rd_bytes(e0) / 1e9:.3f} GB read in {ta:.3f} ms = {rd_bytes(e0) / 1e9 / ta:.2f} TB/s; sweep B: "
            f"{rd_bytes(e1) / 1e9:.3f} GB read + {w1 / 1e9:.3f} GB written in {tb:.3f} ms = {(rd_bytes(e1) + w1) / 1e9 / tb:.2f} TB/s "
            "(K cache = 1.074 GB)", ""]
    # ---- 3. SQ counters, sparse / dense / gather launches
    out += ["## 3. SQ counters of k_attention: sparse launch | dense launch | gather probe",
            "commands: the sq1, sq2, sq3 runs of bench_counters.py's header", ""]
    agg = [collections.defaultdict(float) for _ in range(3)]
    for run in ("sq1", "sq2", "sq3"):
        a_ = pick(dispatches(run, base), ATT)
        for i, c in enumerate((a_[0], a_[1], a_[-1])):
            for k, v in c.items():
                if k == "GRBM_GUI_ACTIVE":
                    agg[i].setdefault("GRBM_GUI_ACTIVE", v)
                else:
                    agg[i][k] = v
    for k in sorted(agg[0]):
        out.append(f"  {k:30s} {agg[0][k]:20,.0f} {agg[1][k]:20,.0f} {agg[2][k]:20,.0f}")
    out.append("")
    for i, (nm, ms) in enumerate((("sparse", kt_sparse_ms), ("dense", kt_dense_ms), ("gather", kt_gather_ms))):
        a = agg[i]
        cyc = a["GRBM_GUI_ACTIVE"] / 8
        out += [f"{nm}: GRBM_GUI_ACTIVE / 8 XCDs = {cyc / 1e6:.1f} M cycles over {ms:.2f} ms (kernel trace) -> clock {cyc / (ms * 1e-3) / 1e9:.2f} GHz "
                "(nominal 2.4; counter runs serialise the launch, the clock is indicative)",
                f"   MFMA busy {a['SQ_VALU_MFMA_BUSY_CYCLES'] / 1024 / cyc * 100:.1f}% of the clocked cycles (32 cycles per MFMA on 1024 SIMDs); "
                f"VALU active {a['SQ_ACTIVE_INST_VALU'] * 4 / 1024 / cyc * 100:.1f}% (MFMA issue included); "
                f"LDS index unit active {a['SQ_LDS_IDX_ACTIVE'] / 256 / cyc * 100:.1f}% of the cycles of a CU",
                f"   per MFMA: {a['SQ_INSTS_VALU'] / a['SQ_INSTS_MFMA']:.2f} VALU (MFMA included), {a['SQ_INSTS_VALU_TRANS_F32'] / a['SQ_INSTS_MFMA']:.2f} "
                f"transcendental, {a['SQ_INSTS_SALU'] / a['SQ_INSTS_MFMA']:.2f} SALU, {a['SQ_INSTS_LDS'] / a['SQ_INSTS_MFMA']:.2f} LDS, "
                f"{a['SQ_INSTS_VMEM'] / a['SQ_INSTS_MFMA']:.3f} VMEM instructions; LDS bytes read {a['SQ_INSTS_LDS_LOAD_BANDWIDTH'] * 64 / a['SQ_INSTS_MFMA']:.0f} per MFMA "
                f"= {a['SQ_INSTS_LDS_LOAD_BANDWIDTH'] * 64 / 256 / cyc:.1f} B/clk per CU",
                f"   wave cycles in s_waitcnt {a['SQ_WAIT_INST_ANY'] / a['SQ_WAVE_CYCLES'] * 100:.1f}% (of which on LDS "
                f"{a['SQ_WAIT_INST_LDS'] / a['SQ_WAVE_CYCLES'] * 100:.1f}%), waiting for anything {a['SQ_WAIT_ANY'] / a['SQ_WAVE_CYCLES'] * 100:.1f}%; "
                f"LDS bank conflicts {a['SQ_LDS_BANK_CONFLICT']:.0f}, LDS data FIFO full {a['SQ_LDS_DATA_FIFO_FULL']:.0f}, command FIFO full {a['SQ_LDS_CMD_FIFO_FULL']:.0f} cycles"]
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)
    open(os.path.join(ROOT, "profiles", "vs_kernels_7b_1m_last_chunk.txt"), "w").write("\n".join(out) + "\n")
    json.dump({"kernel": "k_attention", "workload": "7b_1m last chunk", "kernel_source_sha": bench.kernel_source_hash(),
               "hbm_bytes_per_launch": hbm, "read_bytes": sparse_rd, "written_bytes": sparse_wr,
               "dense_read_bytes": dense_rd,
               "gather_probe": {"hbm_bytes": gather_rd + gather_wr, "read_bytes": gather_rd, "written_bytes": gather_wr,
                                "kernel_ms": kt_gather_ms},
               "expression": "32 n32 + 128 n128 + 64 (n - n32 - n128) over TCC_EA0_RDREQ*_sum, + WRITE_SIZE KiB"},
              open(os.path.join(ROOT, "profiles", "traffic_k_attention_7b_1m.json"), "w"), indent=1)
    print("\n".join(out))


if __name__ == "__main__":
    main()
