"""Turns rocprofv3 output of bench.py into the short text summaries kept with the measurements.

    python -m paper_2201_12465_amd.profile_summary kernel-trace <dir> [--workload NAME] > summary.txt
    python -m paper_2201_12465_amd.profile_summary traffic <bench_fetch_dir> <bench_write_dir> \
           <copy_fetch_dir> <copy_write_dir> [--workload NAME] > summary.txt

kernel-trace: <dir> is the -d directory of
    rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -- python3 bench.py ...
traffic: the four directories come from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` (one
counter per run) around `python3 bench.py --no-kernel-timing --no-cpu-baseline ...` and around
`python3 bench.py --copy-calibration`.  The counters are in KiB per dispatch; each is scaled by
(bytes the plain copy kernel is known to move) / (what the same counter reads for it), and the
per-class lines `traffic <class> bytes_per_launch <bytes>` are what bench.py reports as
roofline.traffic.
    python -m paper_2201_12465_amd.profile_summary mfma <dir> [--workload NAME] > summary.txt
mfma: <dir> is the -d directory of one counter run (SQ block + GRBM_GUI_ACTIVE, see MFMA_COUNTERS) around
the same bench command; per kernel it prints the share of the chip's MFMA issue cycles that were busy
(the matrix-core utilisation the roofline fraction is cross-checked against), the share of the
wavefronts' resident cycles spent waiting, and LDS bank conflicts.
    python -m paper_2201_12465_amd.profile_summary l2 <dir> [--workload NAME] > summary.txt
l2: <dir> is the -d directory of one counter run (L2_COUNTERS: the L2 and vector-L1 blocks) around the same
bench command; per kernel it prints the L2 hit rate, the average latency of a vector-L1 read request to
L2, and how much of the time the L1 had requests pending -- the evidence for where a GEMM's operand
traffic waits.
Only text parsing happens here: nothing touches the GPU.
"""
import argparse
import collections
import csv
import glob
import re
import sys

COPY_BYTES = 256 << 20


def classify(name: str) -> str:
    """Kernel class (as in fl_kernel_class_t) of a kernel name, mangled or demangled."""
    n = name
    if "copy_kernel" in n:
        return "copy"
    if "gemm_bf16_pipe" in n:
        m = re.search(r"gemm_bf16_pipe(?:<|ILb)(true|false|1|0)(?:, |ELb)(true|false|1|0)", n)
        if m:
            a, bb = (x in ("true", "1") for x in m.groups())
            return {(True, True): "gemm_nt", (True, False): "gemm_nn", (False, False): "gemm_tn"}.get((a, bb), "gemm")
        return "gemm_nt"
    if "gemm_f32_small" in n:
        m = re.search(r"gemm_f32_small(?:<|ILb)(true|false|1|0)(?:, |ELb)(true|false|1|0)", n)
        if m:
            a, bb = (x in ("true", "1") for x in m.groups())
            return {(True, True): "gemm_nt", (True, False): "gemm_nn", (False, False): "gemm_tn"}.get((a, bb), "gemm")
        return "gemm"
    if "gemm_kernel" in n:
        m = re.search(r"gemm_kernelI\w+?Lb([01])ELb([01])E", n)
        if m:
            a, bb = m.group(1) == "1", m.group(2) == "1"
        else:  # demangled: <T, AKC, BKC, tile height, dropout>
            bools = re.findall(r"\b(true|false)\b", n)
            if "bool, E" in n:
                # a known demangler slip: "<__bf16, true, ..." comes out as "<bool _Accum, bool, E, ..."
                # (the element type and AKC = true are swallowed); BKC is the first boolean that is left
                a, bb = True, bools[0] == "true"
            else:
                a, bb = bools[0] == "true", bools[1] == "true"
        return {(True, True): "gemm_nt", (True, False): "gemm_nn", (False, False): "gemm_tn"}.get((a, bb), "gemm")
    table = (("reduce_partials", "splitk_reduce"), ("reduce_batch", "splitk_reduce"), ("colsum", "colsum"), ("attn_fwd", "attn_fwd"),
             ("attn_bwd", "attn_bwd"), ("attn_delta", "attn_bwd"), ("ln_fwd", "ln_fwd"), ("ln_bwd", "ln_bwd"),
             ("opt_step", "optimizer"), ("zero_tensors", "optimizer"), ("transpose_tiles", "wt_transpose"))
    for key, cls in table:
        if key in n:
            return cls
    return "other"


def ours(name: str) -> bool:
    return "fl::" in name or "_ZN2fl" in name


def short(name: str, width: int = 72) -> str:
    n = name.replace("void ", "").replace("fl::(anonymous namespace)::", "").replace("_ZN2fl12_GLOBAL__N_1", "")
    return n[:width]


def kernel_trace(args) -> int:
    files = glob.glob(args.dir + "/**/*kernel_stats.csv", recursive=True)
    if not files:
        print(f"no *kernel_stats.csv under {args.dir}", file=sys.stderr)
        return 1
    rows = [r for r in csv.DictReader(open(files[0])) if ours(r["Name"])]
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("# made by (from /tmp, TMPDIR=/tmp, on one MI355X):")
    print(f"#   rocprofv3 --kernel-trace --stats --output-format csv -d <dir> -- python3 bench.py "
          f"--workload {args.workload} --steps 50 --warmup 10 --no-cpu-baseline --no-kernel-timing --no-grad-overlap")
    print(f"#   python3 -m paper_2201_12465_amd.profile_summary kernel-trace <dir> --workload {args.workload}")
    print(f"workload {args.workload}; kernels of this library only; durations in microseconds")
    print(f"{'class':14s} {'kernel':72s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'share':>6s}")
    per_class = collections.defaultdict(lambda: [0, 0.0])
    for r in sorted(rows, key=lambda r: -float(r["TotalDurationNs"])):
        c = classify(r["Name"])
        per_class[c][0] += int(r["Calls"])
        per_class[c][1] += float(r["TotalDurationNs"])
        print(f"{c:14s} {short(r['Name']):72s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:9.2f} "
              f"{float(r['MinNs']) / 1e3:9.2f} {float(r['MaxNs']) / 1e3:9.2f} "
              f"{100 * float(r['TotalDurationNs']) / total:5.1f}%")
    print()
    for c, (calls, ns) in sorted(per_class.items(), key=lambda kv: -kv[1][1]):
        print(f"class {c:14s} calls {calls:6d} avg_us {ns / calls / 1e3:9.2f} share {100 * ns / total:5.1f}%")
    return 0


def load_counter(d: str) -> dict:
    acc = collections.defaultdict(list)
    for f in glob.glob(d + "/**/*counter_collection.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            acc[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return acc


def traffic(args) -> int:
    print("# made by (from /tmp, TMPDIR=/tmp, on one MI355X; C = FETCH_SIZE, then WRITE_SIZE, one counter per run):")
    print("#   rocprofv3 --pmc C --output-format csv -d <copy_C> -- python3 bench.py --copy-calibration")
    print(f"#   rocprofv3 --pmc C --output-format csv -d <bench_C> -- python3 bench.py --workload {args.workload} "
          f"--steps 6 --warmup 2 --no-cpu-baseline --no-kernel-timing --no-grad-overlap")
    print(f"#   python3 -m paper_2201_12465_amd.profile_summary traffic <bench_FETCH_SIZE> <bench_WRITE_SIZE> "
          f"<copy_FETCH_SIZE> <copy_WRITE_SIZE> --workload {args.workload}")
    print("# FETCH_SIZE / WRITE_SIZE count what the L2 caches of the 8 XCDs exchange with the memory side (the")
    print("# shared last-level cache or HBM), in KiB per dispatch; an operand panel used by several XCDs is")
    print("# fetched once by each of them, so a GEMM's figure exceeds its algorithmic bytes by construction.")
    factor = {}
    for which, d, known in (("FETCH_SIZE", args.copy_fetch, COPY_BYTES), ("WRITE_SIZE", args.copy_write, COPY_BYTES)):
        v = [x for k, xs in load_counter(d).items() if classify(k) == "copy" for x in xs]
        if not v:
            print(f"no copy_kernel dispatches under {d}", file=sys.stderr)
            return 1
        factor[which] = known / (sum(v) / len(v) * 1024.0)
        print(f"calibration {which}: copy kernel of {known} bytes reads {sum(v) / len(v):.1f} KiB "
              f"over {len(v)} launches -> factor {factor[which]:.4f}")
    fetch, write = load_counter(args.bench_fetch), load_counter(args.bench_write)
    print(f"workload {args.workload}; per launch, KiB as counted and bytes after scaling")
    print(f"{'class':14s} {'kernel':72s} {'n':>5s} {'FETCH_KiB':>11s} {'WRITE_KiB':>11s} {'hbm_bytes':>13s}")
    per_class = collections.defaultdict(lambda: [0, 0.0])
    for k in sorted(set(fetch) | set(write)):
        if not ours(k) or classify(k) == "copy":
            continue
        fv, wv = fetch.get(k, []), write.get(k, [])
        f = sum(fv) / len(fv) if fv else 0.0
        w = sum(wv) / len(wv) if wv else 0.0
        n = max(len(fv), len(wv))
        by = (f * factor["FETCH_SIZE"] + w * factor["WRITE_SIZE"]) * 1024.0
        c = classify(k)
        per_class[c][0] += n
        per_class[c][1] += by * n
        print(f"{c:14s} {short(k):72s} {n:5d} {f:11.1f} {w:11.1f} {by:13.0f}")
    print()
    for c, (n, tot) in sorted(per_class.items()):
        print(f"traffic {c} bytes_per_launch {tot / n:.0f}")
    return 0


MFMA_COUNTERS = ("SQ_WAVES", "SQ_BUSY_CYCLES", "SQ_WAVE_CYCLES", "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS",
                 "SQ_ACTIVE_INST_VALU", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_LDS_BANK_CONFLICT", "GRBM_GUI_ACTIVE")
SIMDS = 1024          # 256 compute units x 4
MFMA_CYCLES = {"bf16": 32, "f32": 64}      # issue cycles of one 32x32 MFMA (x16 bf16: 32768 flop; x2 f32: 4096 flop)
MFMA_FLOP = {"bf16": 32768.0, "f32": 4096.0}


def mfma(args) -> int:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    info = {}
    for f in glob.glob(args.dir + "/**/*counter_collection.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            k = r["Kernel_Name"]
            if not ours(k):
                continue
            acc[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
            info[k] = (r.get("Workgroup_Size", "?"), r.get("LDS_Block_Size", "?"), r.get("VGPR_Count", "?"),
                       r.get("Accum_VGPR_Count", "?"), r.get("Scratch_Size", "?"))
    if not acc:
        print(f"no counter_collection.csv with this library's kernels under {args.dir}", file=sys.stderr)
        return 1
    # GRBM_GUI_ACTIVE arrives summed over the accelerator dies (XCCs), each of which counts its own clocks
    xcc = 8
    for f in glob.glob(args.dir + "/**/*agent_info.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            if r.get("Agent_Type") == "GPU" and r.get("Num_Xcc", "").isdigit():
                xcc = int(r["Num_Xcc"])
    print("# made by (from /tmp, TMPDIR=/tmp, on one MI355X):")
    print(f"#   rocprofv3 --pmc {' '.join(MFMA_COUNTERS)} --output-format csv -d <dir> -- python3 bench.py "
          f"--workload {args.workload} --steps 3 --warmup 2 --no-cpu-baseline --no-kernel-timing --no-grad-overlap")
    print(f"#   python3 -m paper_2201_12465_amd.profile_summary mfma <dir> --workload {args.workload}")
    print("# Per dispatch, averaged over the launches of a kernel (each kernel runs alone under counter collection).")
    print(f"# gui_cyc   GRBM_GUI_ACTIVE / {xcc} (the counter is the sum over the {xcc} dies): clocks the dispatch kept the GPU busy;")
    print("#           under counter collection a dispatch lasts about 20 % longer than in the kernel trace")
    print("# mfma_busy SQ_VALU_MFMA_BUSY_CYCLES summed over the SIMDs: issue cycles the matrix cores were occupied")
    print(f"# mfma_util mfma_busy / (gui_cyc x {SIMDS} SIMDs): 1.0 = every matrix core busy on every clock, i.e. the")
    print("#           dense peak (2.5 PFLOP/s bf16: 32768 flop per 32x32x16 MFMA, 32 issue cycles each)")
    print("# wait      SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES: share of the wavefronts' resident cycles spent at s_waitcnt")
    print("# wait_lds  SQ_WAIT_INST_LDS / SQ_WAVE_CYCLES: the part of it waiting for LDS")
    print("# valu      SQ_ACTIVE_INST_VALU / SQ_WAVE_CYCLES (counter units as delivered: compare kernels, not 1.0)")
    print("# conflict  SQ_LDS_BANK_CONFLICT / SQ_BUSY_CYCLES: LDS bank-conflict cycles per busy SQ cycle")
    print(f"workload {args.workload}")
    print(f"{'class':13s} {'kernel':60s} {'n':>4s} {'wg':>4s} {'lds':>6s} {'vgpr':>4s} {'agpr':>4s} {'scr':>4s} "
          f"{'gui_cyc':>9s} {'mfma_busy':>11s} {'mfma_util':>9s} {'wait':>6s} {'wait_lds':>8s} {'valu':>6s} {'conflict':>8s}")
    per_class = collections.defaultdict(lambda: [0.0, 0.0])
    rows = []
    for k, cs in acc.items():
        avg = {c: (sum(v) / len(v) if v else 0.0) for c, v in cs.items()}
        g = avg.get("GRBM_GUI_ACTIVE", 0.0) / xcc
        mb = avg.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0)
        wc = avg.get("SQ_WAVE_CYCLES", 0.0) or 1.0
        n = len(cs.get("GRBM_GUI_ACTIVE", [])) or len(next(iter(cs.values())))
        rows.append((g * n, k, n, g, mb, avg, wc))
        c = classify(k)
        per_class[c][0] += mb * n
        per_class[c][1] += g * n
    for _, k, n, g, mb, avg, wc in sorted(rows, reverse=True):
        wg, lds, vg, ag, scr = info[k]
        print(f"{classify(k):13s} {short(k, 60):60s} {n:4d} {wg:>4s} {lds:>6s} {vg:>4s} {ag:>4s} {scr:>4s} "
              f"{g:9.0f} {mb:11.0f} {mb / (g * SIMDS) if g else 0:9.3f} {avg.get('SQ_WAIT_INST_ANY', 0) / wc:6.2f} "
              f"{avg.get('SQ_WAIT_INST_LDS', 0) / wc:8.2f} {avg.get('SQ_ACTIVE_INST_VALU', 0) / wc:6.2f} "
              f"{avg.get('SQ_LDS_BANK_CONFLICT', 0) / (avg.get('SQ_BUSY_CYCLES', 0) or 1):8.3f}")
    print()
    for c, (mb, g) in sorted(per_class.items(), key=lambda kv: -kv[1][1]):
        if mb:
            print(f"mfma_util {c} {mb / (g * SIMDS):.3f}")
    return 0


L2_COUNTERS = ("TCC_HIT_sum", "TCC_MISS_sum", "TCC_EA0_RDREQ_sum", "TCP_TCC_READ_REQ_sum",
               "TCP_TCC_READ_REQ_LATENCY_sum", "TCP_PENDING_STALL_CYCLES_sum", "GRBM_GUI_ACTIVE")


def l2(args) -> int:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in glob.glob(args.dir + "/**/*counter_collection.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            if ours(r["Kernel_Name"]):
                acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    if not acc:
        print(f"no counter_collection.csv with this library's kernels under {args.dir}", file=sys.stderr)
        return 1
    xcc = 8
    for f in glob.glob(args.dir + "/**/*agent_info.csv", recursive=True):
        for r in csv.DictReader(open(f)):
            if r.get("Agent_Type") == "GPU" and r.get("Num_Xcc", "").isdigit():
                xcc = int(r["Num_Xcc"])
    print("# made by (from /tmp, TMPDIR=/tmp, on one MI355X):")
    print(f"#   rocprofv3 --pmc {' '.join(L2_COUNTERS)} --output-format csv -d <dir> -- python3 bench.py "
          f"--workload {args.workload} --steps 3 --warmup 2 --no-cpu-baseline --no-kernel-timing --no-grad-overlap")
    print(f"#   python3 -m paper_2201_12465_amd.profile_summary l2 <dir> --workload {args.workload}")
    print("# Per dispatch, averaged over the launches of a kernel (each kernel runs alone under counter collection).")
    print(f"# gui_cyc      GRBM_GUI_ACTIVE / {xcc}: clocks the dispatch kept the GPU busy")
    print("# l2_hit       TCC_HIT / (TCC_HIT + TCC_MISS): share of L2 requests served from the L2 of the requesting die")
    print("# l2_req_MB    TCP_TCC_READ_REQ x 64 bytes: what the vector L1 caches asked the L2 for")
    print("# mem_rd_MB    TCC_EA0_RDREQ x 64 bytes (upper bound: 32-byte requests count as one): L2 misses sent to the memory side")
    print("# rd_latency   TCP_TCC_READ_REQ_LATENCY / TCP_TCC_READ_REQ: average clocks from an L1 read request to its answer")
    print("# l1_pending   TCP_PENDING_STALL_CYCLES summed over the 256 L1s / (gui_cyc x 256)")
    print(f"workload {args.workload}")
    print(f"{'class':13s} {'kernel':60s} {'n':>4s} {'gui_cyc':>9s} {'l2_hit':>7s} {'l2_req_MB':>10s} {'mem_rd_MB':>10s} "
          f"{'rd_latency':>10s} {'l1_pending':>10s}")
    rows = []
    for k, cs in acc.items():
        a = {c: (sum(v) / len(v) if v else 0.0) for c, v in cs.items()}
        g = a.get("GRBM_GUI_ACTIVE", 0.0) / xcc
        n = len(cs.get("GRBM_GUI_ACTIVE", [])) or len(next(iter(cs.values())))
        rows.append((g * n, k, n, g, a))
    for _, k, n, g, a in sorted(rows, reverse=True):
        hit, miss = a.get("TCC_HIT_sum", 0.0), a.get("TCC_MISS_sum", 0.0)
        req = a.get("TCP_TCC_READ_REQ_sum", 0.0)
        print(f"{classify(k):13s} {short(k, 60):60s} {n:4d} {g:9.0f} {hit / (hit + miss) if hit + miss else 0:7.3f} "
              f"{req * 64 / 1e6:10.1f} {a.get('TCC_EA0_RDREQ_sum', 0.0) * 64 / 1e6:10.1f} "
              f"{a.get('TCP_TCC_READ_REQ_LATENCY_sum', 0.0) / req if req else 0:10.0f} "
              f"{a.get('TCP_PENDING_STALL_CYCLES_sum', 0.0) / (g * 256) if g else 0:10.2f}")
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    k = sub.add_parser("kernel-trace")
    k.add_argument("dir")
    k.add_argument("--workload", default="cfg3_bert_base_bf16")
    t = sub.add_parser("traffic")
    for n in ("bench_fetch", "bench_write", "copy_fetch", "copy_write"):
        t.add_argument(n)
    t.add_argument("--workload", default="cfg3_bert_base_bf16")
    m = sub.add_parser("mfma")
    m.add_argument("dir")
    m.add_argument("--workload", default="cfg3_bert_base_bf16")
    q = sub.add_parser("l2")
    q.add_argument("dir")
    q.add_argument("--workload", default="cfg3_bert_base_bf16")
    a = ap.parse_args()
    return {"kernel-trace": kernel_trace, "traffic": traffic, "mfma": mfma, "l2": l2}[a.cmd](a)


if __name__ == "__main__":
    sys.exit(main())
