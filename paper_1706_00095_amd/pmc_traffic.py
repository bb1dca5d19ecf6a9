#!/usr/bin/env python3
"""HBM traffic per kernel launch from two rocprofv3 counter runs of bench.py.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d <dirF> -o f -- python3 bench.py <args>
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d <dirW> -o w -- python3 bench.py <args>
    python3 paper_1706_00095_amd/pmc_traffic.py <dirF>/f_counter_collection.csv <dirW>/w_counter_collection.csv \
            <out.json> <out.txt> "<args>"

Each counter is scaled by what it reads for the 256 MiB plain copy bench.py runs first
(cg::debug_copy_kernel: 256 MiB fetched, 256 MiB written).  Kernel names are mapped to the labels
the library's per-launch profile uses, and the result is the mean over a label's launches.

    python3 paper_1706_00095_amd/pmc_traffic.py --merge <step.json> <update_only.json> <out.json>

joins the summary of a whole-step run with that of a `bench.py --update-only` run, whose
reduce_sgd_kernel<K> entries become standalone_update_K<K> (the stand-alone eight-bucket launches;
<K,tree> entries standalone_update_K<K>_tree).
"""
import collections
import csv
import json
import os
import re
import sys

COPY_BYTES = 256 << 20


def label(name):
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    math = {"0": "", "1": ",bf16", "2": ",bf16x3"}      # last template argument of the two big kernels: the arithmetic
    m = re.match(r"cg::igemm_patch_kernel<(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d)>", name)
    if m:
        wm, _, tm, _, _, nsl = map(int, m.groups()[:6])
        return f"igemm_patch_kernel<{wm * tm * 32}x128,{nsl}{math[m.group(7)]}>"
    m = re.match(r"cg::igemm_patch16_kernel<(\d+), (\d+), (\d+)>", name)
    if m:
        tm, _, nsl = map(int, m.groups())
        return f"igemm_patch16_kernel<{tm * 16}x128,{nsl}>"
    m = re.match(r"cg::igemm_wgrad_kernel<(\d+), (\d+), (\d+), (\d+), (\d+), (\d+), (\d+)>", name)
    if m:
        wm, _, tm, _, _, cpb, nsl = map(int, m.groups())
        return f"igemm_wgrad_kernel<{wm * tm * 32}x128,{cpb},{nsl}>"
    m = re.match(r"cg::igemm_kernel<(\d+), (\d+), (\d+), (\d+), (\d+), cg::(\w+)<(\d+)(?:, (\w+))?>, cg::(\w+)<(\d+)(?:, (\w+))?>, (\d)>", name)
    if m:
        wm, wn, tm, tn = (int(m.group(i)) for i in (1, 2, 3, 4))
        code = {"KLoader4": "4", "KLoader": "k", "RowsLoader": "r"}
        return (f"igemm_kernel<{wm * tm * 32}x{wn * tn * 32},{code[m.group(6)]}{code[m.group(9)]}"
                f"{'c' if m.group(11) == 'true' else '-'}{math[m.group(12)]}>")
    m = re.match(r"cg::reduce_sgd_kernel<(\d+), (\w+)>", name)
    if m:       # as the library's own launch log names it: <K> left to right, <K,tree> tree association
        return f"reduce_sgd_kernel<{m.group(1)}{',tree' if m.group(2) == 'true' else ''}>"
    m = re.match(r"cg::(\w+)(<[^(]*>)?", name)
    if m:
        return m.group(1) + (m.group(2) or "").replace(" ", "")
    return None


def load(path):
    d = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if "cg::" not in r["Kernel_Name"]:
            continue
        lab = label(r["Kernel_Name"])
        if lab:
            d[lab].append(float(r["Counter_Value"]))
    return d


def merge(step_json, update_json, out_json):
    a, b = json.load(open(step_json)), json.load(open(update_json))
    for lab, v in b["kernels"].items():
        m = re.match(r"reduce_sgd_kernel<(\d+)(,tree)?>", lab)
        if m:
            a["kernels"][f"standalone_update_K{m.group(1)}{'_tree' if m.group(2) else ''}"] = v
    a["note"] = ("bytes per launch behind L2 (FETCH_SIZE / WRITE_SIZE scaled by a 256 MiB copy); in-step kernels from the "
                 "one-stream run, standalone_update_K* from bench.py --update-only; the .txt summaries beside this file "
                 "give the commands")
    a["update_only_command_args"] = b["command_args"]
    json.dump(a, open(out_json, "w"), indent=1)


def main():
    if sys.argv[1] == "--merge":
        return merge(*sys.argv[2:5])
    fpath, wpath, out_json, out_txt, args = sys.argv[1:6]
    f, w = load(fpath), load(wpath)
    kf = COPY_BYTES / f["debug_copy_kernel"][0]
    kw = COPY_BYTES / w["debug_copy_kernel"][0]
    res = {}
    for lab in sorted(f, key=lambda k: -sum(f[k])):
        fb = sum(f[lab]) / len(f[lab]) * kf
        wb = sum(w.get(lab, [0.0])) / max(len(w.get(lab, [0.0])), 1) * kw
        res[lab] = dict(fetch_bytes=fb, write_bytes=wb, launches=len(f[lab]))
    json.dump(dict(command_args=args, scale_fetch_bytes_per_count=kf, scale_write_bytes_per_count=kw, kernels=res),
              open(out_json, "w"), indent=1)
    with open(out_txt, "w") as o:
        o.write("# HBM traffic per kernel launch (bytes fetched from / written to memory behind L2), mean over the launches of a label\n")
        o.write("# commands (from the repository root on the MI355X box), one counter per run:\n")
        o.write(f"#   rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d {os.path.dirname(fpath)} -o f -- python3 bench.py {args}\n")
        o.write(f"#   rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d {os.path.dirname(wpath)} -o w -- python3 bench.py {args}\n")
        o.write(f"#   python3 paper_1706_00095_amd/pmc_traffic.py {fpath} {wpath} <json> <txt> '<args>'\n")
        o.write(f"# scale from the 256 MiB copy (cg::debug_copy_kernel): {kf:.1f} bytes per FETCH_SIZE count, {kw:.1f} bytes per WRITE_SIZE count\n")
        o.write(f"{'kernel label':44s} {'launches':>8s} {'fetch MB':>10s} {'write MB':>10s}\n")
        for lab, v in res.items():
            o.write(f"{lab:44s} {v['launches']:8d} {v['fetch_bytes'] / 1e6:10.1f} {v['write_bytes'] / 1e6:10.1f}\n")


if __name__ == "__main__":
    main()
