"""Turns two rocprofv3 counter runs of gemm_driver (one with --pmc FETCH_SIZE, one with --pmc WRITE_SIZE, CSV
output) into the per-kernel traffic figures bench.py reports as `roofline.traffic`.

    python -m paper_2403_17031_amd.pmc_summary FETCH.csv WRITE.csv ROWS COMMIT OUT.json

Both counters read KiB per dispatch.  They are scaled by what the same counter reads for the driver's copy kernel,
which moves exactly 1 GiB each way: factor = 1,048,576 KiB / reading.  The result (bytes per launch for every GEMM
epilogue class, their mean, and that mean per GEMM row) goes to OUT.json with the commit it was measured at; a
markdown table of the same numbers is printed."""
import collections
import csv
import json
import re
import sys

GIB_KIB = 1048576.0
EPI = {"0": "bias", "1": "bias+GELU (FC1)", "2": "bias+residual (out-projection + FC2)", "3": "raw fp32",
       "5": "QKV: bias, rotary turn, q rows and K/V cache slots"}


def per_kernel(path, counter):
    tot, n = collections.defaultdict(float), collections.Counter()
    for r in csv.DictReader(open(path)):
        if r.get("Counter_Name") != counter:
            continue
        tot[r["Kernel_Name"]] += float(r["Counter_Value"])
        n[r["Kernel_Name"]] += 1
    return {k: tot[k] / n[k] for k in tot}


def main():
    fetch_csv, write_csv, rows, commit, out = sys.argv[1:6]
    rows = int(rows)
    f, w = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    copy_f = next(v for k, v in f.items() if "copy_yardstick" in k)
    copy_w = next(v for k, v in w.items() if "copy_yardstick" in k)
    ff, fw = GIB_KIB / copy_f, GIB_KIB / copy_w
    res = {"commit": commit, "gemm_rows": rows, "fetch_scale": ff, "write_scale": fw, "kernels": {}}
    print("| kernel | FETCH_SIZE KiB (raw) | read, scaled | WRITE_SIZE KiB (raw) | written, scaled |")
    print("|---|---|---|---|---|")
    total = []
    for k in sorted(f):
        if "gemm_f16_dma_kernel" not in k:
            continue
        # the epilogue is the kernel's first template argument: "<5, 8>" demangled, "ILi5ELi8E" mangled
        m = re.search(r"gemm_f16_dma_kernel(?:<|ILi)(\d+)", k)
        epi = m.group(1) if m else "?"
        rd, wr = f[k] * ff * 1024.0, w.get(k, 0.0) * fw * 1024.0
        res["kernels"][EPI.get(epi, epi)] = {"read_bytes": rd, "written_bytes": wr}
        total.append(rd + wr)
        print(f"| `{k[:48]}` ({EPI.get(epi, epi)}) | {f[k]:,.0f} | {rd / 1e9:.2f} GB | {w.get(k, 0.0):,.0f} | {wr / 1e9:.2f} GB |")
    print(f"| copy yardstick (1 GiB each way) | {copy_f:,.0f} | factor {ff:.3f} | {copy_w:,.0f} | factor {fw:.3f} |")
    res["mean_bytes_per_launch"] = sum(total) / len(total)
    res["bytes_per_gemm_row"] = res["mean_bytes_per_launch"] / rows
    print(f"\nmean over the {len(total)} products: {res['mean_bytes_per_launch'] / 1e9:.2f} GB per launch, "
          f"{res['bytes_per_gemm_row']:,.0f} bytes per row")
    json.dump(res, open(out, "w"), indent=1)


if __name__ == "__main__":
    main()
