"""Host logic of the HBM-traffic tool: counter files -> calibrated bytes per launch, tied to a source digest."""
import csv
import json
import os

from paper_2201_05587_amd import traffic

SYM = "tt::contract_async_kernel<1, 1, 64, 64, 32, 32, 32, 16>"


def write_counters(directory, counter, rows):
    os.makedirs(directory, exist_ok=True)
    with open(os.path.join(directory, "run_counter_collection.csv"), "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=["Kernel_Name", "Counter_Name", "Counter_Value"])
        w.writeheader()
        for name, value in rows:
            w.writerow(dict(Kernel_Name=name, Counter_Name=counter, Counter_Value=value))


def test_summarise_scales_by_the_copy_and_lookup_follows_the_digest(tmp_path, monkeypatch):
    out = str(tmp_path / "out")
    copy_name = "void at::native::vectorized_elementwise_kernel<4, copy>(int)"
    units = traffic.COPY_BYTES / 1024 * 1.25   # a counter that over-reads by 25 %
    for leg, counter in (("copy_fetch", "FETCH_SIZE"), ("copy_write", "WRITE_SIZE")):
        write_counters(os.path.join(out, leg), counter,
                       [(copy_name, units)] * traffic.COPY_LAUNCHES + [("void fill_kernel(int)", 8.0)])
    kname = f"void {SYM}(tt::ContractArgs)"
    write_counters(os.path.join(out, "fetch"), "FETCH_SIZE", [(kname, 1000.0), (kname, 3000.0), ("void other(int)", 5.0)])
    write_counters(os.path.join(out, "write"), "WRITE_SIZE", [(kname, 500.0), (kname, 500.0)])
    monkeypatch.setattr(traffic, "HERE", str(tmp_path))
    os.makedirs(tmp_path / "tuned")
    os.makedirs(tmp_path / "csrc")
    (tmp_path / "csrc" / "k.hip").write_text("kernel v1")
    path = traffic.summarise(out, "cfgX")
    doc = json.load(open(path))
    k = doc["kernels"][SYM]
    assert abs(k["fetch_bytes_per_launch"] - 2000.0 * 1024 / 1.25) < 1e-6
    assert abs(k["write_bytes_per_launch"] - 500.0 * 1024 / 1.25) < 1e-6
    assert list(doc["kernels"]) == [SYM]
    assert abs(traffic.lookup("cfgX", SYM) - 2500.0 * 1024 / 1.25) < 1e-6
    assert traffic.lookup("cfgX", "tt::contract_kernel<0>") is None
    assert traffic.lookup("cfgY", SYM) is None
    (tmp_path / "csrc" / "k.hip").write_text("kernel v2")   # the kernel changed: the figure no longer applies
    assert traffic.lookup("cfgX", SYM) is None
