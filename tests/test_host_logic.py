"""Host-side logic that needs no GPU: the traffic-reading store, bench.py's algorithmic work
formulas, and the synthetic query streams."""
import csv
import importlib.util
import json
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_algorithmic_bytes_and_flops_match_the_stated_formulas():
    from paper_2510_25979_amd import synth
    b = _bench()
    w2, w3, w4 = synth.WORKLOADS[2], synth.WORKLOADS[3], synth.WORKLOADS[4]
    # workload 2: 32,768 tiles x (20,480 map + 16,384 V + 16,384 O) bytes
    assert b.apply_bytes(w2, 64) == 32768 * (20480 + 16384 + 16384) == 1_744_830_464
    assert b.apply_bytes(w2, 64, dense_equivalent=True) == 32768 * (32768 + 16384 + 16384)
    # workload 3: V is shared by the four query heads of a KV head
    assert b.apply_bytes(w3, 64) == 64 * 32 * 32 * (20480 + 32768 // 4 + 32768)
    # workload 4: S (S + 32) bytes of causal map per head
    assert b.apply_bytes(w4, 16) == 512 * (1024 * 1056 + 2 * 262144) == 822_083_584
    assert b.exact_bytes(w2, 64) == 32768 * 4 * 16384
    assert b.exact_bytes(w3, 128) == 128 * 32 * 32 * 32768 * (2 + 2 / 4)
    # two products of 2 D flops per visible score
    assert b.exact_flops(w4, 16) == 4.0 * (1024 * 1025 // 2) * 128 * 512
    assert b.exact_flops(w4, 16, dense_equivalent=True) == 4.0 * 1024 * 1024 * 128 * 512
    assert b.apply_kernel_name(w2) == "apply_bf16_kernel" and b.apply_kernel_name(w4) == "apply_bf16_long_kernel"


def _write_counter_csv(path, counter, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as f:
        wr = csv.DictWriter(f, fieldnames=["Dispatch_Id", "Kernel_Name", "Counter_Name", "Counter_Value"])
        wr.writeheader()
        for i, (name, value) in enumerate(rows):
            wr.writerow({"Dispatch_Id": i + 1, "Kernel_Name": name, "Counter_Name": counter,
                         "Counter_Value": value})


def test_traffic_store_scales_by_the_copy_probe_and_forgets_other_revisions(tmp_path, monkeypatch):
    from paper_2510_25979_amd import traffic
    monkeypatch.setattr(traffic, "DATA", str(tmp_path / "profiles" / "traffic.json"))
    kern = "void ac::apply_bf16_kernel<64, true, true, false>(ac::ApplyArgs)"
    # the probe, the LAST copy of the run (2^20 KiB), reads as 524,288 (factor 2) and writes as
    # 1,048,576 (factor 1); an earlier copy of another size must not be mistaken for it
    _write_counter_csv(str(tmp_path / "f" / "x" / "1_counter_collection.csv"), "FETCH_SIZE",
                       [("__amd_rocclr_copyBuffer", 77), (kern, 1000), (kern, 1010), (kern, 990),
                        ("__amd_rocclr_copyBuffer", 524288)])
    _write_counter_csv(str(tmp_path / "w" / "x" / "1_counter_collection.csv"), "WRITE_SIZE",
                       [("__amd_rocclr_copyBuffer", 99), (kern, 500), (kern, 500), (kern, 500),
                        ("__amd_rocclr_copyBuffer", 1048576)])
    monkeypatch.setattr(sys, "argv", ["traffic", "--fetch", str(tmp_path / "f"), "--write", str(tmp_path / "w"),
                                      "--kernel", "apply_bf16_kernel", "--workload", "w", "--layout", "packed"])
    traffic.main()
    entry = traffic.lookup("apply_bf16_kernel", "w", "packed")
    assert entry["read_bytes"] == 1000 * 2 * 1024 and entry["written_bytes"] == 500 * 1024
    assert entry["bytes"] == 2500 * 1024 and entry["revision"] == traffic.source_revision("apply_bf16_kernel")
    assert traffic.lookup("apply_bf16_kernel", "other", "packed") is None
    # a reading taken on other kernel sources is not handed out
    data = json.load(open(traffic.DATA))
    data["apply_bf16_kernel|w|packed"]["revision"] = "0" * 16
    json.dump(data, open(traffic.DATA, "w"))
    assert traffic.lookup("apply_bf16_kernel", "w", "packed") is None
    # a reading belongs to the file that defines the kernel (and the shared headers), so the
    # long reuse kernel shares apply.hip's revision and the exact kernel has its own
    assert traffic.source_file("apply_bf16_long_kernel") == "apply.hip"
    assert traffic.source_file("exact_bf16_kernel") == "exact.hip"
    assert traffic.source_revision("apply_bf16_long_kernel") == traffic.source_revision("apply_bf16_kernel")
    assert traffic.source_revision("exact_bf16_kernel") != traffic.source_revision("apply_bf16_kernel")
    with pytest.raises(ValueError):
        traffic.source_file("nosuch_kernel")


def test_query_stream_batches_differ_but_share_the_popularity_order():
    import torch
    from paper_2510_25979_amd import synth
    w = synth.WORKLOADS[5].scaled(n_entries=200, n_emb=2000, batch=512)
    emb, raw, map_of = synth.make_embeddings(w)
    assert map_of is not None and int(map_of.max()) == 199
    q0, p0 = synth.make_queries(w, raw, batch_id=0)
    q0b, p0b = synth.make_queries(w, raw, batch_id=0)
    q1, p1 = synth.make_queries(w, raw, batch_id=1)
    assert torch.equal(q0, q0b) and torch.equal(p0, p0b)          # seeded
    assert not torch.equal(p0, p1)                                 # another batch, other draws
    e0, e1 = (p0 % 200).tolist(), (p1 % 200).tolist()
    top0 = max(set(e0), key=e0.count)
    top1 = max(set(e1), key=e1.count)
    assert top0 == top1                                            # the same entry is the most popular
    assert len(set(e0)) < 200 and abs(len(set(e0)) - synth.expected_unique_zipf(w)) < 25
