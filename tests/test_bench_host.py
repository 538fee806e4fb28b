"""Host logic of bench.py: the algorithmic bytes and flops of a verify step against figures worked out by hand from the
workload descriptions, the single-GPU rule, and the workload table against the configurations the metric is quoted on."""
import json
import os
import subprocess
import sys

import workload as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_algorithmic_bytes_and_flops_by_hand():
    # 135M class: 30 layers, d 576, 9 / 3 heads of 64, ffn 1536, vocab 49152, bf16, batch 1, k 8, prompt 512, generate 256
    c = W.get_config("cfg2")
    per_layer = 576 * (576 + 2 * 192) + 576 * 576 + 3 * 576 * 1536          # qkv, output, gate + up + down
    weights = (30 * per_layer + 49152 * 576) * 2
    assert weights == 268959744
    kv_tok = 30 * 2 * 192 * 2                                               # bytes of one cached position, all layers
    total, parts = bench.algorithmic_bytes_verify(c, 512 + 128)
    assert parts == {"weights": weights, "kv_read": 640 * kv_tok, "kv_write": 9 * kv_tok}
    assert total == weights + 649 * kv_tok and round(total / 1e6, 1) == 283.9
    gemm, attn = bench.algorithmic_flops_verify(c, 640)
    assert gemm == 2.0 * (30 * per_layer + 49152 * 576) * 9
    assert attn == 4.0 * 30 * 9 * 576 * 640
    # 3B class: 36 layers, d 2048, 16 / 2 heads of 128, ffn 11008, vocab 151936, batch 256, k 4, prompt 512, generate 128
    c = W.get_config("cfg5")
    per_layer = 2048 * (2048 + 2 * 256) + 2048 * 2048 + 3 * 2048 * 11008
    total, parts = bench.algorithmic_bytes_verify(c, 512 + 64)
    assert parts["weights"] == (36 * per_layer + 151936 * 2048) * 2 == 6171394048
    assert parts["kv_write"] == 256 * 5 * 36 * 2 * 256 * 2 == 47185920
    assert parts["kv_read"] == 256 * 576 * 36 * 2 * 256 * 2
    gemm, _ = bench.algorithmic_flops_verify(c, 576)
    assert gemm == 2.0 * (36 * per_layer + 151936 * 2048) * 1280 and round(gemm / 1e12, 2) == 7.90
    # fp32 configuration: 4 bytes per element
    c = W.get_config("cfg1")
    _, parts = bench.algorithmic_bytes_verify(c, 96)
    assert parts["weights"] == (2 * (128 * (128 + 2 * 128) + 128 * 128 + 3 * 128 * 512) + 512 * 128) * 4


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr


def test_workload_table_matches_the_configurations_of_the_metric():
    base = json.load(open(os.path.join(ROOT, "BASELINE.json")))
    text = base["configs"]
    assert len(text) == 5
    want = {
        "cfg1": dict(n_layers=2, d_model=128, n_heads=4, d_ffn=512, vocab=512, n_max=3, k=4, batch=1, prompt_len=64, gen_len=64),
        "cfg2": dict(n_layers=30, d_model=576, n_heads=9, n_kv_heads=3, d_ffn=1536, vocab=49152, n_max=4, k=8, batch=1, prompt_len=512, gen_len=256),
        "cfg3": dict(n_layers=24, d_model=896, n_heads=14, n_kv_heads=2, d_ffn=4864, vocab=151936, n_max=4, k=6, batch=32, prompt_len=1024, gen_len=256),
        "cfg4": dict(n_layers=28, d_model=1536, n_heads=12, n_kv_heads=2, d_ffn=8960, vocab=151936, n_max=5, k=8, batch=64),
        "cfg5": dict(n_layers=36, d_model=2048, n_heads=16, n_kv_heads=2, d_ffn=11008, vocab=151936, batch=256, k=4),
    }
    for i, (name, fields) in enumerate(want.items()):
        c = W.get_config(name)
        for key, value in fields.items():
            assert getattr(c, key) == value, (name, key)
            # every number of the table appears in the configuration's description (thousands separators removed)
            assert str(value) in text[i].replace(",", ""), (name, key, value)
