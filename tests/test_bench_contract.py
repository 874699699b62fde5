"""CPU-only checks of bench.py's contract that need no GPU: more than one GPU is refused with a
message (this build has no cross-GPU step), and the host-side work accounting it reports from
matches the workload's definition."""
import os
import subprocess
import sys

import numpy as np

from paper_2504_18154_amd import accounting as acc
from paper_2504_18154_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for extra_env, argv in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "2"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *argv], env=env, capture_output=True, text=True,
                           timeout=120)
        assert r.returncode != 0
        assert "ONE GPU" in r.stderr
        assert r.stdout.strip() == ""


def test_benchmark_workloads_and_their_work():
    """The two batches bench.py times are the 30B-scale configurations, and their algorithmic
    work follows Table 2 (decode: every cached K/V byte once; prefill: causal pairs)."""
    db, pb = wl.config2_decode_30b(), wl.config3_prefill_30b()
    assert (db.B, db.model.Hq, db.model.Hkv, db.model.D, db.model.layers) == (128, 40, 8, 128, 64)
    assert db.ctx_len.min() >= 512 and db.ctx_len.max() <= 4096
    assert pb.B == 16 and pb.q_len.min() >= 128 and pb.q_len.max() <= 4096
    kv = int(db.ctx_len.sum()) * acc.kv_bytes_per_token(1, db.model.Hkv, db.model.D, 2)   # one layer: 4096 B per token
    total = acc.decode_bytes(db.ctx_len, db.model.Hq, db.model.Hkv, db.model.D, 16)
    qo = 2 * db.B * db.model.Hq * db.model.D * 2
    table = 4 * int(np.sum((db.ctx_len + 15) // 16))
    assert total == kv + qo + table
    pairs = sum(int(s) * (int(s) + 1) // 2 for s in pb.q_len)
    assert acc.prefill_flops_causal(pb.q_len, pb.model.Hq, pb.model.D) == 4 * pb.model.Hq * pb.model.D * pairs
