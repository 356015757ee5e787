"""The seeded input generators: shapes, structure and determinism of the five configurations
(reduced contexts on the CPU)."""
import numpy as np
import torch

from paper_2407_15891_amd.workloads import make_workload, retrieval_pairs_stack


def test_shapes_masks_and_windows():
    w1 = make_workload(1, "cpu")
    assert (w1.B, w1.Hq, w1.Hkv, w1.d, w1.N, w1.dtype) == (1, 8, 8, 64, 2048, torch.float32)
    assert w1.mask.tolist() == [1, 0, 0, 0, 0, 1, 0, 0] and (w1.n_sink, w1.window) == (4, 256)
    assert float(w1.K[:, :, :4].abs().mean()) > 2.5 * float(w1.K[:, :, 4:].abs().mean())   # sink keys x4
    for cfg, hq, hkv, n_ret, steps in ((2, 32, 32, 5, 64), (3, 32, 8, 2, 1), (4, 64, 8, 1, 1)):
        w = make_workload(cfg, "cpu", materialize=False)
        assert (w.Hq, w.Hkv, w.d, w.dtype) == (hq, hkv, 128, torch.bfloat16)
        assert int(w.mask.sum()) == n_ret and w.decode_steps == steps
    assert make_workload(2, "cpu", materialize=False).window == 6553          # floor(0.20 * 32768)
    assert make_workload(3, "cpu", materialize=False).window == 19660         # max(4096, floor(0.15 * 131072))
    assert make_workload(3, "cpu", context=8192, materialize=False).window == 4096
    w4 = make_workload(4, "cpu", materialize=False)
    assert w4.window == 2048 and w4.B == 16 and w4.seq_lens.min() >= 8192 and w4.seq_lens.max() <= 65536
    assert len(set(w4.seq_lens.tolist())) > 8                                 # ragged


def test_config2_outlier_channels():
    w = make_workload(2, "cpu", context=512)
    for t in (w.K, w.V):
        col = t.float().abs().mean(dim=(0, 2))                                # [H, d]
        big = (col > 4 * col.median(dim=1, keepdim=True).values).sum(1)
        assert (big == 4).all()


def test_config5_stack_masks():
    table = retrieval_pairs_stack(32, 8, 0.15, 5000)
    assert table.shape == (32, 8) and table.sum() == 38
    for layer in (0, 7, 31):
        assert (make_workload(5, "cpu", layer=layer, materialize=False).mask == table[layer]).all()


def test_determinism_and_step_inputs():
    a = make_workload(3, "cpu", context=300, batch=2)
    b = make_workload(3, "cpu", context=300, batch=2)
    assert torch.equal(a.K, b.K) and torch.equal(a.V, b.V) and (a.mask == b.mask).all()
    qa, ka, va = a.step_inputs(5)
    qb, kb, vb = b.step_inputs(5)
    assert torch.equal(qa, qb) and torch.equal(ka, kb) and torch.equal(va, vb)
    assert not torch.equal(qa, a.step_inputs(6)[0])
    assert a.step_inputs(0, append=False)[1] is None
    assert not torch.equal(a.K, make_workload(3, "cpu", context=300, batch=2, layer=1).K)
    assert np.isclose(a.scale, 128 ** -0.5)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: any other --gpus value ends with a message and a non-zero status
    before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_algorithmic_bytes_of_configuration_3_by_hand():
    """The numerators of the roofline figures, against arithmetic done by hand for configuration 3
    (Table 2 settings at 131072 tokens: 4 sinks, window 19660; 4 sequences x 8 KV heads, 2 of them
    retrieval): a compressed head keeps 4 + 19660 rows, a retrieval head all 131072."""
    import os
    import sys

    import paper_2407_15891_amd as razor
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench

    w = make_workload(3, "cpu", materialize=False)
    desc = np.zeros(w.B * w.Hkv, razor.DESC_DTYPE)
    sizes = razor.RazorSizes()
    p = razor.RazorParams(w.B, w.Hq, w.Hkv, w.d, w.n_sink, w.window, 0, 1, razor.RAZOR_BF16, razor.RAZOR_F32,
                          w.scale, 0, 0, 0, None, None)
    assert razor.razor_plan(p, w.seq_lens, w.mask, desc, None, sizes) == 0
    kept_rows = 4 * (2 * 131072 + 6 * (4 + 19660))
    assert int(desc["rows"].sum()) == kept_rows == 1_520_512
    row_bytes = 2 * 128 * 2                                      # K and V, 128 bf16 each
    by_hand = (kept_rows * row_bytes                              # every cached row once
               + 4 * 6 * 2 * 128 * 4                              # khat, vhat (fp32) of the 24 compressed heads
               + 4 * 32 * 128 * 2 + 4 * 32 * 128 * 2              # Q in, O out (bf16)
               + 32 * 48)                                         # the table
    assert bench.algorithmic_bytes_decode(desc, w.d, 2, w.B, w.Hq, 2) == by_hand == 778_593_792
    src_rows = 4 * 8 * 131072
    assert bench.algorithmic_bytes_compress(desc, w.seq_lens, w.Hkv, w.d, 2) == \
        (src_rows + kept_rows) * row_bytes + 32 * 2 * 128 * 4
