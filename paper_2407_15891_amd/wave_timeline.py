"""Load-balance check of the decode streaming kernel: per-wavefront start / located / end
times from the debug build of the library (`librazor_timeline.so`, compiled with
-DRAZOR_TIMELINE by `__graft_entry__.build()`), which stamps the 100 MHz wall clock in every
wave and leaves the stamps behind the last partial-state slot of the workspace.

    python -m paper_2407_15891_amd.wave_timeline --config 4 [--workers 1024]

Prints when the waves finish (median, p90, max, max / mean), how finish time depends on the
number of head segments a wave crossed, and the per-XCD medians.
"""
import argparse
import os
import sys


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4])
    ap.add_argument("--workers", type=int, default=1024)
    args = ap.parse_args()
    here = os.path.dirname(os.path.abspath(__file__))
    lib = os.path.join(here, "librazor_timeline.so")
    if not os.path.exists(lib):
        sys.exit(f"{lib} not found: run `python __graft_entry__.py` first")
    sys.path.insert(0, os.path.dirname(here))
    import numpy as np
    import torch
    import paper_2407_15891_amd as razor
    from paper_2407_15891_amd.workloads import make_workload

    assert razor._lib is None, "the product library is already loaded in this process"
    razor.LIB_PATH = lib                        # load the debug twin instead
    W = args.workers
    w = make_workload(args.config, "cuda:0", max_new=64)
    caches = []
    for _ in range(3):                          # rotate so that no launch finds its cache in the memory-side cache
        c = razor.RazorCache.from_workload(w, n_workers=W)
        c.compress(w.K, w.V)
        caches.append(c)
    Q, k, v = w.step_inputs(0)
    for it in range(12):
        caches[it % 3].decode(Q, k, v)
    torch.cuda.synchronize()
    c = caches[(12 - 1) % 3]
    g, D = w.Hq // w.Hkv, w.d
    n_heads = w.B * w.Hkv
    slots = razor.RAZOR_MAX_WORKERS + n_heads
    r256 = lambda x: (x + 255) // 256 * 256
    acc_off = r256((n_heads + 2) * 4) + r256(n_heads * 4) + r256(slots * g * 2 * 4)
    off = acc_off + 7000 * g * D * 4            # where the debug build leaves its stamps
    raw = c.workspace[off: off + W * 32].cpu().numpy().view(np.int64).reshape(W, 4)
    desc = c.desc()
    total_blocks = int(((desc["rows"] + 15) // 16).sum())
    per = max(2, -(-total_blocks // W))
    active = min(W, -(-total_blocks // per))
    raw = raw[:active]
    us = (raw[:, :3] - raw[:, 0].min()).astype(np.float64) / 100.0
    print(f"config {args.config}: {w.name}; {n_heads} (sequence, KV head) pairs, {total_blocks} blocks, "
          f"{active} waves x {per} blocks")
    for i, name in enumerate(["start", "located", "end"]):
        col = us[:, i]
        print(f"  {name:8s} min {col.min():8.2f}  p50 {np.median(col):8.2f}  p90 {np.percentile(col, 90):8.2f}  "
              f"max {col.max():8.2f} us")
    busy = us[:, 2] - us[:, 0]
    print(f"  wave busy time: mean {busy.mean():.2f} us, max {busy.max():.2f} us, max / mean {busy.max() / busy.mean():.3f}")
    segs = raw[:, 3]
    for s in sorted(set(segs.tolist())):
        sel = segs == s
        print(f"  waves crossing {s} head segment(s): {int(sel.sum()):5d}, end p50 {np.median(us[sel, 2]):7.2f} "
              f"max {us[sel, 2].max():7.2f} us")
    wg = np.arange(active) // 4
    cu_busy = np.array([busy[wg == x].max() for x in range(wg.max() + 1)])
    print(f"  workgroup (= compute unit) busy time: mean {cu_busy.mean():.2f} us, max {cu_busy.max():.2f} us, "
          f"max / mean {cu_busy.max() / cu_busy.mean():.3f}")
    print("  median end per XCD (workgroup id mod 8): " +
          " ".join(f"{np.median(us[(wg % 8) == x, 2]):.1f}" for x in range(8)))


if __name__ == "__main__":
    main()
