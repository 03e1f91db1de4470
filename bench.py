#!/usr/bin/env python3
"""Benchmark of the STA forward hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input:
sta_tile_permute(Q), (K), (V) -> sta_forward -> sta_untile(O), all through the
C-ABI library, inputs resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is the layer's effective TFLOP/s over kept
tiles (4*P^2*D flop per kept (query tile, key tile) pair) for the whole step;
`roofline` is for the dominant kernel (sta_forward) from HIP-event timing of
the kernel alone; `cpu_baseline` is the fp64 oracle timed on the host cores on
a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2502_04507_amd as sta  # noqa: E402
import synth_inputs as syn  # noqa: E402

BF16_MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0

# HBM-side bytes per sta_forward launch from rocprofv3 FETCH_SIZE + WRITE_SIZE passes, each scaled by what the
# same counter reads for a plain copy of known size (FETCH_SIZE x2.0, WRITE_SIZE x1.0 on this machine); summary in
# profiles/sta_forward_C4_w3x3x3_pmc.txt.  Only workloads that were actually profiled have an entry.
MEASURED_FORWARD_TRAFFIC_BYTES = {
    ("C4", ((3, 3, 3),)): 6.39e9 + 0.708e9,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C4", help="C1..C5 or C4dense")
    ap.add_argument("--window", default=None, help="override: uniform window in tiles, e.g. 3,3,3")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense (full-window) comparison run")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-backward", action="store_true", help="skip the gradient entry point's timing")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target oracle time")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line, time sta_forward for a list of uniform windows and the "
                         "per-head mixed table on the 30x48x80 grid (speedup-versus-sparsity curve), one JSON line")
    ap.add_argument("--extras", action="store_true",
                    help="instead of the benchmark line, time the entry points built on top of the attention kernel "
                         "(log-denominator output, recall, per-head MSE, mask search) on the workload, one JSON line")
    ap.add_argument("--backward", action="store_true",
                    help="instead of the benchmark line, time the gradient entry point (sta_backward) on the workload, "
                         "one JSON line")
    ap.add_argument("--profile-only", default=None, choices=[None, "forward", "permute", "layer", "copy", "backward"],
                    help="run only this part (for rocprofv3), print nothing else; 'copy' is a plain "
                         "device copy of one tensor, the known-size reference for the traffic counters")
    return ap.parse_args()


class Layer:
    """Device buffers of one attention layer call and the calls of the path."""

    def __init__(self, w, device, split=True):
        self.w = w
        self.split = split
        self.q, self.k, self.v = syn.make_qkv_device(w, device)      # raster inputs, resident in HBM
        shape = self.q.shape
        mk = lambda: torch.empty(shape, dtype=torch.bfloat16, device=device)
        self.qt, self.kt, self.vt, self.ot, self.o = mk(), mk(), mk(), mk(), mk()
        self.windows = w.window_tiles
        # scratch with which sta_forward splits the work items of the ragged last round of workgroups
        self.ws = torch.empty(max(sta.sta_workspace_bytes(w.B, w.H, w.D, w.grid, w.tile), 16), dtype=torch.uint8,
                              device=device)

    def permute_in(self):
        w = self.w
        sta.sta_tile_permute(self.q, self.qt, w.grid, w.tile)
        sta.sta_tile_permute(self.k, self.kt, w.grid, w.tile)
        sta.sta_tile_permute(self.v, self.vt, w.grid, w.tile)

    def forward(self, windows=None):
        w = self.w
        sta.sta_forward(self.qt, self.kt, self.vt, self.ot, w.grid, w.tile, windows or self.windows,
                        workspace=self.ws if self.split else None)

    def untile(self):
        sta.sta_untile(self.ot, self.o, self.w.grid, self.w.tile)

    def step(self):
        self.permute_in()
        self.forward()
        self.untile()


def event_time_ms(fn, iters, warmup=1):
    """Average duration of fn() in ms from HIP events on the launch stream."""
    for _ in range(warmup):
        fn()
    stream = torch.cuda.current_stream()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record(stream)
    for _ in range(iters):
        fn()
    stop.record(stream)
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def cpu_baseline(w, target_seconds):
    """Oracle (as it stands) on the host cores, bounded sample of the same workload."""
    from oracle import sta_oracle as orc
    g = torch.Generator().manual_seed(w.seed)
    # one head's worth of the workload's inputs is enough for a bounded sample
    q, k, v = (torch.randn((w.N, w.D), generator=g).to(torch.bfloat16).float().numpy() for _ in range(3))
    win_tokens = orc.window_tiles_to_tokens(w.window_tiles[0], w.tile)
    counts, _ = orc.key_tiles(w.grid, w.tile, win_tokens)
    rng = np.random.default_rng(1)
    cores = orc.num_threads()

    def run(nq):
        idx = np.sort(rng.integers(0, w.N, size=nq)).astype(np.int64)
        t0 = time.perf_counter()
        orc.attention(q, k, v, w.grid, w.tile, win_tokens, query_idx=idx)
        return time.perf_counter() - t0, idx

    t_cal, _ = run(4 * cores)
    nq = int(max(4 * cores, min(w.N, target_seconds / max(t_cal, 1e-6) * 4 * cores)))
    t, idx = run(nq)
    order = orc.tile_order(w.grid, w.tile)
    tile_of_raster = np.empty(w.N, dtype=np.int64)
    tile_of_raster[order] = np.repeat(np.arange(w.n_tiles), w.P)
    kept_keys = counts[tile_of_raster[idx]].astype(np.float64) * w.P
    flops = float((4.0 * w.D * kept_keys).sum())
    return {
        "value": flops / t / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
        "sample": "%d random query tokens of head 0 of %s (all %d key tokens visited per query, fp64), %.1f s"
                  % (nq, w.name, w.N, t),
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported. Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    sta.load_library()          # fails loudly when the HIP library is not built
    device = "cuda:0"
    torch.cuda.set_device(0)

    w = syn.workload(args.workload)
    if args.window:
        w = syn.with_window(w, tuple(int(x) for x in args.window.split(",")))
    layer = Layer(w, device)
    flops = sta.sta_kept_flops(w.B, w.H, w.D, w.grid, w.tile, w.window_tiles)
    tensor_bytes = w.B * w.H * w.N * w.D * 2

    if args.sweep:
        layer.permute_in()
        dense_w = tuple(w.tile_grid)
        rows = []
        dense_ms = None
        windows = [dense_w, (5, 5, 5), (5, 3, 5), (3, 3, 5), (3, 3, 3), (1, 3, 3), (1, 1, 1)]
        for wt in windows:
            table = tuple(tuple(wt) for _ in range(w.H))
            fl = sta.sta_kept_flops(w.B, w.H, w.D, w.grid, w.tile, table)
            ms = event_time_ms(lambda: layer.forward(table), 2 if wt == dense_w else 5, warmup=1)
            if wt == dense_w:
                dense_ms, dense_fl = ms, fl
            rows.append({"window_tiles": "x".join(map(str, wt)), "kept_fraction": fl / dense_fl, "ms": ms,
                         "tflops": fl / ms / 1e9, "frac_of_peak": fl / ms / 1e9 / BF16_MFMA_PEAK_TFLOPS,
                         "speedup_vs_dense": dense_ms / ms, "ideal_speedup": dense_fl / fl})
        mixed = syn.workload("C5").window_tiles
        fl = sta.sta_kept_flops(w.B, w.H, w.D, w.grid, w.tile, mixed)
        ms = event_time_ms(lambda: layer.forward(mixed), 3, warmup=1)
        rows.append({"window_tiles": "C5 per-head mixed", "kept_fraction": fl / dense_fl, "ms": ms,
                     "tflops": fl / ms / 1e9, "frac_of_peak": fl / ms / 1e9 / BF16_MFMA_PEAK_TFLOPS,
                     "speedup_vs_dense": dense_ms / ms, "ideal_speedup": dense_fl / fl})
        print(json.dumps({"sweep": "sta_forward on grid 30x48x80, tile 6x8x8, H=24, D=128, bf16", "rows": rows}))
        return

    if args.extras:
        layer.permute_in()
        H = w.H
        lse_w = torch.empty((w.B, H, w.N), dtype=torch.float32, device=device)
        lse_f = torch.empty_like(lse_w)
        full = tuple(tuple(w.tile_grid) for _ in range(H))
        fwd_ms = event_time_ms(layer.forward, 5)
        lse_ms = event_time_ms(lambda: sta.sta_forward_lse(layer.qt, layer.kt, layer.vt, layer.ot, lse_w, w.grid, w.tile,
                                                           w.window_tiles), 5)
        sta.sta_forward_lse(layer.qt, layer.kt, layer.vt, layer.o, lse_f, w.grid, w.tile, full)
        mean = torch.empty((w.B * H,), dtype=torch.float32, device=device)
        ws = torch.empty(sta.sta_head_mse_workspace_bytes(w.B, H), dtype=torch.uint8, device=device)
        recall_ms = event_time_ms(lambda: sta.sta_attention_recall(lse_w, lse_f, w.grid, ws, mean), 20)
        mse = torch.empty((H,), dtype=torch.float32, device=device)
        mse_ms = event_time_ms(lambda: sta.sta_head_mse(layer.ot, layer.o, w.grid, ws, mse), 20)
        patterns = [(1, 3, 3), (3, 3, 3), (3, 3, 5)]
        losses = torch.empty((len(patterns), H), dtype=torch.float32, device=device)
        best = torch.empty((H,), dtype=torch.int32, device=device)
        search_ms = event_time_ms(lambda: sta.sta_mask_search(layer.qt, layer.kt, layer.vt, w.grid, w.tile, patterns,
                                                              layer.q, layer.k, ws, losses, best), 2, warmup=1)
        torch.cuda.synchronize()
        search_flops = sum(sta.sta_kept_flops(w.B, H, w.D, w.grid, w.tile, tuple(tuple(p) for _ in range(H)))
                           for p in patterns + [tuple(w.tile_grid)])
        print(json.dumps({
            "extras": "%s: B=%d H=%d D=%d grid=%s tile=%s" % (w.name, w.B, H, w.D, w.grid, w.tile),
            "sta_forward_ms": fwd_ms, "sta_forward_lse_ms": lse_ms,
            "sta_attention_recall_ms": recall_ms,
            "sta_attention_recall_GBs": 2.0 * lse_w.numel() * 4 / (recall_ms * 1e-3) / 1e9,
            "sta_head_mse_ms": mse_ms, "sta_head_mse_GBs": 2.0 * tensor_bytes / (mse_ms * 1e-3) / 1e9,
            "sta_head_mse_frac_hbm": 2.0 * tensor_bytes / (mse_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "sta_mask_search_patterns": ["x".join(map(str, p)) for p in patterns],
            "sta_mask_search_ms": search_ms, "sta_mask_search_tflops": search_flops / (search_ms * 1e-3) / 1e12,
            "mean_recall_first_heads": [float(x) for x in mean[:4].cpu()],
            "best_first_heads": [int(x) for x in best[:4].cpu()],
        }))
        return

    bwd = None
    if args.backward or args.profile_only == "backward":
        layer.permute_in()
        lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=device)
        sta.sta_forward_lse(layer.qt, layer.kt, layer.vt, layer.ot, lse, w.grid, w.tile, w.window_tiles)
        d_o = layer.q                                   # any N(0,1) bf16 tensor of the right shape serves as dO
        d_q, d_k, d_v = layer.k, layer.v, layer.o       # raster inputs are no longer needed: reuse as outputs
        bws = torch.empty(sta.sta_backward_workspace_bytes(w.B, w.H, w.grid), dtype=torch.uint8, device=device)
        bwd = lambda: sta.sta_backward(layer.qt, layer.kt, layer.vt, layer.ot, d_o, lse, d_q, d_k, d_v, w.grid, w.tile,
                                       w.window_tiles, bws)
    if args.backward:
        ms = event_time_ms(bwd, max(args.steps // 4, 2), warmup=1)
        torch.cuda.synchronize()
        pairs_flops = sta.sta_kept_flops(w.B, w.H, w.D, w.grid, w.tile, w.window_tiles)     # 4*P^2*D per kept pair
        print(json.dumps({
            "backward": "%s: B=%d H=%d D=%d grid=%s tile=%s" % (w.name, w.B, w.H, w.D, w.grid, w.tile),
            "sta_backward_ms": ms,
            "products_needed": 5, "products_executed": 7,
            "tflops_needed": 2.5 * pairs_flops / (ms * 1e-3) / 1e12,
            "tflops_executed": 3.5 * pairs_flops / (ms * 1e-3) / 1e12,
            "frac_of_peak_needed": 2.5 * pairs_flops / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
            "frac_of_peak_executed": 3.5 * pairs_flops / (ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
            "note": "S and dP are computed in both the dQ kernel and the dK/dV kernel (7 matrix products per kept "
                    "block against the 5 the chain rule needs); the forward pass is not included",
        }))
        return

    if args.profile_only:
        fn = {"backward": bwd, "forward": layer.forward, "permute": lambda: (layer.permute_in(), layer.untile()),
              "layer": layer.step, "copy": lambda: layer.qt.copy_(layer.q)}[args.profile_only]
        layer.permute_in()
        for _ in range(args.warmup + args.steps):
            fn()
        torch.cuda.synchronize()
        return

    # ---- the timed region: exactly K steps bracketed by synchronize ---------------
    for _ in range(args.warmup):
        layer.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layer.step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- per-kernel durations from HIP events on the launch stream ----------------
    iters = max(3, min(args.steps, 20))
    fwd_ms = event_time_ms(layer.forward, iters)
    perm_ms = event_time_ms(lambda: sta.sta_tile_permute(layer.q, layer.qt, w.grid, w.tile), iters)
    untile_ms = event_time_ms(layer.untile, iters)
    copy_ms = event_time_ms(lambda: layer.qt.copy_(layer.q), iters)      # plain device copy of the same tensor
    fwd_tflops = flops / (fwd_ms * 1e-3) / 1e12
    perm_gbs = 2.0 * tensor_bytes / (perm_ms * 1e-3) / 1e9
    untile_gbs = 2.0 * tensor_bytes / (untile_ms * 1e-3) / 1e9
    copy_gbs = 2.0 * tensor_bytes / (copy_ms * 1e-3) / 1e9

    out = {
        "metric": "STA fwd effective TFLOP/s (kept tiles) + ms/layer at 115,200 tokens, d=128",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": "%s: B=%d H=%d D=%d grid=%s tile=%s window_tiles=%s" % (
                w.name, w.B, w.H, w.D, "x".join(map(str, w.grid)), "x".join(map(str, w.tile)),
                "x".join(map(str, w.window_tiles[0])) if len(set(w.window_tiles)) == 1 else "per-head mixed"),
            "tokens": w.N, "kept_tflop": flops / 1e12,
            "step": "tile_permute(Q,K,V) + sta_forward + untile(O)",
        },
        "roofline": {
            "kernel": "sta_forward", "bound": "mfma",
            "achieved": fwd_tflops, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": fwd_tflops / BF16_MFMA_PEAK_TFLOPS,
            "traffic": MEASURED_FORWARD_TRAFFIC_BYTES.get((w.name, tuple(sorted(set(w.window_tiles))))),
            "traffic_unit": "bytes per launch (null = this workload was not profiled)",
            "algorithmic_bytes": 4 * tensor_bytes,
        },
        "kernels": {
            "sta_forward_ms": fwd_ms, "sta_forward_tflops": fwd_tflops,
            "sta_tile_permute_ms": perm_ms, "sta_tile_permute_GBs": perm_gbs,
            "sta_tile_permute_frac_hbm": perm_gbs / HBM_PEAK_GBS,
            "sta_untile_ms": untile_ms, "sta_untile_GBs": untile_gbs,
            "sta_untile_frac_hbm": untile_gbs / HBM_PEAK_GBS,
            "plain_copy_ms": copy_ms, "plain_copy_GBs": copy_gbs,
            "sta_tile_permute_frac_of_plain_copy": perm_gbs / copy_gbs,
            "sta_untile_frac_of_plain_copy": untile_gbs / copy_gbs,
        },
        "paper_context": "H100 bf16, same shape: STA w=(18,24,24) 25.38 ms, MFU 58.79%; dense FA3 265.28 ms "
                         "(paper Table 2; other hardware, context only)",
    }

    if not args.no_dense and w.name.startswith("C4") and len(set(w.window_tiles)) == 1:
        dense_windows = tuple(tuple(w.tile_grid) for _ in range(w.H))
        dense_flops = sta.sta_kept_flops(w.B, w.H, w.D, w.grid, w.tile, dense_windows)
        dense_ms = event_time_ms(lambda: layer.forward(dense_windows), 2, warmup=1)
        out["dense_same_kernel"] = {
            "ms": dense_ms, "tflops": dense_flops / (dense_ms * 1e-3) / 1e12,
            "speedup_sparse_vs_dense": dense_ms / fwd_ms, "ideal_speedup": dense_flops / flops,
            "kernel_efficiency": (flops / fwd_ms) / (dense_flops / dense_ms),
        }

    # What the matrix pipes deliver on this chip, this run, for the attention kernels' MFMA instruction alone:
    # with constant operands (little switching, the clock stays high) and with N(0,1) bf16 operands.
    sink = torch.empty(512 * 256, dtype=torch.float32, device=device)
    probe = {}
    for label, operands in (("constant_operands", torch.ones(8192, dtype=torch.bfloat16, device=device)),
                            ("random_operands", layer.qt.reshape(-1)[:8192].contiguous())):
        probe_flops = sta.sta_probe_mfma(operands, 10000, 512, sink)
        probe_ms = event_time_ms(lambda: sta.sta_probe_mfma(operands, 10000, 512, sink), 3)
        probe[label + "_tflops"] = probe_flops / (probe_ms * 1e-3) / 1e12
    probe["sta_forward_frac_of_random_operand_rate"] = fwd_tflops / probe["random_operands_tflops"]
    probe["what"] = ("v_mfma_f32_32x32x16_bf16 only, 2 waves per SIMD on all CUs, no memory traffic; the nominal "
                     "peak in `roofline` assumes 2.4 GHz, which the chip does not hold on random data")
    out["mfma_probe"] = probe

    if not args.no_backward and w.D == 128 and w.P % 128 == 0:
        lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=device)
        sta.sta_forward_lse(layer.qt, layer.kt, layer.vt, layer.ot, lse, w.grid, w.tile, w.window_tiles)
        bws = torch.empty(sta.sta_backward_workspace_bytes(w.B, w.H, w.grid), dtype=torch.uint8, device=device)
        # dO: any N(0,1) bf16 tensor of the right shape; the raster inputs are not needed any more and hold the outputs
        bwd_ms = event_time_ms(lambda: sta.sta_backward(layer.qt, layer.kt, layer.vt, layer.ot, layer.q, lse, layer.k,
                                                        layer.v, layer.o, w.grid, w.tile, w.window_tiles, bws), 3)
        out["backward"] = {
            "sta_backward_ms": bwd_ms, "matrix_products_needed": 5, "matrix_products_executed": 7,
            "tflops_needed": 2.5 * flops / (bwd_ms * 1e-3) / 1e12,
            "tflops_executed": 3.5 * flops / (bwd_ms * 1e-3) / 1e12,
            "frac_of_peak_executed": 3.5 * flops / (bwd_ms * 1e-3) / 1e12 / BF16_MFMA_PEAK_TFLOPS,
        }

    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(w, args.cpu_seconds)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
