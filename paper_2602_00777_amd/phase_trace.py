"""Per-phase timing of the hot kernels from a tuning build of the library.

The product library carries no timing code.  A tuning build does (``csrc/trace.h``: thread 0
of every workgroup stamps the 100 MHz wall clock at a few fixed points); build one next to the
product library and point this tool at it:

    HYLRA_EXTRA_FLAGS="-DHYLRA_TRACE -fgpu-rdc" HYLRA_LIB_OUT=/tmp/libhylra_trace.so \\
        python -m paper_2602_00777_amd.build
    python -m paper_2602_00777_amd.phase_trace --lib /tmp/libhylra_trace.so --workload long_131k

For one Full layer (streaming kernel, then the selection) and one Reuse layer of the workload
it prints, over the workgroups of the launch, the median / 90th percentile / maximum duration
of every phase and when the phase ended, counted from the first workgroup's first stamp.
The stamps cost a little: read the phases against each other, and take absolute kernel times
from rocprofv3 on the product library.
"""
from __future__ import annotations

import argparse
import ctypes

import numpy as np
import torch

ROWS = 8192         # workgroups per region of the trace buffer (csrc/trace.h)

FULL_PHASES = [(0, "workgroup start"), (5, "first tile requested, queue set up"), (1, "streaming loop done"),
               (2, "barrier after the loop"), (3, "scores written out"), (4, "partials stored, histogram flushed")]
SCAN_PHASES = [(4, "rows and histogram requested"), (5, "level-1 threshold picked"), (2, "rows counted"),
               (3, "list entries placed"), (6, "barrier"), (7, "list (and headers) sent")]
EMIT_PHASES = [(8, "headers polled / start"), (9, "lists loaded, level-2 histogram"), (10, "level-2 threshold picked"),
               (11, "rows classified"), (12, "candidates ranked"), (13, "indices written")]
REUSE_COUNTER = [(0, "workgroup start"), (1, "row loop entered"), (2, "rows loaded and consumed"),
                 (3, "partial stored (issue)"), (4, "stores acknowledged, barrier"), (5, "arrival counter answered"),
                 (6, "last workgroup: partials merged, output written")]
REUSE_PACKETS = [(0, "workgroup start"), (1, "row loop entered"), (2, "rows loaded and consumed"),
                 (3, "waves done (thread 0)"), (4, "states staged, packets sent"), (5, "packets polled, barrier"),
                 (6, "slice merged, output written")]
REUSE_SINGLE = [(0, "workgroup start"), (1, "row loop entered"), (2, "rows loaded and consumed (last sweep)")]


def report(title, t, phases):
    """t: [workgroups, 16] stamps in microseconds (0 = not stamped)."""
    slots = [s for s, _ in phases]
    ok = np.all(t[:, slots[:2]] > 0, axis=1)
    t = t[ok]
    if t.shape[0] == 0:
        print("%s: no workgroup stamped" % title)
        return
    base = t[:, slots[0]].min()
    last = max(t[:, s][t[:, s] > 0].max() for s in slots if np.any(t[:, s] > 0))
    print("%s: %d workgroups, first stamp to last %.1f us" % (title, t.shape[0], last - base))
    prev = slots[0]
    v = t[:, prev] - base
    print("   %-48s                          at med %6.2f max %6.2f" % (phases[0][1], np.median(v), v.max()))
    for s, label in phases[1:]:
        have = (t[:, s] > 0) & (t[:, prev] > 0)
        if not np.any(have):
            continue
        d, e = (t[:, s] - t[:, prev])[have], (t[:, s] - base)[have]
        print("   %-48s dur med %5.2f p90 %5.2f max %5.2f | ends med %6.2f max %6.2f  (n=%d)" % (
            label, np.median(d), np.percentile(d, 90), d.max(), np.median(e), e.max(), have.sum()))
        prev = s


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--lib", required=True, help="library built with -DHYLRA_TRACE -fgpu-rdc")
    ap.add_argument("--workload", default="llama3_8b_32k")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value")
    args = ap.parse_args(argv)

    from paper_2602_00777_amd import binding, synth

    binding.LIB_PATH = args.lib
    lib = binding.load_library()
    if not hasattr(lib, "hylra_debug_set_trace"):
        raise SystemExit("%s is not a tuning build (no hylra_debug_set_trace)" % args.lib)
    dev = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    policy = w.policy()
    full_l = int(np.flatnonzero(policy == synth.FULL)[0])
    reuse_l = int(np.flatnonzero(policy == synth.REUSE)[0])
    planted = synth.planted_positions(synth.scaled(w, n_layers=reuse_l + 1))
    qf, Kf, Vf = synth.make_layer(w, full_l, planted[full_l], dev)
    qr, Kr, Vr = synth.make_layer(w, reuse_l, planted[reuse_l], dev)
    trace = torch.zeros(2 * ROWS * 16, dtype=torch.int64, device=dev)

    def stamps():
        torch.cuda.synchronize()
        t = trace.cpu().numpy().reshape(2, ROWS, 16).astype(np.float64) / 100.0
        trace.zero_()
        torch.cuda.synchronize()
        return t

    print("workload %s: %s" % (w.name, w.description))
    with binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k) as ctx:
        for kv in args.opt:
            name, value = kv.split("=")
            ctx.set_option(name, int(value))
        for _ in range(3):
            _, idx = ctx.full_attn_topk(qf, Kf, Vf, w.top_k)
            ctx.reuse_sparse_attn(qr, Kr, Vr, idx)
        torch.cuda.synchronize()
        lib.hylra_debug_set_trace(ctypes.c_void_p(trace.data_ptr()))
        ctx.full_attn_topk(qf, Kf, Vf, w.top_k)
        t = stamps()
        report("Full layer, streaming kernel", t[0], FULL_PHASES)
        launches = ctx.get_info("last_topk_launches")
        sel = t[1]
        scan_rows = sel[:, 7] > 0
        emit_rows = sel[:, 13] > 0
        report("selection, scan part (%d launch%s)" % (launches, "" if launches == 1 else "es"), sel[scan_rows], SCAN_PHASES)
        report("selection, emit part", sel[emit_rows], EMIT_PHASES)
        if np.any(scan_rows) and np.any(emit_rows):
            print("   scan part's first stamp to emit part's last: %.1f us" % (sel[emit_rows][:, 13].max() - sel[scan_rows][:, 4].min()))
        ctx.reuse_sparse_attn(qr, Kr, Vr, idx)
        t = stamps()
        merge = ctx.get_info("last_reuse_merge")
        how = {1: ("arrival counter", REUSE_COUNTER), 2: ("packets", REUSE_PACKETS), 3: ("one workgroup per pair", REUSE_SINGLE)}.get(merge)
        if how:
            report("Reuse layer (%d partials per pair, %d rows per wave tile, merge: %s)" % (
                ctx.get_info("last_reuse_splits"), ctx.get_info("last_reuse_wave_rows"), how[0]), t[0], how[1])
        lib.hylra_debug_set_trace(ctypes.c_void_p(0))


if __name__ == "__main__":
    main()
