"""In-kernel phase timers of the two kernels of a batched LSTM step (profiling build).

    python -m paper_1802_00150_amd.build --phase-timing
    AMQ_LIBRARY=paper_1802_00150_amd/libamq_phases.so python -m paper_1802_00150_amd.phase_timing [B H k]

The profiling build writes the shader clock at marked points of workgroup (0, 0) into a device buffer
(one row of 32 marks per wave).  This script runs the on-line quantizer and the fused products + cell
kernel at a recurrent step's shape (default: batch 64, hidden 1024, 3-bit) and prints, per kernel, the
cycles between consecutive marks of wave 0 (median over repeated launches) and the spread over waves.
The timers cost a scalar memory-time read, a wait and a store per mark, so the sums run a few per cent
above the un-instrumented kernels; the split between phases is what they are for.
"""
import ctypes as C
import sys

import numpy as np
import torch

from . import binding

QUANT_MARKS = [(0, "start"), (1, "vector in registers"), (2, "greedy initialisation done (Eq. 4)"),
               (4, "cycle 1: reduction of B^T w and Gram counts"), (5, "cycle 1: k x k solve (Eq. 5)"),
               (6, "cycle 1: sorted code table"), (7, "cycle 1: code assignment (Alg. 1)"),
               (8, "cycle 2: reduction"), (9, "cycle 2: solve"), (10, "cycle 2: code table"),
               (11, "cycle 2: code assignment"), (31, "codes and coefficients stored")]
STEP_MARKS = [(0, "start"), (1, "operand requests issued"),
              (9, "own share of the activation operands expanded and written"), (2, "barrier: activation operands complete"),
              (3, "weight words arrived and written to the private piece of LDS"), (4, "weight words in operand layout"),
              (10, "first operands ready"), (5, "contraction done (matrix cores)"),
              (6, "coefficient epilogue done"), (7, "x/h exchange (barrier)"), (8, "cell applied, stores issued")]


def _report(name, names, samples, row0, origin_row=None):
    """origin_row: row whose mark 0 is the time origin (default: wave 0 of the reported kernel; for a step
    that runs as one launch the quantizer's wave 0, which puts both roles on one time line)."""
    allrows = np.asarray(samples, np.int64)
    samples = allrows[:, row0:row0 + 8]   # [launch, wave, mark]
    print(name)
    start = samples[:, 0, names[0][0]] if origin_row is None else allrows[:, origin_row, 0]
    nwaves = [w for w in range(samples.shape[1]) if (samples[:, w, names[0][0]] != 0).all()]
    print("  %-58s %s" % ("cycles after wave 0 started, per wave:", " ".join("%6d" % w for w in nwaves)))
    for i, label in names:
        row = []
        for w in nwaves:
            ok = (samples[:, w, i] != 0).all()
            row.append("%6.0f" % np.median(samples[:, w, i] - start) if ok else "     -")
        print("  %-58s %s" % (label, " ".join(row)))


def main():
    B, H, k = (int(a) for a in sys.argv[1:4]) if len(sys.argv) >= 4 else (64, 1024, 3)
    L = binding.lib()
    if not hasattr(L, "amq_debug_set_phase_buffer"):
        raise SystemExit("this is not the profiling build: build with --phase-timing and set AMQ_LIBRARY")
    L.amq_debug_set_phase_buffer.argtypes = [C.c_void_p]
    dev = "cuda:0"
    s = torch.cuda.current_stream().cuda_stream
    g = torch.Generator().manual_seed(1)
    buf = torch.zeros((16, 32), dtype=torch.int64, device=dev)
    wpr = binding.wpr(H)
    h = torch.tanh(torch.randn(B, H, generator=g)).to(dev)
    x = torch.randn(B, H, generator=g).to(dev)
    c = torch.randn(B, H, generator=g).to(dev)
    W = [(torch.randn(4 * H, H, generator=g) * 0.02).to(dev) for _ in range(2)]
    (Wxp, ax), (Whp, ah) = [binding.quantize_weights(w, k, 2) for w in W]
    P = torch.empty((k, B, wpr), dtype=torch.int32, device=dev)
    be = torch.empty((B, k), device=dev)
    Xp, bx = binding.quantize_activations(x, k, 2)
    Hp, bh = binding.quantize_activations(h, k, 2)
    ho, co = torch.empty_like(c), torch.empty_like(c)

    ws = binding.lstm_workspace(H, H, B, k, dev)

    def step():   # one whole step: the quantizer launch (x_t and h_{t-1}), then products + cell
        L.amq_lstm_step(Wxp.data_ptr(), ax.data_ptr(), Whp.data_ptr(), ah.data_ptr(), H, H, k, None, x.data_ptr(),
                        h.data_ptr(), c.data_ptr(), B, k, 2, ho.data_ptr(), co.data_ptr(), ws.data_ptr(), ws.numel(), s)

    samples = []
    for it in range(40):
        L.amq_debug_set_phase_buffer(None)
        for _ in range(3):
            step()
        buf.zero_()
        torch.cuda.synchronize()
        L.amq_debug_set_phase_buffer(buf.data_ptr())
        step()
        torch.cuda.synchronize()
        if it >= 5:
            samples.append(buf.cpu().numpy().copy())
    L.amq_debug_set_phase_buffer(None)
    _report("on-line quantizer, %d vectors of %d, %d-bit, T=2" % (2 * B, H, k), QUANT_MARKS, samples, 0)
    _report("products + LSTM cell, 4H x 2H = %d x %d, batch %d, W%d/A%d" % (4 * H, 2 * H, B, k, k), STEP_MARKS,
            samples, 8)
    # the split step of a sequence with given inputs: the marks left are those of the last step's launches
    # (front launch: only the vectors of h to quantize; back launch: h-side sums + cell)
    xs = torch.randn(3, B, H, generator=g).to(dev)
    wss = binding.lstm_sequence_workspace(H, H, B, k, dev)
    hh, cc = h.clone(), c.clone()

    def sequence():
        L.amq_lstm_sequence(Wxp.data_ptr(), ax.data_ptr(), Whp.data_ptr(), ah.data_ptr(), H, H, k, None, xs.data_ptr(), 3,
                            hh.data_ptr(), cc.data_ptr(), B, k, 2, None, wss.data_ptr(), wss.numel(), s)

    samples = []
    for it in range(40):
        L.amq_debug_set_phase_buffer(None)
        for _ in range(2):
            sequence()
        buf.zero_()
        torch.cuda.synchronize()
        L.amq_debug_set_phase_buffer(buf.data_ptr())
        sequence()
        torch.cuda.synchronize()
        if it >= 5:
            samples.append(buf.cpu().numpy().copy())
    L.amq_debug_set_phase_buffer(None)
    _report("split step, front launch of the last step: quantizer of h (%d vectors)" % B, QUANT_MARKS, samples, 0)
    _report("split step, back launch: h-side sums + stored x-side sums + cell", STEP_MARKS, samples, 8)


if __name__ == "__main__":
    main()
