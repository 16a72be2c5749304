#!/usr/bin/env python3
"""What one MI355X sustains for the instruction mix of the attention step with nothing else in the
way (paper_2501_15383_amd/csrc/vs_ceiling.hip): no global memory traffic, no barriers, no tile walk.
Each line runs one variant for about 0.3 s on all compute units (two workgroups of four waves each,
the occupancy of the attention kernel) and prints the bf16 MFMA rate.  The attention kernel's own
rate on issued tiles belongs next to the line "1 fragment + 3 fma + 1 exp, random operands".

    python3 bench_ceiling.py > profiles/stream_ceiling_mi355x.txt
"""
import ctypes as C
import os
import sys

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(ROOT, "paper_2501_15383_amd", "libvs_ceiling.so")

VARIANTS = [(0, "MFMA + 1 LDS fragment,                  small-integer operands"),
            (1, "MFMA + 1 LDS fragment,                  random operands"),
            (2, "MFMA + 1 fragment + 3 fma + 1 exp,      small-integer operands"),
            (3, "MFMA + 1 fragment + 3 fma + 1 exp,      random operands   <- the mix of the attention step"),
            (4, "MFMA + 1 fragment + 2 fma + 1 exp,      random operands"),
            (5, "MFMA + 1 fragment + 4 fma + 1 exp,      random operands")]

STEP_VARIANTS = [(0, "fused step, LDS tiles left as they are (no copies)"),
                 (2, "fused step + the global -> LDS copy of K (16 KiB per workgroup and step)"),
                 (1, "fused step + the copies of K and V (32 KiB per step)   <- what the kernel's step does")]


def main():
    if not os.path.exists(LIB):
        raise SystemExit(f"{LIB} is missing: build it with python -c 'import __graft_entry__ as g; g.build()'")
    lib = C.CDLL(LIB)
    lib.vsc_launch.restype = C.c_int
    lib.vsc_launch.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
    assert torch.cuda.is_available(), "bench_ceiling.py needs a GPU"
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    blocks, iters = 2 * n_cu, 400000
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    print("# instruction-mix ceiling, written by bench_ceiling.py (one MI355X, %d compute units, %d workgroups of 256 threads,"
          % (n_cu, blocks))
    print("# %d x 16 MFMAs per wave; bf16 v_mfma_f32_32x32x16 = 32768 FLOP; nominal dense bf16 peak 2500 TFLOP/s)" % iters)
    for rep in range(2):
        for var, name in VARIANTS:
            assert lib.vsc_launch(var, blocks, 1000, out.data_ptr(), st) == 0
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            assert lib.vsc_launch(var, blocks, iters, out.data_ptr(), st) == 0
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            tf = blocks * 4 * iters * 16 * 32768.0 / (ms * 1e-3) / 1e12
            print(f"pass {rep}  {name:92s} {ms:8.1f} ms  {tf:7.1f} TFLOP/s  {100 * tf / 2500:5.1f} % of nominal")
            sys.stdout.flush()
    # the fused step of k_attention on its own (same LDS layouts, interleaving and dependences; no walk, no masks)
    lib.vsc_step_src_bytes.restype = C.c_size_t
    lib.vsc_launch_step.restype = C.c_int
    lib.vsc_launch_step.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    n_src = int(lib.vsc_step_src_bytes())
    src = (torch.rand(n_src // 2, device="cuda") - 0.5).to(torch.bfloat16)       # random values, as K and V hold
    step_iters = 150000
    print("# the arithmetic stream of one steady-state step of k_attention (32 MFMAs per wave and step), stand-alone;")
    print("# the kernel's own rate on a dense list (dense_tflops of bench.py) belongs next to the line with both copies")
    for rep in range(2):
        for var, name in STEP_VARIANTS:
            assert lib.vsc_launch_step(var, blocks, 1000, out.data_ptr(), src.data_ptr(), n_src, st) == 0
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            assert lib.vsc_launch_step(var, blocks, step_iters, out.data_ptr(), src.data_ptr(), n_src, st) == 0
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            tf = blocks * 4 * step_iters * 32 * 32768.0 / (ms * 1e-3) / 1e12
            print(f"pass {rep}  {name:92s} {ms:8.1f} ms  {tf:7.1f} TFLOP/s  {100 * tf / 2500:5.1f} % of nominal")
            sys.stdout.flush()


if __name__ == "__main__":
    main()
