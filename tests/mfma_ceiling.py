#!/usr/bin/env python3
"""Matrix-pipe ceilings for the instruction mix of the GEMM scoring kernel (tests/csrc/probe.hip,
probe_mfma_ceiling_kernel): what `v_mfma_f32_32x32x16_bf16` sustains on this machine from registers
only, with the A operand re-read from LDS for every 32-key sub-tile, and with the scale / document-max
epilogue on top.  The numbers bound what score_gemm_kernel can reach; see profiles/mfma_ceiling.txt."""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))


def main():
    lib = ctypes.CDLL(os.path.join(HERE, "libmsa_probe.so"))
    lib.probe_mfma_ceiling.restype = ctypes.c_float
    lib.probe_mfma_ceiling.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    scratch = torch.zeros(1024, dtype=torch.float32, device="cuda")
    names = {0: "registers only", 1: "A operand from LDS", 2: "A from LDS + scale/max epilogue",
             3: "same, two accumulator sets"}
    iters = 2048
    for mode in (0, 1, 2, 3):
        for blocks in (256, 512):
            ms = lib.probe_mfma_ceiling(mode, blocks, iters, ctypes.c_void_p(scratch.data_ptr()))
            assert ms > 0
            tflops = blocks * 4 * iters * 32 * 32768.0 / ms / 1e9
            print(f"{names[mode]:34s} {blocks // 256} workgroup(s) per CU: {ms:7.3f} ms  {tflops:7.1f} TFLOP/s "
                  f"({tflops / 2500:.2f} of 2.5 PFLOP/s)", flush=True)


if __name__ == "__main__":
    main()
