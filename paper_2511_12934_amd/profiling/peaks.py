"""Achievable peaks of this MI355X, beside the published ones the roofline fractions are quoted against: what a
bf16 MFMA loop shaped like the scoring kernels' inner loops delivers (operands in registers or the A operand read
from LDS per MFMA; zero, constant or random operand values), and what a plain device copy and a read-only pass
deliver from HBM.  Prints a table and, last, the machine-readable lines ``bench.py`` looks for:

    achievable_peak mfma_bf16 <TFLOP/s>      (random operands, A from LDS: the MLP chain's situation)
    achievable_peak hbm <GB/s>               (copy, bytes read + bytes written)

    python3 -m paper_2511_12934_amd.profiling.peaks
"""
from __future__ import annotations

import ctypes as C
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libaif_calib.so")


def main() -> None:
    import torch
    if not torch.cuda.is_available():
        sys.exit("peaks needs a GPU")
    if not os.path.exists(LIB):
        sys.exit(f"{LIB} is missing: run python -m paper_2511_12934_amd.build")
    lib = C.CDLL(LIB)
    vp = C.c_void_p
    lib.aifcal_mfma.restype = C.c_int
    lib.aifcal_mfma.argtypes = [vp, vp, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.aifcal_copy.restype = C.c_int
    lib.aifcal_copy.argtypes = [vp, vp, C.c_size_t, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.aifcal_fill.restype = C.c_int
    lib.aifcal_fill.argtypes = [vp, C.c_size_t, C.c_int, C.POINTER(C.c_double)]
    g = torch.Generator(device="cuda").manual_seed(1234)
    n = 16 * 64 * 8
    operands = {
        "zero": (torch.zeros(n, dtype=torch.bfloat16, device="cuda"), torch.zeros(n, dtype=torch.bfloat16, device="cuda")),
        "constant": (torch.full((n,), 0.5, dtype=torch.bfloat16, device="cuda"), torch.full((n,), 1.25, dtype=torch.bfloat16, device="cuda")),
        "random N(0,1)": (torch.randn(n, device="cuda", generator=g).to(torch.bfloat16), torch.randn(n, device="cuda", generator=g).to(torch.bfloat16)),
        "random N(0,0.1)": ((torch.randn(n, device="cuda", generator=g) * 0.1).to(torch.bfloat16), (torch.randn(n, device="cuda", generator=g) * 0.1).to(torch.bfloat16)),
    }
    print(f"{'MFMA loop (bf16 32x32x16, 4 accumulators per wave)':58s} {'TFLOP/s':>9s} {'of 2500':>8s} {'clock MHz':>10s}")
    best = {}
    for from_lds in (0, 1):
        for waves in (1, 2):
            for name, (a, b) in operands.items():
                tf, mhz = C.c_double(0), C.c_double(0)
                # about 40 ms of MFMAs per measurement: long enough for the board's power management to settle
                rc = lib.aifcal_mfma(a.data_ptr(), b.data_ptr(), from_lds, waves, 160000 // waves, C.byref(tf), C.byref(mhz))
                assert rc == 0, "aifcal_mfma failed"
                label = f"A from {'LDS' if from_lds else 'registers'}, {waves} wave(s)/SIMD, operands {name}"
                print(f"{label:58s} {tf.value:9.1f} {tf.value / 2500:8.3f} {mhz.value:10.0f}", flush=True)
                best[(from_lds, name)] = max(best.get((from_lds, name), 0.0), tf.value)
    nbytes = 1 << 30
    src = torch.randint(0, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    cp, rd = C.c_double(0), C.c_double(0)
    assert lib.aifcal_copy(src.data_ptr(), dst.data_ptr(), nbytes, 20, C.byref(cp), C.byref(rd)) == 0
    assert bool((dst[-7:] == src[-7:]).all())
    wr = C.c_double(0)
    assert lib.aifcal_fill(dst.data_ptr(), nbytes, 20, C.byref(wr)) == 0
    print(f"\n1 GiB, 16 B per lane: copy {cp.value:.0f} GB/s read + written ({cp.value / 8000:.3f} of 8000); "
          f"read-only pass {rd.value:.0f} GB/s ({rd.value / 8000:.3f}); write-only pass {wr.value:.0f} GB/s ({wr.value / 8000:.3f})")
    lib.aifcal_coissue.restype = C.c_int
    lib.aifcal_coissue.argtypes = [C.POINTER(C.c_double)]
    ns = (C.c_double * 8)()
    assert lib.aifcal_coissue(ns) == 0
    labels = ["1 MFMA", "1 MFMA + 4 v_fma_f32", "1 MFMA + 4 v_exp_f32", "1 MFMA + 4 v_fma_f32 + 4 v_exp_f32",
              "1 MFMA + 8 v_fma_f32 + 8 v_exp_f32", "4 v_fma_f32 + 4 v_exp_f32 (no MFMA)", "8 v_fma_f32 + 8 v_exp_f32 (no MFMA)",
              "16 v_fma_f32 (no MFMA)"]
    print("\nVector-ALU work beside the matrix cores (independent instructions, 3 waves per SIMD, constant operands): ns per group per SIMD")
    for lb, v in zip(labels, ns):
        print(f"  {lb:40s} {v:7.2f}")
    print(f"  => v_fma_f32 {ns[7] / 16:.2f} ns, v_exp_f32 {(ns[6] - ns[7] / 2) / 8:.2f} ns; an MFMA under which the vector work does not fit "
          f"adds {ns[4] - ns[6]:.2f} ns (of its {ns[0]:.2f}) to the vector work's time")
    lib.aifcal_valu_costs.restype = C.c_int
    lib.aifcal_valu_costs.argtypes = [C.POINTER(C.c_double)]
    vc = (C.c_double * 8)()
    assert lib.aifcal_valu_costs(vc) == 0
    print("\nOne kind of vector instruction at a time (16 independent ones per group, 3 waves per SIMD): ns each per SIMD,")
    print("and what one MFMA (14 ns of the matrix cores) per group adds to the group's time")
    for i, nm in enumerate(["v_fma_f32", "v_exp_f32", "v_cvt_pk_bf16_f32", "v_dot2c_f32_bf16"]):
        print(f"  {nm:20s} {vc[i] / 16:5.2f} ns   + MFMA: {vc[4 + i] - vc[i]:+6.2f} ns per group")
    lib.aifcal_attn_loop.restype = C.c_int
    lib.aifcal_attn_loop.argtypes = [vp, vp, C.POINTER(C.c_double)]
    rows = ["whole loop, 3 waves per SIMD", "whole loop, 2 waves per SIMD", "whole loop, 1 wave per SIMD", "without the row sums",
            "without the exponentials", "without the conversions", "without the LDS reads", "MFMAs alone",
            "row sums as 8 v_dot2c_f32_bf16 of the rounded weights", "whole loop once more",
            "two candidate tiles a wave, 2 waves per SIMD"]
    print("\nThe resident attention kernel's key-tile loop in isolation (heads of 64: 8 MFMAs, 16 v_exp_f32, 8 v_cvt_pk_bf16_f32,")
    print("16 v_add_f32, 8 LDS fragment reads per 32-key tile): ns per key tile and SIMD (3 waves per SIMD unless stated)")
    print(f"  {'':48s} {'zeros':>8s} {'N(0,0.1)':>9s}")
    kvz, qz = torch.zeros(64 * 1024, dtype=torch.bfloat16, device="cuda"), torch.zeros(32 * 1024, dtype=torch.bfloat16, device="cuda")
    kvr = (torch.randn(64 * 1024, device="cuda", generator=g) * 0.1).to(torch.bfloat16)
    qr = (torch.randn(32 * 1024, device="cuda", generator=g) * 0.1).to(torch.bfloat16)
    lz, lr = (C.c_double * 11)(), (C.c_double * 11)()
    assert lib.aifcal_attn_loop(kvz.data_ptr(), qz.data_ptr(), lz) == 0
    assert lib.aifcal_attn_loop(kvr.data_ptr(), qr.data_ptr(), lr) == 0
    for i, nm in enumerate(rows):
        print(f"  {nm:48s} {lz[i]:8.1f} {lr[i]:9.1f}")
    print(f"\nachievable_peak mfma_bf16 {best[(1, 'random N(0,0.1)')]:.1f}")
    print(f"achievable_peak hbm {cp.value:.0f}")
    print(f"achievable_peak hbm_read {rd.value:.0f}")
    print(f"achievable_peak hbm_write {wr.value:.0f}")


if __name__ == "__main__":
    main()
