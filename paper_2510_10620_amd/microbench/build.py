"""Builds the standalone gfx950 micro-benchmarks in this folder (no torch, no library):

    python -m paper_2510_10620_amd.microbench.build      # -> paper_2510_10620_amd/microbench/bin/<name>

  isa_probe          semantics of ds_read_b64_tr_b16 and the 32x32x16 / 16x16x32 bf16 MFMA operand layouts
  clock_mfma_peak    shader clock and the rate of v_mfma_f32_32x32x16_bf16, on constants and on data-like operands
  mfma_chains        cycles per MFMA when 1..8 accumulators are updated round-robin (dependent-issue cost)
  lds_bandwidth      ds_read_b128 / ds_read_b64 / ds_read_b64_tr_b16 bytes per clock per CU
  lds_patterns       ds_read_b128 rate of the kernels' swizzled tile layout against other layouts
  mfma_valu_overlap  whether vector-ALU instructions run in the shadow of MFMAs, in one wave and across two waves of a SIMD
  valu_rates         cycles per wave instruction of v_fma / v_exp / v_max3 / v_cvt_pk_bf16, one and two waves per SIMD
  lds_copy_issue     cycles a wave spends issuing 4 or 8 global_load_lds_dwordx4, alone and with the workgroup's other waves
  hbm_stream         GB/s of plain read-only, write-only and copy kernels (what the HBM-bound kernels can be held against)
  loop_ingredients   MFMA rate of the attention inner-loop skeleton as LDS operands, softmax ALU work
                     and the barrier are added one by one
They were used to choose the LDS layout and to bound what the kernel structure can reach.
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build():
    out = os.path.join(HERE, "bin")
    os.makedirs(out, exist_ok=True)
    for f in sorted(os.listdir(HERE)):
        if f.endswith(".hip"):
            exe = os.path.join(out, f[:-4])
            cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                   "-Wno-unused-result", "-o", exe, os.path.join(HERE, f)]
            r = subprocess.run(cmd, capture_output=True, text=True)
            if r.returncode != 0:
                raise RuntimeError(r.stderr)
            print("built", exe)


if __name__ == "__main__":
    build()
