"""Probe, not part of the library: timing-only builds of the attention kernels with one ingredient
removed, to see what each costs and whether the costs overlap.  The variants compute WRONG results
on purpose (operands never loaded, arithmetic skipped); every address stays in bounds and every
loop still ends, so they are safe to time.  A patched copy of csrc/ is compiled into a library of
its own; select it with BSA_LIB=<path> and time it with probes/time_attn.py.

    python -m paper_2509_01085_amd.probes.elimination <out.so> <fwd|dkv> <MODE[,MODE...]>

Modes: NODMA (tiles / records are not loaded), NOCOMPUTE (no wavefront multiplies anything),
NOBARRIER (no workgroup barrier in the tile loop), NOSOFTMAX (no exponentials, maxima or sums),
NOLDS (forward only: matrix operands come from registers instead of LDS), NOMFMA (one vector
multiply-add in place of every matrix instruction)."""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ROOT = os.path.dirname(PKG)
SOURCES = ["bsa_api.hip", "bsa_pool_prune.hip", "bsa_select.hip", "bsa_attn_generic.hip", "bsa_attn_pipe.hip", "bsa_probe.hip"]


def patch_fwd(k: str, modes) -> str:
    def rep(a, b):
        nonlocal k
        assert a in k, a
        k = k.replace(a, b)

    if "NODMA" in modes:
        rep("      if (jn >= 0) {\n        issue(jn, (t + NB - 1) & (NB - 1));", "      if (jn >= 0) {\n        if (jn < 0) issue(jn, (t + NB - 1) & (NB - 1));")
        rep("      if (jb >= 0) {\n        issue(jb, k);", "      if (jb >= 0) {\n        if (jb < 0) issue(jb, k);")
    if "NOCOMPUTE" in modes:
        rep("    const bool mine = mbits != 0;", "    const bool mine = mbits != 0 && a.n_keep > 1000;")
    if "NOBARRIER" in modes:
        rep("    raw_barrier();  // tile t visible to all", "    // (no barrier)")
    if "NOSOFTMAX" in modes:
        rep("        s[0][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[0][r], c2, -mnew));\n        s[1][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[1][r], c2, -mnew));",
            "        s[0][r] = s[0][r] * c2;\n        s[1][r] = s[1][r] - c2;")
        rep("        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);", "        for (int r = 0; r < 1; ++r) mx = fmaxf(mx, s[kt][r]);")
    if "NOLDS" in modes:
        rep("        if (f < 2 * DS) return lds_frag(reinterpret_cast<const uint16_t*>(Kb + 32 * (f / DS) * RB + koffs[f % DS]));", "        if (f >= 0) return qf[f % DS];")
    if "NOMFMA" in modes:
        rep("        s[f / DS] = mfma32(fr[f % RING], qf[f % DS], s[f / DS]);", "        s[f / DS][f % 16] += __builtin_bit_cast(f32x4, fr[f % RING])[0];")
        rep("        o[v % DT] = mfma32(fr[f % RING], pf[v / DT], o[v % DT]);",
            "        o[v % DT][f % 16] += __builtin_bit_cast(f32x4, fr[f % RING])[0] * __builtin_bit_cast(f32x4, pf[v / DT])[1];")
    return k


def patch_dkv(k: str, modes) -> str:
    def rep(a, b):
        nonlocal k
        assert a in k, a
        k = k.replace(a, b)

    if "NODMA" in modes:
        rep("      if (n < NFULL) dma16_raw(src, tid16, dst);\n      else if (NTAIL && wave == 0 && lane < NTAIL) dma16_raw(src, tid16, dst);",
            "      if (n < NFULL && dib[k] < -5) dma16_raw(src, tid16, dst);")
        rep("    for (int n = 0; n < NFULL; ++n) dma16(src + n * (NT * 16), dst + n * (NT * 16));\n    if (NTAIL && wave == 0 && lane < NTAIL) dma16(src + NFULL * (NT * 16), dst + NFULL * (NT * 16));",
            "    for (int n = 0; n < NFULL; ++n) if (ib < -5) dma16(src, dst);")
    if "NOCOMPUTE" in modes:
        rep("    const bool mine = mbits != 0;", "    const bool mine = mbits != 0 && a.n_keep > 1000;")
    if "NOBARRIER" in modes:
        rep("    raw_barrier();  // ... for every wavefront; and every wavefront is done with the previous step's slots", "    // (no barrier)")
    if "NOSOFTMAX" in modes:
        rep("          const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[4 * r4 + e], c2, -l4[e]));", "          const float pv = sacc[4 * r4 + e] * c2;")
        rep("          dp[4 * r4 + e] = pv * (dp[4 * r4 + e] - d4[e]);", "          dp[4 * r4 + e] = dp[4 * r4 + e] - d4[e];")
    if "NOMFMA" in modes:
        rep("        if (f & 2) dp = mfma32(fr[f % RING], fr[(f + 1) % RING], dp);\n        else sacc = mfma32(fr[f % RING], fr[(f + 1) % RING], sacc);",
            "        if (f & 2) dp[f % 16] += __builtin_bit_cast(f32x4, fr[f % RING])[0] * __builtin_bit_cast(f32x4, fr[(f + 1) % RING])[1];\n"
            "        else sacc[f % 16] += __builtin_bit_cast(f32x4, fr[f % RING])[0] * __builtin_bit_cast(f32x4, fr[(f + 1) % RING])[1];")
        rep("        if (v & 1) dk[dt] = mfma32(fr[f % RING], h ? df1 : df0, dk[dt]);\n        else dv[dt] = mfma32(fr[f % RING], h ? pf1 : pf0, dv[dt]);",
            "        if (v & 1) dk[dt][f % 16] += __builtin_bit_cast(f32x4, fr[f % RING])[0] * __builtin_bit_cast(f32x4, h ? df1 : df0)[1];\n"
            "        else dv[dt][f % 16] += __builtin_bit_cast(f32x4, fr[f % RING])[0] * __builtin_bit_cast(f32x4, h ? pf1 : pf0)[1];")
    return k


def main():
    out, which, modes = os.path.abspath(sys.argv[1]), sys.argv[2], sys.argv[3].split(",")
    dst = out + ".src"
    shutil.rmtree(dst, ignore_errors=True)
    shutil.copytree(os.path.join(PKG, "csrc"), dst)
    p = os.path.join(dst, "bsa_attn_pipe.hip")
    s = open(p).read()
    if which == "fwd":
        i = s.index("template <int D, bool SPLITQ, bool COMBINE, bool PACK>\n__global__ __launch_bounds__(SPLITQ ? 512 : 256, 2) void fwd_pipe_kernel")
        j = s.index("// Backward, same streaming scheme.")
        s = s[:i] + patch_fwd(s[i:j], modes) + s[j:]
    else:
        i = s.index("template <int D, int NQT, bool PACK>\n__global__ __launch_bounds__(512, 1) void bwd_dkv_pipe_kernel")
        j = s.index("// Finishes the split units of the dK/dV launch")
        s = s[:i] + patch_dkv(s[i:j], modes) + s[j:]
    open(p, "w").write(s)
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + dst, "-Wno-inline-asm", "-Wno-unused-result"]

    def comp(f):
        o = os.path.join(dst, f + ".o")
        r = subprocess.run(["hipcc", *flags, "-c", os.path.join(dst, f), "-o", o], capture_output=True, text=True)
        if r.returncode:
            raise SystemExit(r.stderr[-3000:])
        return o

    with ThreadPoolExecutor(6) as ex:
        objs = list(ex.map(comp, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs])
    shutil.rmtree(dst, ignore_errors=True)
    print("built", out)


if __name__ == "__main__":
    main()
