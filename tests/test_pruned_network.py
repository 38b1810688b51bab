"""Facts the paper prints about pruning and truncation (Sec. 3.3, Fig. 5), checked on the library's own code.

The pruned transform networks of the kernels (`dft_prune_out`, `dft_prune_in`, `RegFFT` in csrc/fft_regs.h) are
templates.  The first test instantiates them for the paper's 4-point example, compiles them for gfx950 with the
library's flags and counts the floating-point additions and subtractions in the instruction stream: one complex
add or subtract (one "operation" of Fig. 5) is two real ones, and a 4-point network needs no multiplies at all.  The second reads the size of the truncated-spectrum buffer that the forward kernel writes.
"""
import os
import re
import shutil
import subprocess
import textwrap

import pytest

from paper_2504_11681_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2504_11681_amd", "csrc")
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_rows(name):
    return [l.split() for l in open(os.path.join(GOLDEN, name)) if l.strip() and l[0] != "#"]


def real_op_counts(tmp_path, kernels):
    """{name: (v_add_f32 + v_sub_f32, multiplies and fused multiply-adds)} of the gfx950 code of `kernels`."""
    src = tmp_path / "networks.hip"
    src.write_text('#include "fft_regs.h"\nusing namespace tfno;\n' + kernels)
    out = tmp_path / "networks.s"
    subprocess.run(["hipcc", "--cuda-device-only", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang",
                    "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", CSRC, "-S", "-o", str(out), str(src)],
                   check=True, capture_output=True, timeout=120)
    counts = {}
    for m in re.finditer(r"^(\w+):[^\n]*\n(.*?)s_endpgm", out.read_text(), flags=re.S | re.M):
        body = m.group(2)
        assert "v_pk_" not in body, "packed FP32 must stay switched off"
        counts[m.group(1)] = (len(re.findall(r"\bv_(?:add|sub)_f32", body)),
                              len(re.findall(r"\bv_(?:mul|fma|fmac|mad|mac)\w*_f32", body)))
    return counts


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc to compile fft_regs.h for gfx950")
def test_pruned_networks_execute_the_operation_counts_the_paper_prints(tmp_path):
    rows = [(int(n), int(kept), int(ops)) for n, kept, ops in golden_rows("pruning_op_counts.txt")]
    assert (4, 1, 3) in rows and (4, 2, 6) in rows and (4, 4, 8) in rows
    fns = ""
    for n, kept, _ in rows:
        fns += textwrap.dedent(f"""
            extern "C" __global__ void fwd_{n}_{kept}(const c64 *in, c64 *out)
            {{
                c64 o[{kept}];
                dft_prune_out<{n}, {kept}, -1>([&](auto t) {{ return in[decltype(t)::value]; }}, o);
                for (int i = 0; i < {kept}; ++i) out[i] = o[i];
            }}""")
    # the full transform of the fused kernels' row stage, and the input-pruned (zero-padded) inverse networks
    fns += textwrap.dedent("""
        extern "C" __global__ void full_4(const c64 *in, c64 *out)
        {
            c64 v[4] = {in[0], in[1], in[2], in[3]}, o[4];
            RegFFT<4, -1, 1>::run(v, o);
            for (int i = 0; i < 4; ++i) out[i] = o[i];
        }
        extern "C" __global__ void inv_4_2(const c64 *in, c64 *out)
        {
            c64 v[2] = {in[0], in[1]};
            dft_prune_in<4, 2, +1>(v, [&](auto t, c64 val) { out[decltype(t)::value] = val; });
        }
        extern "C" __global__ void inv_4_1(const c64 *in, c64 *out)
        {
            c64 v[1] = {in[0]};
            dft_prune_in<4, 1, +1>(v, [&](auto t, c64 val) { out[decltype(t)::value] = val; });
        }""")
    counts = real_op_counts(tmp_path, fns)
    for n, kept, ops in rows:
        adds, muls = counts[f"fwd_{n}_{kept}"]
        assert (adds, muls) == (2 * ops, 0), (n, kept, adds, muls)       # Fig. 5: 8, 3 and 6 complex operations
    assert counts["full_4"] == (16, 0)
    # zero padding is the mirror image on the input side (Sec. 3.3): two non-zero inputs of four need 4 operations,
    # a single one none (its four outputs are copies)
    assert counts["inv_4_2"] == (8, 0) and counts["inv_4_1"] == (0, 0)


def test_forward_kernel_writes_a_quarter_of_the_spectrum_for_64_of_256():
    """Sec. 3.3: keeping 64 of 256 bins removes 75 % of the forward transform's global writes.  The forward kernel of
    the CGEMM + iFFT variant writes exactly the buffer tfno_workspace_bytes(1, 4, ...) describes."""
    binding.lib()
    for n, kept, frac in golden_rows("truncation_traffic.txt"):
        n, kept, frac = int(n), int(kept), float(frac)
        B, C = 512, 128
        truncated = binding.workspace_bytes(1, 4, B, C, C, n, kept)
        full = 8 * B * C * n
        assert truncated > 0 and 1.0 - truncated / full == frac
