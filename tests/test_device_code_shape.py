"""The copy kernel's loop keeps its shape in the generated code (CPU only: hipcc cross-compiles).

gather_kernel's loop holds four workgroup barriers.  A compiler that threads a
lone lane's path across the loop's back edge duplicates parts of the loop body,
barriers included, and lanes then no longer meet at the same barrier (seen once
while the kernel was written: the workgroup copied one tile for ever).  Every
instance of the kernel must therefore come out with exactly four barrier
instructions, each source barrier once."""
import os
import re
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2512_01357_amd", "csrc", "tangram_api.hip")


def test_every_gather_kernel_instance_has_each_barrier_once(tmp_path):
    from paper_2512_01357_amd.build import HIPCC_FLAGS
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = tmp_path / "device.s"
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    proc = subprocess.run([hipcc] + flags + ["-x", "hip", "--cuda-device-only", "-S", SRC, "-o", str(out)],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout
    lines = out.read_text().split("\n")
    starts = [i for i, ln in enumerate(lines) if re.match(r"^_ZN3tgk\w+:", ln)] + [len(lines)]
    seen = 0
    for a, b in zip(starts, starts[1:]):
        name = lines[a].split(":")[0]
        if "gather_kernel" not in name:
            continue
        body = [ln for ln in lines[a:b] if not ln.lstrip().startswith(";")]
        end = max(i for i, ln in enumerate(body) if "s_endpgm" in ln)
        barriers = sum(1 for ln in body[:end + 1] if re.search(r"\bs_barrier\b", ln))
        assert barriers == 4, (name, barriers)
        seen += 1
    assert seen == 8          # unroll 2, 4, 8, 16, with and without the fingerprint
