"""Every gfx950 kernel of the library must run without scratch memory and without reading the
dispatch packet: both were measured to cost far more than the short decode kernels themselves
(a private array that the compiler failed to keep in registers, or a by-value argument struct
indexed at run time, each silently add microseconds per workgroup).  Checked on the compiler's
assembly output; needs hipcc, not a GPU."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

from paper_2501_04052_amd import build

ALLOWED_SCRATCH = {}      # kernel-name substring -> bytes (none at present)


def _asm(src):
    cmd = [build.hipcc()] + [f for f in build.HIPCC_FLAGS if f != "-fPIC"] + \
          ["--cuda-device-only", "-S", os.path.join(build.CSRC, src), "-o", "-"]
    return subprocess.run(cmd, check=True, capture_output=True, text=True).stdout


def test_no_scratch_no_dispatch_packet():
    with ThreadPoolExecutor(max_workers=6) as ex:
        outs = list(ex.map(_asm, build.SOURCES))
    seen = 0
    for src, text in zip(build.SOURCES, outs):
        for m in re.finditer(r"\.amdhsa_kernel (\S+)(.*?)\.end_amdhsa_kernel", text, re.S):
            name, body = m.group(1), m.group(2)
            seen += 1
            scratch = int(re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body).group(1))
            allowed = max([v for k, v in ALLOWED_SCRATCH.items() if k in name] + [0])
            assert scratch <= allowed, "%s: %s uses %d bytes of scratch" % (src, name, scratch)
            disp = re.search(r"\.amdhsa_user_sgpr_dispatch_ptr (\d+)", body)
            assert disp is None or disp.group(1) == "0", "%s: %s reads the dispatch packet" % (src, name)
    assert seen >= 20
