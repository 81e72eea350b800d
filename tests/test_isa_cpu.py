"""What the compiler made of the balanced decode kernel's publication protocol (no GPU needed).

A cut row's partial travels from one wavefront to another inside a launch: the writer stores
it with device-scope accesses, waits until those stores have completed and only then adds to
the row's counter word; the reader fetches the slot once the counter shows the publication.
The wait is an explicit instruction in the source because a release fence at workgroup scope
compiles to no wait at all on gfx950.  This test compiles the kernel to assembly with the
library's own flags and checks that the wait is there in every instance of the kernel, so that
a compiler or source change that drops it is seen on the CPU and not as a rare wrong result.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2503_13773_amd import build as B

SRC = os.path.join(B.CSRC, "paged_attention_mfma_stream.hip")


def _assembly(tmp_path):
    hipcc = B._hipcc()
    if not (shutil.which(hipcc) or os.path.exists(hipcc)):
        pytest.skip("hipcc not available")
    out = tmp_path / "stream.s"
    flags = [f for f in B.FLAGS if f != "-fPIC"]
    r = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", SRC, "-o", str(out)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    return out.read_text().splitlines()


def test_partial_stores_complete_before_the_publication(tmp_path):
    lines = _assembly(tmp_path)
    kernels, name = {}, None
    for ln in lines:
        m = re.match(r"^(_ZN\S*pa_stream_mfma_kernel\S*):", ln)
        if m:
            name = m.group(1)
            kernels[name] = []
        elif name is not None:
            kernels[name].append(ln.strip())
            if ln.strip().startswith("s_endpgm"):
                name = None
    assert len(kernels) >= 4, sorted(kernels)
    checked = 0
    for name, body in kernels.items():
        # publications are the counter adds whose result is not read back (no sc0 on the add)
        pubs = [i for i, ln in enumerate(body) if ln.startswith("global_atomic_add") and "sc0" not in ln]
        stores = [i for i, ln in enumerate(body) if ln.startswith("buffer_store_dword") and "sc1" in ln]
        if not stores:      # the schedule-building instance streams nothing and publishes nothing
            assert not pubs, name
            continue
        assert pubs, name
        for i in pubs:
            before = [j for j in stores if j < i]
            assert before, (name, body[i])
            between = body[before[-1] + 1:i]
            assert any(re.match(r"s_waitcnt\b.*vmcnt\(0\)", ln) for ln in between), \
                f"{name}: no wait for the partial's stores before `{body[i]}`"
            checked += 1
    assert checked >= 4
