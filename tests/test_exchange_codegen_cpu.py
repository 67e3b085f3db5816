"""The split exchange of the decode kernels is ordered at the instruction level (no fences): its argument rests on
the compiler emitting the agent-scope atomic stores and loads of the partials as write-through / cache-bypassing
instructions (`sc1`) and the ticket as a device atomic.  This test cross-compiles the decode kernels that merge
splits in the launch (8-bit per-head and grouped, 12-bit fused, two-pass and grouped) to gfx950 assembly (no GPU needed) and checks exactly that, so a toolchain that changed the mapping would be noticed."""
import os
import re
import subprocess

import pytest

from paper_2504_03661_amd import build as lib_build

CSRC = lib_build.CSRC


def assembly(source, tmp_path):
    out = tmp_path / (source + ".s")
    flags = [f for f in lib_build.FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + ["--cuda-device-only", "-S", os.path.join(CSRC, source),
                                                                         "-o", str(out)]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-2000:]
    return out.read_text()


def kernels(text):
    """name -> body of every kernel (from its label to the end-of-function label)."""
    out = {}
    for m in re.finditer(r"^(_Z\w+):[^\n]*\n(.*?)^\.Lfunc_end", text, re.S | re.M):
        out[m.group(1)] = m.group(2)
    return out


@pytest.mark.parametrize("source,needle", [("pq_decode.hip", "pq_decode_kernel"), ("pq_decode_grouped.hip", "pq_decode_grouped_kernel"),
                                           ("pq12_decode.hip", "pq12_decode_kernel"), ("pq12_decode.hip", "pq12_values_kernel"),
                                           ("pq12_decode_grouped.hip", "pq12_decode_grouped_kernel")])
def test_partials_travel_with_sc1_and_the_ticket_is_a_device_atomic(source, needle, tmp_path):
    ks = {k: v for k, v in kernels(assembly(source, tmp_path)).items() if needle in k}
    assert ks, "no decode kernel found in the assembly"
    for name, body in ks.items():
        lines = body.splitlines()
        tickets = [i for i, l in enumerate(lines) if re.search(r"\bglobal_atomic_add\b", l)]
        assert len(tickets) == 1, (name, "one ticket per kernel")
        t = tickets[0]
        # publish: 8-byte stores before the ticket, every one of them sc1, then a full wait
        # (a plain 8-byte store may sit there too: the output row of the one-split path, which exchanges nothing)
        stores = [l for l in lines[:t] if re.search(r"\bglobal_store_dwordx2\b.*sc1", l)]
        assert len(stores) >= 2, (name, "the partial's two store instructions")
        waits = [i for i, l in enumerate(lines[:t]) if "s_waitcnt vmcnt(0)" in l]
        last_store = max(i for i, l in enumerate(lines[:t]) if re.search(r"\bglobal_store_dwordx2\b.*sc1", l))
        assert waits and waits[-1] > last_store, (name, "the stores are waited for before the ticket")
        # merge: 8-byte loads after the ticket, all sc1
        loads = [l for l in lines[t:] if re.search(r"\bglobal_load_dwordx2\b", l)]
        assert loads and all("sc1" in l for l in loads), (name, [l for l in loads if "sc1" not in l][:3])
        # counter back to zero: a store after the ticket that is sc1 too
        assert any(re.search(r"\bglobal_store_dword\b.*sc1", l) for l in lines[t:]), (name, "ticket reset")
