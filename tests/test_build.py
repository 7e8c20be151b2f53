"""The build's choice between the two forms of the LDS rank kernel (CPU only).

The streaming form leaves a scalar load in flight between two evaluation statements and is built
only when a check of the generated assembly passes; otherwise the conservative form is built,
whose statements load and wait for their own entries.  Forced here: a failing check must select
the conservative form, and that form's assembly must leave nothing in flight."""
import os
import re
import subprocess

from paper_2301_13441_amd import build as hb
from paper_2301_13441_amd import check_stream_registers as csr


def test_failed_register_check_selects_the_conservative_form(monkeypatch, tmp_path, capsys):
    def fails(*args, **kwargs):
        raise RuntimeError("forced by the test")
    monkeypatch.setattr(csr, "check", fails)
    assert hb.ranklds_variant_flags(list(hb.FLAGS)) == [hb.CONSERVATIVE]
    assert "conservative form" in capsys.readouterr().err

    asm = str(tmp_path / "ranklds_conservative.s")
    subprocess.run([hb.HIPCC, *hb.FLAGS, hb.CONSERVATIVE, "-x", "hip", "-S", "--cuda-device-only",
                    os.path.join(hb.CSRC, hb.RANKLDS), "-o", asm], check=True, stderr=subprocess.DEVNULL)
    text = open(asm).read()
    blocks = re.findall(r"ASMSTART\n(.*?)ASMEND", text, flags=re.S)
    evals = [b for b in blocks if "ds_read_addtid_b32" in b]
    assert len(evals) >= 20
    for b in evals:
        lines = [ln.strip() for ln in b.split("\n") if ln.strip() and not ln.strip().startswith(";")]
        # the statement's own entries are loaded and waited for first; no scalar load follows
        assert lines[0].startswith("s_load_dwordx16") and lines[1] == "s_waitcnt lgkmcnt(0)"
        assert sum(ln.startswith("s_load") for ln in lines) == 1


def test_streaming_form_passes_the_register_check():
    n = csr.check(hb.HIPCC, list(hb.FLAGS), os.path.join(hb.CSRC, hb.RANKLDS), hb.OBJ)
    assert n >= 1
