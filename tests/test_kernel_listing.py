"""Static check of the compiled tiled kernel (no GPU needed): the multiply-adds that take an
operand from the neighbouring lane (their DPP form, written as inline assembly, which the
compiler's hazard pass does not look into) must not follow, within two instructions, a vector
instruction that writes the register they shift."""
import os
import re
import shutil
import subprocess

import pytest

from paper_1802_10280_amd import build as esc_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _vgprs(tok):
    tok = tok.strip().rstrip(",")
    m = re.match(r"^v(\d+)$", tok)
    if m:
        return {int(m.group(1))}
    m = re.match(r"^v\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


def dpp_hazards(listing):
    ins = [l.strip() for l in listing.splitlines()]
    ins = [l for l in ins if re.match(r"^[a-z]\w*\s", l + " ") and not l.endswith(":")]
    checked, bad = 0, []
    for k, l in enumerate(ins):
        if "_dpp" not in l.split()[0]:
            continue
        checked += 1
        src = _vgprs(l.split(None, 1)[1].split(",")[1].split()[0])
        for back in (1, 2):
            if k - back < 0:
                continue
            prev = ins[k - back]
            if prev.startswith("v_") and _vgprs(prev.split(None, 1)[1].split(",")[0]) & src:
                bad.append((prev, l))
    return checked, bad


def test_the_checker_sees_a_planted_hazard():
    text = "v_mov_b32_e32 v5, v9\n\tv_fmac_f32_dpp v1, v5, v2 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:0\n"
    assert dpp_hazards(text) == (1, [("v_mov_b32_e32 v5, v9", "v_fmac_f32_dpp v1, v5, v2 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:0")])
    text = "ds_read_b128 v[4:7], v9\n\ts_nop 0\n\tv_fmac_f32_dpp v1, v5, v2 wave_shl:1 row_mask:0xf bank_mask:0xf bound_ctrl:0\n"
    assert dpp_hazards(text) == (1, [])


def test_no_vector_write_right_before_a_lane_shifted_operand(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc here")
    flags = [f for f in esc_build.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    out = tmp_path / "sconv_tiled.s"
    cmd = [hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-I", esc_build.CSRC, "--cuda-device-only", "-S",
           "-o", str(out), os.path.join(esc_build.CSRC, "sconv_tiled.hip")]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL, timeout=600)
    checked, bad = dpp_hazards(out.read_text())
    assert checked > 1000          # every instantiation carries them
    assert not bad, bad[:5]
