"""The generated header of the kernels is the output of its committed generator."""
import subprocess
import sys
from pathlib import Path

CSRC = Path(__file__).resolve().parent.parent / "paper_2512_23966_amd" / "csrc"


def test_score_asm_header_matches_its_generator():
    res = subprocess.run([sys.executable, str(CSRC / "gen_score_asm.py")], capture_output=True, text=True, check=True, cwd=CSRC)
    assert res.stdout == (CSRC / "score_asm.h").read_text(), "score_asm.h is stale: run `python3 gen_score_asm.py > score_asm.h` in csrc/"
