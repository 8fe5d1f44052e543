"""The load / wait schedule of the main GEMM kernel template, replayed on the host (no GPU).

tests/schedule_check.cpp includes the kernel's own schedule header (plain constexpr C++) and replays prologue and
stages for every instantiated tile shape; this file compiles and runs it, checks that its list of shapes is the
list the sources instantiate, and plants mistakes in a copy of the header to see that the replay catches them."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_08713_amd", "csrc")
CHECK = os.path.join(ROOT, "tests", "schedule_check.cpp")


def build_and_run(tmp_path, include_dir, name="check"):
    exe = str(tmp_path / name)
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-I", include_dir, "-I", CSRC, CHECK, "-o", exe], check=True)
    return subprocess.run([exe], stdout=subprocess.PIPE, text=True)


def test_every_instantiated_shape_holds(tmp_path):
    out = build_and_run(tmp_path, CSRC)
    assert out.returncode == 0 and "all schedules hold" in out.stdout, out.stdout[-2000:]
    checked = set(re.findall(r"ok (RingShape<[0-9, ]*>)", out.stdout))
    used = set()
    for f in os.listdir(CSRC):
        if f.endswith(".hip"):
            used |= set(re.findall(r"RingShape<[0-9, ]*>", open(os.path.join(CSRC, f)).read()))
    assert checked == used, checked ^ used
    # several K lengths each, the shortest (one group of four stages, no loads in the loop) included
    assert len(re.findall(r"nstages=4 ", out.stdout)) == len(used)


MUTATIONS = [
    # a stage of phase 0 lets one load too many fly: the last code load of stage s + 1 may not have landed
    ("return phase == 0 ? issue_count(3) : phase == 2 ? issue_count(1) : 1;",
     "return phase == 0 ? issue_count(3) + 1 : phase == 2 ? issue_count(1) : 1;", "read before a wait"),
    # phases 1 and 3 allow a whole stage's loads instead of its last one
    ("return phase == 0 ? issue_count(3) : phase == 2 ? issue_count(1) : 1;",
     "return phase == 0 ? issue_count(3) : phase == 2 ? issue_count(1) : kCodeDma;", "read before a wait"),
    # the pair of stages is requested one stage too far ahead: into slots that are still being read
    ("return LoadItem{kLoadCode, 3 + (k & 1), k >> 1};", "return LoadItem{kLoadCode, 4 + (k & 1), k >> 1};", "FAIL"),
    # the E8M0 bytes of the next group behind the codes instead of in front of them
    ("if (n < small) return phase == 1 ? LoadItem{kLoadScale, 1, n} : LoadItem{kLoadWords, 2, n};",
     "if (n >= 2 * kCodeDma) return phase == 1 ? LoadItem{kLoadScale, 1, n - 2 * kCodeDma} : LoadItem{kLoadWords, 2, n - 2 * kCodeDma};",
     "FAIL"),
    # the prologue's first wait forgets the second batch of MBS words
    ("static constexpr int prologue_wait_first() { return 1 + kWordDma + 2 * kCodeDma; }",
     "static constexpr int prologue_wait_first() { return 2 + 2 * kWordDma + 2 * kCodeDma; }", "read before a wait"),
    # the MBS words of the group after next requested a group too late
    ("LoadItem{kLoadWords, 2, n}", "LoadItem{kLoadWords, 3, n}", "FAIL"),
]


@pytest.mark.parametrize("old,new,expect", MUTATIONS)
def test_replay_catches_planted_mistakes(tmp_path, old, new, expect):
    text = open(os.path.join(CSRC, "mx_gemm_schedule.h")).read()
    assert text.count(old) >= 1, old
    mutated = tmp_path / "inc"
    mutated.mkdir()
    shutil.copy(os.path.join(CSRC, "mx_constants.h"), mutated / "mx_constants.h")
    (mutated / "mx_gemm_schedule.h").write_text(text.replace(old, new))
    try:
        out = build_and_run(tmp_path, str(mutated), "mutant")
    except subprocess.CalledProcessError:
        return  # the mutant no longer compiles (a static_assert caught it): also a catch
    assert out.returncode != 0 and expect in out.stdout, out.stdout[-1500:]
