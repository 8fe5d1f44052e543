"""The load / wait schedules of the GEMM kernels, replayed on the host (no GPU).

tests/schedule_check.cpp includes the kernels' own schedule headers (plain constexpr C++: mx_gemm_schedule.h for the
main kernel template, mx_gemm_f8_schedule.h for the kernel on 8-bit and 6-bit operands) and replays prologue and
stages for every instantiated tile shape and form; this file compiles and runs it, checks that its list of shapes is
the list the sources instantiate, and plants mistakes in copies of the headers to see that the replay catches them."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_08713_amd", "csrc")
CHECK = os.path.join(ROOT, "tests", "schedule_check.cpp")


HEADERS = ("mx_constants.h", "mx_gemm_schedule.h", "mx_gemm_f8_schedule.h")


def build_and_run(tmp_path, include_dir, name="check"):
    exe = str(tmp_path / name)
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-I", include_dir, CHECK, "-o", exe], check=True, stderr=subprocess.PIPE, text=True)
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
    assert len(re.findall(r"ok RingShape<[0-9, ]*> nstages=4 ", out.stdout)) == len(used)
    # the kernel for 8-bit and 6-bit operands: its three forms, with and without MBS words
    forms = set(re.findall(r"ok (F8Schedule<[a-zA-Z, ]*>)", out.stdout))
    assert forms == {"F8Schedule<%s, %s>" % (f, m) for f in ("general", "fast", "six") for m in ("MBS", "no MBS")}, forms


MUTATIONS = [
    # the barrier opens the stages that issue nothing instead of those that issue the loads
    ("static constexpr bool has_barrier(int phase) { return phase % 2 == 1; }",
     "static constexpr bool has_barrier(int phase) { return phase % 2 == 0; }", "FAIL"),
    # a barrier in the first stage of a group only
    ("static constexpr bool has_barrier(int phase) { return phase % 2 == 1; }",
     "static constexpr bool has_barrier(int phase) { return phase == 1; }", "FAIL"),
    # a stage with a barrier lets its youngest load fly: the stage after reads it without a wait of its own
    ("static constexpr int wait_count(int phase) { return has_barrier(phase) ? 0 : 63; }",
     "static constexpr int wait_count(int phase) { return has_barrier(phase) ? 1 : 63; }", "read before a wait"),
    # the pair of stages is requested one stage too far ahead: into slots that are still being read
    ("return LoadItem{kLoadCode, 3 + (k & 1), k >> 1};", "return LoadItem{kLoadCode, 4 + (k & 1), k >> 1};", "FAIL"),
    # the prologue's wait lets one load of stage 1 fly, which stage 0 reads without a wait of its own
    ("static constexpr int prologue_wait_first() { return kWordDma + 2 * kCodeDma; }",
     "static constexpr int prologue_wait_first() { return 1 + kWordDma + 2 * kCodeDma; }", "read before a wait"),
    # the MBS words of the group after next requested a group too late
    ("LoadItem{kLoadWords, 2, n}", "LoadItem{kLoadWords, 3, n}", "FAIL"),
    # the E8M0 bytes of the next group requested in phase 3 instead of phase 1: not published when first read
    ("if (n < small) return phase == 1 ? LoadItem{kLoadScale, 1, n} : LoadItem{kLoadWords, 2, n};",
     "if (n < small) return phase == 3 ? LoadItem{kLoadScale, 1, n} : LoadItem{kLoadWords, 2, n};", "FAIL"),
]


F8_MUTATIONS = [
    # the general form's wait counts the two MBS-word loads whether or not the call has words: without them the two
    # youngest code loads of the stage about to be read may still fly (a mistake this kernel once had)
    ("        return kLoads;\n    }\n\n    // ---- the prologue",
     "        return kForm == kF8General ? kCodeDma + kRegScales + 2 : kLoads;\n    }\n\n    // ---- the prologue", "read before a wait"),
    # a stage lets one load too many fly
    ("        return kLoads;\n    }\n\n    // ---- the prologue", "        return kLoads + 1;\n    }\n\n    // ---- the prologue", "read before a wait"),
    # 6-bit: before a group's second stage one load more than the two group loads may fly: the last piece of plane 2
    # (letting both group loads fly would still hold: the E8M0 bytes are read two stages later)
    ("if (kForm == kF8Six) return p == 1 ? 1 : kCodeDma;", "if (kForm == kF8Six) return p == 1 ? 3 : kCodeDma;", "read before a wait"),
    # 6-bit: a plane's worth more in flight everywhere
    ("if (kForm == kF8Six) return p == 1 ? 1 : kCodeDma;", "if (kForm == kF8Six) return p == 1 ? 1 : 2 * kCodeDma;", "read before a wait"),
    # 6-bit: plane L of the next group loaded during stage L instead of L + 1, while stage L + 1's fragments are read from it
    ("return F8LoadItem{kF8Code, 3 + (p - 1), n};", "return F8LoadItem{kF8Code, 3 + p, n};", "FAIL"),
    # fast form: the group loads behind the stage's codes instead of ahead of them
    ("if (p == 0 && n < 2) return F8LoadItem{n == 0 ? kF8GroupScale : kF8GroupWords, 1, 0};\n        if (kForm == kF8Fast) return F8LoadItem{kF8Code, 3, n - (p == 0 ? 2 : 0)};",
     "if (kForm == kF8Fast && p == 0 && n >= kCodeDma) return F8LoadItem{n == kCodeDma ? kF8GroupScale : kF8GroupWords, 1, 0};\n"
     "        if (kForm == kF8Fast) return F8LoadItem{kF8Code, 3, n};\n"
     "        if (p == 0 && n < 2) return F8LoadItem{n == 0 ? kF8GroupScale : kF8GroupWords, 1, 0};", None),
    # the group loads requested for the group after next: a buffer that is still being read
    ("return F8LoadItem{n == 0 ? kF8GroupScale : kF8GroupWords, 1, 0};", "return F8LoadItem{n == 0 ? kF8GroupScale : kF8GroupWords, 2, 0};", "FAIL"),
    # the codes of stage s + 4 instead of s + 3: into a slot whose stage has not been read yet
    ("return F8LoadItem{kF8Code, 3, n - kRegScales - kRegWords};", "return F8LoadItem{kF8Code, 4, n - kRegScales - kRegWords};", "FAIL"),
    # the prologue's wait lets the loads of all three stages fly
    ("return kForm == kF8Six ? 0 : 2 * kLoads;", "return kForm == kF8Six ? 0 : 3 * kLoads;", "read before a wait"),
]


def run_mutant(tmp_path, header, old, new, expect):
    """Replay with `old` replaced by `new` in a copy of `header` (the other headers copied as they are).  A mutant that
    a static_assert of the headers rejects counts as caught; any other compile error is a mistake of the test."""
    mutated = tmp_path / "inc"
    mutated.mkdir()
    for h in HEADERS:
        text = open(os.path.join(CSRC, h)).read()
        if h == header:
            assert text.count(old) >= 1, old
            text = text.replace(old, new)
        (mutated / h).write_text(text)
    try:
        out = build_and_run(tmp_path, str(mutated), "mutant")
    except subprocess.CalledProcessError as e:
        assert "static assertion failed" in e.stderr, e.stderr[-1500:]
        return None
    if expect is not None:
        assert out.returncode != 0 and expect in out.stdout, out.stdout[-1500:]
    return out


@pytest.mark.parametrize("old,new,expect", F8_MUTATIONS)
def test_replay_catches_planted_mistakes_in_the_8_bit_kernel(tmp_path, old, new, expect):
    out = run_mutant(tmp_path, "mx_gemm_f8_schedule.h", old, new, expect)
    if expect is None and out is not None:
        # a harmless reordering: the group loads behind the codes still land a stage later under the same wait...
        # unless the wait then covers them: the replay decides, and says which
        assert ("all schedules hold" in out.stdout) != (out.returncode != 0)


@pytest.mark.parametrize("old,new,expect", MUTATIONS)
def test_replay_catches_planted_mistakes(tmp_path, old, new, expect):
    run_mutant(tmp_path, "mx_gemm_schedule.h", old, new, expect)


def test_unmutated_copy_of_the_headers_holds(tmp_path):
    """The mutation harness itself: copies of the headers, nothing replaced, compile and hold."""
    out = run_mutant(tmp_path, "mx_constants.h", "constexpr int kWave = 64;", "constexpr int kWave = 64;", None)
    assert out is not None and out.returncode == 0 and "all schedules hold" in out.stdout
