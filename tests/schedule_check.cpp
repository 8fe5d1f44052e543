// Host-side replay of the load schedules of the GEMM kernels (no GPU): for every instantiated tile shape, with and
// without MBS words, and several K lengths, the prologue and every stage are replayed in the order the kernel
// issues its direct-to-LDS loads, waits (s_waitcnt vmcnt) and passes its barriers, and these are checked:
//   1. whatever a stage reads from LDS that another wavefront loaded - the codes of stage s + 1, the E8M0 bytes of
//      that stage's group - was retired by a wait of its loader before a barrier that the reader has passed (a
//      wavefront's loads complete in the order it issued them, so "all but the n youngest" have landed; every
//      wavefront runs the same schedule); the MBS words a wavefront converts are its own rows' and need the wait only;
//   2. no load is issued into a slot whose contents another wavefront may still read (wavefronts are at most as
//      far apart as the barriers allow), or that holds a stage not yet consumed;
//   3. everything that is read was loaded, exactly once, and no load asks for a stage past the end of K;
//   4. every wait count fits the 6-bit counter.
// Prints one line per case; exits 1 at the first violation.  Compiled and run by tests/test_gemm_schedule.py.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <tuple>
#include <vector>

#include "mx_gemm_f8_schedule.h"
#include "mx_gemm_schedule.h"

namespace {

struct Issued {
    mx::LoadItem item;  // absolute: what = stage (codes) or group (others)
    int at_stage;       // -1 = prologue
};

[[noreturn]] void fail(const char* shape, int nstages, const char* why, int a = 0, int b = 0, int c = 0) {
    std::printf("FAIL %s nstages=%d: %s (%d, %d, %d)\n", shape, nstages, why, a, b, c);
    std::exit(1);
}

template <typename S>
void check(const char* name, int nstages) {
    constexpr int C = S::kCodeDma, Sc = S::kScaleDma, W = S::kMbs ? S::kM8Dma : 0;
    using Sched = mx::RingSchedule<C, Sc, W>;
    std::vector<Issued> issued;
    size_t landed = 0;     // loads [0, landed) have been retired by a wait
    size_t published = 0;  // ... and a barrier has been passed since: the other wavefronts' copies may be read
    auto wait = [&](int n) {
        if (n < 0 || n > 63) fail(name, nstages, "wait count outside the 6-bit counter", n);
        const size_t keep = (size_t)n < issued.size() ? issued.size() - (size_t)n : 0;
        if (keep > landed) landed = keep;
    };
    auto barrier = [&]() { published = landed; };
    // how often each piece was issued, and whether it has landed
    auto find = [&](int kind, int what, int index) -> int {
        int pos = -1, count = 0;
        for (size_t k = 0; k < issued.size(); ++k)
            if (issued[k].item.kind == kind && issued[k].item.what == what && issued[k].item.index == index) {
                pos = (int)k;
                ++count;
            }
        if (count > 1) fail(name, nstages, "a piece is loaded twice", kind, what, index);
        return pos;
    };
    auto need = [&](int kind, int what, int count, int reader_stage, bool own_rows = false) {
        for (int i = 0; i < count; ++i) {
            const int pos = find(kind, what, i);
            if (pos < 0) fail(name, nstages, "a piece that is read was never loaded", kind, what, reader_stage);
            if ((size_t)pos >= landed) fail(name, nstages, "a piece is read before a wait has retired its load", kind, what, reader_stage);
            if (!own_rows && (size_t)pos >= published) fail(name, nstages, "a piece is read before a barrier has published it", kind, what, reader_stage);
        }
    };
    // Between two barriers the wavefronts are at most this far apart: one that has just passed the barrier of stage
    // t and one that is about to reach the next barrier.  While stage t issues, readers may be anywhere in
    // [t, next barrier stage - 1], reading the stage after the one they are in.
    auto next_barrier_after = [&](int t) {
        for (int u = t + 1;; ++u)
            if (u >= nstages || Sched::has_barrier(u % 4)) return u;
    };
    auto issue = [&](mx::LoadItem abs, int t) {
        if (abs.kind == mx::kLoadCode) {
            if (abs.what >= nstages) fail(name, nstages, "codes requested past the end of K", abs.what, t);
            if (t >= 0) {
                if (!Sched::has_barrier(t % 4)) fail(name, nstages, "loads issued in a stage that no barrier opens", abs.what, t);
                // slot what % 4 held stage what - 4, read during stage what - 5: every wavefront has finished stage
                // t - 1 behind the barrier of stage t.  Readers between this barrier and the next read the stages
                // t + 1 .. next barrier stage, and what is loaded now must not be needed before it is published
                const int last_reader = next_barrier_after(t) - 1;  // reads stage last_reader + 1
                bool ok = abs.what - 5 <= t - 1 && abs.what > last_reader + 1;
                for (int u = t; u <= last_reader; ++u) ok = ok && (abs.what % 4) != ((u + 1) % 4);
                if (!ok) fail(name, nstages, "codes loaded into a slot that is still in use", abs.what, t);
            }
        } else if (abs.kind == mx::kLoadScale) {
            // group G goes where group G - 2 was, whose bytes are last read during stage 4 (G - 2) + 2
            if (t >= 0 && !(4 * (abs.what - 2) + 2 <= t - 1)) fail(name, nstages, "E8M0 bytes loaded into a slot still in use", abs.what, t);
        } else {
            // group G goes where group G - 2 was, whose words are last read (by the sigma conversion) during stage 4 (G - 2) + 1 at the latest
            if (t >= 0 && !(4 * (abs.what - 2) + 1 <= t - 1)) fail(name, nstages, "MBS words loaded into a slot still in use", abs.what, t);
        }
        issued.push_back({abs, t});
    };
    const int ngroups = nstages / 4;
    // ---- prologue
    for (int n = 0; n < Sched::prologue_count(); ++n) issue(Sched::prologue_item(n), -1);
    wait(Sched::prologue_wait_first());
    barrier();
    // first LDS reads: E8M0 bytes and MBS words of group 0 (sigma tables of stages 0 and 1), codes of stage 0
    need(mx::kLoadScale, 0, Sc, -1);
    need(mx::kLoadWords, 0, W, -1, true);
    need(mx::kLoadCode, 0, C, -1);
    // ---- the loop
    const int n_issue = nstages - 4 > 0 ? (nstages - 4 + 3) / 4 * 4 : 0;
    for (int s = 0; s < nstages; ++s) {
        const int phase = s % 4;
        const bool does_issue = s < n_issue;
        if (Sched::has_barrier(phase)) {
            wait(Sched::wait_count(phase));
            barrier();
        }
        // reads of this stage
        if (s + 1 < nstages) {
            need(mx::kLoadCode, s + 1, C, s);
            need(mx::kLoadScale, (s + 1) / 4, Sc, s);
        }
        // a stage without a barrier converts the MBS words of the stages s + 2 and s + 3 (its own rows)
        if (!Sched::has_barrier(phase))
            for (int y = s + 2; y <= s + 3; ++y)
                if (y < nstages) need(mx::kLoadWords, y / 4, W, s, true);
        if (does_issue)
            for (int n = 0; n < Sched::issue_count(phase); ++n) {
                mx::LoadItem it = Sched::issue_item(phase, n);
                it.what += it.kind == mx::kLoadCode ? s : s / 4;
                // (past the last group the kernel fetches the last group again: the slot rule still applies, but the
                // load brings nothing new)
                const bool repeat = it.kind != mx::kLoadCode && it.what >= ngroups;
                issue(it, s);
                if (repeat) issued.back().item.index += 1000;
            }
    }
    // The sigma tables (LDS written by the workgroup itself, four tables): a stage without a barrier converts the
    // words of the stages s + 2 and s + 3; the table of stage y is read at the start of stage y - 1, behind that
    // stage's barrier if it has one.  A barrier must lie between, and the table's former contents (stage y - 4, read
    // at the start of stage y - 5) must be out of use for every wavefront, i.e. a barrier must also lie between that
    // read and the write.
    if (W > 0)
        for (int y = 2; y < nstages; ++y) {
            const int conv = !Sched::has_barrier((y - 2) % 4) ? y - 2 : y - 3;
            if (conv < 0 || Sched::has_barrier(conv % 4)) fail(name, nstages, "no stage converts the words of a stage", y);
            bool published_before_read = false, old_out_of_use = y - 5 < 0;
            for (int b = conv + 1; b <= y - 1; ++b) published_before_read = published_before_read || Sched::has_barrier(b % 4);
            for (int b = y - 5 + 1; b <= conv; ++b) old_out_of_use = old_out_of_use || (b >= 0 && Sched::has_barrier(b % 4));
            if (!published_before_read) fail(name, nstages, "a sigma table is read before a barrier has published it", y, conv);
            if (!old_out_of_use) fail(name, nstages, "a sigma table is overwritten while it may still be read", y, conv);
        }
    // everything of every stage and group was loaded
    for (int y = 0; y < nstages; ++y)
        for (int i = 0; i < C; ++i)
            if (find(mx::kLoadCode, y, i) < 0) fail(name, nstages, "codes of a stage never loaded", y, i);
    std::printf("ok %s nstages=%d loads/wavefront: codes %d per stage, E8M0 %d and words %d per group; barrier and wait in phases", name, nstages, C, Sc, W);
    for (int p = 0; p < 4; ++p)
        if (Sched::has_barrier(p)) std::printf(" %d (vmcnt %d)", p, Sched::wait_count(p));
    std::printf("\n");
}

template <typename S>
void check_all(const char* name) {
    static_assert(S::kLdsBytes <= 160 * 1024, "LDS");
    for (int nstages : {4, 8, 12, 16, 64, 256}) check<S>(name, nstages);
}

// ---- the kernel for 8-bit and 6-bit operands (mx_gemm_f8.hip), same rules ------------------------------------
struct F8Issued {
    mx::F8LoadItem item;  // absolute
    int at_stage;
    bool repeat;          // past the end of K the kernel fetches the last stage, group or plane again
};

template <int kForm, bool kMbs>
void check_f8(const char* name, int nstages) {
    using Sched = mx::F8Schedule<kForm, kMbs>;
    constexpr int C = Sched::kCodeDma;
    constexpr bool kGroups = kForm != mx::kF8General, kSix = kForm == mx::kF8Six;
    std::vector<F8Issued> issued;
    size_t landed = 0;
    auto wait = [&](int n) {
        if (n < 0 || n > 63) fail(name, nstages, "wait count outside the 6-bit counter", n);
        const size_t keep = (size_t)n < issued.size() ? issued.size() - (size_t)n : 0;
        if (keep > landed) landed = keep;
    };
    auto find = [&](int kind, int what, int index) -> int {
        int pos = -1, count = 0;
        for (size_t k = 0; k < issued.size(); ++k)
            if (!issued[k].repeat && issued[k].item.kind == kind && issued[k].item.what == what && issued[k].item.index == index) {
                pos = (int)k;
                ++count;
            }
        if (count > 1) fail(name, nstages, "a piece is loaded twice", kind, what, index);
        return pos;
    };
    auto need = [&](int kind, int what, int count, int reader_stage) {
        for (int i = 0; i < count; ++i) {
            const int pos = find(kind, what, i);
            if (pos < 0) fail(name, nstages, "a piece that is read was never loaded", kind, what, reader_stage);
            if ((size_t)pos >= landed) fail(name, nstages, "a piece is read before a wait has retired its load", kind, what, reader_stage);
        }
    };
    const int ngroups = nstages / 4, nplanes = 3 * ngroups;
    auto issue = [&](mx::F8LoadItem abs, int t) {
        bool repeat = false;
        if (abs.kind == mx::kF8Code && !kSix) {
            // stage y goes into slot y % 3 where stage y - 3 was, whose fragments are read during stage y - 4: free
            // from the barrier of stage y - 3 on
            if (abs.what >= nstages) { repeat = true; abs.what = nstages - 1; }
            else if (t >= 0 && !(abs.what - 3 <= t)) fail(name, nstages, "codes loaded into a slot that is still in use", abs.what, t);
            if (t >= 0 && abs.what <= t + 1 && !repeat) fail(name, nstages, "codes requested too late", abs.what, t);
        } else if (abs.kind == mx::kF8Code) {
            // plane 3 g + L goes where plane 3 (g - 1) + L was, last read for the fragments of stage L + 1 of group
            // g - 1, during stage L of that group: free from the barrier of stage 4 (g - 1) + L + 1 on
            if (abs.what >= nplanes) { repeat = true; abs.what -= 3; }
            const int g = abs.what / 3, L = abs.what % 3;
            if (t >= 0 && !(4 * (g - 1) + L + 1 <= t)) fail(name, nstages, "plane loaded into a slot that is still in use", abs.what, t);
        } else if (abs.kind == mx::kF8GroupScale) {
            // group G goes where group G - 2 was, last read (for stage 4 (G - 2) + 3) during stage 4 (G - 2) + 2
            if (abs.what >= ngroups) { repeat = true; abs.what = ngroups - 1; }
            if (t >= 0 && !(4 * (abs.what - 2) + 3 <= t)) fail(name, nstages, "E8M0 bytes loaded into a buffer still in use", abs.what, t);
        }
        issued.push_back({abs, t, repeat});
    };
    // what the fragments of stage y are read from
    auto need_stage = [&](int y, int reader) {
        if (!kSix) { need(mx::kF8Code, y, C, reader); return; }
        const int g = y / 4, q = y % 4;
        for (int plane = (6 * q) / 8; plane <= (6 * q + 5) / 8; ++plane) need(mx::kF8Code, 3 * g + plane, C, reader);
    };
    for (int n = 0; n < Sched::prologue_count(); ++n) issue(Sched::prologue_item(n), -1);
    wait(Sched::prologue_wait());
    need_stage(0, -1);
    if (kGroups) need(mx::kF8GroupScale, 0, 1, -1);
    for (int s = 0; s < nstages; ++s) {
        const int p = s % 4;
        wait(Sched::stage_wait(p));
        if (s + 1 < nstages) {
            need_stage(s + 1, s);
            if (kGroups) need(mx::kF8GroupScale, (s + 1) / 4, 1, s);
        }
        for (int n = 0; n < Sched::issue_count(p); ++n) {
            mx::F8LoadItem it = Sched::issue_item(p, n);
            if (it.kind == mx::kF8Code) it.what += kSix ? 3 * (s / 4) : s;
            else if (it.kind == mx::kF8GroupScale || it.kind == mx::kF8GroupWords) it.what += s / 4;
            else it.what += s;
            issue(it, s);
        }
    }
    if (kSix) {
        for (int y = 0; y < nplanes; ++y)
            for (int i = 0; i < C; ++i)
                if (find(mx::kF8Code, y, i) < 0) fail(name, nstages, "a plane was never loaded", y, i);
    } else {
        for (int y = 0; y < nstages; ++y)
            for (int i = 0; i < C; ++i)
                if (find(mx::kF8Code, y, i) < 0) fail(name, nstages, "codes of a stage never loaded", y, i);
    }
    std::printf("ok %s nstages=%d loads/wavefront and stage: %d codes; waits %d %d %d %d\n", name, nstages, C, Sched::stage_wait(0),
                Sched::stage_wait(1), Sched::stage_wait(2), Sched::stage_wait(3));
}

template <int kForm, bool kMbs>
void check_f8_all(const char* name) {
    // the general form takes any number of stages, the fast forms whole groups of four
    if (kForm == mx::kF8General)
        for (int nstages : {1, 2, 3, 4, 5, 7, 12, 61, 256}) check_f8<kForm, kMbs>(name, nstages);
    else
        for (int nstages : {4, 8, 12, 16, 20, 64, 256}) check_f8<kForm, kMbs>(name, nstages);
}

}  // namespace

#define SHAPE(...) check_all<mx::RingShape<__VA_ARGS__>>("RingShape<" #__VA_ARGS__ ">")

int main() {
    // every shape the library instantiates (tests/test_gemm_schedule.py compares this list with the sources)
    SHAPE(2, 2, 4, 4, 0);
    SHAPE(2, 2, 4, 2, 0);
    SHAPE(2, 2, 2, 2, 0);
    SHAPE(2, 2, 4, 2, 0, 1);
    SHAPE(2, 2, 2, 2, 0, 1);
    SHAPE(2, 2, 2, 2, 0, 2);
    SHAPE(4, 2, 2, 2, 3);
    SHAPE(2, 4, 4, 1, 1);
    SHAPE(2, 4, 4, 1, 2);
    SHAPE(2, 4, 2, 1, 3);
    SHAPE(2, 4, 2, 1, 1);
    SHAPE(2, 4, 2, 1, 2);
    SHAPE(4, 2, 2, 2, 3, 1);
    SHAPE(2, 4, 2, 1, 3, 1);
    SHAPE(2, 4, 2, 1, 3, 2);
    // the forms of the kernel for 8-bit and 6-bit operands, with and without MBS words
    check_f8_all<mx::kF8General, false>("F8Schedule<general, no MBS>");
    check_f8_all<mx::kF8General, true>("F8Schedule<general, MBS>");
    check_f8_all<mx::kF8Fast, false>("F8Schedule<fast, no MBS>");
    check_f8_all<mx::kF8Fast, true>("F8Schedule<fast, MBS>");
    check_f8_all<mx::kF8Six, false>("F8Schedule<six, no MBS>");
    check_f8_all<mx::kF8Six, true>("F8Schedule<six, MBS>");
    std::printf("all schedules hold\n");
    return 0;
}
