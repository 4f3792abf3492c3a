// Four threads drive the host-only entry points of libmoc at once (layout bookkeeping of the outer
// loop, argument checks, the per-thread error string). Built with -fsanitize=thread on the host side
// (tests/test_host_sanitizers.py): a data race in the library's host state is reported by the
// sanitizer; a wrong result or an error string that leaked from another thread fails an expectation.
// No call below reaches the device. Prints "ok <n>".
#include <atomic>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/moc.h"

static std::atomic<int> g_checks{0}, g_failed{0};
#define EXPECT(cond)                                                                          \
    do {                                                                                      \
        ++g_checks;                                                                           \
        if (!(cond)) {                                                                        \
            std::fprintf(stderr, "thread %d line %d: %s (last error: %s)\n", id, __LINE__, #cond, moc_last_error()); \
            ++g_failed;                                                                       \
            return;                                                                           \
        }                                                                                     \
    } while (0)

static void worker(int id) {
    // a stream of `shots` shots, each [caption of 8 | 2 chunks of 16]; the thread's own shot count
    const int shots = 2 + id;
    std::vector<int32_t> off{0}, shot, win, spans;
    for (int s = 0; s < shots; ++s) {
        spans.push_back(off.back()); off.push_back(off.back() + 8); spans.push_back(off.back());
        shot.push_back(s); win.push_back(3 * s);
        for (int c = 0; c < 2; ++c) { off.push_back(off.back() + 16); shot.push_back(s); win.push_back(3 * s + 1 + c); }
    }
    const int C = (int)shot.size(), T = shots;
    for (int rep = 0; rep < 200; ++rep) {
        std::vector<int32_t> seg(C + 1), cap(C);
        int32_t P = 0;
        EXPECT(moc_outer_segments(C, off.data(), shot.data(), spans.data(), T, seg.data(), cap.data(), &P) == MOC_OK);
        EXPECT(P == 2 * shots);
        for (int j = 0; j < P; ++j) EXPECT(cap[j] == (j % 2 == 0) && seg[j] == (j / 2) * 40 + (j % 2) * 8);
        // keep every caption and the last shot
        std::vector<int32_t> kept;
        for (int j = 0; j < P; j += 2) kept.push_back(j);
        kept.push_back(P - 1);
        std::vector<int32_t> o_off(C + 1), o_shot(C), o_win(C), o_spans(2 * (T + (int)kept.size() + 1)), rg(2 * kept.size());
        int32_t oC = 0, oT = 0;
        EXPECT(moc_reduce_layout(C, off.data(), shot.data(), win.data(), spans.data(), T, P, seg.data(), (int)kept.size(),
                                 kept.data(), o_off.data(), o_shot.data(), o_win.data(), o_spans.data(), &oC, &oT,
                                 rg.data()) == MOC_OK);
        EXPECT(oC == shots + 2 && oT == shots && o_off[oC] == 8 * shots + 32);
        EXPECT(rg[2 * (kept.size() - 1)] == (shots - 1) * 40 + 8 && rg[2 * (kept.size() - 1) + 1] == 32);
        // an error of this thread's own: the message must be the one this thread caused
        if (id % 2 == 0) {
            int32_t bad_kept[2] = {1, 0};
            EXPECT(moc_reduce_layout(C, off.data(), shot.data(), win.data(), spans.data(), T, P, seg.data(), 2, bad_kept,
                                     o_off.data(), o_shot.data(), o_win.data(), o_spans.data(), &oC, &oT, rg.data()) != MOC_OK);
            EXPECT(std::strstr(moc_last_error(), "kept") != nullptr);
        } else {
            size_t n = 0;
            EXPECT(moc_outer_workspace_bytes(0, 64, 4, &n) == MOC_ERR_SHAPE);
            EXPECT(std::strstr(moc_last_error(), "kept") == nullptr && std::strlen(moc_last_error()) > 0);
        }
        EXPECT(moc_prof_enable(0) == MOC_OK);
    }
}

int main() {
    std::vector<std::thread> th;
    for (int id = 0; id < 4; ++id) th.emplace_back(worker, id);
    for (auto &t : th) t.join();
    if (g_failed.load()) return 1;
    std::printf("ok %d\n", g_checks.load());
    return 0;
}
