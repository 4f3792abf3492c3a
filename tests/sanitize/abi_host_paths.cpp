// Drives the host half of libmoc (argument validation, layout bookkeeping, error strings) without a
// GPU. Built with -fsanitize=address,undefined on the host side (tests/test_host_sanitizers.py);
// every call below returns before any device work, so a sanitizer report here is a bug in the host
// code of the library. Prints "ok <n>" when all expectations held.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/moc.h"

static int g_checks = 0;
#define EXPECT(cond)                                                            \
    do {                                                                        \
        ++g_checks;                                                             \
        if (!(cond)) {                                                          \
            std::fprintf(stderr, "line %d: %s (last error: %s)\n", __LINE__, #cond, moc_last_error()); \
            return 1;                                                           \
        }                                                                       \
    } while (0)

static int meta_rc(std::vector<int32_t> off, std::vector<int32_t> shot, const std::vector<int32_t> *win,
                   std::vector<int32_t> spans) {
    moc_meta *m = nullptr;
    const int C = (int)off.size() - 1;
    int rc = moc_chunk_meta(off.back(), C, off.data(), shot.data(), win ? win->data() : nullptr,
                            spans.empty() ? nullptr : spans.data(), (int)spans.size() / 2, nullptr, &m);
    if (rc == 0) moc_meta_destroy(m);      // only where a GPU is present
    return rc;
}

int main() {
    for (int code = -10; code <= 0; ++code) EXPECT(std::strlen(moc_status_string(code)) > 0);
    EXPECT(std::strcmp(moc_status_string(-99), "unknown status") == 0);

    // stage (a): every rejection happens before the first device call
    EXPECT(meta_rc({0, 4, 4, 9}, {0, 0, 0}, nullptr, {}) == MOC_ERR_OFFSETS);
    EXPECT(meta_rc({1, 4, 9}, {0, 0}, nullptr, {}) == MOC_ERR_OFFSETS);
    EXPECT(meta_rc({0, 4, 9}, {1, 0}, nullptr, {}) == MOC_ERR_SHOT);
    EXPECT(meta_rc({0, 4, 9}, {0, 0}, nullptr, {0, 3}) == MOC_ERR_TEXT_SPAN);
    EXPECT(meta_rc({0, 4, 9}, {0, 0}, nullptr, {4, 4}) == MOC_ERR_TEXT_SPAN);
    EXPECT(meta_rc({0, 4, 9}, {0, 0}, nullptr, {4, 9, 0, 4}) == MOC_ERR_TEXT_SPAN);
    EXPECT(meta_rc({0, 4, 9}, {0, 0}, nullptr, {0, 12}) == MOC_ERR_TEXT_SPAN);
    std::vector<int32_t> w1{7, 8, 7}, w2{3, 3};
    EXPECT(meta_rc({0, 4, 9, 12}, {0, 0, 0}, &w1, {}) == MOC_ERR_WINDOW);
    EXPECT(meta_rc({0, 4, 9}, {0, 1}, &w2, {}) == MOC_ERR_WINDOW);
    {
        moc_meta *m = nullptr;
        int32_t off[2] = {0, 4}, shot[1] = {0};
        EXPECT(moc_chunk_meta(4, 1, nullptr, shot, nullptr, nullptr, 0, nullptr, &m) == MOC_ERR_NULL);
        EXPECT(moc_chunk_meta(0, 0, off, shot, nullptr, nullptr, 0, nullptr, &m) == MOC_ERR_SHAPE);
        EXPECT(moc_chunk_meta(4, 1, off, shot, nullptr, nullptr, 0, nullptr, nullptr) == MOC_ERR_NULL);
        EXPECT(moc_chunk_meta(4, 1, off, shot, nullptr, nullptr, 2, nullptr, &m) == MOC_ERR_NULL);
    }
    // calls that need a handle reject its absence first
    size_t n = 0;
    EXPECT(moc_attn_workspace_bytes(nullptr, 1, 1, 128, 4, 0, 0, &n) == MOC_ERR_NULL);
    EXPECT(moc_route_workspace_bytes(nullptr, 1, 1, 128, 4, 0, &n) == MOC_ERR_NULL);
    EXPECT(moc_route(nullptr, 1, 1, 128, 0, nullptr, nullptr, 4, 1, nullptr, nullptr, nullptr, 0, nullptr) == MOC_ERR_NULL);
    EXPECT(moc_attn_fwd(nullptr, 1, 1, 128, 0, nullptr, nullptr, nullptr, nullptr, 4, 0.1f, nullptr, nullptr, nullptr, 0,
                        nullptr) == MOC_ERR_NULL);
    EXPECT(moc_attn_bwd(nullptr, 1, 1, 128, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 4, 0.1f,
                        nullptr, nullptr, nullptr, nullptr, 0, nullptr) == MOC_ERR_NULL);
    EXPECT(moc_attn_bwd_after_fwd(nullptr, 1, 1, 128, 0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 4,
                                  0.1f, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == MOC_ERR_NULL);
    EXPECT(moc_route_perturbed(nullptr, 1, 1, 128, 0, nullptr, nullptr, 4, 1, 0.5f, 1.f, 2, 1, nullptr, nullptr, nullptr,
                               0, nullptr) == MOC_ERR_NULL);
    EXPECT(moc_route_static(nullptr, 1, 1, 128, 0, nullptr, nullptr, 4, 1, nullptr, nullptr, nullptr) == MOC_ERR_NULL);
    EXPECT(moc_meta_copy_tables(nullptr, nullptr, nullptr, nullptr) == MOC_ERR_NULL);
    EXPECT(moc_meta_destroy(nullptr) == MOC_OK);

    // probes
    float ms = 0.f;
    double units = 0.0;
    void *fake = (void *)0x1000;         // never dereferenced: every call below is rejected on the host
    EXPECT(moc_probe(0, nullptr, 64, 1, nullptr, &ms, &units) == MOC_ERR_NULL);
    EXPECT(moc_probe(10, fake, 64, 1, nullptr, &ms, &units) == MOC_ERR_SHAPE);
    EXPECT(moc_probe(0, fake, 64, 0, nullptr, &ms, &units) == MOC_ERR_SHAPE);
    EXPECT(moc_probe(0, (void *)0x1004, 64, 1, nullptr, &ms, &units) == MOC_ERR_ALIGN);
    EXPECT(moc_probe(0, fake, 16, 1, nullptr, &ms, &units) == MOC_ERR_WORKSPACE);
    EXPECT(moc_probe(1, fake, 4096, 1, nullptr, &ms, &units) == MOC_ERR_WORKSPACE);

    // outer loop: workspace size, argument checks, host tables
    EXPECT(moc_outer_workspace_bytes(100, 16, 4, &n) == MOC_OK && n > 0);
    EXPECT(moc_outer_workspace_bytes(100, 12, 4, &n) == MOC_ERR_SHAPE);
    EXPECT(moc_outer_workspace_bytes(100, 16, 0, &n) == MOC_ERR_SHAPE);
    EXPECT(moc_outer_workspace_bytes(100, 16, 5000, &n) == MOC_ERR_SHAPE);
    EXPECT(moc_outer_workspace_bytes(100, 16, 4, nullptr) == MOC_ERR_NULL);
    {
        int32_t off[4] = {0, 10, 40, 100}, bad1[4] = {0, 10, 10, 100}, bad2[4] = {0, 10, 40, 99};
        int32_t sel[3], kept[3], nk = 0;
        auto call = [&](const int32_t *o, int g, int M, void *x, int dtype, size_t wsb) {
            return moc_outer_route(100, 16, dtype, x, 3, o, nullptr, g, M, 1, (float *)fake, (float *)fake, sel, kept, &nk,
                                   fake, wsb, nullptr);
        };
        EXPECT(call(off, 3, 1, fake, 0, 1u << 30) == MOC_ERR_SHAPE);
        EXPECT(call(off, -1, 1, fake, 0, 1u << 30) == MOC_ERR_SHAPE);
        EXPECT(call(off, 1, 4, fake, 0, 1u << 30) == MOC_ERR_SHAPE);
        EXPECT(call(bad1, 1, 1, fake, 0, 1u << 30) == MOC_ERR_OFFSETS);
        EXPECT(call(bad2, 1, 1, fake, 0, 1u << 30) == MOC_ERR_OFFSETS);
        EXPECT(call(off, 1, 1, fake, 7, 1u << 30) == MOC_ERR_DTYPE);
        EXPECT(call(off, 1, 1, nullptr, 0, 1u << 30) == MOC_ERR_NULL);
        EXPECT(call(off, 1, 1, (void *)0x1004, 0, 1u << 30) == MOC_ERR_ALIGN);
        EXPECT(call(off, 1, 1, fake, 0, 16) == MOC_ERR_WORKSPACE);
        int32_t rg_bad[4] = {0, 5, 90, 20}, rg_ok[4] = {0, 5, 90, 10};
        EXPECT(moc_gather_rows(1, 100, 64, fake, 2, rg_bad, fake, fake, 64, nullptr) == MOC_ERR_OFFSETS);
        EXPECT(moc_gather_rows(1, 100, 60, fake, 2, rg_ok, fake, fake, 64, nullptr) == MOC_ERR_SHAPE);
        EXPECT(moc_gather_rows(1, 100, 64, fake, 2, rg_ok, fake, fake, 16, nullptr) == MOC_ERR_WORKSPACE);
        EXPECT(moc_gather_rows(1, 100, 64, nullptr, 2, rg_ok, fake, fake, 64, nullptr) == MOC_ERR_NULL);
        EXPECT(moc_gather_rows(1, 100, 64, fake, 0, nullptr, fake, fake, 0, nullptr) == MOC_OK);
    }
    // segments and reduced layout: 3 shots of [caption 8 | 4 video chunks of 8]
    {
        std::vector<int32_t> off{0}, shot, win, spans;
        for (int s = 0; s < 3; ++s) {
            spans.push_back(off.back());
            off.push_back(off.back() + 8);
            spans.push_back(off.back());
            shot.push_back(s);
            win.push_back(100 * s);
            for (int c = 0; c < 4; ++c) { off.push_back(off.back() + 8); shot.push_back(s); win.push_back(100 * s + 1 + c / 2); }
        }
        const int C = (int)shot.size();
        std::vector<int32_t> seg(C + 1), cap(C);
        int32_t P = 0;
        EXPECT(moc_outer_segments(C, off.data(), shot.data(), spans.data(), 3, seg.data(), cap.data(), &P) == MOC_OK);
        EXPECT(P == 6 && seg[0] == 0 && seg[1] == 8 && seg[2] == 40 && seg[3] == 48 && seg[6] == 120);
        EXPECT(cap[0] == 1 && cap[1] == 0 && cap[2] == 1 && cap[5] == 0);
        int32_t kept[4] = {0, 2, 4, 5};
        std::vector<int32_t> o_off(C + 1), o_shot(C), o_win(C), o_spans(2 * (3 + 4)), ranges(8);
        int32_t oC = 0, oT = 0;
        EXPECT(moc_reduce_layout(C, off.data(), shot.data(), win.data(), spans.data(), 3, P, seg.data(), 4, kept,
                                 o_off.data(), o_shot.data(), o_win.data(), o_spans.data(), &oC, &oT, ranges.data()) == MOC_OK);
        EXPECT(oC == 7 && oT == 3 && o_off[7] == 56 && o_spans[4] == 16 && o_spans[5] == 24 && ranges[6] == 88 && ranges[7] == 32);
        EXPECT(o_shot[2] == 2 && o_win[3] == 201 && o_win[6] == 202);
        // all chunks kept, no windows given
        std::vector<int32_t> all(P);
        for (int j = 0; j < P; ++j) all[j] = j;
        std::vector<int32_t> ranges_all(2 * P), o_spans2(2 * (3 + P));
        EXPECT(moc_reduce_layout(C, off.data(), shot.data(), nullptr, spans.data(), 3, P, seg.data(), P, all.data(),
                                 o_off.data(), o_shot.data(), o_win.data(), o_spans2.data(), &oC, &oT, ranges_all.data()) == MOC_OK);
        EXPECT(oC == C && oT == 3 && o_off[C] == 120 && o_win[C - 1] == C - 1);
        int32_t bad_seg[3] = {0, 12, 120}, k0[1] = {0}, k_desc[2] = {1, 0};
        EXPECT(moc_reduce_layout(C, off.data(), shot.data(), nullptr, spans.data(), 3, 2, bad_seg, 1, k0, o_off.data(),
                                 o_shot.data(), o_win.data(), o_spans2.data(), &oC, &oT, ranges_all.data()) == MOC_ERR_OFFSETS);
        EXPECT(moc_reduce_layout(C, off.data(), shot.data(), nullptr, spans.data(), 3, P, seg.data(), 2, k_desc, o_off.data(),
                                 o_shot.data(), o_win.data(), o_spans2.data(), &oC, &oT, ranges_all.data()) == MOC_ERR_SHAPE);
        EXPECT(moc_reduce_layout(C, off.data(), shot.data(), nullptr, spans.data(), 3, P, seg.data(), 0, k0, o_off.data(),
                                 o_shot.data(), o_win.data(), o_spans2.data(), &oC, &oT, ranges_all.data()) == MOC_ERR_SHAPE);
        int32_t bad_span[2] = {3, 8};
        EXPECT(moc_outer_segments(C, off.data(), shot.data(), bad_span, 1, seg.data(), cap.data(), &P) == MOC_ERR_TEXT_SPAN);
        EXPECT(moc_outer_segments(C, off.data(), shot.data(), nullptr, 0, seg.data(), cap.data(), &P) == MOC_OK && P == 3);
    }
    // profiling switches work without a device
    EXPECT(moc_prof_enable(0) == MOC_OK);
    EXPECT(moc_prof_read(-1, nullptr, 0, nullptr, nullptr) == 0);
    std::printf("ok %d\n", g_checks);
    return 0;
}
