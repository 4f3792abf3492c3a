// C ABI of libmoc: argument validation, layout tables (stage a), workspace
// layout, and dispatch to the kernel launchers. No kernel code in this file.
#include <algorithm>
#include <atomic>
#include <cstdio>
#include <map>
#include <mutex>
#include <cstring>
#include <new>
#include <cmath>
#include <string>
#include <unordered_set>
#include <vector>

#include "moc_internal.h"

namespace {

thread_local std::string g_err;

int fail(int code, const std::string &detail) {
    g_err = detail;
    return code;
}

int hip_fail(hipError_t e, const char *what) {
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return MOC_ERR_HIP;
}

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_common(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int32_t topk, int dtype) {
    if (!meta) return fail(MOC_ERR_NULL, "meta is NULL");
    if (dtype != MOC_BF16 && dtype != MOC_F32) return fail(MOC_ERR_DTYPE, "dtype must be MOC_BF16 or MOC_F32");
    if (B <= 0 || H <= 0) return fail(MOC_ERR_SHAPE, "B and H must be positive");
    if (d != 64 && d != 128) return fail(MOC_ERR_SHAPE, "d must be 64 or 128");
    if (topk < 0 || topk > MOC_MAX_TOPK) return fail(MOC_ERR_SHAPE, "topk out of range [0, MOC_MAX_TOPK]");
    if ((long long)meta->N * std::max(topk, 1) >= (1LL << 31)) return fail(MOC_ERR_SHAPE, "N * topk must be < 2^31");
    if (meta->N >= (1 << 26)) return fail(MOC_ERR_SHAPE, "N must be < 2^26");
    if ((long long)B * H * meta->N * (topk + 1) >= (1LL << 31))
        return fail(MOC_ERR_SHAPE, "B * H * N * (topk + 1) must be < 2^31");
    if ((long long)B * H > 65535) return fail(MOC_ERR_SHAPE, "B * H must be <= 65535");
    if (topk > 0 && meta->C > moc::kMaxListChunks)
        return fail(MOC_ERR_SHAPE, "routing needs C <= 16384 (the list builder's histogram)");
    return MOC_OK;
}

struct ProfRec { const char *name; hipEvent_t e0, e1; };
std::mutex g_prof_mu;
std::vector<ProfRec> g_prof;
std::vector<hipEvent_t> g_prof_pool;
std::atomic<bool> g_prof_on{false};

hipEvent_t prof_event() {
    if (!g_prof_pool.empty()) { hipEvent_t e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

void prof_clear_locked() {
    for (auto &r : g_prof) { g_prof_pool.push_back(r.e0); g_prof_pool.push_back(r.e1); }
    g_prof.clear();
}

bool bad_scale(float s) { return !(s > 0.f) || !std::isfinite(s); }

// What the last moc_attn_fwd left in a workspace: moc_attn_bwd_after_fwd reuses the lists only when
// its own arguments name the same call.
struct ListTag { const moc_meta *meta; const int32_t *sel; int32_t B, H, topk; void *stream; };
std::mutex g_tag_mu;
std::map<const void *, ListTag> g_tags;

void tag_set(const void *ws, const ListTag &t) {
    std::lock_guard<std::mutex> lk(g_tag_mu);
    if (g_tags.size() > 64) g_tags.clear();
    g_tags[ws] = t;
}
void tag_drop(const void *ws) {
    std::lock_guard<std::mutex> lk(g_tag_mu);
    g_tags.erase(ws);
}
void tag_drop_meta(const moc_meta *m) {
    std::lock_guard<std::mutex> lk(g_tag_mu);
    for (auto it = g_tags.begin(); it != g_tags.end();)
        if (it->second.meta == m) it = g_tags.erase(it); else ++it;
}
bool tag_matches(const void *ws, const ListTag &t) {
    std::lock_guard<std::mutex> lk(g_tag_mu);
    auto it = g_tags.find(ws);
    if (it == g_tags.end()) return false;
    const ListTag &u = it->second;
    return u.meta == t.meta && u.sel == t.sel && u.B == t.B && u.H == t.H && u.topk == t.topk && u.stream == t.stream;
}

}  // namespace

namespace moc {

bool prof_on() { return g_prof_on.load(std::memory_order_relaxed); }

void prof_begin(const char *name, hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    ProfRec r{name, prof_event(), prof_event()};
    (void)hipEventRecord(r.e0, st);
    g_prof.push_back(r);
}

void prof_end(hipStream_t st) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof.empty()) (void)hipEventRecord(g_prof.back().e1, st);
}

AttnWs attn_ws_layout(const moc_meta *m, int BH, int d, int topk, bool with_bwd) {
    AttnWs L{};
    size_t off = 0;
    const size_t C = m->C, N = m->N, slots = (size_t)topk + 1;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.cnt = take((size_t)BH * C * 4);
    L.list_off = take((size_t)BH * (C + 1) * 4);
    L.tile_off = take((size_t)BH * (C + 1) * 4);
    L.vmask = take((size_t)BH * N * 4);
    L.gsum = take((size_t)BH * 32 * C * 4);
    L.cnt_blk = take((size_t)BH * ((N + kRowsPerBlk - 1) / kRowsPerBlk) * C * 4);
    L.qlist = take((size_t)BH * N * std::max(topk, 1) * 4);
    L.plse = take((size_t)BH * N * slots * 4);
    L.po = take((size_t)BH * N * slots * d * 2);
    if (with_bwd) {
        L.delta = take((size_t)BH * N * 4);
        L.stats2 = take(((size_t)BH * N + 1) * 8);     // (lse2, delta) pairs + one pair holding (+inf, 0)
        L.gstats2 = take((size_t)BH * N * std::max(topk, 1) * 8);
        L.tpart_k = take((size_t)BH * m->n_partials * kKeyTile * d * 4);
        L.tpart_v = take((size_t)BH * m->n_partials * kKeyTile * d * 4);
    }
    L.total = off;
    return L;
}

RouteWs route_ws_layout(const moc_meta *m, int BH, int d, int, int) {
    RouteWs L{};
    L.Cpad = (m->C + 31) / 32 * 32;
    L.kb_split = 0;
    L.total = align_up((size_t)BH * 3 * L.Cpad * d * 2);
    return L;
}

}  // namespace moc

extern "C" {

const char *moc_status_string(int s) {
    switch (s) {
        case MOC_OK: return "ok";
        case MOC_ERR_NULL: return "null pointer";
        case MOC_ERR_SHAPE: return "bad shape";
        case MOC_ERR_OFFSETS: return "bad chunk offsets";
        case MOC_ERR_TEXT_SPAN: return "bad text span";
        case MOC_ERR_WINDOW: return "bad window ids";
        case MOC_ERR_DTYPE: return "bad dtype";
        case MOC_ERR_WORKSPACE: return "workspace missing or too small";
        case MOC_ERR_ALIGN: return "pointer not 16-byte aligned";
        case MOC_ERR_HIP: return "HIP error";
        case MOC_ERR_SHOT: return "shot ids decrease";
        default: return "unknown status";
    }
}

const char *moc_last_error(void) { return g_err.c_str(); }

int moc_prof_enable(int on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    prof_clear_locked();
    g_prof_on.store(on != 0);
    return MOC_OK;
}

int moc_prof_read(int32_t index, char *name, size_t name_cap, int32_t *launches, float *total_ms) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    // aggregate by kernel name, in order of first appearance
    std::vector<const char *> order;
    std::map<std::string, std::pair<int, double>> agg;
    for (auto &r : g_prof) {
        hipError_t e = hipEventSynchronize(r.e1);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, r.e0, r.e1);
        if (e != hipSuccess) return hip_fail(e, "moc_prof_read");
        auto it = agg.find(r.name);
        if (it == agg.end()) { order.push_back(r.name); agg[r.name] = {1, ms}; }
        else { it->second.first += 1; it->second.second += ms; }
    }
    if (index < 0) return (int)order.size();           // number of distinct kernels
    if (index >= (int)order.size()) return fail(MOC_ERR_SHAPE, "profile index out of range");
    const auto &a = agg[order[index]];
    if (name && name_cap) { std::strncpy(name, order[index], name_cap - 1); name[name_cap - 1] = 0; }
    if (launches) *launches = a.first;
    if (total_ms) *total_ms = (float)a.second;
    return MOC_OK;
}

int moc_probe(int32_t kind, void *buf, size_t bytes, int32_t iters, void *stream, float *ms, double *units) {
    if (!buf || !ms || !units) return fail(MOC_ERR_NULL, "moc_probe: NULL argument");
    if (kind < MOC_PROBE_COPY || kind > MOC_PROBE_COPY_VIA_REGISTERS) return fail(MOC_ERR_SHAPE, "moc_probe: unknown kind");
    if (iters <= 0) return fail(MOC_ERR_SHAPE, "moc_probe: iters must be positive");
    if (misaligned(buf)) return fail(MOC_ERR_ALIGN, "moc_probe: buffer must be 16-byte aligned");
    if (kind == MOC_PROBE_COPY && bytes < 32) return fail(MOC_ERR_WORKSPACE, "moc_probe: copy needs at least 32 bytes");
    if (kind != MOC_PROBE_COPY && bytes < (size_t)moc::kProbeMfmaGrid * 512 * sizeof(float))
        return fail(MOC_ERR_WORKSPACE, "moc_probe: mfma needs a 512 KiB buffer");
    if (kind >= MOC_PROBE_LDS_READ && bytes < ((size_t)1 << 20))
        return fail(MOC_ERR_WORKSPACE, "moc_probe: the compute-unit probes need a 1 MiB buffer");
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return hip_fail(e, "moc_probe");
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e, "moc_probe"); }
    e = moc::launch_probe(kind, buf, bytes, iters, (hipStream_t)stream, e0, e1, units);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e == hipSuccess ? MOC_OK : hip_fail(e, "moc_probe");
}

int moc_chunk_meta(int32_t N, int32_t C, const int32_t *off, const int32_t *shot, const int32_t *window,
                   const int32_t *spans, int32_t T, void *stream, moc_meta **out) {
    using namespace moc;
    if (!out) return fail(MOC_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (!off || !shot) return fail(MOC_ERR_NULL, "chunk_offsets / chunk_shot is NULL");
    if (T < 0 || (T > 0 && !spans)) return fail(MOC_ERR_NULL, "text_spans is NULL with T > 0");
    if (N <= 0 || C <= 0 || C > N) return fail(MOC_ERR_SHAPE, "need 0 < C <= N");
    if (off[0] != 0 || off[C] != N) return fail(MOC_ERR_OFFSETS, "offsets must start at 0 and end at N");
    for (int j = 0; j < C; ++j)
        if (off[j + 1] <= off[j]) return fail(MOC_ERR_OFFSETS, "offsets must be strictly increasing");
    for (int j = 1; j < C; ++j)
        if (shot[j] < shot[j - 1]) return fail(MOC_ERR_SHOT, "chunk_shot must be non-decreasing");

    // text spans: sorted, disjoint, non-empty, chunk-aligned
    std::vector<int32_t> kind(C, 0);
    {
        int prev_end = 0;
        for (int s = 0; s < T; ++s) {
            int a = spans[2 * s], b = spans[2 * s + 1];
            if (a < 0 || b > N || a >= b) return fail(MOC_ERR_TEXT_SPAN, "text span empty or out of range");
            if (a < prev_end) return fail(MOC_ERR_TEXT_SPAN, "text spans must be sorted and disjoint");
            prev_end = b;
            const int32_t *pa = std::lower_bound(off, off + C + 1, a);
            const int32_t *pb = std::lower_bound(off, off + C + 1, b);
            if (*pa != a || *pb != b) return fail(MOC_ERR_TEXT_SPAN, "text span is not a union of whole chunks");
            for (int j = int(pa - off); j < int(pb - off); ++j) kind[j] = 1;
        }
    }

    // dense window ids; equal ids must be contiguous and inside one shot
    std::vector<int32_t> win(C), wfirst, wlast;
    {
        std::unordered_set<int32_t> seen;
        for (int j = 0; j < C; ++j) {
            bool fresh = (j == 0) || !window || window[j] != window[j - 1];
            if (fresh) {
                if (window && !seen.insert(window[j]).second)
                    return fail(MOC_ERR_WINDOW, "equal window ids must be contiguous");
                wfirst.push_back(j);
                wlast.push_back(j);
            } else {
                if (shot[j] != shot[wfirst.back()]) return fail(MOC_ERR_WINDOW, "a window spans two shots");
                wlast.back() = j;
            }
            win[j] = int32_t(wfirst.size()) - 1;
        }
    }
    const int W = int(wfirst.size());

    // forced-link key ranges per window: union of all text spans and the window's own tokens
    std::vector<int32_t> arange_off(W + 1, 0);
    std::vector<KeyRange> aranges;
    std::vector<AnchorTile> atiles;
    for (int w = 0; w < W; ++w) {
        std::vector<std::pair<int, int>> iv;
        for (int s = 0; s < T; ++s) iv.emplace_back(spans[2 * s], spans[2 * s + 1]);
        const int ws = off[wfirst[w]], we = off[wlast[w] + 1];
        iv.emplace_back(ws, we);
        std::sort(iv.begin(), iv.end());
        std::vector<std::pair<int, int>> merged;
        for (auto &p : iv) {
            if (!merged.empty() && p.first <= merged.back().second)
                merged.back().second = std::max(merged.back().second, p.second);
            else
                merged.push_back(p);
        }
        for (auto &p : merged) aranges.push_back(KeyRange{p.first, p.second - p.first});
        arange_off[w + 1] = int32_t(aranges.size());
        for (int q0 = ws; q0 < we; q0 += kBM) atiles.push_back(AnchorTile{q0, std::min(kBM, we - q0), w, 0});
    }

    // key-stationary backward items. Caption key tiles come first, ordered by query segment: the
    // tiles that walk the same segment of queries are neighbours in the list, run at the same time
    // on one XCD and share those Q / dO rows in its L2 instead of each fetching them from HBM.
    std::vector<KvItem> kvitems;
    std::vector<TextTile> ttiles;
    int n_partials = 0;
    const int nseg = (N + kTextSeg - 1) / kTextSeg;
    for (int j = 0; j < C; ++j)
        if (kind[j])
            for (int k0 = off[j]; k0 < off[j + 1]; k0 += kKeyTile) {
                ttiles.push_back(TextTile{k0, std::min(kKeyTile, off[j + 1] - k0), n_partials, nseg});
                n_partials += nseg;
            }
    for (int s = 0; s < nseg; ++s)
        for (const TextTile &tt : ttiles)
            kvitems.push_back(KvItem{tt.key_start, tt.key_len, s * kTextSeg, std::min(kTextSeg, N - s * kTextSeg), -1,
                                     tt.first_partial + s, 0, 0});
    for (int j = 0; j < C; ++j) {
        if (kind[j]) continue;
        for (int k0 = off[j]; k0 < off[j + 1]; k0 += kKeyTile) {
            const int klen = std::min(kKeyTile, off[j + 1] - k0);
            const int w = win[j];
            const int ws = off[wfirst[w]], we = off[wlast[w] + 1];
            kvitems.push_back(KvItem{k0, klen, ws, we - ws, j, -1, 0, 0});
        }
    }

    std::vector<uint32_t> textmask((C + 31) / 32, 0u);
    for (int j = 0; j < C; ++j)
        if (kind[j]) textmask[j >> 5] |= 1u << (j & 31);

    moc_meta *m = new (std::nothrow) moc_meta();
    if (!m) return fail(MOC_ERR_HIP, "host allocation failed");
    m->N = N; m->C = C; m->T = T; m->W = W;
    m->n_atiles = int32_t(atiles.size());
    m->n_ranges = int32_t(aranges.size());
    m->n_kvitems = int32_t(kvitems.size());
    m->n_text_tiles = int32_t(ttiles.size());
    m->n_partials = n_partials;
    m->h_off.assign(off, off + C + 1);
    for (int j = 0; j < C; ++j) m->max_chunk_len = std::max(m->max_chunk_len, off[j + 1] - off[j]);
    m->h_kind = kind;
    m->h_win = win;

    // one device allocation, one blocking upload
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + std::max<size_t>(bytes, 16)); return r; };
    const size_t o_off = take((size_t)(C + 1) * 4), o_kind = take((size_t)C * 4), o_win = take((size_t)C * 4),
                 o_wf = take((size_t)W * 4), o_wl = take((size_t)W * 4), o_aro = take((size_t)(W + 1) * 4),
                 o_ar = take(aranges.size() * sizeof(KeyRange)), o_at = take(atiles.size() * sizeof(AnchorTile)),
                 o_kv = take(kvitems.size() * sizeof(KvItem)), o_tt = take(ttiles.size() * sizeof(TextTile)),
                 o_tm = take(textmask.size() * 4), o_ntb = take((size_t)(C + 1) * 4), o_rw = take((size_t)C * 4),
                 o_cof = take((size_t)N * 4);
    const size_t upload = o_cof;  // chunk_of is filled on the device
    std::vector<char> host(upload, 0);
    auto put = [&](size_t at, const void *src, size_t bytes) { if (bytes) std::memcpy(host.data() + at, src, bytes); };
    put(o_off, off, (size_t)(C + 1) * 4);
    put(o_kind, kind.data(), (size_t)C * 4);
    put(o_win, win.data(), (size_t)C * 4);
    put(o_wf, wfirst.data(), (size_t)W * 4);
    put(o_wl, wlast.data(), (size_t)W * 4);
    put(o_aro, arange_off.data(), (size_t)(W + 1) * 4);
    put(o_ar, aranges.data(), aranges.size() * sizeof(KeyRange));
    put(o_at, atiles.data(), atiles.size() * sizeof(AnchorTile));
    put(o_kv, kvitems.data(), kvitems.size() * sizeof(KvItem));
    put(o_tt, ttiles.data(), ttiles.size() * sizeof(TextTile));
    put(o_tm, textmask.data(), textmask.size() * 4);
    std::vector<int32_t> ntb(C + 1, 0);
    for (int j = 0; j < C; ++j) ntb[j + 1] = ntb[j] + (kind[j] ? 0 : 1);
    put(o_ntb, ntb.data(), (size_t)(C + 1) * 4);
    std::vector<int32_t> rwin(C);
    for (int j = 0; j < C; ++j) rwin[j] = kind[j] ? -1 : win[j];
    put(o_rw, rwin.data(), (size_t)C * 4);

    hipError_t e = hipMalloc(&m->d_base, o);
    if (e != hipSuccess) { delete m; return hip_fail(e, "hipMalloc(meta tables)"); }
    m->d_bytes = o;
    char *base = static_cast<char *>(m->d_base);
    m->d_off = reinterpret_cast<int32_t *>(base + o_off);
    m->d_kind = reinterpret_cast<int32_t *>(base + o_kind);
    m->d_win = reinterpret_cast<int32_t *>(base + o_win);
    m->d_wfirst = reinterpret_cast<int32_t *>(base + o_wf);
    m->d_wlast = reinterpret_cast<int32_t *>(base + o_wl);
    m->d_arange_off = reinterpret_cast<int32_t *>(base + o_aro);
    m->d_aranges = reinterpret_cast<KeyRange *>(base + o_ar);
    m->d_atiles = reinterpret_cast<AnchorTile *>(base + o_at);
    m->d_kvitems = reinterpret_cast<KvItem *>(base + o_kv);
    m->d_text_tiles = reinterpret_cast<TextTile *>(base + o_tt);
    m->d_textmask = reinterpret_cast<uint32_t *>(base + o_tm);
    m->d_ntb = reinterpret_cast<int32_t *>(base + o_ntb);
    m->d_rwin = reinterpret_cast<int32_t *>(base + o_rw);
    m->d_chunk_of = reinterpret_cast<int32_t *>(base + o_cof);

    hipStream_t st = static_cast<hipStream_t>(stream);
    e = hipMemcpy(m->d_base, host.data(), upload, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = launch_chunk_of(m, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        (void)hipFree(m->d_base);
        delete m;
        return hip_fail(e, "moc_chunk_meta upload");
    }
    *out = m;
    return MOC_OK;
}

int moc_meta_destroy(moc_meta *m) {
    if (!m) return MOC_OK;
    tag_drop_meta(m);
    hipError_t e = m->d_base ? hipFree(m->d_base) : hipSuccess;
    delete m;
    return e == hipSuccess ? MOC_OK : hip_fail(e, "hipFree(meta tables)");
}

int moc_meta_copy_tables(const moc_meta *m, int32_t *chunk_of, int32_t *kind, int32_t *win) {
    if (!m) return fail(MOC_ERR_NULL, "meta is NULL");
    hipError_t e = hipSuccess;
    if (chunk_of) e = hipMemcpy(chunk_of, m->d_chunk_of, (size_t)m->N * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess && kind) e = hipMemcpy(kind, m->d_kind, (size_t)m->C * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess && win) e = hipMemcpy(win, m->d_win, (size_t)m->C * 4, hipMemcpyDeviceToHost);
    return e == hipSuccess ? MOC_OK : hip_fail(e, "moc_meta_copy_tables");
}

int moc_route_workspace_bytes(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int32_t topk, int dtype,
                              size_t *bytes) {
    if (!bytes) return fail(MOC_ERR_NULL, "bytes is NULL");
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    *bytes = moc::route_ws_layout(meta, B * H, d, topk, dtype).total;
    return MOC_OK;
}

int moc_route(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
              int32_t topk, int32_t causal, float *pooled_k, int32_t *sel, void *workspace, size_t workspace_bytes,
              void *stream) {
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    if (!q || !k || !pooled_k || (!sel && topk > 0)) return fail(MOC_ERR_NULL, "q, k, pooled_k or sel is NULL");
    if (misaligned(q) || misaligned(k) || misaligned(pooled_k) || misaligned(sel))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const moc::RouteWs RL = moc::route_ws_layout(meta, B * H, d, topk, dtype);
    if (!workspace || workspace_bytes < RL.total) return fail(MOC_ERR_WORKSPACE, "route workspace too small");
    if (misaligned(workspace)) return fail(MOC_ERR_ALIGN, "workspace must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *kb_split = static_cast<char *>(workspace) + RL.kb_split;
    hipError_t e = moc::launch_pool(meta, B * H, d, dtype, k, pooled_k, kb_split, RL.Cpad, st);
    if (e != hipSuccess) return hip_fail(e, "pool kernel");
    if (topk > 0) {
        e = moc::launch_route(meta, B * H, d, dtype, q, kb_split, RL.Cpad, topk, causal, sel, topk, st);
        if (e != hipSuccess) return hip_fail(e, "route kernel");
    }
    return MOC_OK;
}

int moc_route_fused(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
                    int32_t topk, int32_t causal, float *pooled_k, int32_t *sel, void *workspace, size_t workspace_bytes,
                    void *stream) {
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    if (dtype != MOC_BF16) return fail(MOC_ERR_DTYPE, "moc_route_fused takes bf16 tensors");
    if (topk < 1) return fail(MOC_ERR_SHAPE, "moc_route_fused needs topk >= 1");
    if (!q || !k || !pooled_k || !sel) return fail(MOC_ERR_NULL, "q, k, pooled_k or sel is NULL");
    if (misaligned(q) || misaligned(k) || misaligned(pooled_k) || misaligned(sel))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const moc::RouteWs RL = moc::route_ws_layout(meta, B * H, d, topk, dtype);
    if (!workspace || workspace_bytes < RL.total) return fail(MOC_ERR_WORKSPACE, "route workspace too small");
    if (misaligned(workspace)) return fail(MOC_ERR_ALIGN, "workspace must be 16-byte aligned");
    void *kb_split = static_cast<char *>(workspace) + RL.kb_split;
    hipError_t e = moc::launch_route_fused(meta, B * H, d, q, k, pooled_k, kb_split, RL.Cpad, topk, causal, sel,
                                           static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e, "fused route kernel");
    return MOC_OK;
}

int moc_route_fused_status(int32_t *timed_out) {
    if (!timed_out) return fail(MOC_ERR_NULL, "timed_out is NULL");
    int t = 0;
    hipError_t e = moc::fused_wait_flag(&t);
    if (e != hipSuccess) return hip_fail(e, "moc_route_fused_status");
    *timed_out = t;
    return MOC_OK;
}

int moc_route_perturbed(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
                        int32_t topk, int32_t causal, float p_max, float lambda, int32_t max_in, uint64_t seed,
                        float *pooled_k, int32_t *sel, void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    if (max_in < 0 || topk + max_in > MOC_MAX_TOPK)
        return fail(MOC_ERR_SHAPE, "need 0 <= max_in and topk + max_in <= MOC_MAX_TOPK");
    if (!(p_max >= 0.f && p_max <= 1.f)) return fail(MOC_ERR_SHAPE, "p_max must lie in [0, 1]");
    if (!(lambda >= 0.f) || !std::isfinite(lambda)) return fail(MOC_ERR_SHAPE, "lambda must be finite and >= 0");
    const int width = topk + max_in;
    rc = check_common(meta, B, H, d, width, dtype);     // the N * width limits of the attention calls
    if (rc) return rc;
    if (!q || !k || !pooled_k || (!sel && width > 0)) return fail(MOC_ERR_NULL, "q, k, pooled_k or sel is NULL");
    if (misaligned(q) || misaligned(k) || misaligned(pooled_k) || misaligned(sel))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const moc::RouteWs RL = moc::route_ws_layout(meta, B * H, d, topk, dtype);
    if (!workspace || workspace_bytes < RL.total) return fail(MOC_ERR_WORKSPACE, "route workspace too small");
    if (misaligned(workspace)) return fail(MOC_ERR_ALIGN, "workspace must be 16-byte aligned");
    // Poisson by inversion: thresholds floor(CDF(j) * 2^32), pmf(j) = pmf(j-1) * lambda / j
    uint64_t thr[MOC_MAX_TOPK] = {};
    {
        double term = std::exp(-(double)lambda), cdf = 0.0;
        for (int j = 0; j < max_in; ++j) {
            if (j > 0) term = term * (double)lambda / j;
            cdf += term;
            thr[j] = (uint64_t)std::floor(std::min(cdf, 1.0) * 4294967296.0);
        }
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *kb_split = static_cast<char *>(workspace) + RL.kb_split;
    hipError_t e = moc::launch_pool(meta, B * H, d, dtype, k, pooled_k, kb_split, RL.Cpad, st);
    if (e != hipSuccess) return hip_fail(e, "pool kernel");
    if (width == 0) return MOC_OK;
    if (topk > 0) {
        e = moc::launch_route(meta, B * H, d, dtype, q, kb_split, RL.Cpad, topk, causal, sel, width, st);
        if (e != hipSuccess) return hip_fail(e, "route kernel");
    }
    e = moc::launch_perturb(meta, B * H, topk, max_in, causal, p_max, thr, seed, sel, st);
    if (e != hipSuccess) return hip_fail(e, "perturb kernel");
    return MOC_OK;
}

namespace {
struct OuterWs { size_t table, partial, total; };
OuterWs outer_ws_layout(int N, int D, int P) {
    OuterWs L{};
    L.table = 0;
    L.partial = align_up((size_t)(4 * (size_t)P + 4) * 4);
    L.total = L.partial + ((size_t)N / 64 + (size_t)P + 1) * (size_t)D * 4;
    return L;
}
int check_outer(int32_t N, int32_t D, int32_t P) {
    if (N <= 0 || P <= 0 || P > N) return fail(MOC_ERR_SHAPE, "need 0 < P <= N");
    if (P > moc::kMaxSegments) return fail(MOC_ERR_SHAPE, "too many segments");
    if (D <= 0 || D % 8 != 0) return fail(MOC_ERR_SHAPE, "D must be a positive multiple of 8");
    return MOC_OK;
}
}  // namespace

int moc_outer_workspace_bytes(int32_t N, int32_t D, int32_t P, size_t *bytes) {
    if (!bytes) return fail(MOC_ERR_NULL, "bytes is NULL");
    int rc = check_outer(N, D, P);
    if (rc) return rc;
    *bytes = outer_ws_layout(N, D, P).total;
    return MOC_OK;
}

int moc_outer_route(int32_t N, int32_t D, int dtype, const void *x, int32_t P, const int32_t *seg_offsets,
                    const int32_t *mandatory, int32_t g, int32_t M, int32_t causal, float *seg_mean, float *scores,
                    int32_t *selected, int32_t *kept, int32_t *n_kept, void *workspace, size_t workspace_bytes,
                    void *stream) {
    int rc = check_outer(N, D, P);
    if (rc) return rc;
    if (dtype != MOC_BF16 && dtype != MOC_F32) return fail(MOC_ERR_DTYPE, "dtype must be MOC_BF16 or MOC_F32");
    if (!x || !seg_offsets || !seg_mean || !scores || !kept || !n_kept || (!selected && M > 0))
        return fail(MOC_ERR_NULL, "a required pointer is NULL");
    if (g < 0 || g >= P) return fail(MOC_ERR_SHAPE, "g must name a segment");
    if (M < 0 || M > P) return fail(MOC_ERR_SHAPE, "need 0 <= M <= P");
    if (seg_offsets[0] != 0 || seg_offsets[P] != N) return fail(MOC_ERR_OFFSETS, "segment offsets must run from 0 to N");
    for (int j = 0; j < P; ++j)
        if (seg_offsets[j + 1] <= seg_offsets[j]) return fail(MOC_ERR_OFFSETS, "segment offsets must be strictly increasing");
    if (misaligned(x) || misaligned(seg_mean) || misaligned(workspace))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const OuterWs L = outer_ws_layout(N, D, P);
    if (!workspace || workspace_bytes < L.total) return fail(MOC_ERR_WORKSPACE, "outer-route workspace too small");

    // host table: offsets, first tile of each segment, candidate flags
    const int tile = 64;
    std::vector<int32_t> tab(4 * (size_t)P + 4, 0);
    int32_t *h_off = tab.data(), *h_tb = h_off + (P + 1), *h_cand = h_tb + (P + 1);
    int max_tiles = 0;
    for (int j = 0; j < P; ++j) {
        const int nt = (seg_offsets[j + 1] - seg_offsets[j] + tile - 1) / tile;
        h_off[j] = seg_offsets[j];
        h_tb[j + 1] = h_tb[j] + nt;
        max_tiles = std::max(max_tiles, nt);
        h_cand[j] = (j != g && !(mandatory && mandatory[j]) && (!causal || j < g)) ? 1 : 0;
    }
    h_off[P] = N;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    int32_t *d_tab = reinterpret_cast<int32_t *>(ws + L.table);
    hipError_t e = hipMemcpyAsync(d_tab, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) return hip_fail(e, "moc_outer_route table upload");
    int32_t *d_sel = d_tab + (3 * (size_t)P + 2);
    e = moc::launch_outer(D, dtype, x, P, max_tiles, g, M, d_tab, d_tab + (P + 1), d_tab + 2 * (P + 1),
                          reinterpret_cast<float *>(ws + L.partial), seg_mean, scores, d_sel, st);
    if (e != hipSuccess) return hip_fail(e, "outer-route kernels");
    if (M > 0) {
        e = hipMemcpyAsync(selected, d_sel, (size_t)M * 4, hipMemcpyDeviceToHost, st);
        if (e != hipSuccess) return hip_fail(e, "moc_outer_route selection download");
    }
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return hip_fail(e, "moc_outer_route");
    // reduced stream: mandatory segments, selected segments and g, in stream order
    std::vector<char> in(P, 0);
    in[g] = 1;
    for (int j = 0; j < P; ++j) if (mandatory && mandatory[j]) in[j] = 1;
    for (int r = 0; r < M; ++r) if (selected[r] >= 0) in[selected[r]] = 1;
    int n = 0;
    for (int j = 0; j < P; ++j) if (in[j]) kept[n++] = j;
    *n_kept = n;
    return MOC_OK;
}

int moc_gather_rows(int32_t outer, int32_t n_src_rows, int32_t row_bytes, const void *src, int32_t n_ranges,
                    const int32_t *ranges, void *dst, void *workspace, size_t workspace_bytes, void *stream) {
    if (outer <= 0 || n_src_rows <= 0 || n_ranges < 0) return fail(MOC_ERR_SHAPE, "outer, n_src_rows must be positive");
    if (row_bytes <= 0 || row_bytes % 16 != 0) return fail(MOC_ERR_SHAPE, "row_bytes must be a positive multiple of 16");
    if (n_ranges == 0) return MOC_OK;
    if (!ranges) return fail(MOC_ERR_NULL, "ranges is NULL");
    // empty ranges contribute no rows and are left out of the device table
    std::vector<int32_t> tab((size_t)n_ranges * 4, 0);
    long long n_dst = 0;
    int n_tab = 0;
    for (int r = 0; r < n_ranges; ++r) {
        const int32_t s0 = ranges[2 * r], len = ranges[2 * r + 1];
        if (s0 < 0 || len < 0 || (long long)s0 + len > n_src_rows) return fail(MOC_ERR_OFFSETS, "range outside the source");
        if (len == 0) continue;
        if (n_dst + len >= (1LL << 31)) return fail(MOC_ERR_SHAPE, "reduced stream too long");
        tab[4 * n_tab] = s0; tab[4 * n_tab + 1] = len; tab[4 * n_tab + 2] = (int32_t)n_dst;
        n_dst += len;
        ++n_tab;
    }
    if (n_tab == 0) return MOC_OK;
    if (!src || !dst) return fail(MOC_ERR_NULL, "src or dst is NULL");
    if (misaligned(src) || misaligned(dst) || misaligned(workspace))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    if (!workspace || workspace_bytes < (size_t)n_tab * 16) return fail(MOC_ERR_WORKSPACE, "need 16 bytes per range");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(workspace, tab.data(), (size_t)n_tab * 16, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = moc::launch_gather(outer, n_src_rows, n_dst, row_bytes, src, dst, workspace, n_tab, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);      // the table lives on this call's stack
    return e == hipSuccess ? MOC_OK : hip_fail(e, "moc_gather_rows");
}

int moc_outer_segments(int32_t C, const int32_t *off, const int32_t *shot, const int32_t *spans, int32_t T,
                       int32_t *seg_offsets, int32_t *is_caption, int32_t *P) {
    if (!off || !shot || !seg_offsets || !is_caption || !P) return fail(MOC_ERR_NULL, "a required pointer is NULL");
    if (T < 0 || (T > 0 && !spans)) return fail(MOC_ERR_NULL, "text_spans is NULL with T > 0");
    if (C <= 0) return fail(MOC_ERR_SHAPE, "need C > 0");
    if (off[0] != 0) return fail(MOC_ERR_OFFSETS, "offsets must start at 0");
    for (int j = 0; j < C; ++j)
        if (off[j + 1] <= off[j]) return fail(MOC_ERR_OFFSETS, "offsets must be strictly increasing");
    // a chunk starts a segment if a caption span starts or ends there, or the shot changes
    std::vector<char> cut(C + 1, 0), text(C, 0);
    cut[0] = cut[C] = 1;
    for (int s = 0; s < T; ++s) {
        const int a = spans[2 * s], b = spans[2 * s + 1];
        const int32_t *pa = std::lower_bound(off, off + C + 1, a), *pb = std::lower_bound(off, off + C + 1, b);
        if (a >= b || pa == off + C + 1 || pb == off + C + 1 || *pa != a || *pb != b)
            return fail(MOC_ERR_TEXT_SPAN, "text span is not a union of whole chunks");
        cut[pa - off] = cut[pb - off] = 1;
        for (int j = int(pa - off); j < int(pb - off); ++j) text[j] = 1;
    }
    for (int j = 1; j < C; ++j)
        if (shot[j] != shot[j - 1]) cut[j] = 1;
    int n = 0;
    for (int j = 0; j < C; ++j)
        if (cut[j]) { seg_offsets[n] = off[j]; is_caption[n] = text[j]; ++n; }
    seg_offsets[n] = off[C];
    *P = n;
    return MOC_OK;
}

int moc_reduce_layout(int32_t C, const int32_t *off, const int32_t *shot, const int32_t *window,
                      const int32_t *spans, int32_t T, int32_t P, const int32_t *seg_offsets, int32_t n_kept,
                      const int32_t *kept, int32_t *out_offsets, int32_t *out_shot, int32_t *out_window,
                      int32_t *out_spans, int32_t *out_C, int32_t *out_T, int32_t *out_ranges) {
    if (!off || !shot || !seg_offsets || !kept || !out_offsets || !out_shot || !out_window || !out_C || !out_T ||
        !out_ranges)
        return fail(MOC_ERR_NULL, "a required pointer is NULL");
    if (T < 0 || (T > 0 && (!spans || !out_spans))) return fail(MOC_ERR_NULL, "text spans missing with T > 0");
    if (C <= 0 || P <= 0 || n_kept <= 0 || n_kept > P) return fail(MOC_ERR_SHAPE, "need C, P > 0 and 0 < n_kept <= P");
    if (off[0] != 0 || seg_offsets[0] != 0 || seg_offsets[P] != off[C])
        return fail(MOC_ERR_OFFSETS, "chunk and segment offsets must cover the same stream");
    for (int j = 0; j < C; ++j)
        if (off[j + 1] <= off[j]) return fail(MOC_ERR_OFFSETS, "offsets must be strictly increasing");
    for (int r = 0; r < n_kept; ++r) {
        if (kept[r] < 0 || kept[r] >= P) return fail(MOC_ERR_SHAPE, "kept names no segment");
        if (r > 0 && kept[r] <= kept[r - 1]) return fail(MOC_ERR_SHAPE, "kept must ascend");
    }
    int nc = 0, nt = 0, pos = 0;
    out_offsets[0] = 0;
    for (int r = 0; r < n_kept; ++r) {
        const int a = seg_offsets[kept[r]], b = seg_offsets[kept[r] + 1];
        const int32_t *pa = std::lower_bound(off, off + C + 1, a), *pb = std::lower_bound(off, off + C + 1, b);
        if (a >= b || pa == off + C + 1 || pb == off + C + 1 || *pa != a || *pb != b)
            return fail(MOC_ERR_OFFSETS, "segment boundaries must be chunk boundaries");
        out_ranges[2 * r] = a;
        out_ranges[2 * r + 1] = b - a;
        const int shift = pos - a;           // stream position -> reduced position inside this segment
        for (int j = int(pa - off); j < int(pb - off); ++j) {
            out_shot[nc] = shot[j];
            out_window[nc] = window ? window[j] : j;
            out_offsets[++nc] = off[j + 1] + shift;
        }
        // the part of every caption span that lies inside the segment stays a caption span
        for (int s = 0; s < T; ++s) {
            const int lo = std::max(spans[2 * s], a), hi = std::min(spans[2 * s + 1], b);
            if (lo < hi) { out_spans[2 * nt] = lo + shift; out_spans[2 * nt + 1] = hi + shift; ++nt; }
        }
        pos += b - a;
    }
    *out_C = nc;
    *out_T = nt;
    return MOC_OK;
}

namespace {
// Scratch of moc_route_static: the three bf16 planes of the pooled keys. One copy per GPU, held
// until the process ends. In host code the array's name is only a handle for hipGetSymbolAddress:
// the device address is looked up once per device and every launch takes that pointer.
constexpr size_t kStaticScratchBytes = (size_t)MOC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(MOC_ERR_HIP, "device ordinal out of range");
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        if (!p) return fail(MOC_ERR_HIP, "hipGetSymbolAddress returned NULL");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MOC_OK;
}
}  // namespace

int moc_route_static(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
                     int32_t topk, int32_t causal, float *pooled_k, int32_t *sel, void *stream) {
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    if (!q || !k || !pooled_k || (!sel && topk > 0)) return fail(MOC_ERR_NULL, "q, k, pooled_k or sel is NULL");
    if (misaligned(q) || misaligned(k) || misaligned(pooled_k) || misaligned(sel))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const moc::RouteWs RL = moc::route_ws_layout(meta, B * H, d, topk, dtype);
    if (RL.total > kStaticScratchBytes)
        return fail(MOC_ERR_WORKSPACE, "moc_route_static: B * H * 3 * roundup(C, 32) * d * 2 bytes exceed "
                                       "MOC_STATIC_SCRATCH_BYTES; use moc_route with a workspace");
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void *kb_split = static_cast<char *>(ws) + RL.kb_split;
    // the pooling pass writes every row of the planes it is about to use (pad rows included), so
    // nothing of an earlier call's contents is read
    hipError_t e = moc::launch_pool(meta, B * H, d, dtype, k, pooled_k, kb_split, RL.Cpad, st);
    if (e != hipSuccess) return hip_fail(e, "pool kernel");
    if (topk > 0) {
        e = moc::launch_route(meta, B * H, d, dtype, q, kb_split, RL.Cpad, topk, causal, sel, topk, st);
        if (e != hipSuccess) return hip_fail(e, "route kernel");
    }
    return MOC_OK;
}

int moc_attn_workspace_bytes(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int32_t topk, int dtype,
                             int with_bwd, size_t *bytes) {
    if (!bytes) return fail(MOC_ERR_NULL, "bytes is NULL");
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    *bytes = moc::attn_ws_layout(meta, B * H, d, topk, with_bwd != 0).total;
    return MOC_OK;
}

namespace {

int attn_bwd_impl(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
                  const void *v, const void *o, const float *lse, const void *d_o, const int32_t *sel, int32_t topk,
                  float softmax_scale, void *dq, void *dk, void *dv, void *workspace, size_t workspace_bytes,
                  void *stream, bool reuse_lists) {
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    if (bad_scale(softmax_scale)) return fail(MOC_ERR_SHAPE, "softmax_scale must be finite and positive");
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv || (!sel && topk > 0))
        return fail(MOC_ERR_NULL, "a tensor pointer is NULL");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) || misaligned(d_o) ||
        misaligned(dq) || misaligned(dk) || misaligned(dv) || misaligned(sel))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const moc::AttnWs L = moc::attn_ws_layout(meta, B * H, d, topk, true);
    if (!workspace || workspace_bytes < L.total) return fail(MOC_ERR_WORKSPACE, "attention workspace too small (with_bwd)");
    if (misaligned(workspace)) return fail(MOC_ERR_ALIGN, "workspace must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    const ListTag tag{meta, sel, B, H, topk, stream};
    if (topk > 0 && !(reuse_lists && tag_matches(workspace, tag))) {
        e = moc::launch_build_lists(meta, B * H, topk, sel, static_cast<char *>(workspace), L, st);
        if (e != hipSuccess) { tag_drop(workspace); return hip_fail(e, "list kernels"); }
    }
    tag_drop(workspace);     // the backward leaves the workspace to whoever comes next
    e = moc::launch_attn_bwd(meta, B * H, d, dtype, q, k, v, o, lse, d_o, topk, softmax_scale, dq, dk, dv,
                             static_cast<char *>(workspace), L, st);
    if (e != hipSuccess) return hip_fail(e, "attention backward kernels");
    return MOC_OK;
}

}  // namespace

int moc_attn_fwd(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
                 const void *v, const int32_t *sel, int32_t topk, float softmax_scale, void *o, float *lse,
                 void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_common(meta, B, H, d, topk, dtype);
    if (rc) return rc;
    if (bad_scale(softmax_scale)) return fail(MOC_ERR_SHAPE, "softmax_scale must be finite and positive");
    if (!q || !k || !v || !o || !lse || (!sel && topk > 0)) return fail(MOC_ERR_NULL, "a tensor pointer is NULL");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o) || misaligned(lse) || misaligned(sel))
        return fail(MOC_ERR_ALIGN, "device pointers must be 16-byte aligned");
    const moc::AttnWs L = moc::attn_ws_layout(meta, B * H, d, topk, false);
    if (!workspace || workspace_bytes < L.total) return fail(MOC_ERR_WORKSPACE, "attention workspace too small");
    if (misaligned(workspace)) return fail(MOC_ERR_ALIGN, "workspace must be 16-byte aligned");
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    tag_drop(workspace);
    if (topk > 0) {
        e = moc::launch_build_lists(meta, B * H, topk, sel, static_cast<char *>(workspace), L, st);
        if (e != hipSuccess) return hip_fail(e, "list kernels");
    }
    e = moc::launch_attn_fwd(meta, B * H, d, dtype, q, k, v, topk, softmax_scale, o, lse,
                             static_cast<char *>(workspace), L, st);
    if (e != hipSuccess) return hip_fail(e, "attention forward kernels");
    if (topk > 0) tag_set(workspace, ListTag{meta, sel, B, H, topk, stream});
    return MOC_OK;
}

int moc_attn_bwd(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q, const void *k,
                 const void *v, const void *o, const float *lse, const void *d_o, const int32_t *sel, int32_t topk,
                 float softmax_scale, void *dq, void *dk, void *dv, void *workspace, size_t workspace_bytes,
                 void *stream) {
    return attn_bwd_impl(meta, B, H, d, dtype, q, k, v, o, lse, d_o, sel, topk, softmax_scale, dq, dk, dv, workspace,
                         workspace_bytes, stream, false);
}

int moc_attn_bwd_after_fwd(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype, const void *q,
                           const void *k, const void *v, const void *o, const float *lse, const void *d_o,
                           const int32_t *sel, int32_t topk, float softmax_scale, void *dq, void *dk, void *dv,
                           void *workspace, size_t workspace_bytes, void *stream) {
    return attn_bwd_impl(meta, B, H, d, dtype, q, k, v, o, lse, d_o, sel, topk, softmax_scale, dq, dk, dv, workspace,
                         workspace_bytes, stream, true);
}

}  // extern "C"
