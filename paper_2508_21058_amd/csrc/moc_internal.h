// Host-side structures and kernel launchers of libmoc (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "../../include/moc.h"

namespace moc {

constexpr int kBM = 128;         // queries per workgroup in the query-stationary passes
constexpr int kKeyTile = 128;    // keys per workgroup in the key-stationary pass (4 waves x 32)
constexpr int kTextSeg = 16384;   // queries per partial of a text key tile in the key-stationary pass
constexpr int kRowsPerBlk = 256; // queries per block of the list builder (one wave and one histogram column each)
constexpr int kMaxListChunks = 16384;   // chunks the list builder's LDS histogram holds

// One query tile of the forced-link pass: queries [q_start, q_start+q_count)
// all belong to window `win` and share its key ranges.
struct AnchorTile { int32_t q_start, q_count, win, pad; };

// A contiguous key range [start, start+len).
struct KeyRange { int32_t start, len; };

// One workgroup of the key-stationary backward pass.
//   keys [key_start, key_start+key_len), key_len <= kKeyTile
//   contiguous query source [q_start, q_start+q_len)
//   chunk >= 0: additionally the routed-query list of that chunk
//   partial >= 0: write fp32 partial sums to that slot instead of dk/dv
struct KvItem { int32_t key_start, key_len, q_start, q_len, chunk, partial, pad0, pad1; };

// A text key tile and the partial slots to sum for it.
struct TextTile { int32_t key_start, key_len, first_partial, n_partials; };

}  // namespace moc

struct moc_meta {
    int32_t N = 0, C = 0, T = 0, W = 0;
    int32_t n_atiles = 0, n_ranges = 0, n_kvitems = 0, n_text_tiles = 0, n_partials = 0;
    int32_t max_chunk_len = 0;
    void *d_base = nullptr;
    size_t d_bytes = 0;
    int32_t *d_off = nullptr;        // [C+1]
    int32_t *d_kind = nullptr;       // [C] 1 = text
    int32_t *d_win = nullptr;        // [C] dense window id
    int32_t *d_rwin = nullptr;       // [C] window id of a video chunk, -1 for a caption chunk
    int32_t *d_wfirst = nullptr;     // [W] first chunk of window
    int32_t *d_wlast = nullptr;      // [W] last chunk of window (inclusive)
    int32_t *d_chunk_of = nullptr;   // [N]
    uint32_t *d_textmask = nullptr;  // [ceil(C/32)] bit j%32 of word j/32 set: chunk j is text
    int32_t *d_ntb = nullptr;        // [C+1] number of non-text chunks with index < j
    int32_t *d_arange_off = nullptr; // [W+1] into d_aranges
    moc::KeyRange *d_aranges = nullptr;
    moc::AnchorTile *d_atiles = nullptr;
    moc::KvItem *d_kvitems = nullptr;
    moc::TextTile *d_text_tiles = nullptr;
    std::vector<int32_t> h_off, h_kind, h_win;
};

namespace moc {

// Optional per-kernel timing with HIP events on the launch stream (off by
// default; switched on through moc_prof_enable). A Scope brackets one launch.
bool prof_on();
void prof_begin(const char *name, hipStream_t st);
void prof_end(hipStream_t st);
struct ProfScope {
    hipStream_t st;
    bool on;
    ProfScope(const char *name, hipStream_t s) : st(s), on(prof_on()) { if (on) prof_begin(name, s); }
    ~ProfScope() { if (on) prof_end(st); }
};
#define MOC_PROF(name, st) ::moc::ProfScope moc_prof_scope_(name, st)

// Drop-off / drop-in on rows of width topk + max_in whose first topk columns hold the routed chunks.
hipError_t launch_perturb(const moc_meta *m, int BH, int topk, int max_in, int causal, float p_max,
                          const uint64_t *thr, uint64_t seed, int32_t *sel, hipStream_t st);

// Outer-loop routing over [N, D] features: per-segment means, scores against segment g, top-M on the device.
constexpr int kMaxSegments = 4096;
hipError_t launch_outer(int D, int dtype, const void *x, int P, int max_tiles, int g, int M, const int32_t *d_seg_off,
                        const int32_t *d_tile_base, const int32_t *d_cand, float *partial, float *mean,
                        float *scores, int32_t *d_selected, hipStream_t st);
// dst[o][..] = rows of src[o] listed by `n_ranges` records (src row, length, dst row, pad) on the device.
hipError_t launch_gather(int outer, long long n_src_rows, long long n_dst_rows, int row_bytes, const void *src,
                         void *dst, const void *d_ranges, int n_ranges, hipStream_t st);

// Machine probes (streaming copy, MFMA loop); see moc_probe.
constexpr int kProbeMfmaGrid = 256;
hipError_t launch_probe(int kind, void *buf, size_t bytes, int iters, hipStream_t st, hipEvent_t e0, hipEvent_t e1,
                        double *units);

// Layout of the attention workspace (byte offsets); shared by fwd and bwd.
struct AttnWs {
    size_t cnt, list_off, tile_off, vmask, gsum, cnt_blk, qlist, plse, po, delta, stats2, gstats2, tpart_k, tpart_v, total;
};
AttnWs attn_ws_layout(const moc_meta *m, int BH, int d, int topk, bool with_bwd);

// Route workspace: pooled keys split into three bf16 planes (hi, mid, lo with
// hi + mid + lo == the fp32 value), [BH][3][Cpad][d], Cpad = C rounded up to 32, pad rows zero.
struct RouteWs { size_t kb_split, total; int Cpad; };
RouteWs route_ws_layout(const moc_meta *m, int BH, int d, int topk, int dtype);

hipError_t launch_chunk_of(const moc_meta *m, hipStream_t st);

hipError_t launch_pool(const moc_meta *m, int BH, int d, int dtype, const void *k, float *kbar, void *kb_split,
                       int Cpad, hipStream_t st);

hipError_t launch_route(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *kb_split, int Cpad,
                        int topk, int causal, int32_t *sel, int sel_stride, hipStream_t st);

// pooling + scoring + top-k in one launch (bf16 storage); see route_fused_kernel
hipError_t launch_route_fused(const moc_meta *m, int BH, int d, const void *q, const void *k, float *kbar,
                              void *kb_split, int Cpad, int topk, int causal, int32_t *sel, hipStream_t st);
hipError_t fused_wait_flag(int *timed_out);

// counts -> offsets -> inverse lists (per head and chunk: the queries that routed to it)
hipError_t launch_build_lists(const moc_meta *m, int BH, int topk, const int32_t *sel, char *ws,
                              const AttnWs &L, hipStream_t st);

// (both read the lists and the slot masks launch_build_lists left in the workspace)
hipError_t launch_attn_fwd(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *k,
                           const void *v, int topk, float scale, void *o, float *lse, char *ws, const AttnWs &L,
                           hipStream_t st);

hipError_t launch_attn_bwd(const moc_meta *m, int BH, int d, int dtype, const void *q, const void *k,
                           const void *v, const void *o, const float *lse, const void *d_o, int topk, float scale,
                           void *dq, void *dk, void *dv, char *ws, const AttnWs &L, hipStream_t st);

}  // namespace moc
