/*
 * moc.h - C ABI of the Mixture-of-Contexts (MoC) sparse attention layer for
 * AMD MI355X (gfx950 / CDNA4).
 *
 * The layer (paper Sec. 3) has four stages, one entry point each:
 *   (a) moc_chunk_meta  content-aligned chunk tables            (Sec. 3.2, 3.3)
 *   (b,c) moc_route     mean-pooled chunk keys, query-chunk scores, per-query
 *                       top-k with forced links and the causal routing mask
 *                                                           (Eq. 3; Sec. 3.2, 3.3)
 *   (d) moc_attn_fwd    softmax attention over the tokens of the forced and the
 *                       routed chunks only                         (Eq. 2)
 *       moc_attn_bwd    its backward, the selection being a constant (Sec. 3.1)
 *
 * Conventions
 *   - All tensors are contiguous, head-major [B, H, N, d] (Sec. 3.3 "head-major
 *     order"); B samples share ONE layout; K/V heads = Q heads.
 *   - "HOST" pointers are read before the call returns. "DEVICE" pointers are
 *     hipMalloc'ed memory owned by the caller; they must be 16-byte aligned.
 *   - Every call only enqueues work on `stream` (a hipStream_t, may be NULL for
 *     the default stream) and returns without synchronising, except
 *     moc_chunk_meta / moc_meta_copy_tables, which also do small blocking
 *     copies, and the calls whose own comment says that they wait for their
 *     work (moc_outer_route, moc_gather_rows, moc_route_fused_status,
 *     moc_prof_read, moc_probe).
 *   - The library allocates device memory only inside moc_chunk_meta (a few
 *     small tables owned by the moc_meta handle). All other scratch space is a
 *     caller-owned workspace whose size the *_workspace_bytes calls report;
 *     the one exception is moc_route_static, whose scratch is a static device
 *     array of MOC_STATIC_SCRATCH_BYTES inside the library.
 *   - Return value: MOC_OK (0) or a negative moc_status. Nothing throws, aborts
 *     or prints. All argument checks happen before any device work.
 *     moc_last_error() returns a thread-local detail string of the last failure.
 *   - d must be 64 or 128; 0 <= topk <= MOC_MAX_TOPK; N < 2^26; N * max(topk,1) < 2^31;
 *     B * H * N * (topk + 1) < 2^31.
 */
#ifndef MOC_H_
#define MOC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOC_MAX_TOPK 32

typedef enum moc_dtype {
    MOC_BF16 = 0, /* bfloat16 storage for q/k/v/o/dO/dq/dk/dv */
    MOC_F32 = 1   /* float32 storage; attention contractions still run on bf16
                     matrix cores (operands rounded to nearest-even), routing
                     scores are accumulated in fp32 from the fp32 values */
} moc_dtype;

typedef enum moc_status {
    MOC_OK = 0,
    MOC_ERR_NULL = -1,      /* a required pointer is NULL */
    MOC_ERR_SHAPE = -2,     /* N, C, B, H <= 0; d not in {64,128}; topk out of range; N*topk overflow */
    MOC_ERR_OFFSETS = -3,   /* chunk_offsets not strictly increasing from 0 to N */
    MOC_ERR_TEXT_SPAN = -4, /* a text span is empty, out of range, overlapping, unsorted or not chunk-aligned */
    MOC_ERR_WINDOW = -5,    /* equal window ids not contiguous, or a window spans two shots */
    MOC_ERR_DTYPE = -6,     /* dtype is neither MOC_BF16 nor MOC_F32 */
    MOC_ERR_WORKSPACE = -7, /* workspace NULL or smaller than *_workspace_bytes reports */
    MOC_ERR_ALIGN = -8,     /* a device pointer is not 16-byte aligned */
    MOC_ERR_HIP = -9,       /* a HIP runtime call or kernel launch failed */
    MOC_ERR_SHOT = -10      /* chunk_shot decreases */
} moc_status;

const char *moc_status_string(int status);
const char *moc_last_error(void);

/* Opaque handle: owns only small device tables derived from the layout
 * (token->chunk map, chunk kind / window tables, forced-link key ranges,
 * query-tile lists of the forced-link pass). Reusable across layers, heads and
 * steps that share the layout. Not tied to a stream after creation returns. */
typedef struct moc_meta moc_meta;

/*
 * Stage (a): chunk tables (Sec. 3.3: boundary tags -> bucketize + prefix-sum
 * tables -> content-aligned variable-length chunks; Sec. 3.2 forced links).
 *   N, C            tokens and chunks of the flattened stream
 *   chunk_offsets   HOST [C+1], off[0] = 0 < off[1] < ... < off[C] = N
 *   chunk_shot      HOST [C], non-decreasing shot id per chunk
 *   chunk_window    HOST [C] or NULL. Chunks with equal id form one local
 *                   window and are mandatory for each other's queries (forced
 *                   intra-shot link). Equal ids must be contiguous and lie in one
 *                   shot. NULL: every chunk is its own window.
 *   text_spans,T    HOST [T][2] token ranges [start,end) of caption spans,
 *                   sorted, disjoint, each a union of whole chunks. Every query
 *                   attends all of them (forced cross-modal link). T may be 0.
 *   out             receives the handle; free with moc_meta_destroy.
 */
int moc_chunk_meta(int32_t N, int32_t C, const int32_t *chunk_offsets, const int32_t *chunk_shot,
                   const int32_t *chunk_window, const int32_t *text_spans, int32_t T,
                   void *stream, moc_meta **out);
int moc_meta_destroy(moc_meta *meta);

/* Test hook for stage (a): blocking copy of the device tables to HOST arrays
 * (any may be NULL): chunk_of [N], chunk_kind [C] (1 = text, 0 = video),
 * chunk_window [C] (dense ids in order of first appearance). */
int moc_meta_copy_tables(const moc_meta *meta, int32_t *chunk_of, int32_t *chunk_kind,
                         int32_t *chunk_window);

/*
 * Stages (b)+(c): routing.
 *   pooled_k  DEVICE out [B,H,C,d] fp32: arithmetic mean of each chunk's keys
 *             (the descriptor phi of Eq. 3), text chunks included.
 *   sel       DEVICE out [B,H,N,topk] int32: for every query the routed chunks,
 *             best score first, ties to the lower chunk index, -1 padded when
 *             fewer than topk candidates exist. Candidates of query i in chunk
 *             c(i): chunks that are neither text nor in c(i)'s window, and, when
 *             causal != 0, have index < c(i). Score = q . pooled_k (no 1/sqrt d).
 *   q, k      DEVICE in [B,H,N,d] of `dtype`.
 *   workspace DEVICE scratch of moc_route_workspace_bytes bytes.
 */
int moc_route_workspace_bytes(const moc_meta *meta, int32_t B, int32_t H, int32_t d,
                              int32_t topk, int dtype, size_t *bytes);
int moc_route(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
              const void *q, const void *k, int32_t topk, int32_t causal,
              float *pooled_k, int32_t *sel, void *workspace, size_t workspace_bytes,
              void *stream);

/*
 * moc_route for callers that cannot allocate device memory or carry a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same arguments and results as moc_route (bit for bit), no
 * workspace: the scratch that pass needs (the pooled keys split into three bf16
 * planes, B * H * 3 * roundup(C, 32) * d * 2 bytes) lives in a static device
 * array of MOC_STATIC_SCRATCH_BYTES that every GPU the library runs on holds
 * until the process ends. Larger shapes are rejected with MOC_ERR_WORKSPACE.
 * The call allocates nothing and frees nothing. All calls on one GPU share that
 * array: calls that may overlap on one GPU (different streams or threads) race
 * and must be serialised by the caller; calls on one stream are ordered.
 */
#define MOC_STATIC_SCRATCH_BYTES (16u << 20)
int moc_route_static(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
                     const void *q, const void *k, int32_t topk, int32_t causal,
                     float *pooled_k, int32_t *sel, void *stream);

/*
 * Stages (b)+(c) in ONE kernel launch (Sec. 5 names the fusion of routing as
 * future work): same arguments, workspace and results as moc_route, bit for
 * bit; bf16 tensors and topk >= 1 only. Inside the launch the first workgroups
 * pool all chunks and every workgroup waits, for a bounded time, until the
 * pooled keys are complete before it scores. The completion counter is a static
 * device word of the library: fused launches must not overlap on one GPU.
 * moc_route_fused_status (blocking) reports, and clears, whether any such wait
 * ever ran out (then that call's sel is not valid); it never has in testing.
 * On the benchmark shapes the fused launch is not faster than moc_route's two
 * launches (figures in the design notes); moc_route stays the default.
 */
int moc_route_fused(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
                    const void *q, const void *k, int32_t topk, int32_t causal,
                    float *pooled_k, int32_t *sel, void *workspace, size_t workspace_bytes,
                    void *stream);
int moc_route_fused_status(int32_t *timed_out);

/*
 * Routing with the two training-time regularisers of Sec. 3.2 ("Context
 * Drop-off", "Context Drop-in") applied to every (batch, head, query) row after
 * the top-k of moc_route:
 *   drop-off  p = u * p_max with u uniform in [0, 1); floor(p * topk) of the
 *             routed chunks (at most all of them), chosen uniformly without
 *             replacement, are removed; the others keep their order.
 *   drop-in   m ~ Poisson(lambda), truncated at max_in and at the number of
 *             chunks available, is drawn by inversion; m chunks are added,
 *             chosen uniformly without replacement from the query's routing
 *             candidates that moc_route did not select for it (a chunk removed
 *             by drop-off does not come back).
 *   sel       DEVICE out [B,H,N,topk + max_in] int32: surviving routed chunks
 *             (best first), then the added chunks in the order drawn, then -1.
 *             Pass it to moc_attn_fwd / moc_attn_bwd with topk + max_in as
 *             their topk. Requires topk + max_in <= MOC_MAX_TOPK.
 *   p_max     in [0, 1]; lambda >= 0, finite; both 0 reproduce moc_route.
 *   seed      the random words of row (b, h, i) are the Philox4x32-10 stream
 *             with key (seed low word, seed high word) and counter
 *             (i, b*H + h, block, 0); draw t is word t mod 4 of block t / 4:
 *             draw 0 -> u = (draw >> 8) * 2^-24, draw 1 -> m = #{j < max_in :
 *             draw >= floor(CDF(j) * 2^32)}, then one draw per removal
 *             (entry floor(draw * n / 2^32) of the n still alive) and one per
 *             addition (entry floor(draw * n / 2^32) of the n available chunks
 *             in ascending index order). floor(p * topk) is evaluated in single
 *             precision as (u * p_max) * topk. The same seed gives the same
 *             rows on every call.
 * Everything else (pooled_k, q, k, workspace of moc_route_workspace_bytes with
 * the same topk, errors) is as for moc_route.
 */
int moc_route_perturbed(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
                        const void *q, const void *k, int32_t topk, int32_t causal,
                        float p_max, float lambda, int32_t max_in, uint64_t seed,
                        float *pooled_k, int32_t *sel, void *workspace, size_t workspace_bytes,
                        void *stream);

/*
 * Outer-loop context routing (App. "Outer Loop Context Routing"): a coarse
 * selection of whole segments (e.g. shots) before the layer runs.
 *   x            DEVICE in [N, D] of `dtype`: token features; D a multiple of 8.
 *   seg_offsets  HOST [P+1]: segment j = rows [seg_offsets[j], seg_offsets[j+1]),
 *                strictly increasing from 0 to N; P <= 4096.
 *   mandatory    HOST [P] or NULL: non-zero marks segments that are always kept
 *                (e.g. the global caption) and never compete.
 *   g            the segment being generated; its mean feature is the query.
 *   seg_mean     DEVICE out [P, D] fp32: arithmetic mean of each segment's rows.
 *   scores       DEVICE out [P] fp32: <seg_mean[j], seg_mean[g]> for every j.
 *   selected     HOST out [M]: the M best-scoring candidates, best first, ties
 *                to the lower index, -1 padded. Candidates: segments other than
 *                g that are not mandatory and, when causal != 0, precede g.
 *   kept, n_kept HOST out [P], [1]: the segments of the reduced stream
 *                (mandatory, selected and g) in ascending order.
 *   workspace    DEVICE scratch of moc_outer_workspace_bytes(N, D, P) bytes.
 * The call returns after the work on `stream` has finished (its results are
 * needed on the host). Sums are formed in a fixed order: same input, same bits.
 *
 * moc_gather_rows builds the reduced stream of any row-major tensor: src is
 * DEVICE [outer][n_src_rows][row_bytes], dst DEVICE [outer][sum of lengths]
 * [row_bytes]; ranges HOST [n_ranges][2] = (first row, length) in the order the
 * rows are to appear (a length of 0 is allowed and adds nothing; ranges may
 * overlap or repeat); row_bytes a multiple of 16; workspace DEVICE scratch of
 * at least 16 * n_ranges bytes. Also returns after the copy has finished.
 *
 * Layout bookkeeping of the outer loop, host arrays only, no device work:
 * moc_outer_segments cuts the stream into the segments the outer router sees:
 *   a new segment starts wherever a caption span starts or ends and wherever
 *   the shot id changes, so every caption span is a segment of its own and the
 *   video chunks of a shot between two captions form one segment.
 *   seg_offsets HOST out [up to C+1], is_caption HOST out [up to C] (1: the
 *   segment is a caption span), *P the number of segments.
 * moc_reduce_layout builds the layout of the reduced stream made of the kept
 *   segments (ascending, each bounded by chunk boundaries) for moc_chunk_meta:
 *   chunks move as a whole and keep their shot and window ids; the part of a
 *   caption span inside a kept segment stays a caption span.
 *   out_offsets HOST out [up to C+1], out_shot / out_window [up to C],
 *   out_spans [up to T + n_kept][2], *out_C, *out_T the sizes used; out_ranges HOST out
 *   [n_kept][2] = (first row, length) of every kept segment, the table
 *   moc_gather_rows takes. chunk_window may be NULL (own chunk).
 */
int moc_outer_segments(int32_t C, const int32_t *chunk_offsets, const int32_t *chunk_shot,
                       const int32_t *text_spans, int32_t T, int32_t *seg_offsets,
                       int32_t *is_caption, int32_t *P);
int moc_reduce_layout(int32_t C, const int32_t *chunk_offsets, const int32_t *chunk_shot,
                      const int32_t *chunk_window, const int32_t *text_spans, int32_t T, int32_t P,
                      const int32_t *seg_offsets, int32_t n_kept, const int32_t *kept,
                      int32_t *out_offsets, int32_t *out_shot, int32_t *out_window,
                      int32_t *out_spans, int32_t *out_C, int32_t *out_T, int32_t *out_ranges);
int moc_outer_workspace_bytes(int32_t N, int32_t D, int32_t P, size_t *bytes);
int moc_outer_route(int32_t N, int32_t D, int dtype, const void *x, int32_t P,
                    const int32_t *seg_offsets, const int32_t *mandatory, int32_t g, int32_t M,
                    int32_t causal, float *seg_mean, float *scores, int32_t *selected,
                    int32_t *kept, int32_t *n_kept, void *workspace, size_t workspace_bytes,
                    void *stream);
int moc_gather_rows(int32_t outer, int32_t n_src_rows, int32_t row_bytes, const void *src,
                    int32_t n_ranges, const int32_t *ranges, void *dst, void *workspace,
                    size_t workspace_bytes, void *stream);

/*
 * Stage (d) forward: o_i = softmax(q_i K_Omega^T * softmax_scale) V_Omega with
 * Omega(i) = tokens of all text chunks + the chunks of i's window + the chunks
 * listed in sel[i] (entries < 0 ignored). Forced links are not subject to the
 * causal mask. lse_i = log sum_t exp(logit_it) (natural log).
 *   sel       DEVICE in [B,H,N,topk]; may come from moc_route or from anywhere
 *             else. Omega(i) is a set: an entry that is negative or >= C, names
 *             a caption chunk or a chunk of i's own window (forced links, in
 *             Omega(i) anyway, Sec. 3.3 pre-routing mask), or repeats an earlier
 *             entry of its row is ignored.
 *   softmax_scale  finite and > 0 (1/sqrt(d) in Eq. 1 and 2), else MOC_ERR_SHAPE.
 *   topk > 0 needs C <= 16384 (MOC_ERR_SHAPE otherwise).
 *   o         DEVICE out [B,H,N,d] dtype;  lse DEVICE out [B,H,N] fp32.
 *   workspace DEVICE scratch of moc_attn_workspace_bytes(..., with_bwd) bytes.
 */
int moc_attn_workspace_bytes(const moc_meta *meta, int32_t B, int32_t H, int32_t d,
                             int32_t topk, int dtype, int with_bwd, size_t *bytes);
int moc_attn_fwd(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
                 const void *q, const void *k, const void *v, const int32_t *sel,
                 int32_t topk, float softmax_scale, void *o, float *lse,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Stage (d) backward with Omega fixed (no gradient through scores or top-k):
 *   delta_i = dO_i . o_i,  P_it = exp(logit_it - lse_i),
 *   dV_t = sum_i P_it dO_i,  dS_it = P_it (dO_i . v_t - delta_i),
 *   dQ_i = scale * sum_t dS_it k_t,  dK_t = scale * sum_i dS_it q_i.
 * o, lse are the forward's outputs; dq, dk, dv [B,H,N,d] dtype are fully
 * overwritten. workspace must have been sized with with_bwd = 1.
 * Every sum is formed in a fixed order (the routed queries of a chunk in
 * ascending query index): dq, dk and dv are bit-identical from call to call.
 *
 * moc_attn_bwd_after_fwd is moc_attn_bwd for the usual training step, where it
 * follows a moc_attn_fwd call with the same meta, B, H, sel pointer, topk,
 * workspace and stream: the per-chunk query lists that call left at the head of
 * the workspace are used again instead of being rebuilt from sel. The caller
 * promises that neither the contents of sel nor the workspace were written in
 * between (a workspace sized with with_bwd = 1 serves both calls). If the
 * library did not see such a forward call last on this workspace it rebuilds
 * the lists, i.e. behaves as moc_attn_bwd.
 */
int moc_attn_bwd(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
                 const void *q, const void *k, const void *v, const void *o, const float *lse,
                 const void *d_o, const int32_t *sel, int32_t topk, float softmax_scale,
                 void *dq, void *dk, void *dv, void *workspace, size_t workspace_bytes,
                 void *stream);
int moc_attn_bwd_after_fwd(const moc_meta *meta, int32_t B, int32_t H, int32_t d, int dtype,
                           const void *q, const void *k, const void *v, const void *o,
                           const float *lse, const void *d_o, const int32_t *sel, int32_t topk,
                           float softmax_scale, void *dq, void *dk, void *dv, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * Per-kernel timing (measurement aid, not part of the layer). While enabled,
 * every kernel launch of the library is bracketed by HIP events recorded on the
 * launch stream. moc_prof_enable(on) clears the records. moc_prof_read(-1, ...)
 * returns the number of distinct kernels recorded (>= 0); moc_prof_read(i, ...)
 * waits for the recorded events and returns kernel i's name, launch count and
 * summed duration in milliseconds. Not thread-safe against concurrent launches
 * on other streams.
 */
int moc_prof_enable(int on);
int moc_prof_read(int32_t index, char *name, size_t name_cap, int32_t *launches, float *total_ms);

/*
 * Machine probes (measurement aid, not part of the layer): the rate this GPU
 * sustains on the two resources the layer's kernels are priced against.
 *   MOC_PROBE_COPY  streams the first half of `buf` (device, 16-byte aligned,
 *                   `bytes` long) into the second half, `iters` times;
 *                   *units = bytes read + bytes written.
 *   MOC_PROBE_MFMA  runs `iters` iterations of 16 independent
 *                   v_mfma_f32_32x32x16_bf16 per wave, 8 waves on each of 256
 *                   workgroups; `buf` (>= 512 KiB) receives one float per lane;
 *                   *units = flops issued.
 * The call launches on `stream` (a hipStream_t, NULL = default), waits for the
 * work, and stores the elapsed milliseconds (HIP events around the timed
 * launches, after one untimed pass) in *ms (host). Returns MOC_OK or a
 * negative moc_status; nothing is allocated on the device.
 */
enum moc_probe_kind {
    MOC_PROBE_COPY = 0, MOC_PROBE_MFMA = 1,
    /* Do matrix and vector instructions of different waves of one SIMD overlap? 8 waves on each of
     * 256 workgroups; per iteration waves 0-3 issue 16 v_mfma_f32_32x32x16_bf16 each (kind 2),
     * waves 4-7 issue 64 fma, 16 mul and 16 exp2 each (kind 3), or both run together (kind 4); kind 5
     * puts that vector work into waves 0-3 themselves, interleaved with their matrix instructions.
     * *units = iterations; compare the durations. buf as for MOC_PROBE_MFMA. */
    MOC_PROBE_MFMA4 = 2, MOC_PROBE_VALU4 = 3, MOC_PROBE_MFMA4_VALU4 = 4, MOC_PROBE_MFMA4_VALU_SAME_WAVE = 5,
    /* Data paths inside a compute unit, two workgroups of four waves on each: every wave re-reads 16 KB
     * of LDS per iteration with ds_read_b128 (kind 6) or 8 KB with ds_read_b64_tr_b16 (kind 7), or copies
     * 16 KB per iteration from a cache-resident 64 KB at the start of `buf` into LDS, with
     * global_load_lds_dwordx4 (kind 8) or through registers (kind 9). *units = bytes moved over all
     * compute units. buf >= 1 MiB (its first 64 KB are read, the rest receives one word per lane). */
    MOC_PROBE_LDS_READ = 6, MOC_PROBE_LDS_READ_TRANSPOSED = 7, MOC_PROBE_COPY_TO_LDS_ASYNC = 8,
    MOC_PROBE_COPY_VIA_REGISTERS = 9
};
int moc_probe(int32_t kind, void *buf, size_t bytes, int32_t iters, void *stream, float *ms, double *units);

#ifdef __cplusplus
}
#endif
#endif /* MOC_H_ */
