/*
 * loopserve.h -- C ABI of libloopserve: the per-layer hot path of LoopServe's online-sparsified
 * prefill attention and its decode-time KV retention scorer (arxiv 2507.13681), for AMD MI355X
 * (gfx950).  Plain C, no exceptions cross this boundary.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers on the context's GPU, 16-byte aligned, row-major and
 *     contiguous in the stated shape.  Only ls_shape and scalars are host data.
 *   - The caller owns every tensor.  The library owns only the context and its workspace, which is
 *     allocated once in ls_create; no entry point below allocates or frees device memory.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t, NULL = the default stream) and contain
 *     no host synchronisation; outputs are valid once the stream reaches the end of the call.
 *     Counts (v_cnt, s_cnt, keep_cnt) stay on the device, so score -> select -> prefill chain without
 *     a host round trip.  Calls that share a context must be issued on one stream at a time (they
 *     share the workspace).
 *   - Return value: LS_OK or a negative ls_status; ls_last_error(ctx) then describes the failure.
 *     Argument errors are detected on the host before anything is launched.
 *   - dtype is the storage type of q / k / v / out (bf16 or fp32); tile products accumulate in fp32
 *     and every line weight, count and index output is fp32 / int32 regardless of dtype.
 *   - Query head h reads KV head h / (Hq / Hkv)  (grouped-query attention).
 *   - Positions: the context has n keys at positions 0..n-1; the newest turn is the last n_hat of
 *     them; new-turn row a sits at absolute position n - n_hat + a and sees keys <= that position.
 */
#ifndef LOOPSERVE_H
#define LOOPSERVE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ls_ctx ls_ctx;

typedef enum {
    LS_OK = 0,
    LS_EINVAL = -1,      /* null or misaligned pointer, bad enum */
    LS_ESHAPE = -2,      /* unsupported or inconsistent shape */
    LS_EALPHA = -3,      /* alpha outside [0, 1] */
    LS_EWORKSPACE = -4,  /* context workspace too small for this call */
    LS_EHIP = -5         /* a HIP runtime call failed */
} ls_status;

typedef enum { LS_BF16 = 0, LS_F32 = 1 } ls_dtype;

/* Limits: d in {64, 128}; w <= 256; n <= LS_MAX_N for ls_select / ls_sparse_prefill. */
#define LS_MAX_N 262144
#define LS_MAX_W 256

typedef struct {
    int32_t B;       /* batch */
    int32_t Hq;      /* query heads */
    int32_t Hkv;     /* KV heads, divides Hq */
    int32_t d;       /* head dimension */
    int64_t n;       /* keys in the context (cache length for ls_kv_compress) */
    int64_t n_hat;   /* rows of the newest turn, 1 <= n_hat <= n (ignored by ls_kv_compress) */
    int32_t w;       /* scoring rows: window size (n_obs for ls_kv_compress) */
    int32_t dtype;   /* ls_dtype */
    float scale;     /* logit scale; <= 0 means 1/sqrt(d) */
} ls_shape;

/* Bytes of workspace that every call on `shape` (and ls_kv_compress with `budget`) fits in.
 * Host-only, no GPU needed.  Returns 0 for an invalid shape. */
size_t ls_workspace_bytes(const ls_shape* shape, int32_t budget);

/* Creates a context on GPU `device` with a workspace of `workspace_bytes` (device memory, allocated
 * here, freed by ls_destroy).  The context can serve any shape whose ls_workspace_bytes fits. */
int ls_create(ls_ctx** out, int device, size_t workspace_bytes);
void ls_destroy(ls_ctx* ctx);
/* Message of the last failing call on this context (never NULL; not thread-safe); with ctx == NULL, of the
 * last failing call that takes no context (ls_kv_compress_static). */
const char* ls_last_error(const ls_ctx* ctx);

/*
 * ls_score -- Alg. 2, steps "A = Softmax(Q~ K^T / sqrt(d_k))", SlashSum, VerticalSum (Appendix,
 * Algorithm "Adaptive Prefilling Sparsification"), with the line definitions of Sec. 3.1 (Obs. 1):
 * a vertical line is a key column, a slash line is a diagonal.
 *
 *   q_win  [B,Hq,w,d]   queries of the scoring rows
 *   q_pos  [w] int64    their absolute positions (each clipped to [0, n-1]), device memory; NULL = the last w
 *                       positions n-w .. n-1 (the newest query window)
 *   k      [B,Hkv,n,d]
 * Outputs (fp32):
 *   vert   [B,Hq,n]  vert[b]  = sum_t A[t][b]              (column b)
 *   slash  [B,Hq,n]  slash[o] = sum_t A[t][p_t - o]        (diagonal o = query pos - key pos)
 *   vmax, smax [B,Hq,n]  the largest single entry of each line (the w^max of Alg. 2)
 *   total  [B,Hq]    sum of all entries of A (about w)
 * The softmax is causal (row t sees keys <= p_t).  With q_pos == NULL and w <= 128 all sums are
 * formed in a fixed order (bit-reproducible); otherwise the diagonal sums use fp32 atomics.
 */
int ls_score(ls_ctx* ctx, const ls_shape* shape, const void* q_win, const int64_t* q_pos, const void* k,
             float* vert, float* slash, float* vmax, float* smax, float* total, void* hip_stream);

/*
 * ls_select -- Alg. 2 from Desc_Sort to the end of the while-loop: both line lists are sorted by
 * weight (descending; ties: smaller index first) and the greedy loop takes list heads until the
 * accounted weight reaches alpha * total.  Gain of a slash is w_s - ol_v, of a vertical w_v - ol_s,
 * where ol_* sums w^max of the lines taken from the other list; cost is max(1, length - #taken from
 * the other list) with length min(n_hat, n - index); the slash is taken when gain_s * cost_v >=
 * gain_v * cost_s; gains are not clamped; an empty list defers to the other.  All in binary32.
 *
 *   vert, slash, vmax, smax [B,Hq,n], total [B,Hq]   as produced by ls_score
 * Outputs:
 *   v_idx [B,Hq,cap_v] int32  selected columns, ascending;   v_cnt [B,Hq] int32
 *   s_idx [B,Hq,cap_s] int32  selected diagonals, ascending; s_cnt [B,Hq] int32
 *   accounted [B,Hq] fp32 or NULL: the loop's final sum.
 * A count larger than its capacity means the list was truncated to the smallest `cap` indices
 * (LS_STAT_S_TRUNCATED / LS_STAT_V_TRUNCATED in the status word).
 * With accounted == NULL the loop stops as soon as the result is decided (when no remaining line
 * has a positive gain every line ends up selected); with accounted != NULL it runs to the end.
 * shape->w and dtype are ignored.  n <= LS_MAX_N.
 */
int ls_select(ls_ctx* ctx, const ls_shape* shape, float alpha,
              const float* vert, const float* slash, const float* vmax, const float* smax, const float* total,
              int32_t* v_idx, int32_t* v_cnt, int32_t cap_v,
              int32_t* s_idx, int32_t* s_cnt, int32_t cap_s,
              float* accounted, void* hip_stream);

/*
 * ls_score_window / ls_select_exact -- Alg. 2 with the marginal contribution of a line taken exactly.
 * Sec. 5.1 describes the quantities the loop compares as the marginal contributions of the two list
 * heads; the listing bounds the part of a candidate that is already covered by the sum of w^max of the
 * lines taken from the other list, which is what ls_select computes.  Here that part is added up cell by
 * cell (a diagonal o and a column b share the cell of the scored row at position b + o, if there is one),
 * so gains are never negative, the accounted sum is the weight of the union of the selected lines on the
 * scored rows, and selections that mix columns and diagonals survive.  Opt-in: it needs the window
 * matrix itself (w * n floats per head) and walks the lists one pick at a time.
 *
 * ls_score_window: the softmax step of Alg. 2 with the matrix kept.
 *   q_win, q_pos, k as for ls_score;  a_win [B,Hq,w,n] fp32: A[t][b] for keys b <= p_t, 0 beyond.
 * ls_select_exact: Desc_Sort and the loop.
 *   a_win as above; q_pos [w] int64 device memory or NULL (the last w positions), the same as was scored;
 *   vert, slash [B,Hq,n], total [B,Hq] as produced by ls_score (the lists are ordered by these weights);
 *   outputs, capacities, accounted, status bits and limits as for ls_select (shape->w is used here).
 */
int ls_score_window(ls_ctx* ctx, const ls_shape* shape, const void* q_win, const int64_t* q_pos, const void* k,
                    float* a_win, void* hip_stream);
int ls_select_exact(ls_ctx* ctx, const ls_shape* shape, float alpha, const float* a_win, const int64_t* q_pos,
                    const float* vert, const float* slash, const float* total,
                    int32_t* v_idx, int32_t* v_cnt, int32_t cap_v,
                    int32_t* s_idx, int32_t* s_cnt, int32_t cap_s,
                    float* accounted, void* hip_stream);

/*
 * ls_merge_lines -- the accumulated line set of Alg. 1 (L: the selections of every turn so far), which Sec. 5,
 * Step 1 says can be reused in later dialogue turns.  A column index is a key position and a diagonal index an
 * offset (query position - key position); neither changes when the context grows, so a selection made in an
 * earlier turn is carried into a later one as a union of index sets.  Per (batch, head): v_idx = union of the
 * column lists a and b, s_idx = union of the diagonal lists, each ascending and free of duplicates, with their
 * counts (a count above its capacity: truncated to the smallest indices, LS_STAT_S_TRUNCATED / V_TRUNCATED).
 *   shape: B, Hq and n (the context the result refers to) are used; entries outside [0, n) are dropped
 *          (LS_STAT_MERGE_RANGE).  min(cnt, cap) entries of each input list are read; inputs need not be sorted.
 *   The output lists are valid inputs of ls_sparse_prefill and of a later ls_merge_lines; an output may not
 *   alias an input.
 */
int ls_merge_lines(ls_ctx* ctx, const ls_shape* shape,
                   const int32_t* v_idx_a, const int32_t* v_cnt_a, int32_t cap_va,
                   const int32_t* s_idx_a, const int32_t* s_cnt_a, int32_t cap_sa,
                   const int32_t* v_idx_b, const int32_t* v_cnt_b, int32_t cap_vb,
                   const int32_t* s_idx_b, const int32_t* s_cnt_b, int32_t cap_sb,
                   int32_t* v_idx, int32_t* v_cnt, int32_t cap_v,
                   int32_t* s_idx, int32_t* s_cnt, int32_t cap_s, void* hip_stream);

/*
 * ls_sparse_prefill -- masked attention Softmax(QK^T/sqrt(d_k) - c(1-M)) V of Sec. 2.2 for the
 * rows of the newest turn (Sec. 5, Step 1), with M[a][b] = 1 iff b <= p_a and (b in v_idx or
 * p_a - b in s_idx), masked entries weighing exactly zero, each allowed cell counted once.
 *
 *   q [B,Hq,n_hat,d]; k, v [B,Hkv,n,d]; index lists as written by ls_select (device memory;
 *   min(cnt, cap) entries are read).  v_idx must be strictly ascending with entries in [0, n); a head
 *   whose list is not is computed without its columns and LS_STAT_V_INVALID is set.  s_idx may be in
 *   any order; entries outside [0, n) are ignored (LS_STAT_S_RANGE).
 * Outputs:
 *   out [B,Hq,n_hat,d] in dtype; a row with no allowed cell is all zeros
 *   lse [B,Hq,n_hat] fp32 or NULL: natural log of the softmax denominator (-inf for an empty row)
 * n <= LS_MAX_N.  shape->w is ignored.
 */
int ls_sparse_prefill(ls_ctx* ctx, const ls_shape* shape, const void* q, const void* k, const void* v,
                      const int32_t* v_idx, const int32_t* v_cnt, int32_t cap_v,
                      const int32_t* s_idx, const int32_t* s_cnt, int32_t cap_s,
                      void* out, float* lse, void* hip_stream);

/*
 * ls_kv_compress -- Alg. 3, the re-selection step (Sec. 5.2): for each KV head keep the `budget`
 * cache entries that receive the most attention from the last n_obs = shape->w query rows, summed
 * over the Hq/Hkv query heads of the group; ties go to the smaller index.
 *
 *   q_obs [B,Hq,n_obs,d]  queries at positions len-n_obs .. len-1 (len = shape->n)
 *   k [B,Hkv,len,d]; v [B,Hkv,len,d] or NULL when v_out is NULL
 * Outputs:
 *   keep_idx [B,Hkv,budget] int32 ascending; keep_cnt [B,Hkv] = min(budget, len)
 *   k_out, v_out [B,Hkv,budget,d] compacted copies of the kept rows, or NULL
 * len <= LS_MAX_N (LS_ESHAPE otherwise, before anything is launched).
 */
int ls_kv_compress(ls_ctx* ctx, const ls_shape* shape, int32_t budget,
                   const void* q_obs, const void* k, const void* v,
                   int32_t* keep_idx, int32_t* keep_cnt, void* k_out, void* v_out, void* hip_stream);

/*
 * ls_kv_compress_static -- ls_kv_compress for callers that cannot allocate device memory or hold a
 * context: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs, limits and results as ls_kv_compress on GPU `device`, but no ls_ctx: its
 * intermediate results (softmax partials of the observation rows, the per-group score, the radix
 * histograms and counts of the top-B selection) live in a fixed block of device memory that is part of
 * the library image, ls_static_scratch_bytes() = LS_STATIC_SCRATCH_BYTES bytes on every GPU the
 * library is used on, held until the process ends.  The call allocates and frees nothing (no hipMalloc,
 * hipFree or allocating library routine) and clears what it needs with kernels of its own.
 * A shape that needs more scratch than that (its ls_workspace_bytes says how much) is refused with
 * LS_EWORKSPACE before anything is launched; ls_last_error(NULL) describes the failure.
 * All calls on one GPU share that GPU's block: calls that overlap in time on one GPU (different streams
 * or threads) race and must be ordered by the caller.
 */
#define LS_STATIC_SCRATCH_BYTES (16u << 20)
size_t ls_static_scratch_bytes(void);
int ls_kv_compress_static(int device, const ls_shape* shape, int32_t budget,
                          const void* q_obs, const void* k, const void* v,
                          int32_t* keep_idx, int32_t* keep_cnt, void* k_out, void* v_out, void* hip_stream);

/*
 * ls_decode_attend -- Alg. 3, the Decoding step (Sec. 5.2) seen from one attention layer: the newest
 * token's query attends over the entries its KV head retained at the last ls_kv_compress, followed by
 * the tokens generated since (Alg. 3 adds every generated token to the retained set); all are visible:
 *     out = softmax(scale * q [K_c; K_t]^T) [V_c; V_t].
 *
 *   shape: B, Hq, Hkv, d, dtype (LS_BF16 only), scale are used; n, n_hat, w are ignored.  Hq/Hkv <= 32.
 *   q [B,Hq,d]
 *   k_c, v_c [B,Hkv,cap,d]  retained rows (e.g. k_out / v_out of ls_kv_compress), cap >= 1
 *   cnt [B,Hkv] int32 device memory: the first cnt rows of each [cap,d] block are valid (values are
 *        clamped to [0, cap]; e.g. keep_cnt of ls_kv_compress), or NULL for all cap rows
 *   k_t, v_t [B,Hkv,T,d]    tokens since the retention, in order; T >= 0, NULL allowed when T == 0
 * Outputs:
 *   out [B,Hq,d] in dtype; all zeros when a KV head has no key at all (cnt == 0 and T == 0)
 *   lse [B,Hq] fp32 or NULL: natural log of the softmax denominator (-inf when there is no key)
 * The caller owns every tensor; the call is asynchronous on hip_stream and uses the context's
 * workspace (ls_decode_workspace_bytes).  Returns LS_ESHAPE for fp32 or Hq/Hkv > 32.
 */
int ls_decode_attend(ls_ctx* ctx, const ls_shape* shape, int32_t cap, int32_t T,
                     const void* q, const void* k_c, const void* v_c, const int32_t* cnt,
                     const void* k_t, const void* v_t, void* out, float* lse, void* hip_stream);
/* Host-only: workspace bytes ls_decode_attend needs for these sizes (0 on a bad shape). */
size_t ls_decode_workspace_bytes(const ls_shape* shape, int32_t cap, int32_t T);

/*
 * Timing of the sparse attention kernel itself (the dominant kernel of ls_sparse_prefill), for
 * roofline reports.  After ls_profile_enable(ctx, 1) every ls_sparse_prefill call attaches a pair
 * of HIP events to that one kernel launch on the call's stream: they receive the start and stop
 * time of the dispatch itself, and no marker is put into the stream (this creates two events per
 * call, so leave it off in allocation-free loops).  ls_profile_prefill_kernel_ms waits for the recorded
 * events and returns the mean kernel duration in milliseconds and the number of launches seen since
 * profiling was enabled.  ls_profile_enable(ctx, 0) stops recording and drops the events.
 */
int ls_profile_enable(ls_ctx* ctx, int on);
int ls_profile_prefill_kernel_ms(ls_ctx* ctx, double* mean_ms, int32_t* launches);

/*
 * Device status word.  Conditions that a kernel can only see while it runs are reported without a
 * host round trip: the kernel ORs a bit into a word in device memory that belongs to the context, the
 * call still returns LS_OK, and the outputs are as described for each bit.  ls_poll_status waits for
 * everything queued on `hip_stream`, writes the word to *host_out (host memory) and clears it; it is
 * the one call here that synchronises with the host.  (Serves callers of the four entry points above;
 * no passage of the paper defines it.)
 */
#define LS_STAT_WALK_TIMEOUT 1  /* ls_select: a bounded wait inside the greedy loop gave up; the head concerned reports
                                   every line selected (v_cnt = s_cnt = n), which still meets the coverage target */
#define LS_STAT_S_TRUNCATED  2  /* ls_select: s_cnt > cap_s for some head (s_idx holds the smallest cap_s indices) */
#define LS_STAT_V_TRUNCATED  4  /* ls_select: v_cnt > cap_v for some head */
#define LS_STAT_S_RANGE      8  /* ls_sparse_prefill: s_idx entries outside [0, n) were ignored */
#define LS_STAT_V_INVALID   16  /* ls_sparse_prefill: a head's v_idx was not strictly ascending inside [0, n); that
                                   head's columns were ignored (its diagonals still apply) */
#define LS_STAT_MERGE_RANGE 32  /* ls_merge_lines: input entries outside [0, n) were dropped */
int ls_poll_status(ls_ctx* ctx, int32_t* host_out, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* LOOPSERVE_H */
