// Host-side argument blocks and launchers shared by the translation units of libloopserve.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ls {

struct ScoreArgs {
    const void* q;            // [B,Hq,w,d]
    const void* k;            // [B,Hkv,n,d]
    const int64_t* q_pos;     // [w] or null
    int64_t n;
    int w, G, Hq, Hkv, B, BH, nkb;
    float scale_log2e;
    float* part;              // [BH*w][nkb][2]   per key block max / sum
    float* rowstat;           // [BH*w][2]        row max, 1 / row sum
    float* spart;             // [2][BH][n][2]    diagonal partial sum / max by key-block parity
    float *vert, *slash, *vmax, *smax, *total;
    float* gscore;            // [B*Hkv][n]       group-summed column sums (retention score)
    float* a_win;             // [BH][w][n]       the window matrix itself (mode 3)
};

constexpr int SELECT_HEAD_LINES = 1024;   // lines at the front of each sorted list whose weight and maximum are stored in order

struct SelectArgs {
    int64_t n, n_hat;
    int BH;
    float alpha;
    const float *vert, *slash, *vmax, *smax, *total;
    uint32_t* skey0;          // [2][BH][n] sorted keys of each segment
    int32_t *sidx0, *sidx1;   // [2][BH][n] line indices of each sorted segment (sidx0) and of the merged order (sidx1)
    float *head_w, *head_m;   // [2][BH][SELECT_HEAD_LINES] weight and largest entry of the first lines of each sorted list
    int32_t *v_idx, *v_cnt, *s_idx, *s_cnt;
    int cap_v, cap_s;
    float* accounted;         // may be null
    int32_t* status;          // device status word of the context (bits LS_STAT_*), OR-ed into
    int spin_limit;           // bound of every wait between the waves of walk_kernel
    // exact-overlap variant (run_select_exact) only
    const float* a_win;       // [BH][w][n] window matrix
    const int64_t* q_pos;     // [w] positions of the scored rows, or null (the last w)
    int w;
};

constexpr int64_t TOPB_MAX_LEN = 262144;   // longest score row run_topb takes

struct TopbArgs {
    const float* score;       // [BK][len]
    int64_t len;              // <= TOPB_MAX_LEN
    int budget;
    int32_t *keep_idx, *keep_cnt;
    // filled in by run_topb from its scratch block
    int chunks;
    uint32_t *hist, *state, *cnt;
};

struct PlanArgs {
    int64_t n;
    int words, tab_len;
    const int32_t *v_idx, *v_cnt, *s_idx, *s_cnt;
    int cap_v, cap_s;
    uint32_t* obits;          // [BH][words]
    uint8_t* tab;             // [BH][tab_len]
    uint8_t* hflag;           // [BH]
    uint32_t* cost;           // [BH] estimated tiles per row block (for the work queues)
    uint16_t* pref;           // [BH][tab_len + 1] prefix counts of table entries with a selected diagonal
    int32_t* status;          // device status word of the context (bits LS_STAT_*), OR-ed into
};

// Work queues of the sparse attention kernel: one list of (head, row block) items per XCD.
struct SchedArgs {
    int BH, G, Hq, Hkv, nqb;
    const uint32_t* cost;     // [BH]
    const uint16_t* pref;     // [BH][tab_len + 1]
    const int32_t* v_cnt;     // [BH]
    const uint8_t* hflag;     // [BH]
    int tab_len, cap_v;
    int64_t n, pos0;
    uint32_t* queue;          // [8][BH * nqb] items: bh << 16 | qb
    int32_t* qlen;            // [8]
    int32_t* qhead;           // [8] next item to hand out
};

struct PrefillArgs {
    const void *q, *k, *v;
    void* out;
    float* lse;
    int64_t n, n_hat, pos0;
    int Hq, Hkv, G, BH, nqb, words, tab_len;
    float scale_log2e;
    const uint32_t* obits;
    const uint8_t *tab, *hflag;
    const int32_t *v_idx, *v_cnt;
    int cap_v;
    const uint32_t* queue;    // work queues built by sched_kernel
    const int32_t* qlen;
    int32_t* qhead;
    int qcap;                 // entries per queue
};

struct DecodeArgs {
    const void *q;            // [B][Hq][d]
    const void *kc, *vc;      // [B][Hkv][cap][d] retained entries (first cnt rows valid)
    const void *kt, *vt;      // [B][Hkv][T][d] tokens since the retention
    const int32_t* cnt;       // [B][Hkv] or NULL (all cap rows)
    void* out;                // [B][Hq][d]
    float* lse;               // [B][Hq] or NULL
    float* part;              // [B*Hkv][nsplit][G][d + 2] per-split output, reference, normaliser
    int B, Hq, Hkv, G, cap, T, nsplit, chunk;
    float scale_log2e;
};

// status bits (mirrors of LS_STAT_* in loopserve.h)
constexpr int STAT_WALK_TIMEOUT = 1, STAT_S_TRUNCATED = 2, STAT_V_TRUNCATED = 4, STAT_S_RANGE = 8, STAT_V_INVALID = 16,
              STAT_MERGE_RANGE = 32;
constexpr int WALK_SPIN_DEFAULT = 1 << 22;   // never reached in practice (about a second of polling)

// Lets a kernel use all of a compute unit's LDS (160 KB, less what the kernel declares statically) as
// dynamic LDS; the launches then only have to name the size they need.
template <typename K>
inline hipError_t allow_full_lds(K kernel) {
    hipFuncAttributes fa;
    hipError_t e = hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kernel));
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                               160 * 1024 - (int)fa.sharedSizeBytes);
}

// Once per device, with that device current: lets every kernel that asks for dynamic LDS use the whole 160 KB.
hipError_t init_score_kernels();
hipError_t init_select_kernels();
hipError_t init_prefill_kernels();
hipError_t init_decode_kernels();

hipError_t run_score(const ScoreArgs& a, int dtype, int d, int mode, hipStream_t st);
hipError_t run_decode(const DecodeArgs& a, int d, hipStream_t st);
size_t decode_smem_bytes(int d, int G);
size_t score_lines_smem(int w, int dtype, int d, int mode);
// Union of two selections per head (the accumulated line set of Alg. 1): lists a and b in, ascending unique list out.
struct MergeArgs {
    int64_t n;
    int BH;
    const int32_t *idx_a[2], *cnt_a[2], *idx_b[2], *cnt_b[2];   // [0] diagonals, [1] columns
    int cap_a[2], cap_b[2];
    int32_t *idx[2], *cnt[2];
    int cap[2];
    int32_t* status;
};
hipError_t run_merge_lines(const MergeArgs& a, hipStream_t st);
hipError_t run_select(const SelectArgs& a, hipStream_t st);
hipError_t run_select_exact(const SelectArgs& a, hipStream_t st);   // a_win, q_pos, w set; vmax / smax unused
hipError_t run_topb(const TopbArgs& a, int BK, uint32_t* scratch, hipStream_t st);   // scratch: topb_scratch_words(BK, len) words
size_t topb_scratch_words(int BK, int64_t len);
hipError_t run_gather_rows(const void* src, void* dst, const int32_t* keep_idx, const int32_t* keep_cnt,
                           int BK, int64_t len, int budget, int row_bytes, hipStream_t st);
hipError_t launch_plan(const PlanArgs& a, int BH, hipStream_t st);
hipError_t launch_sched(const SchedArgs& a, hipStream_t st);
// ev0 / ev1 (both or neither): events that receive the start and stop time of the attention kernel's own dispatch
hipError_t launch_prefill(const PrefillArgs& a, int dtype, int d, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
size_t prefill_smem_bytes(int dtype, int d, int words, int tab_len);
int prefill_block_rows();

}  // namespace ls
