// C-ABI entry points of libloopserve: argument checks, workspace carving, kernel dispatch.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <utility>
#include <vector>

#include <mutex>

#include "../../include/loopserve.h"
#include "../../include/loopserve_test_hooks.h"
#include "ls_internal.h"

static_assert(ls::TOPB_MAX_LEN == LS_MAX_N, "ls_kv_compress documents LS_MAX_N as its longest cache");
static_assert(ls::STAT_WALK_TIMEOUT == LS_STAT_WALK_TIMEOUT && ls::STAT_S_TRUNCATED == LS_STAT_S_TRUNCATED &&
              ls::STAT_V_TRUNCATED == LS_STAT_V_TRUNCATED && ls::STAT_S_RANGE == LS_STAT_S_RANGE &&
              ls::STAT_V_INVALID == LS_STAT_V_INVALID && ls::STAT_MERGE_RANGE == LS_STAT_MERGE_RANGE,
              "status bits of the kernels and of the header");

struct ls_ctx {
    int device;
    unsigned char* ws;
    size_t ws_bytes;
    int32_t* status;          // device status word (bits LS_STAT_*), OR-ed into by kernels, read and cleared by ls_poll_status
    int walk_spin_limit;      // bound of the waits inside walk_kernel (test hook)
    char err[256];
    // optional timing of the sparse attention kernel (ls_profile_*): event pairs on the call's stream
    bool profile;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> events;
};

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

int fail(ls_ctx* c, int code, const char* fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Scratch of the entry point that allocates nothing (ls_kv_compress_static): a fixed block of device memory
// that is part of the loaded code object.  Every GPU the library runs on holds its own copy at its own
// address until the process ends; host code reaches it only through the address that hipGetSymbolAddress
// returns on that device (scratch_on[device]), never through the array's name.
constexpr size_t STATIC_SCRATCH_BYTES = LS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
std::vector<unsigned char*> scratch_on;      // per device, filled by init_device_once
char static_err[256] = "";                   // last error of a call that has no context

// Kernel attributes and the scratch address are per device: set once for each device the library is used on,
// with that device current.
hipError_t init_device_once(int device) {
    static std::mutex mu;
    static std::vector<char> done;
    std::lock_guard<std::mutex> lock(mu);
    if ((int)done.size() <= device) { done.resize(device + 1, 0); scratch_on.resize(device + 1, nullptr); }
    if (done[device]) return hipSuccess;
    hipError_t e;
    unsigned char* sp = nullptr;
    if ((e = hipGetSymbolAddress(reinterpret_cast<void**>(&sp), HIP_SYMBOL(scratch))) != hipSuccess) return e;
    scratch_on[device] = sp;
    if ((e = ls::init_score_kernels()) != hipSuccess) return e;
    if ((e = ls::init_select_kernels()) != hipSuccess) return e;
    if ((e = ls::init_prefill_kernels()) != hipSuccess) return e;
    if ((e = ls::init_decode_kernels()) != hipSuccess) return e;
    done[device] = 1;
    return hipSuccess;
}

struct Bump {
    unsigned char* base; size_t cap, off;
    template <typename T> T* take(size_t count) {
        const size_t bytes = up(count * sizeof(T));
        if (off + bytes > cap) { off = cap + 1; return nullptr; }
        T* p = reinterpret_cast<T*>(base + off);
        off += bytes;
        return p;
    }
    bool ok() const { return off <= cap; }
};

// common shape checks; `what` selects which fields matter
const char* check_shape(const ls_shape* s, bool need_nhat, bool need_w, bool cap_n) {
    if (!s) return "shape is NULL";
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0) return "B, Hq, Hkv must be positive";
    if (s->Hq % s->Hkv) return "Hq must be a multiple of Hkv";
    if (s->d != 64 && s->d != 128) return "d must be 64 or 128";
    if (s->dtype != LS_BF16 && s->dtype != LS_F32) return "dtype must be LS_BF16 or LS_F32";
    if (s->n <= 0 || s->n > 2147483000LL) return "n out of range";
    if (cap_n && s->n > LS_MAX_N) return "n exceeds LS_MAX_N";
    if (need_nhat && (s->n_hat <= 0 || s->n_hat > s->n)) return "need 1 <= n_hat <= n";
    if (need_w && (s->w <= 0 || s->w > LS_MAX_W || s->w > s->n)) return "need 1 <= w <= min(n, LS_MAX_W)";
    if ((int64_t)s->B * s->Hq > 65535) return "B * Hq too large";
    return nullptr;
}

inline int nkb_of(int64_t n) { return (int)((n + 127) / 128); }
inline float scale_log2e(const ls_shape* s) {
    const float sc = s->scale > 0.f ? s->scale : 1.0f / sqrtf((float)s->d);
    return sc * 1.44269504088896340736f;
}

// per key block max / sum of every scored row; later the 8 partial totals of every head
inline size_t part_floats(const ls_shape* s) {
    const size_t BH = (size_t)s->B * s->Hq;
    const size_t a = BH * s->w * nkb_of(s->n) * 2, b = BH * 8;
    return a > b ? a : b;
}
size_t ws_score(const ls_shape* s, bool lines) {
    const size_t BH = (size_t)s->B * s->Hq;
    size_t b = up(part_floats(s) * 4) + up(BH * s->w * 2 * 4);
    if (lines) b += up(2 * BH * (size_t)s->n * 2 * 4);
    return b;
}
size_t ws_select(const ls_shape* s) {
    const size_t BH = (size_t)s->B * s->Hq;
    return 3 * up(2 * BH * (size_t)s->n * 4) + 2 * up(2 * BH * ls::SELECT_HEAD_LINES * 4);
}
inline int words_of(int64_t n) { return (int)((n + 31) / 32) + 8; }
inline int tab_len_of(int64_t n) { return (int)(n / 64) + 4; }
size_t ws_prefill(const ls_shape* s) {
    const size_t BH = (size_t)s->B * s->Hq;
    const size_t items = BH * (size_t)(s->n / 128 + 2);          // (head, row block) work items, upper bound
    return up(BH * (size_t)(words_of(s->n) + 1) * 4) + up(BH * (size_t)tab_len_of(s->n)) + up(BH) + up(BH * 4) + up(BH * (size_t)(tab_len_of(s->n) + 1) * 2) +
           up(8 * items * 4) + 2 * up(8 * 4);
}
size_t ws_compress(const ls_shape* s) {
    return ws_score(s, false) + up((size_t)s->B * s->Hkv * (size_t)s->n * 4) +
           up(ls::topb_scratch_words(s->B * s->Hkv, s->n) * 4);
}

}  // namespace

extern "C" {

size_t ls_workspace_bytes(const ls_shape* s, int32_t budget) {
    (void)budget;
    if (check_shape(s, false, false, false)) return 0;
    ls_shape t = *s;
    if (t.w <= 0) t.w = 1;
    size_t m = ws_score(&t, true);
    if (ws_select(&t) > m) m = ws_select(&t);
    if (ws_prefill(&t) > m) m = ws_prefill(&t);
    if (ws_compress(&t) > m) m = ws_compress(&t);
    return m + ALIGN;
}

int ls_create(ls_ctx** out, int device, size_t workspace_bytes) {
    if (!out) return LS_EINVAL;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return LS_EHIP;
    if (hipSetDevice(device) != hipSuccess) return LS_EHIP;
    ls_ctx* c = new (std::nothrow) ls_ctx();
    if (!c) return LS_EINVAL;
    c->device = device; c->ws = nullptr; c->ws_bytes = workspace_bytes; c->err[0] = 0; c->profile = false;
    c->status = nullptr; c->walk_spin_limit = ls::WALK_SPIN_DEFAULT;
    if (init_device_once(device) != hipSuccess) { delete c; return LS_EHIP; }
    {
        void* p = nullptr;
        if (hipMalloc(&p, ALIGN) != hipSuccess || hipMemset(p, 0, ALIGN) != hipSuccess) { if (p) (void)hipFree(p); delete c; return LS_EWORKSPACE; }
        c->status = static_cast<int32_t*>(p);
    }
    if (workspace_bytes) {
        void* p = nullptr;
        if (hipMalloc(&p, workspace_bytes) != hipSuccess) { (void)hipFree(c->status); delete c; return LS_EWORKSPACE; }
        c->ws = static_cast<unsigned char*>(p);
    }
    *out = c;
    return LS_OK;
}

void ls_destroy(ls_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    for (auto& e : c->events) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
    if (c->ws) (void)hipFree(c->ws);
    if (c->status) (void)hipFree(c->status);
    delete c;
}

const char* ls_last_error(const ls_ctx* c) { return c ? c->err : static_err; }

int ls_score(ls_ctx* c, const ls_shape* s, const void* q_win, const int64_t* q_pos, const void* k,
             float* vert, float* slash, float* vmax, float* smax, float* total, void* stream) {
    if (!c) return LS_EINVAL;
    if (const char* m = check_shape(s, false, true, false)) return fail(c, LS_ESHAPE, "ls_score: %s", m);
    if (!q_win || !k || !vert || !slash || !vmax || !smax || !total) return fail(c, LS_EINVAL, "ls_score: NULL tensor");
    if (!aligned16(q_win) || !aligned16(k) || !aligned16(vert) || !aligned16(slash) || !aligned16(vmax) ||
        !aligned16(smax) || (q_pos && (reinterpret_cast<uintptr_t>(q_pos) & 7u)))
        return fail(c, LS_EINVAL, "ls_score: misaligned tensor");
    ls::ScoreArgs a{};
    a.q = q_win; a.k = k; a.q_pos = q_pos; a.n = s->n; a.w = s->w; a.G = s->Hq / s->Hkv; a.Hq = s->Hq;
    a.Hkv = s->Hkv; a.B = s->B; a.BH = s->B * s->Hq; a.nkb = nkb_of(s->n); a.scale_log2e = scale_log2e(s);
    Bump bp{c->ws, c->ws_bytes, 0};
    a.part = bp.take<float>(part_floats(s));
    a.rowstat = bp.take<float>((size_t)a.BH * a.w * 2);
    a.spart = bp.take<float>(2 * (size_t)a.BH * (size_t)a.n * 2);
    if (!bp.ok()) return fail(c, LS_EWORKSPACE, "ls_score: workspace of %zu bytes is too small", c->ws_bytes);
    a.vert = vert; a.slash = slash; a.vmax = vmax; a.smax = smax; a.total = total; a.gscore = nullptr;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_score: hipSetDevice failed");
    const int mode = (q_pos == nullptr && s->w <= 128) ? 0 : 1;
    if (ls::score_lines_smem(s->w, s->dtype, s->d, mode) > 160 * 1024) return fail(c, LS_ESHAPE, "ls_score: w too large for LDS");
    const hipError_t e = ls::run_score(a, s->dtype, s->d, mode, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_score: %s", hipGetErrorString(e));
    return LS_OK;
}

int ls_score_window(ls_ctx* c, const ls_shape* s, const void* q_win, const int64_t* q_pos, const void* k,
                    float* a_win, void* stream) {
    if (!c) return LS_EINVAL;
    if (const char* m = check_shape(s, false, true, false)) return fail(c, LS_ESHAPE, "ls_score_window: %s", m);
    if (!q_win || !k || !a_win) return fail(c, LS_EINVAL, "ls_score_window: NULL tensor");
    if (!aligned16(q_win) || !aligned16(k) || !aligned16(a_win) || (q_pos && (reinterpret_cast<uintptr_t>(q_pos) & 7u)))
        return fail(c, LS_EINVAL, "ls_score_window: misaligned tensor");
    ls::ScoreArgs a{};
    a.q = q_win; a.k = k; a.q_pos = q_pos; a.n = s->n; a.w = s->w; a.G = s->Hq / s->Hkv; a.Hq = s->Hq;
    a.Hkv = s->Hkv; a.B = s->B; a.BH = s->B * s->Hq; a.nkb = nkb_of(s->n); a.scale_log2e = scale_log2e(s);
    Bump bp{c->ws, c->ws_bytes, 0};
    a.part = bp.take<float>(part_floats(s));
    a.rowstat = bp.take<float>((size_t)a.BH * a.w * 2);
    if (!bp.ok()) return fail(c, LS_EWORKSPACE, "ls_score_window: workspace of %zu bytes is too small", c->ws_bytes);
    a.a_win = a_win;
    if (ls::score_lines_smem(s->w, s->dtype, s->d, 3) > 160 * 1024) return fail(c, LS_ESHAPE, "ls_score_window: w too large for LDS");
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_score_window: hipSetDevice failed");
    const hipError_t e = ls::run_score(a, s->dtype, s->d, 3, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_score_window: %s", hipGetErrorString(e));
    return LS_OK;
}

int ls_select_exact(ls_ctx* c, const ls_shape* s, float alpha, const float* a_win, const int64_t* q_pos,
                    const float* vert, const float* slash, const float* total,
                    int32_t* v_idx, int32_t* v_cnt, int32_t cap_v, int32_t* s_idx, int32_t* s_cnt, int32_t cap_s,
                    float* accounted, void* stream) {
    if (!c) return LS_EINVAL;
    if (const char* m = check_shape(s, true, true, true)) return fail(c, LS_ESHAPE, "ls_select_exact: %s", m);
    if (!(alpha >= 0.f && alpha <= 1.f)) return fail(c, LS_EALPHA, "ls_select_exact: alpha %g outside [0, 1]", (double)alpha);
    if (!a_win || !vert || !slash || !total || !v_idx || !v_cnt || !s_idx || !s_cnt)
        return fail(c, LS_EINVAL, "ls_select_exact: NULL tensor");
    if (q_pos && (reinterpret_cast<uintptr_t>(q_pos) & 7u)) return fail(c, LS_EINVAL, "ls_select_exact: misaligned q_pos");
    if (cap_v <= 0 || cap_s <= 0) return fail(c, LS_ESHAPE, "ls_select_exact: capacities must be positive");
    ls::SelectArgs a{};
    a.n = s->n; a.n_hat = s->n_hat; a.BH = s->B * s->Hq; a.alpha = alpha;
    a.vert = vert; a.slash = slash; a.vmax = vert; a.smax = slash; a.total = total;   // the maxima are not used: any readable array
    Bump bp{c->ws, c->ws_bytes, 0};
    const size_t cnt = 2 * (size_t)a.BH * (size_t)a.n;
    a.skey0 = bp.take<uint32_t>(cnt);
    a.sidx0 = bp.take<int32_t>(cnt); a.sidx1 = bp.take<int32_t>(cnt);
    a.head_w = bp.take<float>(2 * (size_t)a.BH * ls::SELECT_HEAD_LINES); a.head_m = bp.take<float>(2 * (size_t)a.BH * ls::SELECT_HEAD_LINES);
    if (!bp.ok()) return fail(c, LS_EWORKSPACE, "ls_select_exact: workspace of %zu bytes is too small", c->ws_bytes);
    a.v_idx = v_idx; a.v_cnt = v_cnt; a.s_idx = s_idx; a.s_cnt = s_cnt; a.cap_v = cap_v; a.cap_s = cap_s;
    a.accounted = accounted; a.status = c->status; a.spin_limit = c->walk_spin_limit;
    a.a_win = a_win; a.q_pos = q_pos; a.w = s->w;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_select_exact: hipSetDevice failed");
    const hipError_t e = ls::run_select_exact(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_select_exact: %s", hipGetErrorString(e));
    return LS_OK;
}

int ls_select(ls_ctx* c, const ls_shape* s, float alpha,
              const float* vert, const float* slash, const float* vmax, const float* smax, const float* total,
              int32_t* v_idx, int32_t* v_cnt, int32_t cap_v, int32_t* s_idx, int32_t* s_cnt, int32_t cap_s,
              float* accounted, void* stream) {
    if (!c) return LS_EINVAL;
    if (const char* m = check_shape(s, true, false, true)) return fail(c, LS_ESHAPE, "ls_select: %s", m);
    if (!(alpha >= 0.f && alpha <= 1.f)) return fail(c, LS_EALPHA, "ls_select: alpha %g outside [0, 1]", (double)alpha);
    if (!vert || !slash || !vmax || !smax || !total || !v_idx || !v_cnt || !s_idx || !s_cnt)
        return fail(c, LS_EINVAL, "ls_select: NULL tensor");
    if (cap_v <= 0 || cap_s <= 0) return fail(c, LS_ESHAPE, "ls_select: capacities must be positive");
    ls::SelectArgs a{};
    a.n = s->n; a.n_hat = s->n_hat; a.BH = s->B * s->Hq; a.alpha = alpha;
    a.vert = vert; a.slash = slash; a.vmax = vmax; a.smax = smax; a.total = total;
    Bump bp{c->ws, c->ws_bytes, 0};
    const size_t cnt = 2 * (size_t)a.BH * (size_t)a.n;
    a.skey0 = bp.take<uint32_t>(cnt);
    a.sidx0 = bp.take<int32_t>(cnt); a.sidx1 = bp.take<int32_t>(cnt);
    a.head_w = bp.take<float>(2 * (size_t)a.BH * ls::SELECT_HEAD_LINES); a.head_m = bp.take<float>(2 * (size_t)a.BH * ls::SELECT_HEAD_LINES);
    if (!bp.ok()) return fail(c, LS_EWORKSPACE, "ls_select: workspace of %zu bytes is too small", c->ws_bytes);
    a.v_idx = v_idx; a.v_cnt = v_cnt; a.s_idx = s_idx; a.s_cnt = s_cnt; a.cap_v = cap_v; a.cap_s = cap_s;
    a.accounted = accounted; a.status = c->status; a.spin_limit = c->walk_spin_limit;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_select: hipSetDevice failed");
    const hipError_t e = ls::run_select(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_select: %s", hipGetErrorString(e));
    return LS_OK;
}

int ls_merge_lines(ls_ctx* c, const ls_shape* s,
                   const int32_t* v_idx_a, const int32_t* v_cnt_a, int32_t cap_va,
                   const int32_t* s_idx_a, const int32_t* s_cnt_a, int32_t cap_sa,
                   const int32_t* v_idx_b, const int32_t* v_cnt_b, int32_t cap_vb,
                   const int32_t* s_idx_b, const int32_t* s_cnt_b, int32_t cap_sb,
                   int32_t* v_idx, int32_t* v_cnt, int32_t cap_v, int32_t* s_idx, int32_t* s_cnt, int32_t cap_s, void* stream) {
    if (!c) return LS_EINVAL;
    if (const char* m = check_shape(s, false, false, true)) return fail(c, LS_ESHAPE, "ls_merge_lines: %s", m);
    if (!v_idx_a || !v_cnt_a || !s_idx_a || !s_cnt_a || !v_idx_b || !v_cnt_b || !s_idx_b || !s_cnt_b || !v_idx || !v_cnt || !s_idx || !s_cnt)
        return fail(c, LS_EINVAL, "ls_merge_lines: NULL tensor");
    if (cap_va <= 0 || cap_sa <= 0 || cap_vb <= 0 || cap_sb <= 0 || cap_v <= 0 || cap_s <= 0)
        return fail(c, LS_ESHAPE, "ls_merge_lines: capacities must be positive");
    ls::MergeArgs a{};
    a.n = s->n; a.BH = s->B * s->Hq; a.status = c->status;
    a.idx_a[0] = s_idx_a; a.cnt_a[0] = s_cnt_a; a.cap_a[0] = cap_sa; a.idx_a[1] = v_idx_a; a.cnt_a[1] = v_cnt_a; a.cap_a[1] = cap_va;
    a.idx_b[0] = s_idx_b; a.cnt_b[0] = s_cnt_b; a.cap_b[0] = cap_sb; a.idx_b[1] = v_idx_b; a.cnt_b[1] = v_cnt_b; a.cap_b[1] = cap_vb;
    a.idx[0] = s_idx; a.cnt[0] = s_cnt; a.cap[0] = cap_s; a.idx[1] = v_idx; a.cnt[1] = v_cnt; a.cap[1] = cap_v;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_merge_lines: hipSetDevice failed");
    const hipError_t e = ls::run_merge_lines(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_merge_lines: %s", hipGetErrorString(e));
    return LS_OK;
}

namespace {
// Where ls_sparse_prefill keeps its per-call state in the workspace (one place, so that the test hook that
// reads the work queues back finds them where the call put them).
struct PrefillCarve {
    uint32_t* obits; uint8_t* hflag; uint32_t* cost; uint16_t* pref; uint32_t* queue; int32_t* qlen; int32_t* qhead; uint8_t* tab;
    int nqb; int64_t pos0; int code;
};
const char* carve_prefill(ls_ctx* c, const ls_shape* s, PrefillCarve& w) {
    const int BH = s->B * s->Hq;
    const int words = words_of(s->n), tab_len = tab_len_of(s->n);
    Bump bp{c->ws, c->ws_bytes, 0};
    w.obits = bp.take<uint32_t>((size_t)BH * (words + 1));
    w.hflag = bp.take<uint8_t>((size_t)BH);
    w.cost = bp.take<uint32_t>((size_t)BH);
    w.pref = bp.take<uint16_t>((size_t)BH * (tab_len + 1));
    const int bm = ls::prefill_block_rows();
    w.pos0 = (s->n - s->n_hat) / bm * bm;
    w.nqb = (int)((s->n - w.pos0 + bm - 1) / bm);
    w.code = LS_ESHAPE;
    if (w.nqb > 65535) return "too many row blocks";
    if (BH > 8192) return "B * Hq exceeds 8192";
    w.queue = bp.take<uint32_t>(8 * (size_t)BH * w.nqb);
    w.qlen = bp.take<int32_t>(8);
    w.qhead = bp.take<int32_t>(8);
    w.tab = bp.take<uint8_t>((size_t)BH * tab_len);
    w.code = LS_EWORKSPACE;
    if (!bp.ok()) return "workspace is too small";
    w.code = LS_OK;
    return nullptr;
}
}  // namespace

int ls_sparse_prefill(ls_ctx* c, const ls_shape* s, const void* q, const void* k, const void* v,
                      const int32_t* v_idx, const int32_t* v_cnt, int32_t cap_v,
                      const int32_t* s_idx, const int32_t* s_cnt, int32_t cap_s,
                      void* out, float* lse, void* stream) {
    if (!c) return LS_EINVAL;
    if (const char* m = check_shape(s, true, false, true)) return fail(c, LS_ESHAPE, "ls_sparse_prefill: %s", m);
    if (!q || !k || !v || !out || !v_idx || !v_cnt || !s_idx || !s_cnt)
        return fail(c, LS_EINVAL, "ls_sparse_prefill: NULL tensor");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
        return fail(c, LS_EINVAL, "ls_sparse_prefill: misaligned tensor");
    if (cap_v <= 0 || cap_s <= 0) return fail(c, LS_ESHAPE, "ls_sparse_prefill: capacities must be positive");
    const int BH = s->B * s->Hq;
    const int words = words_of(s->n), tab_len = tab_len_of(s->n);
    if (ls::prefill_smem_bytes(s->dtype, s->d, words, tab_len) > 160 * 1024)
        return fail(c, LS_ESHAPE, "ls_sparse_prefill: n too large for the LDS bitmaps");
    PrefillCarve w;
    if (const char* m = carve_prefill(c, s, w)) return fail(c, w.code, "ls_sparse_prefill: %s", m);
    uint32_t* obits = w.obits; uint8_t* hflag = w.hflag; uint32_t* cost = w.cost; uint16_t* pref = w.pref;
    uint32_t* queue = w.queue; int32_t* qlen = w.qlen; int32_t* qhead = w.qhead; uint8_t* tab = w.tab;
    const int nqb = w.nqb; const int64_t pos0 = w.pos0;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_sparse_prefill: hipSetDevice failed");
    ls::PlanArgs p{};
    p.n = s->n; p.words = words; p.tab_len = tab_len; p.v_idx = v_idx; p.v_cnt = v_cnt; p.s_idx = s_idx; p.s_cnt = s_cnt;
    p.cap_v = cap_v; p.cap_s = cap_s; p.obits = obits; p.tab = tab; p.hflag = hflag; p.cost = cost; p.pref = pref;
    p.status = c->status;
    hipError_t e = ls::launch_plan(p, BH, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_sparse_prefill(plan): %s", hipGetErrorString(e));
    ls::SchedArgs sa{};
    sa.BH = BH; sa.G = s->Hq / s->Hkv; sa.Hq = s->Hq; sa.Hkv = s->Hkv; sa.nqb = nqb; sa.cost = cost;
    sa.queue = queue; sa.qlen = qlen; sa.qhead = qhead;
    sa.pref = pref; sa.v_cnt = v_cnt; sa.hflag = hflag; sa.tab_len = tab_len; sa.cap_v = cap_v; sa.n = s->n; sa.pos0 = pos0;
    e = ls::launch_sched(sa, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_sparse_prefill(sched): %s", hipGetErrorString(e));
    ls::PrefillArgs a{};
    a.q = q; a.k = k; a.v = v; a.out = out; a.lse = lse; a.n = s->n; a.n_hat = s->n_hat;
    a.queue = queue; a.qlen = qlen; a.qhead = qhead; a.qcap = BH * nqb;
    a.pos0 = pos0;
    a.Hq = s->Hq; a.Hkv = s->Hkv; a.G = s->Hq / s->Hkv; a.BH = BH;
    a.nqb = nqb;
    a.words = words; a.tab_len = tab_len; a.scale_log2e = scale_log2e(s);
    a.obits = obits; a.tab = tab; a.hflag = hflag; a.v_idx = v_idx; a.v_cnt = v_cnt; a.cap_v = cap_v;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (c->profile) {
        if (hipEventCreate(&e0) != hipSuccess) return fail(c, LS_EHIP, "ls_sparse_prefill: hipEventCreate failed");
        if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(c, LS_EHIP, "ls_sparse_prefill: hipEventCreate failed"); }
    }
    e = ls::launch_prefill(a, s->dtype, s->d, static_cast<hipStream_t>(stream), e0, e1);
    if (c->profile) c->events.emplace_back(e0, e1);
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_sparse_prefill: %s", hipGetErrorString(e));
    return LS_OK;
}

namespace {
// Where a call's errors go: the context's message buffer, or the library's own for calls without a context.
struct ErrSink {
    ls_ctx* c;
    int operator()(int code, const char* fmt, ...) const {
        char* dst = c ? c->err : static_err;
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(dst, 256, fmt, ap);
        va_end(ap);
        return code;
    }
};

// ls_kv_compress on an explicit scratch block (the context's workspace, or the static scratch)
int kv_compress_on(const ErrSink& fail, const char* who, int device, unsigned char* ws, size_t ws_bytes,
                   const ls_shape* s, int32_t budget, const void* q_obs, const void* k, const void* v,
                   int32_t* keep_idx, int32_t* keep_cnt, void* k_out, void* v_out, void* stream) {
    if (const char* m = check_shape(s, false, true, false)) return fail(LS_ESHAPE, "%s: %s", who, m);
    if (budget <= 0) return fail(LS_ESHAPE, "%s: budget must be positive", who);
    if (s->n > ls::TOPB_MAX_LEN) return fail(LS_ESHAPE, "%s: cache length %lld exceeds LS_MAX_N", who, (long long)s->n);
    if (ls::score_lines_smem(s->w, s->dtype, s->d, 2) > 160 * 1024) return fail(LS_ESHAPE, "%s: w too large for LDS", who);
    if (!q_obs || !k || !keep_idx || !keep_cnt || (v_out && !v)) return fail(LS_EINVAL, "%s: NULL tensor", who);
    if (!aligned16(q_obs) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
        return fail(LS_EINVAL, "%s: misaligned tensor", who);
    ls::ScoreArgs a{};
    a.q = q_obs; a.k = k; a.q_pos = nullptr; a.n = s->n; a.w = s->w; a.G = s->Hq / s->Hkv; a.Hq = s->Hq;
    a.Hkv = s->Hkv; a.B = s->B; a.BH = s->B * s->Hq; a.nkb = nkb_of(s->n); a.scale_log2e = scale_log2e(s);
    const int BK = s->B * s->Hkv;
    Bump bp{ws, ws_bytes, 0};
    a.part = bp.take<float>(part_floats(s));
    a.rowstat = bp.take<float>((size_t)a.BH * a.w * 2);
    a.gscore = bp.take<float>((size_t)BK * (size_t)a.n);
    uint32_t* tb_scratch = bp.take<uint32_t>(ls::topb_scratch_words(BK, s->n));
    if (!bp.ok()) return fail(LS_EWORKSPACE, "%s: needs %zu bytes of scratch, %zu are there", who, ws_compress(s), ws_bytes);
    if (hipSetDevice(device) != hipSuccess) return fail(LS_EHIP, "%s: hipSetDevice failed", who);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = ls::run_score(a, s->dtype, s->d, 2, st);
    if (e != hipSuccess) return fail(LS_EHIP, "%s(score): %s", who, hipGetErrorString(e));
    ls::TopbArgs t{};
    t.score = a.gscore; t.len = s->n; t.budget = budget; t.keep_idx = keep_idx; t.keep_cnt = keep_cnt;
    e = ls::run_topb(t, BK, tb_scratch, st);
    if (e != hipSuccess) return fail(LS_EHIP, "%s(topb): %s", who, hipGetErrorString(e));
    const int row_bytes = s->d * (s->dtype == LS_BF16 ? 2 : 4);
    if (k_out) {
        e = ls::run_gather_rows(k, k_out, keep_idx, keep_cnt, BK, s->n, budget, row_bytes, st);
        if (e != hipSuccess) return fail(LS_EHIP, "%s(gather k): %s", who, hipGetErrorString(e));
    }
    if (v_out) {
        e = ls::run_gather_rows(v, v_out, keep_idx, keep_cnt, BK, s->n, budget, row_bytes, st);
        if (e != hipSuccess) return fail(LS_EHIP, "%s(gather v): %s", who, hipGetErrorString(e));
    }
    return LS_OK;
}
}  // namespace

int ls_kv_compress(ls_ctx* c, const ls_shape* s, int32_t budget, const void* q_obs, const void* k, const void* v,
                   int32_t* keep_idx, int32_t* keep_cnt, void* k_out, void* v_out, void* stream) {
    if (!c) return LS_EINVAL;
    return kv_compress_on(ErrSink{c}, "ls_kv_compress", c->device, c->ws, c->ws_bytes, s, budget, q_obs, k, v,
                          keep_idx, keep_cnt, k_out, v_out, stream);
}

size_t ls_static_scratch_bytes(void) { return STATIC_SCRATCH_BYTES; }

int ls_kv_compress_static(int device, const ls_shape* s, int32_t budget, const void* q_obs, const void* k, const void* v,
                          int32_t* keep_idx, int32_t* keep_cnt, void* k_out, void* v_out, void* stream) {
    const ErrSink fail{nullptr};
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev)
        return fail(LS_EHIP, "ls_kv_compress_static: no GPU %d", device);
    if (hipSetDevice(device) != hipSuccess) return fail(LS_EHIP, "ls_kv_compress_static: hipSetDevice failed");
    const hipError_t e = init_device_once(device);      // first call on this device: kernel attributes, scratch address
    if (e != hipSuccess) return fail(LS_EHIP, "ls_kv_compress_static: %s", hipGetErrorString(e));
    return kv_compress_on(fail, "ls_kv_compress_static", device, scratch_on[device], STATIC_SCRATCH_BYTES, s, budget,
                          q_obs, k, v, keep_idx, keep_cnt, k_out, v_out, stream);
}

namespace {
// split of the key axis for ls_decode_attend: chunks of whole 128-key rounds (4 waves x 32 keys),
// enough workgroups to cover the chip about twice (more, shorter chunks measured slower: more partials to merge)
void decode_split(const ls_shape* s, int32_t cap, int32_t T, int* nsplit, int* chunk) {
    const int64_t L = (int64_t)cap + T;
    const int64_t rounds = (L + 127) / 128;
    int64_t want = 512 / ((int64_t)s->B * s->Hkv);
    if (want < 1) want = 1;
    if (want > rounds) want = rounds;
    const int64_t per = (rounds + want - 1) / want;
    *chunk = (int)(per * 128);
    *nsplit = (int)((rounds + per - 1) / per);
}
}  // namespace

size_t ls_decode_workspace_bytes(const ls_shape* s, int32_t cap, int32_t T) {
    if (!s || s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv || (s->d != 64 && s->d != 128) || cap < 1 || T < 0) return 0;
    int nsplit, chunk;
    decode_split(s, cap, T, &nsplit, &chunk);
    return up((size_t)s->B * s->Hq * nsplit * (s->d + 2) * 4) + ALIGN;
}

int ls_decode_attend(ls_ctx* c, const ls_shape* s, int32_t cap, int32_t T, const void* q, const void* k_c, const void* v_c,
                     const int32_t* cnt, const void* k_t, const void* v_t, void* out, float* lse, void* stream) {
    if (!c) return LS_EINVAL;
    if (!s) return fail(c, LS_ESHAPE, "ls_decode_attend: shape is NULL");
    if (s->B <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->Hq % s->Hkv) return fail(c, LS_ESHAPE, "ls_decode_attend: need positive B, Hq, Hkv with Hkv dividing Hq");
    if (s->d != 64 && s->d != 128) return fail(c, LS_ESHAPE, "ls_decode_attend: d must be 64 or 128");
    if (s->dtype != LS_BF16) return fail(c, LS_ESHAPE, "ls_decode_attend: dtype must be LS_BF16");
    if (s->Hq / s->Hkv > 32) return fail(c, LS_ESHAPE, "ls_decode_attend: at most 32 query heads per KV head");
    if ((int64_t)s->B * s->Hkv > 65535) return fail(c, LS_ESHAPE, "ls_decode_attend: B * Hkv too large");
    if (cap < 1 || T < 0 || (int64_t)cap + T > 2147483000LL / 256) return fail(c, LS_ESHAPE, "ls_decode_attend: need cap >= 1, T >= 0, cap + T < 2^23");
    if (!q || !k_c || !v_c || !out || (T > 0 && (!k_t || !v_t))) return fail(c, LS_EINVAL, "ls_decode_attend: NULL tensor");
    if (!aligned16(q) || !aligned16(k_c) || !aligned16(v_c) || !aligned16(k_t) || !aligned16(v_t) || !aligned16(out))
        return fail(c, LS_EINVAL, "ls_decode_attend: misaligned tensor");
    ls::DecodeArgs a{};
    a.q = q; a.kc = k_c; a.vc = v_c; a.kt = k_t; a.vt = v_t; a.cnt = cnt; a.out = out; a.lse = lse;
    a.B = s->B; a.Hq = s->Hq; a.Hkv = s->Hkv; a.G = s->Hq / s->Hkv; a.cap = cap; a.T = T;
    a.scale_log2e = scale_log2e(s);
    decode_split(s, cap, T, &a.nsplit, &a.chunk);
    if (ls::decode_smem_bytes(s->d, a.G) > 160 * 1024) return fail(c, LS_ESHAPE, "ls_decode_attend: group too large for LDS");
    Bump bp{c->ws, c->ws_bytes, 0};
    a.part = bp.take<float>((size_t)s->B * s->Hq * a.nsplit * (s->d + 2));
    if (!bp.ok()) return fail(c, LS_EWORKSPACE, "ls_decode_attend: workspace of %zu bytes is too small", c->ws_bytes);
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_decode_attend: hipSetDevice failed");
    hipError_t e = ls::run_decode(a, s->d, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(c, LS_EHIP, "ls_decode_attend: %s", hipGetErrorString(e));
    return LS_OK;
}

int ls_profile_enable(ls_ctx* c, int on) {
    if (!c) return LS_EINVAL;
    (void)hipSetDevice(c->device);
    for (auto& e : c->events) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
    c->events.clear();
    c->profile = on != 0;
    return LS_OK;
}

int ls_profile_prefill_kernel_ms(ls_ctx* c, double* mean_ms, int32_t* launches) {
    if (!c || !mean_ms || !launches) return LS_EINVAL;
    double tot = 0.0;
    int cnt = 0;
    for (auto& e : c->events) {
        if (hipEventSynchronize(e.second) != hipSuccess) return fail(c, LS_EHIP, "ls_profile: hipEventSynchronize failed");
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, e.first, e.second) != hipSuccess) return fail(c, LS_EHIP, "ls_profile: hipEventElapsedTime failed");
        tot += ms; ++cnt;
    }
    *mean_ms = cnt ? tot / cnt : 0.0;
    *launches = cnt;
    return LS_OK;
}

int ls_poll_status(ls_ctx* c, int32_t* host_out, void* stream) {
    if (!c || !host_out) return LS_EINVAL;
    if (hipSetDevice(c->device) != hipSuccess) return fail(c, LS_EHIP, "ls_poll_status: hipSetDevice failed");
    hipStream_t st = static_cast<hipStream_t>(stream);
    int32_t word = 0;
    // stream-ordered: read the word behind everything queued so far, then clear it
    if (hipMemcpyAsync(&word, c->status, sizeof(word), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipMemsetAsync(c->status, 0, sizeof(word), st) != hipSuccess || hipStreamSynchronize(st) != hipSuccess)
        return fail(c, LS_EHIP, "ls_poll_status: reading the status word failed");
    *host_out = word;
    return LS_OK;
}

int ls_debug_set_walk_spin_limit(ls_ctx* c, int32_t limit) {
    if (!c) return LS_EINVAL;
    c->walk_spin_limit = limit < 0 ? ls::WALK_SPIN_DEFAULT : limit;
    return LS_OK;
}

/* Debug / test hook: the eight work queues the last ls_sparse_prefill call on this context built
 * (host_queue: [8][B*Hq*nqb] item words = (head << 16) | row block, host_qlen: [8]); synchronises the stream. */
int ls_debug_copy_prefill_queues(ls_ctx* c, const ls_shape* s, uint32_t* host_queue, int32_t* host_qlen, int32_t* nqb_out, void* stream) {
    if (!c || !s || !host_queue || !host_qlen || !nqb_out) return LS_EINVAL;
    if (check_shape(s, true, false, true)) return LS_ESHAPE;
    PrefillCarve w;
    if (carve_prefill(c, s, w)) return w.code;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t items = (size_t)s->B * s->Hq * w.nqb;
    if (hipSetDevice(c->device) != hipSuccess) return LS_EHIP;
    if (hipMemcpyAsync(host_queue, w.queue, 8 * items * sizeof(uint32_t), hipMemcpyDeviceToHost, st) != hipSuccess) return LS_EHIP;
    if (hipMemcpyAsync(host_qlen, w.qlen, 8 * sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess) return LS_EHIP;
    if (hipStreamSynchronize(st) != hipSuccess) return LS_EHIP;
    *nqb_out = w.nqb;
    return LS_OK;
}

/* Debug / test hook: the group-summed retention score of the last ls_kv_compress call on this
 * context lives at the start of the third workspace block; exposed so tests can compare scores. */
int ls_debug_copy_compress_score(ls_ctx* c, const ls_shape* s, float* dst_device, void* stream) {
    if (!c || !s || !dst_device) return LS_EINVAL;
    const size_t BH = (size_t)s->B * s->Hq;
    const size_t off = up(part_floats(s) * 4) + up(BH * s->w * 2 * 4);
    const size_t bytes = (size_t)s->B * s->Hkv * (size_t)s->n * 4;
    if (off + bytes > c->ws_bytes) return LS_EWORKSPACE;
    if (hipMemcpyAsync(dst_device, c->ws + off, bytes, hipMemcpyDeviceToDevice, static_cast<hipStream_t>(stream)) != hipSuccess)
        return LS_EHIP;
    return LS_OK;
}

}  // extern "C"
