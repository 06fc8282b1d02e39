// C ABI of the TTT attention library: argument validation, workspace layout, launch sequencing.
// No arithmetic of the method lives here; see include/ttt_attn.h for the contract.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/ttt_attn.h"
#include "../../include/ttt_loss.h"
#include "../../include/ttt_qkv.h"
#include "ttt_args.hpp"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Everything that can be checked from the parameter block alone.
int check_params(const ttt_attn_params* p) {
    if (!p) return fail(TTT_ERR_INVALID_ARG, "params is NULL");
    if (p->dtype != TTT_F32 && p->dtype != TTT_BF16) return fail(TTT_ERR_UNSUPPORTED, "dtype %d is not TTT_F32/TTT_BF16", p->dtype);
    if (p->head_dim != 64 && p->head_dim != 128) return fail(TTT_ERR_UNSUPPORTED, "head_dim %d is not 64 or 128", p->head_dim);
    if (p->k < 1 || p->k > TTT_MAX_STEPS) return fail(TTT_ERR_INVALID_ARG, "k=%d outside 1..%d", p->k, TTT_MAX_STEPS);
    if (p->step_begin < 0 || p->step_end > p->k || p->step_begin > p->step_end)
        return fail(TTT_ERR_INVALID_ARG, "step range [%d,%d) not inside [0,%d)", p->step_begin, p->step_end, p->k);
    if (p->total_tokens < 0 || p->n_docs < 0) return fail(TTT_ERR_INVALID_ARG, "negative total_tokens or n_docs");
    if (p->total_tokens > 0 && p->n_docs == 0) return fail(TTT_ERR_INVALID_ARG, "tokens without documents");
    if (p->hq < 1 || p->hkv < 1 || p->hq % p->hkv != 0)
        return fail(TTT_ERR_INVALID_ARG, "hq=%d must be a positive multiple of hkv=%d", p->hq, p->hkv);
    if (!(p->softmax_scale > 0.f) || !std::isfinite(p->softmax_scale))
        return fail(TTT_ERR_INVALID_ARG, "softmax_scale must be positive and finite");
    const int64_t st[4] = {p->q_stride_token, p->q_stride_head, p->kv_stride_token, p->kv_stride_head};
    for (int i = 0; i < 4; ++i)
        if (st[i] < p->head_dim || st[i] % 8 != 0)
            return fail(TTT_ERR_INVALID_ARG, "stride %d = %lld must be >= head_dim and a multiple of 8 elements", i, (long long)st[i]);
    return TTT_OK;
}

int check_cu(const ttt_attn_params* p, const int32_t* cu_dev, const int32_t* cu_host) {
    if (!cu_dev || !cu_host) return fail(TTT_ERR_INVALID_ARG, "cu_seqlens pointer is NULL");
    if (cu_host[0] != 0) return fail(TTT_ERR_INVALID_ARG, "cu_seqlens[0] = %d, expected 0", cu_host[0]);
    for (int r = 0; r < p->n_docs; ++r)
        if (cu_host[r + 1] < cu_host[r]) return fail(TTT_ERR_INVALID_ARG, "cu_seqlens decreases at document %d", r);
    if (cu_host[p->n_docs] != p->total_tokens)
        return fail(TTT_ERR_INVALID_ARG, "cu_seqlens[n_docs] = %d, expected total_tokens = %d", cu_host[p->n_docs], p->total_tokens);
    return TTT_OK;
}

int check_ptr(const void* p, const char* what, int step) {
    if (!p) return fail(TTT_ERR_INVALID_ARG, "%s[%d] is NULL but the call needs it", what, step);
    if (!aligned16(p)) return fail(TTT_ERR_INVALID_ARG, "%s[%d] is not 16-byte aligned", what, step);
    return TTT_OK;
}

struct Layout {
    size_t tok_start, tok_end, delta, lse2, dk0, dv0, dkl, dvl, total;
};

Layout make_layout(const ttt_attn_params* p, int pass) {
    Layout L{};
    const size_t T = (size_t)p->total_tokens;
    size_t off = 0;
    L.tok_start = off; off += align256(T * sizeof(int));
    L.tok_end = off;   off += align256(T * sizeof(int));
    if (pass != TTT_PASS_FWD) {
        const size_t kv = T * (size_t)p->hkv * (size_t)p->head_dim * sizeof(float);
        L.delta = off; off += align256((size_t)p->k * p->hq * T * sizeof(float));
        L.lse2 = off;  off += align256((size_t)p->k * p->hq * T * sizeof(float));
        L.dk0 = off;   off += align256(kv);
        L.dv0 = off;   off += align256(kv);
        if (pass == TTT_PASS_BWD_ACCUM) {
            L.dkl = off; off += align256(kv * (size_t)(p->k - 1));
            L.dvl = off; off += align256(kv * (size_t)(p->k - 1));
        }
    }
    L.total = off > 0 ? off : 256;
    return L;
}

void fill_geometry(ttt::Geometry& g, const ttt_attn_params* p) {
    g.T = p->total_tokens;
    g.k = p->k;
    g.step_begin = p->step_begin;
    g.n_steps = p->step_end - p->step_begin;
    g.hq = p->hq;
    g.hkv = p->hkv;
    g.G = p->hq / p->hkv;
    g.scale = p->softmax_scale;
    g.scale_log2 = p->softmax_scale * 1.44269504088896340736f;
    g.q_st = p->q_stride_token;
    g.q_sh = p->q_stride_head;
    g.kv_st = p->kv_stride_token;
    g.kv_sh = p->kv_stride_head;
    g.lse_st = p->total_tokens;
}

int check_workspace(const void* ws, size_t have, size_t need) {
    if (!ws) return fail(TTT_ERR_WORKSPACE, "workspace is NULL (need %zu bytes)", need);
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(TTT_ERR_WORKSPACE, "workspace is not 256-byte aligned");
    if (have < need) return fail(TTT_ERR_WORKSPACE, "workspace has %zu bytes, need %zu", have, need);
    return TTT_OK;
}

// ---- diagnostics: per-kernel HIP-event timing, off unless a caller turns it on
struct ProfileRecord {
    const char* name;
    hipEvent_t start, stop;
};
std::mutex g_prof_mutex;
std::atomic<bool> g_prof_on{false};   // read by every launch, written under g_prof_mutex
std::vector<ProfileRecord> g_prof_records;
thread_local ProfileRecord g_prof_open = {nullptr, nullptr, nullptr};

}  // namespace

namespace ttt {

void profile_begin(const char* kernel_name, hipStream_t stream) {
    g_prof_open.name = nullptr;
    if (!g_prof_on.load(std::memory_order_relaxed)) return;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return;
    }
    (void)hipEventRecord(a, stream);
    g_prof_open = {kernel_name, a, b};
}

void profile_end(hipStream_t stream) {
    if (!g_prof_open.name) return;
    (void)hipEventRecord(g_prof_open.stop, stream);
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof_records.push_back(g_prof_open);
    g_prof_open.name = nullptr;
}

}  // namespace ttt

// ---- forward without a workspace argument: the token-bounds scratch lives in a file-scope device
// array.  Host code never uses the array's name as an address (on the host it is only a stand-in
// for the symbol): the device address is asked for once per device and kept.
static __device__ __align__(256) int32_t g_static_scratch[2 * TTT_STATIC_MAX_TOKENS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
void* g_static_ptr[kMaxDevices] = {};

// device address of g_static_scratch on the CURRENT device (nullptr + error message on failure)
void* static_scratch_ptr() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        fail(TTT_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
        return nullptr;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        fail(TTT_ERR_UNSUPPORTED, "device index %d outside 0..%d", dev, kMaxDevices - 1);
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
        if (e != hipSuccess || !ptr) {
            fail(TTT_ERR_HIP, "hipGetSymbolAddress(static scratch) on device %d: %s", dev, hipGetErrorString(e));
            return nullptr;
        }
        g_static_ptr[dev] = ptr;
    }
    return g_static_ptr[dev];
}
}  // namespace

extern "C" {

int ttt_attn_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    const int was = g_prof_on.load() ? 1 : 0;
    g_prof_on.store(on != 0);
    return was;
}

int ttt_attn_profile_totals(int capacity, const char** names, float* total_ms, int32_t* launches) {
    std::vector<ProfileRecord> recs;
    {
        std::lock_guard<std::mutex> lock(g_prof_mutex);
        recs.swap(g_prof_records);
    }
    int n = 0;
    for (const ProfileRecord& r : recs) {
        float ms = 0.f;
        const bool ok = hipEventSynchronize(r.stop) == hipSuccess && hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess;
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
        if (!ok) continue;
        int slot = -1;
        for (int i = 0; i < n; ++i)
            if (std::strcmp(names[i], r.name) == 0) slot = i;
        if (slot < 0) {
            if (n >= capacity) continue;
            slot = n++;
            names[slot] = r.name;
            total_ms[slot] = 0.f;
            launches[slot] = 0;
        }
        total_ms[slot] += ms;
        launches[slot] += 1;
    }
    return n;
}

const char* ttt_attn_last_error(void) { return g_err; }

size_t ttt_attn_workspace_bytes(const ttt_attn_params* params, int pass) {
    if (check_params(params) != TTT_OK) return 0;
    if (pass != TTT_PASS_FWD && pass != TTT_PASS_BWD && pass != TTT_PASS_BWD_ACCUM) {
        fail(TTT_ERR_INVALID_ARG, "pass %d is not one of TTT_PASS_*", pass);
        return 0;
    }
    return make_layout(params, pass).total;
}

// A slice of the batch: consecutive documents [doc0, doc0 + n_docs) = tokens [tok0, tok0 + tokens),
// processed with the step range [step_begin, step_end).  The whole batch is one slice.
struct Slice {
    int doc0, n_docs, tok0, tokens, step_begin, step_end;
};

static int fwd_slice(const ttt_attn_params* p, const Slice& sl, const void* const* q, const void* const* k,
                     const void* const* v, const int32_t* cu_dev, const int32_t* cu_host, void* const* o, float* const* lse,
                     char* ws, hipStream_t stream) {
    if (sl.tokens == 0 || sl.step_begin >= sl.step_end) return TTT_OK;
    ttt_attn_params ps = *p;
    ps.total_tokens = sl.tokens;
    ps.n_docs = sl.n_docs;
    ps.step_begin = sl.step_begin;
    ps.step_end = sl.step_end;
    const Layout L = make_layout(&ps, TTT_PASS_FWD);
    int* tok_start = reinterpret_cast<int*>(ws + L.tok_start);
    int* tok_end = reinterpret_cast<int*>(ws + L.tok_end);
    hipError_t e = ttt::launch_tok_bounds(cu_dev + sl.doc0, cu_host[sl.doc0], sl.n_docs, sl.tokens, tok_start, tok_end, stream);
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "token-bounds kernel launch: %s", hipGetErrorString(e));

    const size_t esz = p->dtype == TTT_F32 ? 4 : 2;
    const size_t qoff = (size_t)sl.tok0 * (size_t)p->q_stride_token * esz;
    const size_t kvoff = (size_t)sl.tok0 * (size_t)p->kv_stride_token * esz;
    auto at = [](const void* base, size_t off) { return base ? static_cast<const char*>(base) + off : nullptr; };
    ttt::FwdArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_geometry(a.geo, &ps);
    a.geo.lse_st = p->total_tokens;
    for (int s = 0; s < p->k; ++s) {
        a.q[s] = at(q[s], qoff);
        a.k[s] = at(k[s], kvoff);
        a.v[s] = at(v[s], kvoff);
        a.o[s] = const_cast<char*>(at(o[s], qoff));
        a.lse[s] = lse[s] ? lse[s] + sl.tok0 : nullptr;
    }
    a.tok_start = tok_start;
    e = ttt::launch_fwd(p->dtype, p->head_dim, a, stream);
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "forward kernel launch: %s", hipGetErrorString(e));
    return TTT_OK;
}

// Runs of consecutive documents with the same step count, as slices; steps beyond a document's own
// count are cut off.  doc_steps == NULL: one slice with the call's step range.
static int make_slices(const ttt_attn_params* p, const int32_t* cu_host, const int32_t* doc_steps, std::vector<Slice>& out) {
    out.clear();
    if (!doc_steps) {
        out.push_back(Slice{0, p->n_docs, 0, p->total_tokens, p->step_begin, p->step_end});
        return TTT_OK;
    }
    for (int r = 0; r < p->n_docs;) {
        const int kr = doc_steps[r];
        if (kr < 0 || kr > p->k) return fail(TTT_ERR_INVALID_ARG, "doc_steps[%d] = %d outside 0..k=%d", r, kr, p->k);
        int r1 = r + 1;
        while (r1 < p->n_docs && doc_steps[r1] == kr) ++r1;
        out.push_back(Slice{r, r1 - r, cu_host[r], cu_host[r1] - cu_host[r], p->step_begin, kr < p->step_end ? kr : p->step_end});
        r = r1;
    }
    return TTT_OK;
}

// Everything the forward checks before it touches the workspace or launches anything.
static int fwd_validate(const ttt_attn_params* p, const void* const* q, const void* const* k, const void* const* v,
                        const int32_t* cu_dev, const int32_t* cu_host, void* const* o, float* const* lse, bool& nothing_to_do) {
    nothing_to_do = false;
    int rc = check_params(p);
    if (rc != TTT_OK) return rc;
    if (!q || !k || !v || !o || !lse) return fail(TTT_ERR_INVALID_ARG, "a step-pointer array is NULL");
    rc = check_cu(p, cu_dev, cu_host);
    if (rc != TTT_OK) return rc;
    if (p->total_tokens == 0 || p->step_begin == p->step_end) {
        nothing_to_do = true;
        return TTT_OK;
    }
    for (int j = p->step_begin; j < p->step_end; ++j) {
        if ((rc = check_ptr(q[j], "q", j)) != TTT_OK) return rc;
        if ((rc = check_ptr(o[j], "o", j)) != TTT_OK) return rc;
        if ((rc = check_ptr(lse[j], "lse", j)) != TTT_OK) return rc;
    }
    for (int l = 0; l < p->step_end; ++l) {
        if ((rc = check_ptr(k[l], "k", l)) != TTT_OK) return rc;
        if ((rc = check_ptr(v[l], "v", l)) != TTT_OK) return rc;
    }
    return TTT_OK;
}

static int fwd_checked(const ttt_attn_params* p, const int32_t* doc_steps, const void* const* q, const void* const* k,
                       const void* const* v, const int32_t* cu_dev, const int32_t* cu_host, void* const* o, float* const* lse,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    bool nothing = false;
    int rc = fwd_validate(p, q, k, v, cu_dev, cu_host, o, lse, nothing);
    if (rc != TTT_OK || nothing) return rc;
    const Layout L = make_layout(p, TTT_PASS_FWD);
    if ((rc = check_workspace(workspace, workspace_bytes, L.total)) != TTT_OK) return rc;
    std::vector<Slice> slices;
    if ((rc = make_slices(p, cu_host, doc_steps, slices)) != TTT_OK) return rc;
    for (const Slice& sl : slices)   // slices run one after the other on the stream and share the workspace
        if ((rc = fwd_slice(p, sl, q, k, v, cu_dev, cu_host, o, lse, static_cast<char*>(workspace),
                            static_cast<hipStream_t>(hip_stream))) != TTT_OK)
            return rc;
    return TTT_OK;
}

int ttt_attn_fwd(const ttt_attn_params* p, const void* const* q, const void* const* k, const void* const* v,
                 const int32_t* cu_dev, const int32_t* cu_host, void* const* o, float* const* lse, void* workspace,
                 size_t workspace_bytes, void* hip_stream) {
    return fwd_checked(p, nullptr, q, k, v, cu_dev, cu_host, o, lse, workspace, workspace_bytes, hip_stream);
}

int ttt_attn_fwd_static(const ttt_attn_params* p, const void* const* q, const void* const* k, const void* const* v,
                        const int32_t* cu_dev, const int32_t* cu_host, void* const* o, float* const* lse, void* hip_stream) {
    bool nothing = false;
    int rc = fwd_validate(p, q, k, v, cu_dev, cu_host, o, lse, nothing);
    if (rc != TTT_OK) return rc;
    if (p->total_tokens > TTT_STATIC_MAX_TOKENS)
        return fail(TTT_ERR_WORKSPACE, "total_tokens = %d exceeds TTT_STATIC_MAX_TOKENS = %d of the built-in scratch; use ttt_attn_fwd",
                    p->total_tokens, TTT_STATIC_MAX_TOKENS);
    if (nothing) return TTT_OK;
    const Layout L = make_layout(p, TTT_PASS_FWD);
    if (L.total > sizeof(int32_t) * 2 * (size_t)TTT_STATIC_MAX_TOKENS)
        return fail(TTT_ERR_WORKSPACE, "built-in scratch too small for %d tokens", p->total_tokens);
    void* scratch = static_scratch_ptr();
    if (!scratch) return TTT_ERR_HIP;
    const Slice whole{0, p->n_docs, 0, p->total_tokens, p->step_begin, p->step_end};
    return fwd_slice(p, whole, q, k, v, cu_dev, cu_host, o, lse, static_cast<char*>(scratch), static_cast<hipStream_t>(hip_stream));
}

int ttt_attn_fwd_docsteps(const ttt_attn_params* p, const int32_t* doc_steps_host, const void* const* q, const void* const* k,
                          const void* const* v, const int32_t* cu_dev, const int32_t* cu_host, void* const* o,
                          float* const* lse, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!doc_steps_host) return fail(TTT_ERR_INVALID_ARG, "doc_steps_host is NULL");
    return fwd_checked(p, doc_steps_host, q, k, v, cu_dev, cu_host, o, lse, workspace, workspace_bytes, hip_stream);
}

static int bwd_slice(const ttt_attn_params* p, const Slice& sl, const void* const* q, const void* const* k,
                     const void* const* v, const void* const* o, const float* const* lse, const void* const* d_o,
                     const int32_t* cu_dev, const int32_t* cu_host, void* const* dq, void* const* dk, void* const* dv,
                     int accumulate_dkv, char* ws, hipStream_t stream) {
    if (sl.tokens == 0 || sl.step_begin >= sl.step_end) return TTT_OK;
    ttt_attn_params ps = *p;
    ps.total_tokens = sl.tokens;
    ps.n_docs = sl.n_docs;
    ps.step_begin = sl.step_begin;
    ps.step_end = sl.step_end;
    const int pass = accumulate_dkv ? TTT_PASS_BWD_ACCUM : TTT_PASS_BWD;
    const Layout L = make_layout(&ps, pass);
    int* tok_start = reinterpret_cast<int*>(ws + L.tok_start);
    int* tok_end = reinterpret_cast<int*>(ws + L.tok_end);
    hipError_t e = ttt::launch_tok_bounds(cu_dev + sl.doc0, cu_host[sl.doc0], sl.n_docs, sl.tokens, tok_start, tok_end, stream);
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "token-bounds kernel launch: %s", hipGetErrorString(e));

    const size_t esz = p->dtype == TTT_F32 ? 4 : 2;
    const size_t qoff = (size_t)sl.tok0 * (size_t)p->q_stride_token * esz;
    const size_t kvoff = (size_t)sl.tok0 * (size_t)p->kv_stride_token * esz;
    auto at = [](const void* base, size_t off) { return base ? static_cast<const char*>(base) + off : nullptr; };
    ttt::BwdArgs a;
    std::memset(&a, 0, sizeof(a));
    fill_geometry(a.geo, &ps);
    a.geo.lse_st = p->total_tokens;
    for (int s = 0; s < p->k; ++s) {
        a.q[s] = at(q[s], qoff);
        a.k[s] = at(k[s], kvoff);
        a.v[s] = at(v[s], kvoff);
        a.o[s] = at(o[s], qoff);
        a.lse[s] = lse[s] ? lse[s] + sl.tok0 : nullptr;
        a.d_o[s] = at(d_o[s], qoff);
        a.dq[s] = const_cast<char*>(at(dq[s], qoff));
        a.dk[s] = const_cast<char*>(at(dk[s], kvoff));
        a.dv[s] = const_cast<char*>(at(dv[s], kvoff));
    }
    a.tok_start = tok_start;
    a.tok_end = tok_end;
    a.cu_host = cu_host + sl.doc0;
    a.cu_base = cu_host[sl.doc0];
    a.n_docs = sl.n_docs;
    a.delta = reinterpret_cast<float*>(ws + L.delta);
    a.lse2 = reinterpret_cast<float*>(ws + L.lse2);
    a.dk0_acc = reinterpret_cast<float*>(ws + L.dk0);
    a.dv0_acc = reinterpret_cast<float*>(ws + L.dv0);
    a.accumulate = accumulate_dkv;
    a.carry_reset = accumulate_dkv && ps.step_end == p->k;
    if (accumulate_dkv && p->k > 1) {
        a.dkl_acc = reinterpret_cast<float*>(ws + L.dkl);
        a.dvl_acc = reinterpret_cast<float*>(ws + L.dvl);
    }
    e = ttt::launch_bwd(p->dtype, p->head_dim, a, stream);
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "backward kernel launch: %s", hipGetErrorString(e));
    return TTT_OK;
}

static int bwd_checked(const ttt_attn_params* p, const int32_t* doc_steps, const void* const* q, const void* const* k,
                       const void* const* v, const void* const* o, const float* const* lse, const void* const* d_o,
                       const int32_t* cu_dev, const int32_t* cu_host, void* const* dq, void* const* dk, void* const* dv,
                       int accumulate_dkv, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int rc = check_params(p);
    if (rc != TTT_OK) return rc;
    if (!q || !k || !v || !o || !lse || !d_o || !dq || !dk || !dv) return fail(TTT_ERR_INVALID_ARG, "a step-pointer array is NULL");
    if (accumulate_dkv != 0 && accumulate_dkv != 1) return fail(TTT_ERR_INVALID_ARG, "accumulate_dkv must be 0 or 1");
    rc = check_cu(p, cu_dev, cu_host);
    if (rc != TTT_OK) return rc;
    if (p->total_tokens == 0 || p->step_begin == p->step_end) return TTT_OK;
    for (int j = p->step_begin; j < p->step_end; ++j) {
        if ((rc = check_ptr(q[j], "q", j)) != TTT_OK) return rc;
        if ((rc = check_ptr(o[j], "o", j)) != TTT_OK) return rc;
        if ((rc = check_ptr(lse[j], "lse", j)) != TTT_OK) return rc;
        if ((rc = check_ptr(d_o[j], "d_o", j)) != TTT_OK) return rc;
        if ((rc = check_ptr(dq[j], "dq", j)) != TTT_OK) return rc;
    }
    for (int l = 0; l < p->step_end; ++l) {
        if ((rc = check_ptr(k[l], "k", l)) != TTT_OK) return rc;
        if ((rc = check_ptr(v[l], "v", l)) != TTT_OK) return rc;
        // blocks written by this call: all l < step_end without carry, l in range (and block 0 at the end) with it
        const bool written = !accumulate_dkv || l >= p->step_begin;
        if (written) {
            if ((rc = check_ptr(dk[l], "dk", l)) != TTT_OK) return rc;
            if ((rc = check_ptr(dv[l], "dv", l)) != TTT_OK) return rc;
        }
    }
    const int pass = accumulate_dkv ? TTT_PASS_BWD_ACCUM : TTT_PASS_BWD;
    const Layout L = make_layout(p, pass);
    if ((rc = check_workspace(workspace, workspace_bytes, L.total)) != TTT_OK) return rc;
    std::vector<Slice> slices;
    if ((rc = make_slices(p, cu_host, doc_steps, slices)) != TTT_OK) return rc;
    for (const Slice& sl : slices)
        if ((rc = bwd_slice(p, sl, q, k, v, o, lse, d_o, cu_dev, cu_host, dq, dk, dv, accumulate_dkv,
                            static_cast<char*>(workspace), static_cast<hipStream_t>(hip_stream))) != TTT_OK)
            return rc;
    return TTT_OK;
}

int ttt_attn_bwd(const ttt_attn_params* p, const void* const* q, const void* const* k, const void* const* v,
                 const void* const* o, const float* const* lse, const void* const* d_o, const int32_t* cu_dev,
                 const int32_t* cu_host, void* const* dq, void* const* dk, void* const* dv, int accumulate_dkv,
                 void* workspace, size_t workspace_bytes, void* hip_stream) {
    return bwd_checked(p, nullptr, q, k, v, o, lse, d_o, cu_dev, cu_host, dq, dk, dv, accumulate_dkv, workspace,
                       workspace_bytes, hip_stream);
}

int ttt_attn_bwd_docsteps(const ttt_attn_params* p, const int32_t* doc_steps_host, const void* const* q,
                          const void* const* k, const void* const* v, const void* const* o, const float* const* lse,
                          const void* const* d_o, const int32_t* cu_dev, const int32_t* cu_host, void* const* dq,
                          void* const* dk, void* const* dv, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!doc_steps_host) return fail(TTT_ERR_INVALID_ARG, "doc_steps_host is NULL");
    return bwd_checked(p, doc_steps_host, q, k, v, o, lse, d_o, cu_dev, cu_host, dq, dk, dv, 0, workspace, workspace_bytes,
                       hip_stream);
}

int ttt_loss_bwd_inplace(void* logits, const void* target, const float* grad, int64_t n_rows, int32_t vocab,
                         int64_t logits_row_stride, int64_t target_row_stride, int32_t dtype, void* hip_stream) {
    if (dtype != TTT_F32 && dtype != TTT_BF16) return fail(TTT_ERR_UNSUPPORTED, "dtype %d is not TTT_F32/TTT_BF16", dtype);
    if (n_rows < 0 || vocab < 1) return fail(TTT_ERR_INVALID_ARG, "n_rows=%lld must be >= 0 and vocab=%d >= 1", (long long)n_rows, vocab);
    if (n_rows > 0x7fffffffLL) return fail(TTT_ERR_INVALID_ARG, "n_rows=%lld exceeds the grid limit", (long long)n_rows);
    if (logits_row_stride < vocab || target_row_stride < vocab)
        return fail(TTT_ERR_INVALID_ARG, "row strides (%lld, %lld) must be >= vocab=%d", (long long)logits_row_stride,
                    (long long)target_row_stride, vocab);
    if (n_rows == 0) return TTT_OK;
    if (!logits || !target || !grad) return fail(TTT_ERR_INVALID_ARG, "logits, target or grad is NULL");
    const uintptr_t esz = dtype == TTT_F32 ? 4 : 2;
    if (reinterpret_cast<uintptr_t>(logits) % esz || reinterpret_cast<uintptr_t>(target) % esz || reinterpret_cast<uintptr_t>(grad) % 4)
        return fail(TTT_ERR_INVALID_ARG, "a pointer is not aligned to its element size");
    hipError_t e = ttt::launch_loss_bwd(dtype, logits, target, grad, n_rows, vocab, logits_row_stride, target_row_stride,
                                        static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "loss backward kernel launch: %s", hipGetErrorString(e));
    return TTT_OK;
}

int ttt_qkv_rope_fwd(const void* x, const void* w, const float* cos_tab, const float* sin_tab, const int32_t* pos, void* q,
                     void* k, void* v, int64_t tokens, int32_t hidden_in, int32_t hq, int32_t hkv, int32_t head_dim,
                     int64_t x_row_stride, int64_t w_row_stride, int32_t n_pos, int32_t dtype, void* hip_stream) {
    if (dtype != TTT_BF16) return fail(TTT_ERR_UNSUPPORTED, "dtype %d: the projection kernel is built for TTT_BF16", dtype);
    if (head_dim != 128) return fail(TTT_ERR_UNSUPPORTED, "head_dim=%d: the projection kernel is built for 128", head_dim);
    if (tokens < 0 || tokens > 0x7fffffffLL) return fail(TTT_ERR_INVALID_ARG, "tokens=%lld out of range", (long long)tokens);
    if (hq < 1 || hkv < 1 || hq > 4096 || hkv > 4096) return fail(TTT_ERR_INVALID_ARG, "hq=%d, hkv=%d must be in [1, 4096]", hq, hkv);
    if (hidden_in < 64 || hidden_in % 64) return fail(TTT_ERR_INVALID_ARG, "hidden_in=%d must be a positive multiple of 64", hidden_in);
    if (n_pos < 1) return fail(TTT_ERR_INVALID_ARG, "n_pos=%d must be >= 1", n_pos);
    if (x_row_stride < hidden_in || w_row_stride < hidden_in || x_row_stride % 8 || w_row_stride % 8)
        return fail(TTT_ERR_INVALID_ARG, "row strides (%lld, %lld) must be multiples of 8 and >= hidden_in=%d",
                    (long long)x_row_stride, (long long)w_row_stride, hidden_in);
    if (tokens == 0) return TTT_OK;
    if (!x || !w || !cos_tab || !sin_tab || !pos || !q || !k || !v) return fail(TTT_ERR_INVALID_ARG, "a pointer is NULL");
    const void* ptrs[] = {x, w, cos_tab, sin_tab, q, k, v};
    for (const void* ptr : ptrs)
        if (reinterpret_cast<uintptr_t>(ptr) % 16) return fail(TTT_ERR_INVALID_ARG, "a tensor pointer is not 16-byte aligned");
    if (reinterpret_cast<uintptr_t>(pos) % 4) return fail(TTT_ERR_INVALID_ARG, "pos is not 4-byte aligned");
    hipError_t e = ttt::launch_qkv_rope(x, w, cos_tab, sin_tab, pos, q, k, v, tokens, hidden_in, hq, hkv, hkv, x_row_stride,
                                        w_row_stride, n_pos, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "projection kernel launch: %s", hipGetErrorString(e));
    return TTT_OK;
}

int ttt_o_proj_fwd(const void* o, const void* w, void* out, int64_t tokens, int32_t in_features, int32_t out_features,
                   int64_t o_row_stride, int64_t w_row_stride, int32_t dtype, void* hip_stream) {
    if (dtype != TTT_BF16) return fail(TTT_ERR_UNSUPPORTED, "dtype %d: the projection kernel is built for TTT_BF16", dtype);
    if (tokens < 0 || tokens > 0x7fffffffLL) return fail(TTT_ERR_INVALID_ARG, "tokens=%lld out of range", (long long)tokens);
    if (in_features < 64 || in_features % 64) return fail(TTT_ERR_INVALID_ARG, "in_features=%d must be a positive multiple of 64", in_features);
    if (out_features < 128 || out_features % 128 || out_features > 128 * 8192)
        return fail(TTT_ERR_INVALID_ARG, "out_features=%d must be a multiple of 128 in [128, 1048576]", out_features);
    if (o_row_stride < in_features || w_row_stride < in_features || o_row_stride % 8 || w_row_stride % 8)
        return fail(TTT_ERR_INVALID_ARG, "row strides (%lld, %lld) must be multiples of 8 and >= in_features=%d",
                    (long long)o_row_stride, (long long)w_row_stride, in_features);
    if (tokens == 0) return TTT_OK;
    if (!o || !w || !out) return fail(TTT_ERR_INVALID_ARG, "a pointer is NULL");
    if (reinterpret_cast<uintptr_t>(o) % 16 || reinterpret_cast<uintptr_t>(w) % 16 || reinterpret_cast<uintptr_t>(out) % 16)
        return fail(TTT_ERR_INVALID_ARG, "a tensor pointer is not 16-byte aligned");
    hipError_t e = ttt::launch_qkv_rope(o, w, nullptr, nullptr, nullptr, nullptr, nullptr, out, tokens, in_features, 0, 0,
                                        out_features / 128, o_row_stride, w_row_stride, 1, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(TTT_ERR_HIP, "projection kernel launch: %s", hipGetErrorString(e));
    return TTT_OK;
}

}  // extern "C"
