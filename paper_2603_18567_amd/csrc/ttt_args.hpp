// Kernel argument blocks (host fills, device reads) and the launcher prototypes that connect the
// C-ABI file to the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "ttt_device.hpp"

namespace ttt {

constexpr int kMaxSteps = 32;

struct Geometry {
    int T;               // packed tokens
    int k;               // cache blocks
    int step_begin, n_steps;
    int hq, hkv, G;
    float scale;         // softmax_scale
    float scale_log2;    // softmax_scale * log2(e)
    int64_t q_st, q_sh;  // strides (elements) of Q/O/dO/dQ
    int64_t kv_st, kv_sh;
    int64_t lse_st;      // row (head) stride of LSE_j in elements (the packed token count of the whole batch)
};

struct FwdArgs {
    Geometry geo;
    const void* q[kMaxSteps];
    const void* k[kMaxSteps];
    const void* v[kMaxSteps];
    void* o[kMaxSteps];
    float* lse[kMaxSteps];
    const int* tok_start;   // [T] first token of each token's document
    int n_tiles;            // query tiles over the packed token axis
    int pack_log2;          // log2 of the query heads (of one kv group) that share a workgroup
    int diag_lds;           // 1: the rows of the diagonal keys are staged in LDS (64-row workgroups)
    HeadMap map;
};

struct BwdArgs {
    Geometry geo;
    const void* q[kMaxSteps];
    const void* k[kMaxSteps];
    const void* v[kMaxSteps];
    const void* o[kMaxSteps];
    const float* lse[kMaxSteps];
    const void* d_o[kMaxSteps];
    void* dq[kMaxSteps];
    void* dk[kMaxSteps];
    void* dv[kMaxSteps];
    const int* tok_start;   // [T]
    const int* tok_end;     // [T] one past the last token of each token's document
    float* delta;           // [n_steps][hq][T]  D = <dO, O>
    float* lse2;            // [n_steps][hq][T]  LSE * log2(e), the exponent offset the kernels use
    float* dk0_acc;         // [T][hkv][d] fp32, block-0 partial sums (atomics)
    float* dv0_acc;
    float* dkl_acc;         // [k-1][T][hkv][d] fp32 carry for blocks l>=1 (accumulate mode), else null
    float* dvl_acc;
    int accumulate;         // 0/1
    int carry_reset;        // accumulate mode: this call starts the sweep (carry is overwritten, not read)
    int n_tiles;            // tiles of the kernel being launched
    int n_split;            // dK/dV kernel: ways the (step, head) list of one kv tile is split
    int n_units;            // dK/dV kernel (16-bit): (key tile, query chunk) units per kv head and split
    int chunk_blocks;       // dK/dV kernel (16-bit): 32-row query blocks per chunk (a multiple of 4)
    HeadMap map;
    // host side only (the launchers' work-split model reads the document structure from it)
    const int32_t* cu_host; // cu_seqlens of the documents of this call: n_docs + 1 entries, first entry = cu_base
    int cu_base;
    int n_docs;
};

// launchers (defined in the kernel files); all enqueue on `stream` and return the launch status
hipError_t launch_tok_bounds(const int* cu_dev, int base, int n_docs, int T, int* tok_start, int* tok_end, hipStream_t stream);
hipError_t launch_fwd(int dtype, int head_dim, FwdArgs& a, hipStream_t stream);
hipError_t launch_bwd(int dtype, int head_dim, BwdArgs& a, hipStream_t stream);
hipError_t launch_loss_bwd(int dtype, void* logits, const void* target, const float* grad, int64_t n_rows, int vocab,
                           int64_t logits_row_stride, int64_t target_row_stride, hipStream_t stream);

hipError_t launch_qkv_rope(const void* x, const void* w, const float* cos_tab, const float* sin_tab, const int* pos, void* q,
                           void* k, void* v, int64_t tokens, int hidden_in, int n_q, int n_k, int n_v, int64_t x_st,
                           int64_t w_st, int n_pos, hipStream_t stream);

// Per-device host-side state of the launchers.  A kernel's opt-in to more than 48 KB of dynamic LDS
// is an attribute of (kernel, device): LdsOptIn sets it the first time a kernel instantiation is
// launched on each device (one bit per device index; indices past 63 simply set it every time).
struct LdsOptIn {
    std::atomic<uint64_t> done{0};
    hipError_t ensure(const void* kernel, int bytes) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        const bool tracked = dev >= 0 && dev < 64;
        if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1u)) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e == hipSuccess && tracked) done.fetch_or((uint64_t)1 << dev, std::memory_order_release);
        return e;
    }
};
// compute units of the current device (cached per device index; 256 if the runtime reports none)
inline hipError_t current_device_cu_count(int& n_cu) {
    static std::atomic<int> cache[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && (n_cu = cache[dev].load(std::memory_order_relaxed)) > 0) return hipSuccess;
    if ((e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    if (n_cu <= 0) n_cu = 256;
    if (tracked) cache[dev].store(n_cu, std::memory_order_relaxed);
    return hipSuccess;
}

// Diagnostics (off by default): brackets one kernel launch with HIP events on its stream so that
// a caller can read per-kernel durations afterwards (ttt_attn_profile_totals).
void profile_begin(const char* kernel_name, hipStream_t stream);
void profile_end(hipStream_t stream);
struct ProfileScope {
    hipStream_t stream;
    ProfileScope(const char* name, hipStream_t s) : stream(s) { profile_begin(name, s); }
    ~ProfileScope() { profile_end(stream); }
};

}  // namespace ttt
