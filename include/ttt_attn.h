/*
 * ttt_attn.h -- C ABI of the MI355X (gfx950) training-time-test (TTT) attention library.
 *
 * Operation (EAGLE-3 draft layer unrolled over k TTT steps; Sec. 2.4 "Training-Time Test",
 * Alg. 1 "TTT Attention", Alg. 2 "BlockMask Construction", Sec. 4.2.1 "Sparse Tree Attention"):
 * step j appends its keys/values K_j, V_j (one block of T rows) to the cache and attends with Q_j.
 * Query (step j, token i, head h) reads kv head g = h / (hq/hkv) and sees
 *     block 0 keys at tokens m with  doc_start(i) <= m <= i       (causal prefix part of Alg. 2)
 *     block l keys at token i itself for 1 <= l <= j               (suffix / diagonal part of Alg. 2)
 * with one softmax over all of them:
 *     s = softmax_scale * <Q_j[i,h,:], K_l[m,g,:]>,  LSE_j[h,i] = log sum exp s,
 *     O_j[i,h,:] = sum exp(s - LSE) * V_l[m,g,:].
 * Nothing of size T x T is ever stored: the forward streams K_0/V_0 tiles with an online softmax
 * and keeps only O and LSE; the backward recomputes the probabilities from LSE.  Tiles that the
 * mask hides completely are never visited.
 *
 * The backward is the vector-Jacobian product of that forward for a cotangent dO_j of O_j
 * (LSE carries none):  D = <dO,O>, dp = <dO,V>, ds = p (dp - D),
 *     dQ_j[i,h]  = scale * sum ds * K_l[m,g]
 *     dK_l[m,g]  = scale * sum ds * Q_j[i,h]      dV_l[m,g] = sum p * dO_j[i,h]
 * the last two summed over every (step j, head h in group g, token i) that sees key (l,m).
 *
 * Memory: every tensor and the workspace are caller-owned DEVICE memory; step-pointer arrays and
 * cu_seqlens_host are HOST memory.  The library allocates no device memory, keeps no pointer after
 * a call returns, enqueues all work on `hip_stream` and never synchronises.
 *
 * Layouts (token-major, packed "thd"): Q_j, O_j, dO_j, dQ_j are [T, hq, head_dim]; K_j, V_j, dK_j,
 * dV_j are [T, hkv, head_dim]; element (t,h,c) at t*stride_token + h*stride_head + c (strides in
 * elements, head_dim contiguous).  LSE_j is [hq, T] fp32 contiguous (natural log).  A padded batch
 * [B,S,...] is passed as documents cu_seqlens = {0,S,2S,...}.  Pointers must be 16-byte aligned and
 * strides multiples of 8 elements.
 *
 * Errors: every entry point returns TTT_OK or a negative code and never throws or aborts;
 * ttt_attn_last_error() gives the message of the calling thread's last failure.
 */
#ifndef TTT_ATTN_H
#define TTT_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    TTT_OK = 0,
    TTT_ERR_INVALID_ARG = -1,  /* null pointer for a needed step, bad head counts / step range / strides / alignment, bad cu_seqlens */
    TTT_ERR_UNSUPPORTED = -2,  /* dtype / head_dim combination not built */
    TTT_ERR_WORKSPACE = -3,    /* workspace null or smaller than ttt_attn_workspace_bytes() */
    TTT_ERR_HIP = -4           /* a HIP call or kernel launch failed (checked without synchronising) */
};

enum { TTT_F32 = 0, TTT_BF16 = 1 };

/* Which call a workspace is sized for. */
enum {
    TTT_PASS_FWD = 0,
    TTT_PASS_BWD = 1,        /* ttt_attn_bwd with accumulate_dkv = 0 */
    TTT_PASS_BWD_ACCUM = 2   /* ttt_attn_bwd with accumulate_dkv = 1 (adds the fp32 carry buffers) */
};

/* The paper sweeps the TTT length from 1 to 17 (Sec. 7.2). */
#define TTT_MAX_STEPS 32

typedef struct ttt_attn_params {
    int32_t dtype;            /* TTT_F32 | TTT_BF16; Q,K,V,O,dO,dQ,dK,dV share it. LSE is always fp32. */
    int32_t k;                /* number of TTT steps = cache blocks, 1..TTT_MAX_STEPS */
    int32_t step_begin;       /* query steps handled by this call: [step_begin, step_end) within [0,k) */
    int32_t step_end;
    int32_t total_tokens;     /* T = cu_seqlens[n_docs] */
    int32_t n_docs;           /* documents in the packed batch (zero-length documents allowed) */
    int32_t hq;               /* query heads */
    int32_t hkv;              /* key/value heads; hq % hkv == 0; query head h reads kv head h/(hq/hkv) */
    int32_t head_dim;         /* 64 or 128 */
    float   softmax_scale;    /* the paper's 1/sqrt(d_k); passed explicitly */
    int64_t q_stride_token;   /* strides of Q, O, dO, dQ in elements */
    int64_t q_stride_head;
    int64_t kv_stride_token;  /* strides of K, V, dK, dV in elements */
    int64_t kv_stride_head;
} ttt_attn_params;

/*
 * Bytes of device workspace a call with these parameters needs (`pass` is one of TTT_PASS_*).
 * Returns 0 and sets the error message if the parameters are invalid.  The size depends on
 * total_tokens, head counts, head_dim, k and the pass only.
 */
size_t ttt_attn_workspace_bytes(const ttt_attn_params* params, int pass);

/*
 * Forward of steps [step_begin, step_end)  (Alg. 1 under the mask of Alg. 2, streamed as in
 * Sec. 4.2.1).
 *   q, k, v        host arrays of params->k device pointers (one per step).  Step j reads q[j] and
 *                  k[l], v[l] for l <= j; entries the call does not need may be NULL.
 *   cu_seqlens_dev device int32[n_docs+1]; cu_seqlens_host the same values in host memory
 *                  (validated: starts at 0, non-decreasing, ends at total_tokens).
 *   o, lse         host arrays of params->k device pointers; o[j] ([T,hq,d], params dtype) and
 *                  lse[j] ([hq,T] fp32) are fully overwritten for the steps in range, others untouched.
 *   workspace      device memory of at least ttt_attn_workspace_bytes(params, TTT_PASS_FWD) bytes,
 *                  256-byte aligned; contents need not survive the call.
 *   hip_stream     a hipStream_t (NULL = the default stream).
 * T == 0 or an empty step range is a successful no-op.
 */
int ttt_attn_fwd(const ttt_attn_params* params,
                 const void* const* q, const void* const* k, const void* const* v,
                 const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                 void* const* o, float* const* lse,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Backward of steps [step_begin, step_end): recomputes p = exp(s - LSE) tile by tile (nothing saved
 * but O and LSE, Sec. 4.2.1) and applies the softmax-attention VJP stated at the top of this file.
 *   q, k, v, o, lse, d_o   as in the forward (o, lse are its outputs; d_o[j] is the cotangent of
 *                          o[j]); needed for the steps in range (k, v for l < step_end).
 *   dq                     dq[j] written for the steps in range.
 *   dk, dv                 accumulate_dkv == 0: dk[l], dv[l] for every l < step_end are overwritten
 *                          with the sum over the query steps in range (the total gradient when the
 *                          range is [0,k)); blocks l >= step_end are untouched.
 *                          accumulate_dkv == 1 (step-at-a-time training order): calls must come in
 *                          DESCENDING step order with the SAME workspace, starting with the call
 *                          whose step_end == k (it resets the fp32 carry buffers in the workspace);
 *                          each call adds its steps' contributions to the carry, and writes
 *                          dk[l], dv[l] for the blocks l in [step_begin, step_end), which are
 *                          complete at that point.
 *   workspace              at least ttt_attn_workspace_bytes(params, TTT_PASS_BWD or
 *                          TTT_PASS_BWD_ACCUM) bytes, 256-byte aligned.  In accumulate mode its
 *                          contents carry state between the calls of one backward sweep.
 * dK_0/dV_0 partial sums are combined with fp32 atomics, so the last bits of dk[0], dv[0] can
 * differ between runs; everything else is deterministic.
 */
int ttt_attn_bwd(const ttt_attn_params* params,
                 const void* const* q, const void* const* k, const void* const* v,
                 const void* const* o, const float* const* lse, const void* const* d_o,
                 const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                 void* const* dq, void* const* dk, void* const* dv,
                 int accumulate_dkv,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same two operations with a step count per document ("Impact of Training-Time Test" in the
 * paper's Training Insights: the best TTT length depends on the task, and adjusting it per sample
 * is named as the way forward).  doc_steps_host[r] in 0..k (HOST array, n_docs entries) is the number
 * of TTT steps of document r: its tokens take part in steps j < doc_steps_host[r] only and own the
 * cache blocks l < doc_steps_host[r] only.  For the other (step, document) combinations nothing is
 * read and nothing is written: the rows of such a document in O_j, LSE_j, dQ_j, dK_l, dV_l keep
 * their contents.  Documents are independent, so the call is carried out as one pass per run of
 * consecutive documents with equal step count, one after the other on the stream, sharing the
 * workspace (sized by ttt_attn_workspace_bytes for the whole batch as before); group documents by
 * step count for the fewest passes.  The backward variant has no carry mode (accumulate_dkv = 0).
 * All other arguments, layouts and errors are those of ttt_attn_fwd / ttt_attn_bwd.
 */
int ttt_attn_fwd_docsteps(const ttt_attn_params* params, const int32_t* doc_steps_host, const void* const* q,
                          const void* const* k, const void* const* v, const int32_t* cu_seqlens_dev,
                          const int32_t* cu_seqlens_host, void* const* o, float* const* lse, void* workspace,
                          size_t workspace_bytes, void* hip_stream);
int ttt_attn_bwd_docsteps(const ttt_attn_params* params, const int32_t* doc_steps_host, const void* const* q,
                          const void* const* k, const void* const* v, const void* const* o, const float* const* lse,
                          const void* const* d_o, const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                          void* const* dq, void* const* dk, void* const* dv, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/*
 * ttt_attn_fwd for callers that cannot hand over (or allocate) a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid device allocation.  Same operation, arguments,
 * layouts and errors as ttt_attn_fwd, minus the workspace: the per-token document bounds that the
 * forward kernels read are kept in a device array built into the library (2 x TTT_STATIC_MAX_TOKENS
 * int32 = 4 MiB on every GPU the library runs on, held until the process ends).  The call allocates
 * no device memory and calls no allocating routine.  total_tokens > TTT_STATIC_MAX_TOKENS is
 * rejected with TTT_ERR_WORKSPACE.  All calls on one GPU share that array (it is fully rewritten
 * for the call's tokens before it is read, nothing needs clearing): calls that overlap in time on
 * the same GPU -- different streams or threads -- race; calls on one stream are ordered and safe.
 * The device that owns `hip_stream` must be the current device, as for every launch.
 */
#define TTT_STATIC_MAX_TOKENS 524288
int ttt_attn_fwd_static(const ttt_attn_params* params,
                        const void* const* q, const void* const* k, const void* const* v,
                        const int32_t* cu_seqlens_dev, const int32_t* cu_seqlens_host,
                        void* const* o, float* const* lse, void* hip_stream);

/* Message of the calling thread's most recent failing call ("" if none).  Never NULL. */
const char* ttt_attn_last_error(void);

/*
 * Diagnostics for measurement (not part of the method).  While enabled, ttt_attn_fwd/bwd bracket
 * every kernel they launch with a pair of HIP events on the caller's stream (host-side objects
 * only; still no device allocation and no synchronisation inside fwd/bwd).
 * ttt_attn_profile_enable returns the previous setting.
 * ttt_attn_profile_totals WAITS for the recorded events, adds the elapsed milliseconds up per
 * kernel name into names[i] (static strings) / total_ms[i] / launches[i] for at most `capacity`
 * distinct kernels, forgets the records and returns the number of names written.
 */
int ttt_attn_profile_enable(int on);
int ttt_attn_profile_totals(int capacity, const char** names, float* total_ms, int32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* TTT_ATTN_H */
