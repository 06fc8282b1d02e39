/*
 * ttt_qkv.h -- C ABI of the producer of Q_j, K_j, V_j on MI355X (gfx950): the draft layer's query /
 * key / value projection with the rotary position embedding applied in the epilogue.
 *
 * Operation: the training-time-test attention (Sec. 4.2.1) takes the per-step tensors Q_j, K_j, V_j
 * as given; this call makes them for one step, in the [token, head, head_dim] layout that
 * ttt_attn_fwd / ttt_attn_bwd read, so that no separate rotation or re-layout pass over them exists.
 *     y[t, f] = sum_c x[t, c] * w[f, c]                  f over (hq + 2 hkv) heads of width head_dim
 *     Q and K heads, i < head_dim/2, c = cos_tab[pos[t], i], s = sin_tab[pos[t], i]:
 *         out[i]              = y[i] * c - y[i + head_dim/2] * s
 *         out[i + head_dim/2] = y[i + head_dim/2] * c + y[i] * s
 *     V heads: out = y
 * The paper does not spell this op out; the conventions are those of the model families it trains
 * drafts for: no bias, weight rows ordered Q heads, K heads, V heads, "rotate half" pairing.  The
 * angle table and the per-token position ids are inputs, so base frequency, scaling and the
 * position ids of a TTT step stay with the caller.
 *
 * Arguments (all pointers are caller-owned DEVICE memory, 16-byte aligned except `pos`):
 *   x        [tokens, hidden_in]            bf16, row stride x_row_stride elements (multiple of 8)
 *   w        [(hq + 2 hkv) * head_dim, hidden_in]  bf16, row stride w_row_stride (multiple of 8)
 *   cos_tab, sin_tab  [n_pos, head_dim / 2]  fp32, contiguous
 *   pos      [tokens]                        int32; values outside [0, n_pos) are clamped into it
 *   q [tokens, hq, head_dim], k [tokens, hkv, head_dim], v [tokens, hkv, head_dim]  bf16, contiguous,
 *            fully overwritten
 *   hidden_in a multiple of 64; head_dim = 128; dtype = TTT_BF16 (ttt_attn.h).  Products are
 *   accumulated in fp32 on the matrix cores, the rotation is done in fp32, results are rounded to
 *   bf16 once.
 *
 * The library allocates nothing, enqueues one kernel on `hip_stream` and never synchronises.
 * Errors: returns TTT_OK or a negative TTT_ERR_* code (ttt_attn.h); ttt_attn_last_error() has the
 * message.  tokens = 0 is a no-op.
 */
#ifndef TTT_QKV_H
#define TTT_QKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int ttt_qkv_rope_fwd(const void* x, const void* w, const float* cos_tab, const float* sin_tab, const int32_t* pos, void* q,
                     void* k, void* v, int64_t tokens, int32_t hidden_in, int32_t hq, int32_t hkv, int32_t head_dim,
                     int64_t x_row_stride, int64_t w_row_stride, int32_t n_pos, int32_t dtype, void* hip_stream);

/*
 * The consumer on the other side of the attention: the output projection that reads O_j as the
 * attention kernels wrote it ([tokens, hq * head_dim] is [tokens, hq, head_dim] seen as a matrix):
 *     out[t, f] = sum_c o[t, c] * w[f, c]
 * Same kernel as above without the rotation (the paper names no fusion on this side; the call exists
 * so that the attention block of the draft layer can be driven through this library alone).
 *   o   [tokens, in_features]        bf16, row stride o_row_stride elements (multiple of 8)
 *   w   [out_features, in_features]  bf16, row stride w_row_stride (multiple of 8)
 *   out [tokens, out_features]       bf16, contiguous, fully overwritten
 *   in_features a multiple of 64, out_features a multiple of 128; dtype = TTT_BF16.
 * Memory, stream and error conventions as for ttt_qkv_rope_fwd.
 */
int ttt_o_proj_fwd(const void* o, const void* w, void* out, int64_t tokens, int32_t in_features, int32_t out_features,
                   int64_t o_row_stride, int64_t w_row_stride, int32_t dtype, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TTT_QKV_H */
