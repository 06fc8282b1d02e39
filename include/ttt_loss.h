/*
 * ttt_loss.h -- C ABI of the in-place backward of the log-softmax loss on MI355X (gfx950).
 *
 * Operation (Sec. 4.2.2 "Memory-Efficient Gradient Computation", Alg. 3): for every row r (one token
 * position of one training-time-test step) with logits z[r, 0..V), target weights p[r, 0..V) and
 * upstream gradient g[r], the gradient of the loss  -g[r] * sum_v p[r,v] * log softmax(z[r,:])[v]
 * with respect to the logits,
 *     softmax(z[r,:])[v] * g[r] * sum_u p[r,u]  -  g[r] * p[r,v],
 * is written over the logits: no gradient buffer of the size of the logits exists.  g is one fp32
 * value per row (loss weight / position mask times the upstream scalar; rows with g = 0 become
 * exactly zero); p need not be normalised.
 *
 * Memory: `logits`, `target` and `grad` are caller-owned DEVICE memory; logits and target are
 * [n_rows, vocab] with the given row strides (in elements, vocab contiguous), both of `dtype`
 * (TTT_F32 or TTT_BF16 of ttt_attn.h); arithmetic is fp32.  16-byte aligned pointers with strides
 * that are multiples of 16 bytes take the vectorised path; anything else is handled element by
 * element.  The library allocates nothing, enqueues one kernel on `hip_stream` and never
 * synchronises.  `logits` is read and then overwritten; `target` and `grad` are only read.
 *
 * Errors: returns TTT_OK or a negative TTT_ERR_* code (ttt_attn.h); ttt_attn_last_error() has the
 * message.  n_rows = 0 is a no-op.
 */
#ifndef TTT_LOSS_H
#define TTT_LOSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int ttt_loss_bwd_inplace(void* logits, const void* target, const float* grad, int64_t n_rows, int32_t vocab,
                         int64_t logits_row_stride, int64_t target_row_stride, int32_t dtype, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TTT_LOSS_H */
