// In-place backward of the log-softmax loss (Sec. 4.2.2, Alg. 3) for gfx950: one workgroup of
// 1024 threads per row.  A row of up to kCacheIters * 1024 sixteen-byte vectors (32768 fp32 or
// 65536 bf16 values: the draft vocabularies) is read ONCE into registers -- logits and target --
// reduced (maximum, sum of exponentials, sum of the target) and written back as the gradient, so
// the HBM traffic is the algorithmic 3 * V * element size per row.  Longer rows are streamed twice
// (online maximum / sum in the first sweep).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ttt_attn.h"
#include "../../include/ttt_loss.h"
#include "ttt_args.hpp"

namespace ttt {

constexpr int kLossThreads = 1024;
constexpr int kCacheIters = 8;
constexpr float kLog2eL = 1.44269504088896340736f;

template <typename T> struct LossVec;
template <> struct LossVec<float> {
    static constexpr int N = 4;
    typedef f32x4 raw;
    TTT_DEV static void unpack(const raw& r, float (&o)[N]) {
#pragma unroll
        for (int i = 0; i < N; ++i) o[i] = r[i];
    }
    TTT_DEV static raw pack(const float (&o)[N]) { return raw{o[0], o[1], o[2], o[3]}; }
};
template <> struct LossVec<__bf16> {
    static constexpr int N = 8;
    typedef bf16x8 raw;
    TTT_DEV static void unpack(const raw& r, float (&o)[N]) {
#pragma unroll
        for (int i = 0; i < N; ++i) o[i] = (float)r[i];
    }
    TTT_DEV static raw pack(const float (&o)[N]) {
        raw r;
#pragma unroll
        for (int i = 0; i < N; ++i) r[i] = (__bf16)o[i];
        return r;
    }
};

// block-wide reductions over 16 waves: wave butterflies, then one LDS round
TTT_DEV float wave_max(float v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v = fmaxf(v, __shfl_xor(v, s, 64));
    return v;
}
TTT_DEV float wave_sum(float v) {
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
    return v;
}

// One row: element e of this thread's vector number `it` is column ((it * 1024 + tid) * N + e).
template <typename T, bool VEC, bool CACHED>
__global__ __launch_bounds__(kLossThreads) void ttt_loss_bwd_kernel(T* __restrict__ logits, const T* __restrict__ target,
                                                                    const float* __restrict__ grad, int vocab,
                                                                    int64_t z_stride, int64_t p_stride) {
    using LV = LossVec<T>;
    constexpr int N = LV::N;
    __shared__ float red[3][kLossThreads / 64];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int64_t row = blockIdx.x;
    T* z = logits + row * z_stride;
    const T* p = target + row * p_stride;
    const float g = grad[row];
    const int n_iter = (vocab + N * kLossThreads - 1) / (N * kLossThreads);

    // one 16-byte vector of a row, kept packed in registers; columns past the row's end read as `fill`
    auto load_raw = [&](const T* src, int it, float fill) -> typename LV::raw {
        const int c0 = (it * kLossThreads + tid) * N;
        if (VEC && c0 + N <= vocab) return *reinterpret_cast<const typename LV::raw*>(src + c0);
        float o[N];
#pragma unroll
        for (int e = 0; e < N; ++e) o[e] = c0 + e < vocab ? (float)src[c0 + e] : fill;
        return LV::pack(o);
    };
    auto load = [&](const T* src, int it, float (&o)[N], float fill) { LV::unpack(load_raw(src, it, fill), o); };
    auto store = [&](int it, const float (&o)[N]) {
        const int c0 = (it * kLossThreads + tid) * N;
        if (VEC && c0 + N <= vocab) {
            *reinterpret_cast<typename LV::raw*>(z + c0) = LV::pack(o);
        } else {
#pragma unroll
            for (int e = 0; e < N; ++e)
                if (c0 + e < vocab) z[c0 + e] = (T)o[e];
        }
    };
    auto block_reduce = [&](float a, float b, float c, bool first_is_max, float& ra, float& rb, float& rc) {
        a = first_is_max ? wave_max(a) : wave_sum(a);
        b = wave_sum(b);
        c = wave_sum(c);
        __syncthreads();   // the previous round's readers are done
        if (lane == 0) {
            red[0][wave] = a;
            red[1][wave] = b;
            red[2][wave] = c;
        }
        __syncthreads();
        ra = red[0][0];
        rb = red[1][0];
        rc = red[2][0];
#pragma unroll
        for (int w = 1; w < kLossThreads / 64; ++w) {
            ra = first_is_max ? fmaxf(ra, red[0][w]) : ra + red[0][w];
            rb += red[1][w];
            rc += red[2][w];
        }
    };

    if constexpr (CACHED) {
        typename LV::raw zc[kCacheIters], pc[kCacheIters];
        float m = -INFINITY, sp = 0.f;
#pragma unroll
        for (int it = 0; it < kCacheIters; ++it) {
            if (it < n_iter) {
                zc[it] = load_raw(z, it, -INFINITY);
                pc[it] = load_raw(p, it, 0.f);
                float zv[N], pv[N];
                LV::unpack(zc[it], zv);
                LV::unpack(pc[it], pv);
#pragma unroll
                for (int e = 0; e < N; ++e) {
                    m = fmaxf(m, zv[e]);
                    sp += pv[e];
                }
            }
        }
        float M, SP, unused;
        block_reduce(m, sp, 0.f, true, M, SP, unused);
        const float mc = M * kLog2eL;
        float l = 0.f;
#pragma unroll
        for (int it = 0; it < kCacheIters; ++it) {
            if (it < n_iter) {
                float zv[N];
                LV::unpack(zc[it], zv);
#pragma unroll
                for (int e = 0; e < N; ++e) l += fast_exp2(fmaf(zv[e], kLog2eL, -mc));   // exp(z - max); 0 past the end
            }
        }
        float L, u1, u2;
        block_reduce(l, 0.f, 0.f, false, L, u1, u2);
        const float w = g * SP / L;     // pi * s = exp(z - max) * (s / sum)
#pragma unroll
        for (int it = 0; it < kCacheIters; ++it) {
            if (it < n_iter) {
                float zv[N], pv[N], o[N];
                LV::unpack(zc[it], zv);
                LV::unpack(pc[it], pv);
#pragma unroll
                for (int e = 0; e < N; ++e) o[e] = fmaf(fast_exp2(fmaf(zv[e], kLog2eL, -mc)), w, -pv[e] * g);
                store(it, o);
            }
        }
    } else {
        // first sweep: online maximum and sum of exponentials per thread, merged across the block
        float m = -INFINITY, l = 0.f, sp = 0.f;
        for (int it = 0; it < n_iter; ++it) {
            float zv[N], pv[N];
            load(z, it, zv, -INFINITY);
            load(p, it, pv, 0.f);
            float mx = m;
#pragma unroll
            for (int e = 0; e < N; ++e) mx = fmaxf(mx, zv[e]);
            if (mx > m) {
                l *= m == -INFINITY ? 0.f : fast_exp2((m - mx) * kLog2eL);
                m = mx;
            }
#pragma unroll
            for (int e = 0; e < N; ++e) {
                if (m != -INFINITY) l += fast_exp2((zv[e] - m) * kLog2eL);
                sp += pv[e];
            }
        }
        float M, SP, unused;
        block_reduce(m, sp, 0.f, true, M, SP, unused);
        l *= m == -INFINITY ? 0.f : fast_exp2((m - M) * kLog2eL);
        float L, u1, u2;
        block_reduce(l, 0.f, 0.f, false, L, u1, u2);
        const float w = g * SP / L;
        const float mc = M * kLog2eL;
        for (int it = 0; it < n_iter; ++it) {
            float zv[N], pv[N], o[N];
            load(z, it, zv, -INFINITY);
            load(p, it, pv, 0.f);
#pragma unroll
            for (int e = 0; e < N; ++e) o[e] = fmaf(fast_exp2(fmaf(zv[e], kLog2eL, -mc)), w, -pv[e] * g);
            store(it, o);
        }
    }
}

template <typename T>
static hipError_t launch_loss_t(void* logits, const void* target, const float* grad, int64_t n_rows, int vocab,
                                int64_t zs, int64_t ps, hipStream_t stream) {
    constexpr int N = LossVec<T>::N;
    const bool vec = (reinterpret_cast<uintptr_t>(logits) & 15) == 0 && (reinterpret_cast<uintptr_t>(target) & 15) == 0 &&
                     zs % N == 0 && ps % N == 0;
    const bool cached = (int64_t)vocab <= (int64_t)kCacheIters * kLossThreads * N;
    T* z = static_cast<T*>(logits);
    const T* p = static_cast<const T*>(target);
    const dim3 grid((unsigned)n_rows), block(kLossThreads);
    ProfileScope prof("ttt_loss_bwd_kernel", stream);
    if (vec && cached) hipLaunchKernelGGL((ttt_loss_bwd_kernel<T, true, true>), grid, block, 0, stream, z, p, grad, vocab, zs, ps);
    else if (vec) hipLaunchKernelGGL((ttt_loss_bwd_kernel<T, true, false>), grid, block, 0, stream, z, p, grad, vocab, zs, ps);
    else if (cached) hipLaunchKernelGGL((ttt_loss_bwd_kernel<T, false, true>), grid, block, 0, stream, z, p, grad, vocab, zs, ps);
    else hipLaunchKernelGGL((ttt_loss_bwd_kernel<T, false, false>), grid, block, 0, stream, z, p, grad, vocab, zs, ps);
    return hipGetLastError();
}

hipError_t launch_loss_bwd(int dtype, void* logits, const void* target, const float* grad, int64_t n_rows, int vocab,
                           int64_t zs, int64_t ps, hipStream_t stream) {
    if (dtype == TTT_BF16) return launch_loss_t<__bf16>(logits, target, grad, n_rows, vocab, zs, ps, stream);
    return launch_loss_t<float>(logits, target, grad, n_rows, vocab, zs, ps, stream);
}

}  // namespace ttt
