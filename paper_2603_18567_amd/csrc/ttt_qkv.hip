// Producer of Q_j, K_j, V_j (gfx950): the draft layer's query / key / value projection with the
// rotary position embedding applied in the epilogue, written in the layout the attention kernels
// read ([token, head, head_dim]) -- the tensors that Sec. 4.2.1 takes as given.
//
//   y[t, f] = sum_c x[t, c] w[f, c]            bf16 operands, fp32 accumulation on the matrix cores
//   Q, K heads: (y[i], y[i + d/2]) turned by the angle whose cos / sin the table holds at pos[t]
//   V heads:    y as it is
// With no rotated heads at all the same kernel is the plain projection y = x w^T (the output
// projection that reads O_j).
//
// One workgroup = 256 tokens x 2 heads (256 features), eight waves: wave (wm, wn) owns 64 tokens x
// the 128 features of head wn, i.e. 2 x 4 accumulator blocks of 32 x 32 (a 128-token variant, one
// block of tokens per wave, is taken when it fills the device in fewer, shorter rounds).  The accumulators hold
// y^T (row = feature, lane = token), so the two elements of a rotary pair (features i and i + 64)
// sit in the same lane at the same index of accumulator blocks nb and nb + 2: the rotation needs no
// exchange between lanes.  Both operands are contraction-contiguous in memory, so both are read
// from their LDS tiles as row fragments; 64-column slices of the x and w tiles stream through two
// LDS stages, filled by LDS-DMA copies.  Tiles are numbered so that the workgroups resident on one
// XCD form a block of token tiles x feature tiles: each x and w slice that enters that XCD's L2 is
// used by several of them.
#include "ttt_args.hpp"

namespace ttt {

constexpr double kSmallTileCost = 0.67;   // time of a 128-token tile relative to a 256-token tile (measured)

struct QkvArgs {
    const void* x;
    const void* w;
    const float* cos_tab;
    const float* sin_tab;
    const int* pos;
    void* q;
    void* k;
    void* v;
    int T, Hin, n_pos;
    int n_q, n_k, n_v;    // heads written to q (rotated), k (rotated), v (as they are); weight rows in this order
    int64_t x_st, w_st;   // row strides in elements
    int m_tiles, n_tiles, per_xcd;
    int n_first;          // first 256-feature tile of this launch (a call may be carried out as two launches)
};

template <typename T, int MB>
__global__ __launch_bounds__(512) void ttt_qkv_rope_kernel(const QkvArgs a) {
    static_assert(sizeof(T) == 2, "16-bit operands");
    using E = Elem<T>;
    using frag = typename E::frag;
    constexpr int D = 128;         // head_dim
    constexpr int MT = MB * 128;   // tokens per workgroup: MB blocks of 32 per wave
    constexpr int NT = 256;        // features per workgroup (two heads)
    constexpr int KT = 64;         // contraction slice per stage
    constexpr int NTHR = 512;
    using TL = Tile<T, KT>;
    constexpr int X_BYTES = MT * KT * E::kBytes;
    constexpr int STAGE_BYTES = X_BYTES + NT * KT * E::kBytes;
    typedef __attribute__((address_space(3))) char lds_char;

    extern __shared__ __align__(16) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

    // Workgroup ids go round-robin over the 8 XCDs; the 32 workgroups that an XCD holds at a time
    // (consecutive slots) are the 4 x 8 tiles of one block of the tile grid.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int blocks_n = (a.n_tiles + 7) / 8;
    const int blk = (slot >> 5) * 8 + xcd;              // block number: blocks are dealt out to the XCDs in turn
    const int in_blk = slot & 31;
    const int tm = (blk / blocks_n) * 4 + (in_blk >> 3), tn = (blk % blocks_n) * 8 + (in_blk & 7);
    if (tm >= a.m_tiles || tn >= a.n_tiles) return;
    const int m0 = tm * MT;
    const int n0 = (a.n_first + tn) * NT;
    const int n_feat = (a.n_q + a.n_k + a.n_v) * D;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 3, wn = wave >> 2;
    const int n = lane & 31, hh = lane >> 5;

    const T* X = static_cast<const T*>(a.x);
    const T* W = static_cast<const T*>(a.w);

    // ---- copies of one slice (KT columns) of the two tiles
    TileCopy<T, KT, MT, NTHR> copy_x;
    TileCopy<T, KT, NT, NTHR> copy_w;
    copy_x.init(a.x_st, tid);
    copy_w.init(a.w_st, tid);
    const bool x_inside = m0 + MT <= a.T, w_inside = n0 + NT <= n_feat;
    auto issue = [&](int ks, int s) {
        const uint32_t st = lds0 + s * STAGE_BYTES;
        const int c0 = ks * KT;
        if (x_inside) copy_x.copy(st, X + (int64_t)m0 * a.x_st + c0);
        else tile_load_async<T, KT, MT, NTHR>(smem + s * STAGE_BYTES, X + c0, a.x_st, m0, a.T - 1, tid);
        if (w_inside) copy_w.copy(st + X_BYTES, W + (int64_t)n0 * a.w_st + c0);
        else tile_load_async<T, KT, NT, NTHR>(smem + s * STAGE_BYTES + X_BYTES, W + c0, a.w_st, n0, n_feat - 1, tid);
    };

    // ---- per-lane LDS addresses of the row fragments (stage 0): chunk t of row n of a 32-row block
    uint32_t ra[KT / 16];
    {
        LaneFrags<T, KT> lf;
        lf.init(lane);
#pragma unroll
        for (int t = 0; t < KT / 16; ++t) ra[t] = lds0 + lf.row[t];
    }
    auto ld = [&](uint32_t addr) -> frag {
        return *reinterpret_cast<const __attribute__((address_space(3))) frag*>((uintptr_t)addr);
    };
    constexpr int BLK = 32 * TL::kRowBytes;   // one 32-row block of a tile

    f32x16 acc[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;

    const int n_k = a.Hin / KT;
    auto step = [&](int ks, auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        wait_async_copies();
        __syncthreads();   // slice ks is in LDS for everyone; everyone is done with the other stage
        if (ks + 1 < n_k) issue(ks + 1, ST ^ 1);
        const uint32_t xo = ST * STAGE_BYTES + (wm * MB) * BLK;
        const uint32_t wo = ST * STAGE_BYTES + X_BYTES + (wn * 4) * BLK;
        // the fragments of chunk t + 1 are requested before the matrix instructions of chunk t are issued
        frag xf[KT / 16][MB], wf[KT / 16][4];
        auto request = [&](int t) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) xf[t][mb] = ld(ra[t] + xo + mb * BLK);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) wf[t][nb] = ld(ra[t] + wo + nb * BLK);
        };
        request(0);
#pragma unroll
        for (int t = 0; t < KT / 16; ++t) {
            if (t + 1 < KT / 16) request(t + 1);
            issue_fence();
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) acc[mb][nb] = mma(wf[t][nb], xf[t][mb], acc[mb][nb]);
        }
    };
    issue(0, 0);
    for (int ks = 0; ks < n_k; ks += 2) {
        step(ks, IntC<0>{});
        if (ks + 1 < n_k) step(ks + 1, IntC<1>{});
    }

    // ---- epilogue: rotate, convert, store.  Lane (n, hh) holds, of accumulator block (mb, nb), the
    // features 32 nb + 8 k4 + 4 hh + 0..3 (k4 = 0..3) of token m0 + 64 wm + 32 mb + n.
    const int head = n0 / D + wn;
    if (head >= a.n_q + a.n_k + a.n_v) return;
    const bool rotate = head < a.n_q + a.n_k;
    T* out;
    int64_t out_st;
    if (head < a.n_q) {
        out = static_cast<T*>(a.q) + (int64_t)head * D;
        out_st = (int64_t)a.n_q * D;
    } else if (head < a.n_q + a.n_k) {
        out = static_cast<T*>(a.k) + (int64_t)(head - a.n_q) * D;
        out_st = (int64_t)a.n_k * D;
    } else {
        out = static_cast<T*>(a.v) + (int64_t)(head - a.n_q - a.n_k) * D;
        out_st = (int64_t)a.n_v * D;
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = m0 + wm * (32 * MB) + mb * 32 + n;
        if (m >= a.T) continue;
        T* row = out + (int64_t)m * out_st;
        if (rotate) {
            int p = a.pos[m];
            p = p < 0 ? 0 : (p >= a.n_pos ? a.n_pos - 1 : p);
            const float* cr = a.cos_tab + (int64_t)p * (D / 2);
            const float* sr = a.sin_tab + (int64_t)p * (D / 2);
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int k4 = 0; k4 < 4; ++k4) {
                    const int i0 = 32 * nb + 8 * k4 + 4 * hh;
                    const f32x4 c4 = *reinterpret_cast<const f32x4*>(cr + i0);
                    const f32x4 s4 = *reinterpret_cast<const f32x4*>(sr + i0);
                    float lo[4], hi[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float y0 = acc[mb][nb][4 * k4 + e], y1 = acc[mb][nb + 2][4 * k4 + e];
                        lo[e] = y0 * c4[e] - y1 * s4[e];
                        hi[e] = y1 * c4[e] + y0 * s4[e];
                    }
                    gstore_vec4<T>(row + i0, lo[0], lo[1], lo[2], lo[3]);
                    gstore_vec4<T>(row + D / 2 + i0, hi[0], hi[1], hi[2], hi[3]);
                }
        } else {
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int k4 = 0; k4 < 4; ++k4) {
                    const int i0 = 32 * nb + 8 * k4 + 4 * hh;
                    gstore_vec4<T>(row + i0, acc[mb][nb][4 * k4], acc[mb][nb][4 * k4 + 1], acc[mb][nb][4 * k4 + 2],
                                   acc[mb][nb][4 * k4 + 3]);
                }
        }
    }
}

template <int MB>
static hipError_t launch_qkv_rope_t(QkvArgs& a, hipStream_t stream) {
    using T = __bf16;
    constexpr int MT = MB * 128;
    constexpr int LDS = 2 * (MT + 256) * 64 * 2;
    auto kern = ttt_qkv_rope_kernel<T, MB>;
    static LdsOptIn lds_opt_in;
    if (hipError_t e = lds_opt_in.ensure((const void*)kern, LDS); e != hipSuccess) return e;
    a.m_tiles = (a.T + MT - 1) / MT;
    // blocks of 4 x 8 tiles, dealt out to the 8 XCDs in turn: 32 slots per block and XCD
    const int64_t blocks = (int64_t)((a.m_tiles + 3) / 4) * ((a.n_tiles + 7) / 8);
    a.per_xcd = (int)((blocks + 7) / 8) * 32;
    const int64_t grid = 8 * (int64_t)a.per_xcd;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    ProfileScope prof("ttt_qkv_rope_kernel", stream);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(512), LDS, stream, a);
    return hipGetLastError();
}

// n_q + n_k heads are rotated and go to q and k, n_v heads go to v as they are.  With n_q = n_k = 0 the
// call is a plain projection y = x w^T into v ([tokens, n_v * 128]).
hipError_t launch_qkv_rope(const void* x, const void* w, const float* cos_tab, const float* sin_tab, const int* pos, void* q,
                           void* k, void* v, int64_t tokens, int hidden_in, int n_q, int n_k, int n_v, int64_t x_st,
                           int64_t w_st, int n_pos, hipStream_t stream) {
    // 64 rows of x or w are addressed with 32-bit byte offsets
    if (x_st * 64 * 2 >= (int64_t)1 << 32 || w_st * 64 * 2 >= (int64_t)1 << 32) return hipErrorInvalidValue;
    QkvArgs a;
    a.x = x;
    a.w = w;
    a.cos_tab = cos_tab;
    a.sin_tab = sin_tab;
    a.pos = pos;
    a.q = q;
    a.k = k;
    a.v = v;
    a.T = (int)tokens;
    a.Hin = hidden_in;
    a.n_q = n_q;
    a.n_k = n_k;
    a.n_v = n_v;
    a.n_pos = n_pos;
    a.x_st = x_st;
    a.w_st = w_st;
    const int n_tiles = ((n_q + n_k + n_v) * 128 + 255) / 256;
    // One workgroup per compute unit at a time, so a launch takes rounds x tile time.  Token tiles of
    // 256 rows are the efficient ones; a tile of 128 rows costs a little more than half of one.  The
    // feature tiles are cut into a first part done with 256-row tiles and a rest done with 128-row
    // tiles (either may be empty) so that both launches fill their last round: 4096 tokens x 6144
    // features are 16 x 24 large tiles = one and a half rounds of 256; as 16 x 16 large tiles plus
    // 32 x 8 small ones they are two full rounds costing 1 + 0.67.
    int n_cu = 0;
    if (hipError_t e = current_device_cu_count(n_cu); e != hipSuccess) return e;
    const int64_t m_big = (tokens + 255) / 256, m_small = (tokens + 127) / 128;
    int best_nb = n_tiles;
    double best_cost = -1.;
    for (int nb = n_tiles; nb >= 0; --nb) {
        const double cost = (double)((m_big * nb + n_cu - 1) / n_cu) * 1.0 +
                            (double)((m_small * (n_tiles - nb) + n_cu - 1) / n_cu) * kSmallTileCost +
                            (nb > 0 && nb < n_tiles ? 0.02 : 0.);   // a second launch is not free
        if (best_cost < 0. || cost < best_cost - 1e-9) {
            best_cost = cost;
            best_nb = nb;
        }
    }
    if (best_nb > 0) {
        a.n_first = 0;
        a.n_tiles = best_nb;
        if (hipError_t e = launch_qkv_rope_t<2>(a, stream); e != hipSuccess) return e;
    }
    if (best_nb < n_tiles) {
        a.n_first = best_nb;
        a.n_tiles = n_tiles - best_nb;
        if (hipError_t e = launch_qkv_rope_t<1>(a, stream); e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace ttt
