// Forward TTT attention kernel (gfx950): streams K_0/V_0 tiles through LDS with an online softmax
// (Sec. 4.2.1: nothing of size T x T is stored), then folds in the <= j diagonal keys of the later
// cache blocks (suffix part of Alg. 2) row by row on the vector ALU.
//
// Work split: one workgroup = one tile of QT consecutive packed tokens x one query head x one step.
// Each wave owns QB blocks of 32 query rows and keeps, per lane, everything that belongs to ONE
// query row: scores are computed transposed (S^T = K Q^T) so that the accumulator's column index --
// the lane -- is the query row; running max / sum / rescale are then per-lane scalars and the only
// cross-lane traffic of the softmax is one exchange between the two lane halves.  The same layout
// lets exp(S^T) be fed straight back as the B operand of O^T = V^T P^T.
//
// Tiles are cut over the packed token axis, not per document: a row's visible prefix is
// [tok_start[i], i], so a wave visits the kv tiles that intersect [tok_start[first row], last row]
// and nothing else; tiles strictly inside that range for every row skip the mask code.
#include <type_traits>

#include "ttt_args.hpp"

namespace ttt {

template <typename T, int D, int QB, int NW, int MINB>
__global__ __launch_bounds__(NW * 64, MINB) void ttt_fwd_kernel(const FwdArgs a) {
    using E = Elem<T>;
    using frag = typename E::frag;
    constexpr int KT = 64;                // kv rows per LDS tile
    constexpr int KB = KT / 32;
    constexpr int QT = NW * QB * 32;
    constexpr int DC = D / 16;            // contraction chunks over head_dim
    constexpr int DB = D / 32;            // 32-wide blocks of head_dim
    constexpr int NT = NW * 64;
    constexpr int TILE_BYTES = KT * D * E::kBytes;
    constexpr float kLazy = 8.f;          // log2 of the largest p tolerated before the reference max moves
    constexpr bool kDiagLds = sizeof(T) == 2 && KT == 64;   // diagonal rows may be staged in LDS (64-row tiles)
    constexpr int kDiagSlots = 3;         // blocks whose rows are staged at once

    extern __shared__ __align__(16) char smem[];
    // LDS: K stage 0, K stage 1, V stage 0, V stage 1
    auto sK = [&](int s) -> char* { return smem + s * TILE_BYTES; };
    auto sV = [&](int s) -> char* { return smem + (2 + s) * TILE_BYTES; };

    const Geometry& geo = a.geo;
    int g, rest;
    if (!decode_block(a.map, blockIdx.x, g, rest)) return;
    // The waves of a workgroup are 2^pack_log2 query heads of the kv group x NW >> pack_log2 blocks of
    // rows: heads that share K_0 / V_0 also share the key range, so all waves of a workgroup see
    // (almost) the same number of key tiles and none idles while the tile on the diagonal is finished.
    const int pk = a.pack_log2;
    const int n_hgrp = geo.G >> pk;
    const int hgrp = rest % n_hgrp;
    rest /= n_hgrp;
    const int j = geo.step_begin + rest % geo.n_steps;
    const int tile = a.n_tiles - 1 - rest / geo.n_steps;   // long-prefix tiles first

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = g * geo.G + (hgrp << pk) + (wave & ((1 << pk) - 1));
    const int n = lane & 31, hh = lane >> 5;
    const int Tn = geo.T;   // packed tokens
    const int qt_rows = QT >> pk;   // rows of a workgroup
    const int q_tile0 = tile * qt_rows;
    const int wq0 = q_tile0 + (wave >> pk) * (QB * 32);
    const bool active = wq0 < Tn;

    const T* Qj = static_cast<const T*>(a.q[j]) + (int64_t)h * geo.q_sh;
    const T* K0 = static_cast<const T*>(a.k[0]) + (int64_t)g * geo.kv_sh;
    const T* V0 = static_cast<const T*>(a.v[0]) + (int64_t)g * geo.kv_sh;

    // rows of this lane, their clamped copies and document starts
    int qi[QB], qc[QB], st[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qi[qb] = wq0 + 32 * qb + n;
        qc[qb] = qi[qb] < Tn ? qi[qb] : Tn - 1;
        st[qb] = a.tok_start[qc[qb]];
    }
    const int hi_w = min(wq0 + QB * 32 - 1, Tn - 1);
    const int lo_w = active ? __builtin_amdgcn_readfirstlane(a.tok_start[min(wq0, Tn - 1)]) : 0;
    const int st_hi = active ? __builtin_amdgcn_readfirstlane(a.tok_start[hi_w]) : 0;
    const int lo = __builtin_amdgcn_readfirstlane(a.tok_start[q_tile0]);
    const int hi = min(q_tile0 + qt_rows - 1, Tn - 1);
    const int u_lo = lo / KT, u_hi = hi / KT;

    // Q as the stationary B operand: lane (n,hh) holds Q[row n][16t + 8hh .. +8]
    frag qf[QB][DC];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int t = 0; t < DC; ++t)
            qf[qb][t] = gload_frag<T>(Qj + (int64_t)qc[qb] * geo.q_st + t * 16 + hh * 8);

    f32x16 oacc[QB][DB];
    float m[QB], l[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m[qb] = -INFINITY;
        l[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[qb][db][i] = 0.f;
    }
    const float c = geo.scale_log2;

    LaneFrags<T, D> lf;
    lf.init(lane);

    // K_0 / V_0 rows of tile u -> stage s.  Tiles that lie inside the tensor (all but the last one)
    // take the copy with precomputed lane offsets.
    constexpr bool kFastCopy = sizeof(T) == 2;
    struct NoCopy { TTT_DEV void init(int64_t, int) {} };
    typename std::conditional<kFastCopy, TileCopy<T, D, KT, NT>, NoCopy>::type tile_copy;
    tile_copy.init(geo.kv_st, tid);
    auto load_tile = [&](int s, int u) {
        if constexpr (kFastCopy) {
            if ((u + 1) * KT <= Tn) {
                const int64_t first = (int64_t)u * KT * geo.kv_st;
                tile_copy.copy(lds_addr(sK(s)), K0 + first);
                tile_copy.copy(lds_addr(sV(s)), V0 + first);
                return;
            }
        }
        tile_load_async<T, D, KT, NT>(sK(s), K0, geo.kv_st, u * KT, Tn - 1, tid);
        tile_load_async<T, D, KT, NT>(sV(s), V0, geo.kv_st, u * KT, Tn - 1, tid);
    };

    // one kv tile: wait for its copy, start the next one into the other stage, compute from this one
    auto step = [&](auto stage_c, int u) {
        constexpr int ST = decltype(stage_c)::value;
        wait_async_copies();
        __syncthreads();   // tile u is in LDS for everyone; everyone is done with the other stage
        if (u < u_hi) load_tile(ST ^ 1, u + 1);
        const int kv0 = u * KT;
        if (!(active && kv0 <= hi_w && kv0 + KT - 1 >= lo_w)) return;
        const char* tk = smem + ST * TILE_BYTES;
        const char* tv = smem + (2 + ST) * TILE_BYTES;
        // S^T[kv, q] = K Q^T
        f32x16 sacc[KB][QB];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[kb][qb][i] = 0.f;
#pragma unroll
        for (int t = 0; t < DC; ++t) {
            frag kf[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) kf[kb] = lf.rowwise(tk, kb, t);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) sacc[kb][qb] = mma(kf[kb], qf[qb][t], sacc[kb][qb]);
        }
        // mask (only tiles that touch the diagonal or a document start of this wave's rows)
        if (kv0 + KT - 1 > wq0 || kv0 < st_hi) {
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int kv = kv0 + kb * 32 + acc_row(i, hh);
                        const bool ok = kv <= qi[qb] && kv >= st[qb];
                        sacc[kb][qb][i] = ok ? sacc[kb][qb][i] : -INFINITY;
                    }
        }
        // online softmax, one query row per lane.  The reference maximum m[] is only moved (and O, l
        // rescaled) when a row's tile maximum exceeds it by more than 2^kLazy, so the accumulator
        // rescale is a rare, wave-uniform branch; p stays below 2^kLazy otherwise.
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = sacc[0][qb][0];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kb][qb][i]);
            mx = half_max(mx);
            const bool grow = (mx - m[qb]) * c > kLazy;   // false while everything is masked (-inf)
            if (__any(grow)) {
                const float m_new = grow ? mx : m[qb];
                const float alpha = grow ? fast_exp2((m[qb] - m_new) * c) : 1.f;   // m = -inf -> 0
                m[qb] = m_new;
                l[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[qb][db][i] *= alpha;
            }
            const float mc = m[qb] == -INFINITY ? 0.f : m[qb] * c;
            float sum = 0.f;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float p = fast_exp2(fmaf(sacc[kb][qb][i], c, -mc));
                    sacc[kb][qb][i] = p;
                    sum += p;
                }
            l[qb] += sum;
        }
        // O^T[d, q] += V^T P^T
#pragma unroll
        for (int c4 = 0; c4 < KT / 16; ++c4) {
            frag pf[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) pf[qb] = acc_chunk<T>(sacc[c4 / 2][qb], c4 % 2);
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const frag vf = lf.transposed(tv, c4, db);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = mma(vf, pf[qb], oacc[qb][db]);
            }
        }
    };

    load_tile(0, u_lo);

    // Diagonal keys of blocks 1..j (suffix part of the mask): one key per block and row, taken first
    // so that their global-memory latency overlaps the first tile copy.  Row-wise dot products on
    // the vector ALU.
    auto diag_key = [&](const frag (&dk)[QB][DC], const frag (&dv)[QB][DC]) {
        float s[QB];
        float vv[QB][DB][16];   // the key's value row in accumulator order
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            s[qb] = 0.f;
#pragma unroll
            for (int t = 0; t < DC; ++t) s[qb] = dot8(qf[qb][t], dk[qb][t], s[qb]);
            frags_to_acc_order<T, DC>(dv[qb], vv[qb]);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float sc = half_sum(s[qb]);
            const bool grow = (sc - m[qb]) * c > kLazy;   // always for the first key (m = -inf)
            if (__any(grow)) {
                const float m_new = grow ? sc : m[qb];
                const float alpha = grow ? fast_exp2((m[qb] - m_new) * c) : 1.f;
                m[qb] = m_new;
                l[qb] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[qb][db][i] *= alpha;
            }
            const float p = fast_exp2((sc - m[qb]) * c);
            l[qb] += 0.5f * p;   // the two lane halves are added at the end
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[qb][db][i] = fmaf(p, vv[qb][db][i], oacc[qb][db][i]);
        }
    };
    if (a.diag_lds) {
        // Workgroups of 64 rows (packed heads: all waves of a row block want the same K_l / V_l rows):
        // the rows of up to kDiagSlots blocks are copied into LDS at once, behind the tile stages, so
        // their latency is paid once per group of blocks, not once per block, and once per kv group,
        // not once per head.  j is the same for the whole workgroup: the barriers are uniform.
        if constexpr (kDiagLds) {
            char* dbase = smem + 4 * TILE_BYTES;
            for (int base = 1; base <= j; base += kDiagSlots) {
                const int nb = min(kDiagSlots, j - base + 1);
                if (base > 1) __syncthreads();   // the slots are free again
                for (int i = 0; i < nb; ++i) {
                    const T* Kl = static_cast<const T*>(a.k[base + i]) + (int64_t)g * geo.kv_sh;
                    const T* Vl = static_cast<const T*>(a.v[base + i]) + (int64_t)g * geo.kv_sh;
                    tile_load_async<T, D, 64, NT>(dbase + (2 * i) * TILE_BYTES, Kl, geo.kv_st, q_tile0, Tn - 1, tid);
                    tile_load_async<T, D, 64, NT>(dbase + (2 * i + 1) * TILE_BYTES, Vl, geo.kv_st, q_tile0, Tn - 1, tid);
                }
                wait_async_copies();
                __syncthreads();
                if (active) {
                    const int rb = (wq0 - q_tile0) / 32;   // this wave's first row block inside the workgroup's rows
                    for (int i = 0; i < nb; ++i) {
                        frag dk[QB][DC], dv[QB][DC];
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                            for (int t = 0; t < DC; ++t) {
                                dk[qb][t] = lf.rowwise(dbase + (2 * i) * TILE_BYTES, rb + qb, t);
                                dv[qb][t] = lf.rowwise(dbase + (2 * i + 1) * TILE_BYTES, rb + qb, t);
                            }
                        diag_key(dk, dv);
                    }
                }
            }
        }
    } else if (active && j >= 1) {
        // the fragments of block lb + 1 are requested from global memory before block lb is consumed
        frag dk[QB][DC], dv[QB][DC], nk[QB][DC], nv[QB][DC];
        auto request = [&](int lb, frag (&rk)[QB][DC], frag (&rv)[QB][DC]) {
            const T* Kl = static_cast<const T*>(a.k[lb]) + (int64_t)g * geo.kv_sh;
            const T* Vl = static_cast<const T*>(a.v[lb]) + (int64_t)g * geo.kv_sh;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const T* krow = Kl + (int64_t)qc[qb] * geo.kv_st;
                const T* vrow = Vl + (int64_t)qc[qb] * geo.kv_st;
#pragma unroll
                for (int t = 0; t < DC; ++t) {
                    rk[qb][t] = gload_frag<T>(krow + t * 16 + hh * 8);
                    rv[qb][t] = gload_frag<T>(vrow + t * 16 + hh * 8);
                }
            }
        };
        request(1, dk, dv);
        for (int lb = 1; lb <= j; ++lb) {
            if (lb < j) request(lb + 1, nk, nv);
            diag_key(dk, dv);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int t = 0; t < DC; ++t) {
                    dk[qb][t] = nk[qb][t];
                    dv[qb][t] = nv[qb][t];
                }
        }
    }

    for (int u = u_lo; u <= u_hi; u += 2) {
        step(IntC<0>{}, u);
        if (u + 1 <= u_hi) step(IntC<1>{}, u + 1);
    }

    // normalise; rows go through a wave-private LDS patch (carved out of the tile stages, which
    // everybody has finished reading after this barrier) so that every global store is a full
    // 16-byte piece of a row and a wave instruction covers whole rows
    __syncthreads();
    if (!active) return;
    char* patch = smem + wave * (32 * D * E::kBytes);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float lt = half_sum(l[qb]);
        const float inv = 1.f / lt;
        if (hh == 0 && qi[qb] < Tn) a.lse[j][(int64_t)h * geo.lse_st + qi[qb]] = m[qb] * geo.scale + __logf(lt);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                T* dst = reinterpret_cast<T*>(patch + Tile<T, D>::offset(n, db * 32 + i4 * 8 + hh * 4));
                typename E::vec4 pk;
#pragma unroll
                for (int e = 0; e < 4; ++e) pk[e] = (T)(oacc[qb][db][i4 * 4 + e] * inv);
                *reinterpret_cast<typename E::vec4*>(dst) = pk;
            }
        // the patch is private to the wave: LDS operations of one wave complete in order
        constexpr int PIECES = Tile<T, D>::kPieces;
        T* obase = static_cast<T*>(a.o[j]) + (int64_t)h * geo.q_sh;
#pragma unroll
        for (int it = 0; it < 32 * PIECES / 64; ++it) {
            const int pidx = it * 64 + lane;
            const int r = pidx / PIECES, piece = pidx % PIECES;
            const int row = wq0 + 32 * qb + r;
            const f32x4 val = *reinterpret_cast<const f32x4*>(patch + r * Tile<T, D>::kRowBytes + ((piece ^ Tile<T, D>::swz(r)) * 16));
            if (row < Tn) *reinterpret_cast<f32x4*>(obase + (int64_t)row * geo.q_st + piece * Tile<T, D>::kElemsPerPiece) = val;
        }
    }
}

// first / one-past-last token of each token's document, by binary search in cu_seqlens
// (`cu` may be a slice of a longer cu_seqlens array: `base` = its first entry, subtracted so that
// the bounds count from the slice's first token)
__global__ void ttt_tok_bounds_kernel(const int* __restrict__ cu, int base, int n_docs, int T, int* __restrict__ tok_start,
                                      int* __restrict__ tok_end) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T) return;
    int lo = 0, hi = n_docs;   // find the largest r with cu[r] <= i (then cu[r+1] > i)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] - base <= i) lo = mid; else hi = mid;
    }
    tok_start[i] = cu[lo] - base;
    tok_end[i] = cu[lo + 1] - base;
}

hipError_t launch_tok_bounds(const int* cu_dev, int base, int n_docs, int T, int* tok_start, int* tok_end, hipStream_t stream) {
    if (T <= 0) return hipSuccess;
    ProfileScope prof("ttt_tok_bounds_kernel", stream);
    hipLaunchKernelGGL(ttt_tok_bounds_kernel, dim3((T + 255) / 256), dim3(256), 0, stream, cu_dev, base, n_docs, T,
                       tok_start, tok_end);
    return hipGetLastError();
}

template <typename T, int D, int QB, int NW, int MINB> struct FwdCfg {
    static constexpr int kQT = NW * QB * 32;
    static constexpr int kLds = 4 * 64 * D * (int)sizeof(T);   // two stages of K and V tiles
    static constexpr int kDiagLds = 3 * 2 * 64 * D * (int)sizeof(T);   // three blocks of 64 diagonal K and V rows
};

template <typename T, int D, int QB, int NW, int MINB> static hipError_t launch_fwd_t(FwdArgs& a, hipStream_t stream) {
    using C = FwdCfg<T, D, QB, NW, MINB>;
    auto kern = ttt_fwd_kernel<T, D, QB, NW, MINB>;
    static LdsOptIn lds_opt_in;
    if (hipError_t e = lds_opt_in.ensure((const void*)kern, C::kLds + (sizeof(T) == 2 ? C::kDiagLds : 0)); e != hipSuccess) return e;
    const Geometry& geo = a.geo;
    // as many heads of a kv group per workgroup as divide both the group and the waves (at most 4:
    // a workgroup keeps at least 64 rows)
    a.pack_log2 = 0;
    while ((2 << a.pack_log2) <= 4 && geo.G % (2 << a.pack_log2) == 0 && NW % (2 << a.pack_log2) == 0) ++a.pack_log2;
    const int qt_rows = C::kQT >> a.pack_log2;
    a.n_tiles = (geo.T + qt_rows - 1) / qt_rows;
    a.diag_lds = sizeof(T) == 2 && qt_rows == 64;   // the diagonal rows of a 64-row workgroup go through LDS
    const int lds_bytes = C::kLds + (a.diag_lds ? C::kDiagLds : 0);
    a.map.hkv = geo.hkv;
    a.map.rest_count = a.n_tiles * geo.n_steps * (geo.G >> a.pack_log2);
    int64_t grid;
    if (geo.hkv % 8 == 0) {
        a.map.mode = 1;
        grid = (int64_t)geo.hkv * a.map.rest_count;
    } else if (8 % geo.hkv == 0) {
        a.map.mode = 2;
        const int xp = 8 / geo.hkv;
        grid = 8 * (int64_t)((a.map.rest_count + xp - 1) / xp);
    } else {
        a.map.mode = 0;
        grid = (int64_t)geo.hkv * a.map.rest_count;
    }
    if (grid <= 0) return hipSuccess;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    // the 16-bit kernels address the pieces of up to 64 rows of K or V with 32-bit byte offsets
    if (sizeof(T) == 2 && geo.kv_st * 64 * (int64_t)sizeof(T) >= (int64_t)1 << 32) return hipErrorInvalidValue;
    ProfileScope prof("ttt_fwd_kernel", stream);
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), lds_bytes, stream, a);
    return hipGetLastError();
}

hipError_t launch_fwd(int dtype, int head_dim, FwdArgs& a, hipStream_t stream) {
    if (dtype == 1 && head_dim == 128) return launch_fwd_t<__bf16, 128, 1, 8, 1>(a, stream);
    if (dtype == 1 && head_dim == 64) return launch_fwd_t<__bf16, 64, 2, 4, 1>(a, stream);
    if (dtype == 0 && head_dim == 128) return launch_fwd_t<float, 128, 1, 4, 1>(a, stream);
    if (dtype == 0 && head_dim == 64) return launch_fwd_t<float, 64, 1, 4, 1>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace ttt
