// Backward TTT attention kernels (gfx950).  Nothing but O and LSE was kept by the forward
// (Sec. 4.2.1), so every kernel here recomputes p = exp(s - LSE) from Q and K tile by tile and
// applies the softmax-attention VJP:  D = <dO,O>, dp = <dO,V>, ds = p (dp - D).
//
//   ttt_bwd_pre_kernel   D for every (step, head, token); and the complete dK_l, dV_l of the later
//                        cache blocks l >= 1, which are only ever read on the diagonal (suffix part
//                        of Alg. 2), so one small group of lanes owns each (token, kv head) -- no atomics.
//   ttt_bwd_dq_kernel    query-stationary, same streaming structure as the forward: dQ_j
//                        (ttt_bwd_dq_pipe_kernel: block-pipelined variant for 16-bit types).
//   ttt_bwd_dkv_kernel   key-stationary over block 0: each wave keeps 32 rows of K_0, V_0 as
//                        operands and their dK, dV accumulators in registers while every
//                        (step, head of the group, query tile at or below the diagonal) streams past
//                        through LDS; partial sums of the (step, head) splits meet in fp32 atomics
//                        (ttt_bwd_dkv_p8_kernel: eight equal waves, for 16-bit types).
//   ttt_bwd_finish_kernel  fp32 block-0 sums -> dK_0, dV_0 in the tensor dtype.
#include <algorithm>
#include <functional>
#include <mutex>
#include <queue>
#include <vector>

#include "ttt_args.hpp"

namespace ttt {

constexpr float kLog2e = 1.44269504088896340736f;

// ------------------------------------------------------------------------------------------------
// D and the diagonal blocks' dK_l, dV_l
// ------------------------------------------------------------------------------------------------
template <int LPR> TTT_DEV float group_sum(float v) {
#pragma unroll
    for (int s = 1; s < LPR; s <<= 1) v += __shfl_xor(v, s, 64);
    return v;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void ttt_bwd_pre_kernel(const BwdArgs a) {
    using frag = typename Elem<T>::frag;
    constexpr int LPR = D / 8;       // lanes that share one (token, kv head): 8 elements each
    constexpr int UPB = 256 / LPR;   // (token, kv head) units per workgroup
    extern __shared__ float sD[];    // [UPB][n_steps*G]

    const Geometry& geo = a.geo;
    const int Tn = geo.T, G = geo.G, ns = geo.n_steps, b = geo.step_begin, e = b + ns;
    const int grp = threadIdx.x / LPR, sub = threadIdx.x % LPR;
    const int64_t unit = (int64_t)blockIdx.x * UPB + grp;
    const bool valid = unit < (int64_t)Tn * geo.hkv;
    const int i = valid ? (int)(unit / geo.hkv) : 0;
    const int g = valid ? (int)(unit % geo.hkv) : 0;
    float* myD = sD + grp * (ns * G);

    // phase 1: D_j[h,i] = <dO_j[i,h], O_j[i,h]>
    for (int js = 0; js < ns; ++js) {
        const int j = b + js;
        for (int hg = 0; hg < G; ++hg) {
            const int h = g * G + hg;
            const int64_t off = (int64_t)i * geo.q_st + (int64_t)h * geo.q_sh + sub * 8;
            const frag go = gload_frag<T>(static_cast<const T*>(a.d_o[j]) + off);
            const frag oo = gload_frag<T>(static_cast<const T*>(a.o[j]) + off);
            float d = 0.f;
#pragma unroll
            for (int x = 0; x < 8; ++x) d = fmaf(to_f32<T>(go[x]), to_f32<T>(oo[x]), d);
            d = group_sum<LPR>(d);
            if (sub == 0) {
                myD[js * G + hg] = d;
                if (valid) {
                    const int64_t at = ((int64_t)js * geo.hq + h) * Tn + i;
                    a.delta[at] = d;
                    a.lse2[at] = a.lse[j][(int64_t)h * geo.lse_st + i] * kLog2e;
                }
            }
        }
    }
    __syncthreads();
    if (!valid) return;

    // phase 2: blocks l >= 1 see only the queries at their own token, steps j >= l
    for (int lb = 1; lb < e; ++lb) {
        const int64_t kvoff = (int64_t)i * geo.kv_st + (int64_t)g * geo.kv_sh + sub * 8;
        const frag kf = gload_frag<T>(static_cast<const T*>(a.k[lb]) + kvoff);
        const frag vf = gload_frag<T>(static_cast<const T*>(a.v[lb]) + kvoff);
        float dk[8], dv[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) dk[x] = dv[x] = 0.f;
        for (int j = (lb > b ? lb : b); j < e; ++j) {
            for (int hg = 0; hg < G; ++hg) {
                const int h = g * G + hg;
                const int64_t off = (int64_t)i * geo.q_st + (int64_t)h * geo.q_sh + sub * 8;
                const frag qf = gload_frag<T>(static_cast<const T*>(a.q[j]) + off);
                const frag go = gload_frag<T>(static_cast<const T*>(a.d_o[j]) + off);
                float s = 0.f, dp = 0.f;
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    s = fmaf(to_f32<T>(qf[x]), to_f32<T>(kf[x]), s);
                    dp = fmaf(to_f32<T>(go[x]), to_f32<T>(vf[x]), dp);
                }
                s = group_sum<LPR>(s);
                dp = group_sum<LPR>(dp);
                const float lse = a.lse[j][(int64_t)h * geo.lse_st + i];
                const float p = fast_exp2((s * geo.scale - lse) * kLog2e);
                const float ds = p * (dp - myD[(j - b) * G + hg]) * geo.scale;
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    dk[x] = fmaf(ds, to_f32<T>(qf[x]), dk[x]);
                    dv[x] = fmaf(p, to_f32<T>(go[x]), dv[x]);
                }
            }
        }
        if (a.accumulate) {
            // fp32 carry across the calls of a descending-step sweep; this group owns its slice
            const int64_t coff = (((int64_t)(lb - 1) * Tn + i) * geo.hkv + g) * D + sub * 8;
            float* ck = a.dkl_acc + coff;
            float* cv = a.dvl_acc + coff;
            if (!a.carry_reset) {
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    dk[x] += ck[x];
                    dv[x] += cv[x];
                }
            }
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                ck[x] = dk[x];
                cv[x] = dv[x];
            }
            if (lb < b) continue;   // not complete yet: earlier steps' calls have not run
        }
        T* gk = static_cast<T*>(a.dk[lb]) + kvoff;
        T* gv = static_cast<T*>(a.dv[lb]) + kvoff;
        gstore_vec4<T>(gk, dk[0], dk[1], dk[2], dk[3]);
        gstore_vec4<T>(gk + 4, dk[4], dk[5], dk[6], dk[7]);
        gstore_vec4<T>(gv, dv[0], dv[1], dv[2], dv[3]);
        gstore_vec4<T>(gv + 4, dv[4], dv[5], dv[6], dv[7]);
    }
}

// Sum over an aligned group of LPR (4, 8 or 16) lanes with DPP moves only (no LDS traffic):
// quad butterflies, then the half-row and the row mirror pair up quads and half-rows.
template <int LPR> TTT_DEV float group_sum_dpp(float v) {
    auto mv = [](float x, auto ctrl) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xf, 0xf, true));
    };
    v += mv(v, IntC<0xB1>{});                              // quad_perm [1,0,3,2]
    v += mv(v, IntC<0x4E>{});                              // quad_perm [2,3,0,1]
    if constexpr (LPR >= 8) v += mv(v, IntC<0x141>{});     // row_half_mirror
    if constexpr (LPR >= 16) v += mv(v, IntC<0x140>{});    // row_mirror
    return v;
}

// The same work for 16-bit types and at most KMAX steps, reading every Q_j, dO_j, O_j row exactly
// once: the K_l, V_l rows of this (token, kv head) and their fp32 gradients stay in registers while
// one sweep over (step, head of the group) feeds all of them (the suffix part of Alg. 2 read from the
// key's side: key (l, i) is seen only by the queries (j >= l, i) of Sec. 2.4's unrolled steps).
template <typename T, int D, int KMAX, int PF>
__global__ __launch_bounds__(256) void ttt_bwd_pre_regs_kernel(const BwdArgs a) {
    static_assert(sizeof(T) == 2, "register budget sized for 16-bit elements");
    using frag = typename Elem<T>::frag;
    constexpr int LPR = D / 8;
    constexpr int UPB = 256 / LPR;
    constexpr int NL = KMAX - 1;

    const Geometry& geo = a.geo;
    const int Tn = geo.T, G = geo.G, ns = geo.n_steps, b = geo.step_begin, e = b + ns;
    const int grp = threadIdx.x / LPR, sub = threadIdx.x % LPR;
    const int64_t unit = (int64_t)blockIdx.x * UPB + grp;
    if (unit >= (int64_t)Tn * geo.hkv) return;   // whole aligned lane groups leave together
    const int i = (int)(unit / geo.hkv);
    const int g = (int)(unit % geo.hkv);
    const int64_t kvoff = (int64_t)i * geo.kv_st + (int64_t)g * geo.kv_sh + sub * 8;

    frag kf[NL], vf[NL];
    float dk[NL][8], dv[NL][8];
#pragma unroll
    for (int l = 0; l < NL; ++l) {
        const int lb = l + 1 < e ? l + 1 : 0;     // unused slots read block 0's row (in bounds), never used
        kf[l] = gload_frag<T>(static_cast<const T*>(a.k[lb]) + kvoff);
        vf[l] = gload_frag<T>(static_cast<const T*>(a.v[lb]) + kvoff);
#pragma unroll
        for (int x = 0; x < 8; ++x) dk[l][x] = dv[l][x] = 0.f;
    }

    // One sweep over the (step, head of the group) pairs; the rows of the next PF pairs are requested
    // before a pair is worked on, so that a lane group always has PF requests in flight beside the pair
    // it works on (the kernel is bound by HBM; measured at 4096 tokens, 0.98 GB per launch: no request
    // ahead 4.45 TB/s, one 4.75, two 5.07, four -- with one block fewer in registers -- 5.07).
    const int n_pairs = ns * G;
    frag qf[PF], go[PF], oo[PF];
    float lse_raw[PF];
    auto request = [&](int n, auto slot_c) {
        constexpr int S = decltype(slot_c)::value;
        const int j = b + n / G, h = g * G + n % G;
        const int64_t off = (int64_t)i * geo.q_st + (int64_t)h * geo.q_sh + sub * 8;
        qf[S] = gload_frag<T>(static_cast<const T*>(a.q[j]) + off);
        go[S] = gload_frag<T>(static_cast<const T*>(a.d_o[j]) + off);
        oo[S] = gload_frag<T>(static_cast<const T*>(a.o[j]) + off);
        lse_raw[S] = a.lse[j][(int64_t)h * geo.lse_st + i];
    };
    if (n_pairs > 0) request(0, IntC<0>{});
    if constexpr (PF > 1) if (n_pairs > 1) request(1, IntC<1>{});
    if constexpr (PF > 2) if (n_pairs > 2) request(2, IntC<2>{});
    if constexpr (PF > 3) if (n_pairs > 3) request(3, IntC<3>{});
    static_assert(PF >= 1 && PF <= 4, "prefetch depth");
    for (int n = 0; n < n_pairs; ++n) {
        const int js = n / G, j = b + js, h = g * G + n % G;
        const frag cq = qf[0], cg = go[0], co = oo[0];
        const float lse2 = lse_raw[0] * kLog2e;
#pragma unroll
        for (int s = 0; s + 1 < PF; ++s) {
            qf[s] = qf[s + 1];
            go[s] = go[s + 1];
            oo[s] = oo[s + 1];
            lse_raw[s] = lse_raw[s + 1];
        }
        if (n + PF < n_pairs) request(n + PF, IntC<PF - 1>{});
        const float dsum = group_sum_dpp<LPR>(dot8(cg, co, 0.f));
        if (sub == 0) {
            const int64_t at = ((int64_t)js * geo.hq + h) * Tn + i;
            a.delta[at] = dsum;
            a.lse2[at] = lse2;
        }
        float qx[8], gx[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            qx[x] = to_f32<T>(cq[x]);
            gx[x] = to_f32<T>(cg[x]);
        }
#pragma unroll
        for (int l = 0; l < NL; ++l) {
            if (l + 1 > j) break;              // block l+1 is visible from step j >= l+1 only
            const float s = group_sum_dpp<LPR>(dot8(cq, kf[l], 0.f));
            const float dp = group_sum_dpp<LPR>(dot8(cg, vf[l], 0.f));
            const float p = fast_exp2(s * (geo.scale * kLog2e) - lse2);
            const float ds = p * (dp - dsum) * geo.scale;
#pragma unroll
            for (int x = 0; x < 8; ++x) {
                dk[l][x] = fmaf(ds, qx[x], dk[l][x]);
                dv[l][x] = fmaf(p, gx[x], dv[l][x]);
            }
        }
    }

#pragma unroll
    for (int l = 0; l < NL; ++l) {
        const int lb = l + 1;
        if (lb >= e) break;
        if (a.accumulate) {
            // fp32 carry across the calls of a descending-step sweep; this group owns its slice
            const int64_t coff = (((int64_t)l * Tn + i) * geo.hkv + g) * D + sub * 8;
            f32x4* ck = reinterpret_cast<f32x4*>(a.dkl_acc + coff);
            f32x4* cv = reinterpret_cast<f32x4*>(a.dvl_acc + coff);
            if (!a.carry_reset) {
#pragma unroll
                for (int v4 = 0; v4 < 2; ++v4) {
                    const f32x4 pk = ck[v4], pv = cv[v4];
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        dk[l][4 * v4 + x] += pk[x];
                        dv[l][4 * v4 + x] += pv[x];
                    }
                }
            }
#pragma unroll
            for (int v4 = 0; v4 < 2; ++v4) {
                ck[v4] = f32x4{dk[l][4 * v4], dk[l][4 * v4 + 1], dk[l][4 * v4 + 2], dk[l][4 * v4 + 3]};
                cv[v4] = f32x4{dv[l][4 * v4], dv[l][4 * v4 + 1], dv[l][4 * v4 + 2], dv[l][4 * v4 + 3]};
            }
            if (lb < b) continue;   // not complete yet: earlier steps' calls have not run
        }
        T* gk = static_cast<T*>(a.dk[lb]) + kvoff;
        T* gv = static_cast<T*>(a.dv[lb]) + kvoff;
        gstore_vec4<T>(gk, dk[l][0], dk[l][1], dk[l][2], dk[l][3]);
        gstore_vec4<T>(gk + 4, dk[l][4], dk[l][5], dk[l][6], dk[l][7]);
        gstore_vec4<T>(gv, dv[l][0], dv[l][1], dv[l][2], dv[l][3]);
        gstore_vec4<T>(gv + 4, dv[l][4], dv[l][5], dv[l][6], dv[l][7]);
    }
}

// ------------------------------------------------------------------------------------------------
// dQ: query-stationary
// ------------------------------------------------------------------------------------------------
template <typename T, int D, int QB, int NW>
__global__ __launch_bounds__(NW * 64) void ttt_bwd_dq_kernel(const BwdArgs a) {
    using E = Elem<T>;
    using frag = typename E::frag;
    constexpr int KT = 64;
    constexpr int KB = KT / 32;
    constexpr int QT = NW * QB * 32;
    constexpr int DC = D / 16;
    constexpr int DB = D / 32;
    constexpr int NT = NW * 64;
    constexpr int TILE_BYTES = KT * D * E::kBytes;

    extern __shared__ __align__(16) char smem[];
    auto sK = [&](int s) -> char* { return smem + s * TILE_BYTES; };
    auto sV = [&](int s) -> char* { return smem + (2 + s) * TILE_BYTES; };

    const Geometry& geo = a.geo;
    int g, rest;
    if (!decode_block(a.map, blockIdx.x, g, rest)) return;
    const int hg = rest % geo.G;
    rest /= geo.G;
    const int js = rest % geo.n_steps;
    const int j = geo.step_begin + js;
    const int tile = a.n_tiles - 1 - rest / geo.n_steps;
    const int h = g * geo.G + hg;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int Tn = geo.T;
    const int q_tile0 = tile * QT;
    const int wq0 = q_tile0 + wave * (QB * 32);
    const bool active = wq0 < Tn;

    const T* Qj = static_cast<const T*>(a.q[j]) + (int64_t)h * geo.q_sh;
    const T* dOj = static_cast<const T*>(a.d_o[j]) + (int64_t)h * geo.q_sh;
    const T* K0 = static_cast<const T*>(a.k[0]) + (int64_t)g * geo.kv_sh;
    const T* V0 = static_cast<const T*>(a.v[0]) + (int64_t)g * geo.kv_sh;

    int qi[QB], qc[QB], st[QB];
    float lse2[QB], dl[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        qi[qb] = wq0 + 32 * qb + n;
        qc[qb] = qi[qb] < Tn ? qi[qb] : Tn - 1;
        st[qb] = a.tok_start[qc[qb]];
        lse2[qb] = a.lse[j][(int64_t)h * geo.lse_st + qc[qb]] * kLog2e;
        dl[qb] = a.delta[((int64_t)js * geo.hq + h) * Tn + qc[qb]];
    }
    const int hi_w = min(wq0 + QB * 32 - 1, Tn - 1);
    const int lo_w = active ? __builtin_amdgcn_readfirstlane(a.tok_start[min(wq0, Tn - 1)]) : 0;
    const int st_hi = active ? __builtin_amdgcn_readfirstlane(a.tok_start[hi_w]) : 0;
    const int lo = __builtin_amdgcn_readfirstlane(a.tok_start[q_tile0]);
    const int hi = min(q_tile0 + QT - 1, Tn - 1);
    const int u_lo = lo / KT, u_hi = hi / KT;

    frag qf[QB][DC], gof[QB][DC];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int t = 0; t < DC; ++t) {
            qf[qb][t] = gload_frag<T>(Qj + (int64_t)qc[qb] * geo.q_st + t * 16 + hh * 8);
            gof[qb][t] = gload_frag<T>(dOj + (int64_t)qc[qb] * geo.q_st + t * 16 + hh * 8);
        }

    f32x16 dqacc[QB][DB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) dqacc[qb][db][i] = 0.f;
    const float c = geo.scale_log2;

    tile_load_async<T, D, KT, NT>(sK(0), K0, geo.kv_st, u_lo * KT, Tn - 1, tid);
    tile_load_async<T, D, KT, NT>(sV(0), V0, geo.kv_st, u_lo * KT, Tn - 1, tid);
    int stage = 0;
    for (int u = u_lo; u <= u_hi; ++u) {
        wait_async_copies();
        __syncthreads();
        if (u < u_hi) {
            tile_load_async<T, D, KT, NT>(sK(stage ^ 1), K0, geo.kv_st, (u + 1) * KT, Tn - 1, tid);
            tile_load_async<T, D, KT, NT>(sV(stage ^ 1), V0, geo.kv_st, (u + 1) * KT, Tn - 1, tid);
        }
        const int kv0 = u * KT;
        if (active && kv0 <= hi_w && kv0 + KT - 1 >= lo_w) {
            const char* tk = sK(stage);
            const char* tv = sV(stage);
            f32x16 sacc[KB][QB], pacc[KB][QB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) sacc[kb][qb][i] = pacc[kb][qb][i] = 0.f;
            // S^T = K Q^T and dP^T = V dO^T
#pragma unroll
            for (int t = 0; t < DC; ++t) {
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const frag kf = frag_rowwise<T, D>(tk, kb * 32 + n, t * 16 + hh * 8);
                    const frag vf = frag_rowwise<T, D>(tv, kb * 32 + n, t * 16 + hh * 8);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        sacc[kb][qb] = mma(kf, qf[qb][t], sacc[kb][qb]);
                        pacc[kb][qb] = mma(vf, gof[qb][t], pacc[kb][qb]);
                    }
                }
            }
            const bool need_mask = kv0 + KT - 1 > wq0 || kv0 < st_hi;
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        float p = fast_exp2(fmaf(sacc[kb][qb][i], c, -lse2[qb]));
                        if (need_mask) {
                            const int kv = kv0 + kb * 32 + acc_row(i, hh);
                            p = (kv <= qi[qb] && kv >= st[qb]) ? p : 0.f;
                        }
                        sacc[kb][qb][i] = p * (pacc[kb][qb][i] - dl[qb]);   // dS^T
                    }
            // dQ^T[d, q] += K^T dS^T
#pragma unroll
            for (int c4 = 0; c4 < KT / 16; ++c4) {
                frag sf[QB];
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) sf[qb] = acc_chunk<T>(sacc[c4 / 2][qb], c4 % 2);
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const frag kt = frag_transposed<T, D>(tk, c4 * 16, db * 32, lane);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) dqacc[qb][db] = mma(kt, sf[qb], dqacc[qb][db]);
                }
            }
        }
        stage ^= 1;
    }
    if (!active) return;

    // diagonal keys of blocks 1..j
    for (int lb = 1; lb <= j; ++lb) {
        const T* Kl = static_cast<const T*>(a.k[lb]) + (int64_t)g * geo.kv_sh;
        const T* Vl = static_cast<const T*>(a.v[lb]) + (int64_t)g * geo.kv_sh;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const T* krow = Kl + (int64_t)qc[qb] * geo.kv_st;
            const T* vrow = Vl + (int64_t)qc[qb] * geo.kv_st;
            float s = 0.f, dp = 0.f;
#pragma unroll
            for (int t = 0; t < DC; ++t) {
                const frag kf = gload_frag<T>(krow + t * 16 + hh * 8);
                const frag vf = gload_frag<T>(vrow + t * 16 + hh * 8);
#pragma unroll
                for (int x = 0; x < 8; ++x) {
                    s = fmaf(to_f32<T>(qf[qb][t][x]), to_f32<T>(kf[x]), s);
                    dp = fmaf(to_f32<T>(gof[qb][t][x]), to_f32<T>(vf[x]), dp);
                }
            }
            s += xor32(s);
            dp += xor32(dp);
            const float p = fast_exp2(fmaf(s, c, -lse2[qb]));
            const float ds = p * (dp - dl[qb]);
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const typename E::vec4 kk = gload_vec4<T>(krow + db * 32 + i4 * 8 + hh * 4);
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        dqacc[qb][db][i4 * 4 + x] = fmaf(ds, to_f32<T>(kk[x]), dqacc[qb][db][i4 * 4 + x]);
                }
        }
    }

#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        if (qi[qb] < Tn) {
            T* row = static_cast<T*>(a.dq[j]) + (int64_t)h * geo.q_sh + (int64_t)qi[qb] * geo.q_st;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4)
                    gstore_vec4<T>(row + db * 32 + i4 * 8 + hh * 4, dqacc[qb][db][i4 * 4 + 0] * geo.scale,
                                   dqacc[qb][db][i4 * 4 + 1] * geo.scale, dqacc[qb][db][i4 * 4 + 2] * geo.scale,
                                   dqacc[qb][db][i4 * 4 + 3] * geo.scale);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// dQ: query-stationary, 128-row kv tiles (16-bit element types)
//
// One wave = 32 query rows with Q and dO as stationary B operands; a kv tile has 128 rows = 4
// blocks of 32, each taken through S^T, dP^T, dS^T and the dQ^T update in turn, with the LDS
// fragments of the next matrix instructions requested ahead.  Eight waves (two per SIMD) overlap
// one wave's vector work with the other's matrix work.
// LDS: two stages of [K tile | V tile]; the stage bit is bit 16 of the per-lane addresses.
// ------------------------------------------------------------------------------------------------
template <typename T, int D, int NW>
__global__ __launch_bounds__(NW * 64) void ttt_bwd_dq_pipe_kernel(const BwdArgs a) {
    static_assert(sizeof(T) == 2, "this dQ kernel is for 16-bit elements");
    static_assert(NW == 8, "two waves per SIMD supply the overlap; no other wave count is built");
    using E = Elem<T>;
    using frag = typename E::frag;
    using TL = Tile<T, D>;
    constexpr int KT = 128;
    constexpr int NB = KT / 32;
    constexpr int QT = NW * 32;
    constexpr int DC = D / 16;
    constexpr int DB = D / 32;
    constexpr int NT = NW * 64;
    constexpr int TILE_BYTES = KT * D * E::kBytes;
    constexpr int STAGE_BYTES = 1 << 16;
    static_assert(2 * TILE_BYTES <= STAGE_BYTES, "stage layout");
    constexpr int NE = 2 * DB;   // matrix instructions of one dQ block update
    constexpr int PDR = 2;       // row-wise K / V fragments requested ahead of their matrix instruction
    constexpr int PDT = 2;       // K^T fragments requested ahead
    typedef __attribute__((address_space(3))) char lds_char;

    extern __shared__ __align__(16) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;

    const Geometry& geo = a.geo;
    int g, rest;
    if (!decode_block(a.map, blockIdx.x, g, rest)) return;
    const int hg = rest % geo.G;
    rest /= geo.G;
    const int js = rest % geo.n_steps;
    const int j = geo.step_begin + js;
    const int tile = a.n_tiles - 1 - rest / geo.n_steps;
    const int h = g * geo.G + hg;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int Tn = geo.T;
    const int q_tile0 = tile * QT;
    const int wq0 = q_tile0 + wave * 32;
    const bool active = wq0 < Tn;

    const T* Qj = static_cast<const T*>(a.q[j]) + (int64_t)h * geo.q_sh;
    const T* dOj = static_cast<const T*>(a.d_o[j]) + (int64_t)h * geo.q_sh;
    const T* K0 = static_cast<const T*>(a.k[0]) + (int64_t)g * geo.kv_sh;
    const T* V0 = static_cast<const T*>(a.v[0]) + (int64_t)g * geo.kv_sh;

    const int qi = wq0 + n;
    const int qc = qi < Tn ? qi : Tn - 1;
    const int st = a.tok_start[qc];
    const int64_t at = ((int64_t)js * geo.hq + h) * Tn + qc;
    const float lse2 = a.lse2[at];
    const float dl = a.delta[at];
    const int hi_w = min(wq0 + 31, Tn - 1);
    const int lo_w = active ? __builtin_amdgcn_readfirstlane(a.tok_start[min(wq0, Tn - 1)]) : 0;
    const int st_hi = active ? __builtin_amdgcn_readfirstlane(a.tok_start[hi_w]) : 0;
    const int lo = __builtin_amdgcn_readfirstlane(a.tok_start[q_tile0]);
    const int hi = min(q_tile0 + QT - 1, Tn - 1);
    const int u_lo = lo / KT, u_hi = hi / KT;

    frag qf[DC], gof[DC];
#pragma unroll
    for (int t = 0; t < DC; ++t) {
        qf[t] = gload_frag<T>(Qj + (int64_t)qc * geo.q_st + t * 16 + hh * 8);
        gof[t] = gload_frag<T>(dOj + (int64_t)qc * geo.q_st + t * 16 + hh * 8);
    }
    f32x16 dqacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[db][i] = 0.f;
    const float c = geo.scale_log2;

    uint32_t ra[DC], ta[DB][2];
    {
        LaneFrags<T, D> lf;
        lf.init(lane);
#pragma unroll
        for (int t = 0; t < DC; ++t) ra[t] = lds0 + lf.row[t];
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            ta[db][0] = lds0 + lf.tr[db][0];
            ta[db][1] = lds0 + lf.tr[db][1];
        }
    }
    auto ld_row = [&](int which, int kb, int t) -> frag {   // which: 0 = K tile, 1 = V tile
        return *reinterpret_cast<const __attribute__((address_space(3))) frag*>(
            (uintptr_t)(ra[t] + which * TILE_BYTES + kb * 32 * TL::kRowBytes));
    };
    auto ld_ktr = [&](int kb, int x) -> frag {   // K^T fragment x = c2 * DB + db of block kb
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const int c2 = x / DB, db = x % DB;
        const uint32_t off = (kb * 32 + c2 * 16) * TL::kRowBytes;
        union { s16x4 s[2]; frag v; } u;
        u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(ta[db][0] + off));
        u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(ta[db][1] + off));
        return u.v;
    };
    TileCopy<T, D, KT, NT> tile_copy;
    tile_copy.init(geo.kv_st, tid);
    auto issue = [&](int u, int s) {
        if ((u + 1) * KT <= Tn) {
            const int64_t first = (int64_t)u * KT * geo.kv_st;
            tile_copy.copy(lds0 + s * STAGE_BYTES, K0 + first);
            tile_copy.copy(lds0 + s * STAGE_BYTES + TILE_BYTES, V0 + first);
        } else {
            char* stg = smem + s * STAGE_BYTES;
            tile_load_async<T, D, KT, NT>(stg, K0, geo.kv_st, u * KT, Tn - 1, tid);
            tile_load_async<T, D, KT, NT>(stg + TILE_BYTES, V0, geo.kv_st, u * KT, Tn - 1, tid);
        }
    };

    issue(u_lo, 0);
    int stage = 0;
    for (int u = u_lo; u <= u_hi; ++u) {
        wait_async_copies();
        __syncthreads();
        if (u < u_hi) issue(u + 1, stage ^ 1);
        const int kv0 = u * KT;
        if (active && kv0 <= hi_w && kv0 + KT - 1 >= lo_w) {
            frag ka[DC], va[DC];   // row-wise K / V fragments of the block being scored
            frag tfr[NE];          // K^T fragments of the block being accumulated
            frag sfr[2];           // dS^T operands of the previous block
            f32x16 sacc, pacc;
            auto prime_rows = [&](int kb) {
#pragma unroll
                for (int t = 0; t < PDR; ++t) {
                    ka[t] = ld_row(0, kb, t);
                    va[t] = ld_row(1, kb, t);
                }
            };
            // S^T[kv, q] = K Q^T and dP^T[kv, q] = V dO^T (lane = query row)
            auto score = [&](int kb) {
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[i] = pacc[i] = 0.f;
#pragma unroll
                for (int t = 0; t < DC; ++t) {
                    if (t + PDR < DC) {
                        ka[t + PDR] = ld_row(0, kb, t + PDR);
                        va[t + PDR] = ld_row(1, kb, t + PDR);
                    }
                    issue_fence();
                    sacc = mma(ka[t], qf[t], sacc);
                    pacc = mma(va[t], gof[t], pacc);
                }
            };
            {
                // Two waves per SIMD: no pipelining inside the wave.  One wave's vector work runs
                // while the other wave of the SIMD uses the matrix core (they fall into opposite
                // phases by themselves); blocks that this wave's rows cannot see are skipped.
                bool primed = false;
#pragma unroll
                for (int kb = 0; kb < NB; ++kb) {
                    const int kb0 = kv0 + kb * 32;
                    if (kb0 > hi_w || kb0 + 31 < lo_w) {
                        primed = false;
                        continue;
                    }
                    if (!primed) prime_rows(kb);
                    score(kb);
                    // requests that do not depend on the vector work below
#pragma unroll
                    for (int x = 0; x < PDT; ++x) tfr[x] = ld_ktr(kb, x);
                    primed = kb + 1 < NB && !(kb0 + 32 > hi_w || kb0 + 63 < lo_w);
                    if (primed) prime_rows(kb + 1);
                    issue_fence();
                    const bool need_mask = kb0 + 31 > wq0 || kb0 < st_hi;
                    if (need_mask) {
#pragma unroll
                        for (int x = 0; x < 16; ++x) {
                            const int kv = kb0 + acc_row(x, hh);
                            float p = fast_exp2(fmaf(sacc[x], c, -lse2));
                            p = (kv <= qi && kv >= st) ? p : 0.f;
                            pacc[x] = p * (pacc[x] - dl);   // dS^T
                        }
                    } else {
#pragma unroll
                        for (int x = 0; x < 16; ++x) pacc[x] = fast_exp2(fmaf(sacc[x], c, -lse2)) * (pacc[x] - dl);
                    }
                    sfr[0] = acc_chunk<T>(pacc, 0);
                    sfr[1] = acc_chunk<T>(pacc, 1);
#pragma unroll
                    for (int x = 0; x < NE; ++x) {
                        if (x + PDT < NE) tfr[x + PDT] = ld_ktr(kb, x + PDT);
                        issue_fence();
                        dqacc[x % DB] = mma(tfr[x], sfr[x / DB], dqacc[x % DB]);
                    }
                }
            }
        }
#pragma unroll
        for (int t = 0; t < DC; ++t) ra[t] ^= STAGE_BYTES;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            ta[db][0] ^= STAGE_BYTES;
            ta[db][1] ^= STAGE_BYTES;
        }
        stage ^= 1;
    }
    __syncthreads();   // everybody is done with the tile stages: they become the store patches
    if (!active) return;

    // Diagonal keys of blocks 1..j.  The workgroup's LDS is free now and every wave has 16 KB of it to
    // itself (its store patch lies inside): the K_l / V_l rows of the wave's 32 tokens are copied there
    // by LDS-DMA as whole 256-byte rows (fragment loads straight from global memory would touch 32 rows
    // with 32 bytes each per instruction) and read back as fragments; the copy of block lb + 1 is
    // requested as soon as the fragments of block lb are in registers.
    constexpr int WAVE_LDS = 2 * 32 * D * E::kBytes;
    static_assert(NW * WAVE_LDS <= 2 * STAGE_BYTES, "one region per wave");
    char* wbuf = smem + wave * WAVE_LDS;
    if (j >= 1) {
        frag dk[DC], dv[DC];
        auto request = [&](int lb) {   // straight from global memory (rows past the end clamped)
            const T* krow = static_cast<const T*>(a.k[lb]) + (int64_t)g * geo.kv_sh + (int64_t)qc * geo.kv_st;
            const T* vrow = static_cast<const T*>(a.v[lb]) + (int64_t)g * geo.kv_sh + (int64_t)qc * geo.kv_st;
#pragma unroll
            for (int t = 0; t < DC; ++t) {
                dk[t] = gload_frag<T>(krow + t * 16 + hh * 8);
                dv[t] = gload_frag<T>(vrow + t * 16 + hh * 8);
            }
        };
        auto apply = [&]() {
            float s = 0.f, dp = 0.f;
            uint32_t kk[DC][4];   // the key row in accumulator order, still packed
#pragma unroll
            for (int t = 0; t < DC; ++t) {
                s = dot8(qf[t], dk[t], s);
                dp = dot8(gof[t], dv[t], dp);
            }
            frags_to_acc_order_packed<T, DC>(dk, kk);
            s = half_sum(s);
            dp = half_sum(dp);
            const float p = fast_exp2(fmaf(s, c, -lse2));
            const float ds = p * (dp - dl);
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int i = 0; i < 16; ++i) dqacc[db][i] = fmaf(ds, acc_order_elem<DC>(kk, db, i), dqacc[db][i]);
        };
        if (wq0 + 32 <= Tn) {
            constexpr int NCP = 32 * TL::kPieces / 64;   // copy instructions per 32-row matrix
            uint32_t doff[NCP];                          // this lane's piece: bytes from the first row
            int lane_here = lane;
            asm volatile("" : "+v"(lane_here));          // computed here, not carried through the main loop
#pragma unroll
            for (int it = 0; it < NCP; ++it) {
                const int pidx = it * 64 + lane_here;
                const int r = pidx / TL::kPieces, pos = pidx % TL::kPieces;
                doff[it] = (uint32_t)((r * geo.kv_st + (pos ^ TL::swz(r)) * TL::kElemsPerPiece) * (int64_t)sizeof(T));
            }
            const uint32_t wl = __builtin_amdgcn_readfirstlane(lds0 + wave * WAVE_LDS);
            const int wq0u = __builtin_amdgcn_readfirstlane(wq0);   // wave-uniform copies of per-wave values
            auto copy = [&](int lb) {
                const T* kb = static_cast<const T*>(a.k[lb]) + (int64_t)g * geo.kv_sh + (int64_t)wq0u * geo.kv_st;
                const T* vb = static_cast<const T*>(a.v[lb]) + (int64_t)g * geo.kv_sh + (int64_t)wq0u * geo.kv_st;
#pragma unroll
                for (int it = 0; it < NCP; ++it) {
                    async_copy16(kb, doff[it], wl + it * 1024);
                    async_copy16(vb, doff[it], wl + WAVE_LDS / 2 + it * 1024);
                }
            };
            LaneFrags<T, D> lf;
            lf.init(lane_here);
            copy(1);
            for (int lb = 1; lb <= j; ++lb) {
                wait_async_copies();
#pragma unroll
                for (int t = 0; t < DC; ++t) {
                    dk[t] = lf.rowwise(wbuf, 0, t);
                    dv[t] = lf.rowwise(wbuf + WAVE_LDS / 2, 0, t);
                }
                if (lb < j) {
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the region is read out: refill it
                    copy(lb + 1);
                }
                apply();
            }
        } else {
            for (int lb = 1; lb <= j; ++lb) {
                request(lb);
                apply();
            }
        }
    }

    // scaled rows go through a wave-private LDS patch so that global stores are whole 16-byte pieces
    char* patch = wbuf;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            typename E::vec4 pk;
#pragma unroll
            for (int x = 0; x < 4; ++x) pk[x] = (T)(dqacc[db][i4 * 4 + x] * geo.scale);
            *reinterpret_cast<typename E::vec4*>(patch + TL::offset(n, db * 32 + i4 * 8 + hh * 4)) = pk;
        }
    T* obase = static_cast<T*>(a.dq[j]) + (int64_t)h * geo.q_sh;
#pragma unroll
    for (int it = 0; it < 32 * TL::kPieces / 64; ++it) {
        const int pidx = it * 64 + lane;
        const int r = pidx / TL::kPieces, piece = pidx % TL::kPieces;
        const int row = wq0 + r;
        const f32x4 val = *reinterpret_cast<const f32x4*>(patch + r * TL::kRowBytes + ((piece ^ TL::swz(r)) * 16));
        if (row < Tn) *reinterpret_cast<f32x4*>(obase + (int64_t)row * geo.q_st + piece * TL::kElemsPerPiece) = val;
    }
}

// ------------------------------------------------------------------------------------------------
// dK_0, dV_0: key-stationary
// ------------------------------------------------------------------------------------------------
template <typename T, int D, int NW>
__global__ __launch_bounds__(NW * 64) void ttt_bwd_dkv_kernel(const BwdArgs a) {
    using E = Elem<T>;
    using frag = typename E::frag;
    constexpr int KVT = NW * 32;   // kv rows per workgroup, 32 per wave
    constexpr int QTL = 64;        // query rows per LDS tile
    constexpr int DC = D / 16;
    constexpr int DB = D / 32;
    constexpr int NT = NW * 64;
    constexpr int TILE_BYTES = QTL * D * E::kBytes;
    constexpr int ROWV_BYTES = QTL * 4;
    constexpr int STAGE_BYTES = 2 * TILE_BYTES + 3 * ROWV_BYTES;

    extern __shared__ __align__(16) char smem[];
    auto sQ = [&](int s) -> char* { return smem + s * STAGE_BYTES; };
    auto sG = [&](int s) -> char* { return smem + s * STAGE_BYTES + TILE_BYTES; };
    auto sLse = [&](int s) -> float* { return reinterpret_cast<float*>(smem + s * STAGE_BYTES + 2 * TILE_BYTES); };
    auto sDl = [&](int s) -> float* { return sLse(s) + QTL; };
    auto sSt = [&](int s) -> int* { return reinterpret_cast<int*>(sLse(s) + 2 * QTL); };

    const Geometry& geo = a.geo;
    int g, rest;
    if (!decode_block(a.map, blockIdx.x, g, rest)) return;
    const int sp = rest % a.n_split;
    const int tile = rest / a.n_split;   // low tiles of a document have the longest query range: first

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hh = lane >> 5;
    const int Tn = geo.T;
    const int kv_tile0 = tile * KVT;
    const int wk0 = kv_tile0 + wave * 32;          // first kv row of this wave
    const bool active = wk0 < Tn;
    const int wk_hi = min(wk0 + 31, Tn - 1);
    // query rows that can see this workgroup's / this wave's keys
    const int q_end = __builtin_amdgcn_readfirstlane(a.tok_end[min(kv_tile0 + KVT - 1, Tn - 1)]);
    const int wq_end = active ? __builtin_amdgcn_readfirstlane(a.tok_end[wk_hi]) : 0;
    const int qt_lo = kv_tile0 / QTL;
    const int qt_hi = (q_end - 1) / QTL;
    const int nqt = qt_hi - qt_lo + 1;
    const int n_jh = geo.n_steps * geo.G;
    const int n_c = (n_jh - sp + a.n_split - 1) / a.n_split;   // (step, head) pairs of this split
    const int n_it = n_c * nqt;

    const T* K0 = static_cast<const T*>(a.k[0]) + (int64_t)g * geo.kv_sh;
    const T* V0 = static_cast<const T*>(a.v[0]) + (int64_t)g * geo.kv_sh;
    const int kc = min(wk0 + n, Tn - 1);
    const int kvi = wk0 + n;   // this lane's kv row (accumulator column)
    // K_0, V_0 rows as stationary B operands: lane (n,hh) holds row n, elements 16t + 8hh .. +8
    frag kf[DC], vf[DC];
#pragma unroll
    for (int t = 0; t < DC; ++t) {
        kf[t] = gload_frag<T>(K0 + (int64_t)kc * geo.kv_st + t * 16 + hh * 8);
        vf[t] = gload_frag<T>(V0 + (int64_t)kc * geo.kv_st + t * 16 + hh * 8);
    }
    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dkacc[db][i] = dvacc[db][i] = 0.f;
    const float c = geo.scale_log2;

    // stage loader: query tile `qt` of (step, head) pair number `ci` of this split
    auto issue = [&](int it, int s) {
        const int ci = it / nqt, qt = qt_lo + it % nqt;
        const int jh = sp + ci * a.n_split;
        const int js = jh / geo.G, h = g * geo.G + jh % geo.G;
        const int j = geo.step_begin + js;
        const T* Qj = static_cast<const T*>(a.q[j]) + (int64_t)h * geo.q_sh;
        const T* dOj = static_cast<const T*>(a.d_o[j]) + (int64_t)h * geo.q_sh;
        tile_load_async<T, D, QTL, NT>(sQ(s), Qj, geo.q_st, qt * QTL, Tn - 1, tid);
        tile_load_async<T, D, QTL, NT>(sG(s), dOj, geo.q_st, qt * QTL, Tn - 1, tid);
        if (tid < QTL) {
            const int q = qt * QTL + tid;
            const bool in = q < Tn;
            const int qq = in ? q : Tn - 1;
            // rows past the end get LSE = +inf so that p = 0
            sLse(s)[tid] = in ? a.lse[j][(int64_t)h * geo.lse_st + qq] * kLog2e : INFINITY;
            sDl(s)[tid] = in ? a.delta[((int64_t)js * geo.hq + h) * Tn + qq] : 0.f;
            sSt(s)[tid] = a.tok_start[qq];
        }
    };

    if (n_it > 0) issue(0, 0);
    int stage = 0;
    for (int it = 0; it < n_it; ++it) {
        wait_async_copies();
        __syncthreads();
        if (it + 1 < n_it) issue(it + 1, stage ^ 1);
        const int q0 = (qt_lo + it % nqt) * QTL;
        // this wave's keys are seen by query rows [wk0, wq_end)
        if (active && q0 + QTL - 1 >= wk0 && q0 < wq_end) {
            const char* tq = sQ(stage);
            const char* tg = sG(stage);
            const float* tl = sLse(stage);
            const float* td = sDl(stage);
            const int* ts = sSt(stage);
#pragma unroll
            for (int qb = 0; qb < QTL / 32; ++qb) {
                const int qb0 = q0 + qb * 32;
                if (qb0 + 31 < wk0 || qb0 >= wq_end) continue;
                // fragments are read where they are used (this kernel serves the fp32 instantiation;
                // 16-bit types take ttt_bwd_dkv_p8_kernel)
                frag qa[DC], ga[DC], gt[2][DB], qt[2][DB];
                // S[q, kv] = Q K^T and dP[q, kv] = dO V^T : lane = kv column, values = query rows
                f32x16 sacc, pacc;
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[i] = pacc[i] = 0.f;
#pragma unroll
                for (int t = 0; t < DC; ++t) {
                    qa[t] = frag_rowwise<T, D>(tq, qb * 32 + n, t * 16 + hh * 8);
                    ga[t] = frag_rowwise<T, D>(tg, qb * 32 + n, t * 16 + hh * 8);
                    sacc = mma(qa[t], kf[t], sacc);
                    pacc = mma(ga[t], vf[t], pacc);
                }
                // every row of the block sees every key of the wave iff the block is below the
                // wave's last key and starts its document at or before the wave's first key
                const bool need_mask = qb0 < wk0 + 31 || ts[min(qb * 32 + 31, QTL - 1)] > wk0 || qb0 + 31 >= wq_end;
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) {
                    const int r = qb * 32 + i4 * 8 + hh * 4;
                    const f32x4 l4 = *reinterpret_cast<const f32x4*>(tl + r);
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(td + r);
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int i = i4 * 4 + x;
                        float p = fast_exp2(fmaf(sacc[i], c, -l4[x]));
                        if (need_mask) {
                            const int q = q0 + r + x;
                            p = (kvi <= q && kvi >= ts[r + x]) ? p : 0.f;
                        }
                        sacc[i] = p;                       // P
                        pacc[i] = p * (pacc[i] - d4[x]);   // dS
                    }
                }
                // dV[kv, d] += P^T dO ;  dK[kv, d] += dS^T Q
#pragma unroll
                for (int c2 = 0; c2 < 2; ++c2) {
                    const frag pf = acc_chunk<T>(sacc, c2);
                    const frag sf = acc_chunk<T>(pacc, c2);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        gt[c2][db] = frag_transposed<T, D>(tg, qb * 32 + c2 * 16, db * 32, lane);
                        qt[c2][db] = frag_transposed<T, D>(tq, qb * 32 + c2 * 16, db * 32, lane);
                        dvacc[db] = mma(pf, gt[c2][db], dvacc[db]);
                        dkacc[db] = mma(sf, qt[c2][db], dkacc[db]);
                    }
                }
            }
        }
        stage ^= 1;
    }
    if (!active) return;

    // fp32 partial sums of this split -> block-0 accumulators [T][hkv][D]
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int kv = wk0 + acc_row(i, hh);
            if (kv < Tn) {
                const int64_t off = ((int64_t)kv * geo.hkv + g) * D + db * 32 + n;
                atomicAdd(a.dk0_acc + off, dkacc[db][i]);
                atomicAdd(a.dv0_acc + off, dvacc[db][i]);
            }
        }
}

// ------------------------------------------------------------------------------------------------
// dK_0, dV_0: key-stationary, eight equal waves (16-bit element types)
//
// Measured on MI355X: a wave issues at most one instruction (of any kind) every ~8 cycles, so the
// time of a step is close to 8 cycles x the instructions a wave executes in it, and the two waves of
// a SIMD are worth most as two independent instruction streams doing the same work on different
// data.  Hence: eight equal waves, and as few instructions per block as the arithmetic allows (stage
// offsets as immediates in an unrolled pair of steps, pointers advanced instead of recomputed, LDS
// reads and waits in pairs).  Workgroup = 128
// key rows; wave w owns the 32 keys of pair w & 3 (fp32 dK, dV accumulators in registers) and takes
// every second query block: group w >> 2 = parity of the block.  The K_0 / V_0 rows of the tile sit
// in LDS for the whole tile (row-wise B operands of S = Q K^T and dP = dO V^T); query blocks (Q and
// dO rows, LSE*log2e, D, document start) stream through a two-stage LDS ring, each group copying the
// blocks it will use.  P and dS never leave the registers: the 16 accumulator values of a lane are
// already two A-operand chunks of dV += P^T dO and dK += dS^T Q, whose B operands are read
// transposed from the same stage.  One workgroup barrier per pair of blocks.  The two waves that
// share a key range both add their partial sums to the fp32 accumulators in global memory.
// ------------------------------------------------------------------------------------------------
template <typename T, int D> struct DkvP8 {
    static constexpr int kKeys = 128;
    static constexpr int kBlk = 32 * D * (int)sizeof(T);      // one 32-row block of one matrix
    static constexpr int kSlot = 2 * kBlk;                    // Q block + dO block of one query block
    static constexpr int kStage = 2 * kSlot;                  // one query block per wave group
    static constexpr int kStages = 2;
    static constexpr int kKBase = kStages * kStage;
    static constexpr int kVBase = kKBase + kKeys * D * (int)sizeof(T);
    static constexpr int kVecBase = kVBase + kKeys * D * (int)sizeof(T);
    static constexpr int kVecSlot = 3 * 32 * 4;               // LSE*log2e, D, first token of the document
    static constexpr int kVecStage = 2 * kVecSlot;
    static constexpr int kLds = kVecBase + kStages * kVecStage;
    static constexpr int kChunk = kKeys * 32;                 // 16 columns of all keys, operand-major
};

template <typename T, int D>
__device__ __forceinline__ void dkv_p8_tile(const BwdArgs& a, char* smem, const int g, const int sp, const int tile,
                                            const int chunk) {
    static_assert(sizeof(T) == 2, "this dK/dV kernel is for 16-bit elements");
    using E = Elem<T>;
    using frag = typename E::frag;
    using TL = Tile<T, D>;
    using C = DkvP8<T, D>;
    constexpr int KVT = C::kKeys;
    constexpr int DC = D / 16;
    constexpr int DB = D / 32;
    constexpr int NE = 4 * DB;                // dV / dK matrix instructions per block
    static_assert((C::kStage & (C::kStage - 1)) == 0, "the stage bit is toggled with XOR");
    typedef __attribute__((address_space(3))) char lds_char;
    typedef __attribute__((address_space(3))) frag lds_frag;
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_char*)smem;
    const Geometry& geo = a.geo;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pair = wave & 3, grp = wave >> 2;
    const int n = lane & 31, hh = lane >> 5;
    const int Tn = geo.T;
    const int kv_tile0 = tile * KVT;
    const int wk0 = kv_tile0 + pair * 32;
    const bool active = wk0 < Tn;
    const int wk_hi = min(wk0 + 31, Tn - 1);
    const int q_end = __builtin_amdgcn_readfirstlane(a.tok_end[min(kv_tile0 + KVT - 1, Tn - 1)]);
    const int wq_end = active ? __builtin_amdgcn_readfirstlane(a.tok_end[wk_hi]) : 0;
    const bool wave_split = active && __builtin_amdgcn_readfirstlane(a.tok_start[wk_hi]) > wk0;
    const int kvi = wk0 + n;
    // query blocks of this chunk that see a key of this tile
    const int qb_lo = max(kv_tile0 / 32, chunk * a.chunk_blocks);
    const int nqb = min((q_end - 1) / 32, (chunk + 1) * a.chunk_blocks - 1) - qb_lo + 1;
    if (nqb <= 0) return;
    const int wq_lim = min(wq_end, (qb_lo + nqb) * 32);   // blocks from here on are not this unit's
    const int n_jh = geo.n_steps * geo.G;
    const int n_c = (n_jh - sp + a.n_split - 1) / a.n_split;
    const int nqb2 = (nqb + 1) / 2;           // steps per (step, head) pair: one block per wave group
    const int n_steps2 = n_c * nqb2;
    const float c = geo.scale_log2;

    // K_0, V_0 rows of the tile -> LDS
    {
        const T* K0 = static_cast<const T*>(a.k[0]) + (int64_t)g * geo.kv_sh;
        const T* V0 = static_cast<const T*>(a.v[0]) + (int64_t)g * geo.kv_sh;
        // operand-major layout [chunk of 16 columns][32-key pair][column half][key]: a lane's row
        // fragment of chunk t is at (its own 16 bytes) + t * kChunk, so one address register serves
        // all chunks of K and V, and consecutive lanes read consecutive 16-byte pieces
        for (int u = wave; u < DC * 4; u += 8) {
            const int t = u >> 2, rg = u & 3;
            const int row = min(kv_tile0 + rg * 32 + n, Tn - 1);
            const int64_t off = (int64_t)row * geo.kv_st + (2 * t + hh) * 8;
            const uint32_t dst = lds0 + t * C::kChunk + rg * 1024;
            async_copy16(K0 + off, dst + C::kKBase);
            async_copy16(V0 + off, dst + C::kVBase);
        }
    }

    // per-lane LDS addresses: query-block fragments (this group's slot of stage 0), the pair's K rows
    uint32_t ra[DC], ta[DB][2];
    const uint32_t ka = lds0 + C::kKBase + pair * 1024 + lane * 16;
    static_assert((DC - 1) * C::kChunk + C::kVBase - C::kKBase < 65536, "LDS offsets are 16-bit immediates");
    {
        LaneFrags<T, D> lf;
        lf.init(lane);
#pragma unroll
        for (int t = 0; t < DC; ++t) ra[t] = lds0 + lf.row[t] + grp * C::kSlot;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            ta[db][0] = lds0 + lf.tr[db][0] + grp * C::kSlot;
            ta[db][1] = lds0 + lf.tr[db][1] + grp * C::kSlot;
        }
    }
    const uint32_t va = lds0 + C::kVecBase + grp * C::kVecSlot + hh * 16;
    auto ld = [&](uint32_t addr) -> frag { return *reinterpret_cast<const lds_frag*>((uintptr_t)addr); };
    auto ld_tr = [&](uint32_t stage_off, int which, int c2, int db) -> frag {
        const uint32_t off = stage_off + which * C::kBlk + c2 * 16 * TL::kRowBytes;
        union { s16x4 s[2]; frag v; } u;
        u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(ta[db][0] + off));
        u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(ta[db][1] + off));
        return u.v;
    };
    auto ld_vec = [&](uint32_t off, int i4) -> f32x4 {
        return *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>((uintptr_t)(va + off + i4 * 32));
    };

    // ---- copies: the 256 threads of a group copy the group's next block (32 x kPieces 16-byte
    // pieces per matrix) and its three per-row vectors.  Group grp takes the query blocks
    // qb_lo + 2 nqb2 - 1 - grp - 2 i, i < nqb2, of one (step, head) pair after the other; if the number
    // of blocks is odd, the first block of group 0 lies past every query that sees the tile and is
    // skipped.  The sweep runs from the last query block down to the tile's own: all key tiles of a
    // (kv head, split) start a pair at the same block, so the workgroups that share an XCD read the
    // same Q / dO rows at about the same time and find them in its L2.
    constexpr int NLD = 32 * TL::kPieces / 256;
    const int gw = wave & 3, gt = tid & 255;
    uint32_t src_off[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int pidx = (i * 4 + gw) * 64 + lane;
        const int r = pidx / TL::kPieces, pos = pidx % TL::kPieces;
        src_off[i] = (uint32_t)((r * geo.q_st + (pos ^ TL::swz(r)) * TL::kElemsPerPiece) * (int64_t)sizeof(T));
    }
    const uint32_t vec_off = (uint32_t)(lane & 31) * 4;
    const uint32_t dst0 = __builtin_amdgcn_readfirstlane(lds0 + grp * C::kSlot + gw * 1024);
    const uint32_t vdst0 = __builtin_amdgcn_readfirstlane(lds0 + C::kVecBase + grp * C::kVecSlot);
    const int64_t blk2_stride = (int64_t)64 * geo.q_st;       // two blocks, in elements
    const int qb_top = qb_lo + 2 * nqb2 - 1 - grp;            // this group's first block: the sweep runs downwards
    struct Pos {
        int i, ci;             // block 2 i + grp of (step, head) pair number ci of this split
        const T *q, *g;        // first row of the block in Q_j and dO_j of that head
    };
    const T *head_q = nullptr, *head_g = nullptr;             // of the pair the next request is in
    const float *head_l = nullptr, *head_d = nullptr;
    auto enter_pair = [&](Pos& ps) {
        const int jh = sp + ps.ci * a.n_split;
        const int js = jh / geo.G, h = g * geo.G + jh % geo.G;
        const int j = geo.step_begin + js;
        head_q = static_cast<const T*>(a.q[j]) + (int64_t)h * geo.q_sh;
        head_g = static_cast<const T*>(a.d_o[j]) + (int64_t)h * geo.q_sh;
        const int64_t at = ((int64_t)js * geo.hq + h) * Tn;
        head_l = a.lse2 + at;
        head_d = a.delta + at;
        const int64_t first = (int64_t)qb_top * 32 * geo.q_st;
        ps.q = head_q + first;
        ps.g = head_g + first;
    };
    auto advance = [&](Pos& ps) {
        if (++ps.i == nqb2) {
            ps.i = 0;
            ++ps.ci;
            if (ps.ci < n_c) enter_pair(ps);
        } else {
            ps.q -= blk2_stride;
            ps.g -= blk2_stride;
        }
    };
    auto request = [&](const Pos& ps, auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        const uint32_t st = dst0 + ST * C::kStage;
        const uint32_t vec = vdst0 + ST * C::kVecStage;
        const int row0 = (qb_top - 2 * ps.i) * 32;
        if (row0 + 32 <= Tn) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                async_copy16(ps.q, src_off[i], st + i * 4096);
                async_copy16(ps.g, src_off[i], st + C::kBlk + i * 4096);
            }
            if (gt < 32) {
                async_copy4(head_l + row0, vec_off, vec);
                async_copy4(head_d + row0, vec_off, vec + 128);
                async_copy4(a.tok_start + row0, vec_off, vec + 256);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int pidx = (i * 4 + gw) * 64 + lane;
                const int r = pidx / TL::kPieces, pos = pidx % TL::kPieces;
                const int row = min(row0 + r, Tn - 1);            // rows past the end are masked later
                const int64_t off = (int64_t)row * geo.q_st + (pos ^ TL::swz(r)) * TL::kElemsPerPiece;
                async_copy16(head_q + off, st + i * 4096);
                async_copy16(head_g + off, st + C::kBlk + i * 4096);
            }
            if (gt < 32) {
                const int qq = min(row0 + gt, Tn - 1);
                async_copy4(head_l + qq, vec);
                async_copy4(head_d + qq, vec + 128);
                async_copy4(a.tok_start + qq, vec + 256);
            }
        }
    };
    Pos nxt{0, 0, nullptr, nullptr};
    enter_pair(nxt);
    request(nxt, IntC<0>{});

    f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) dkacc[db][i] = dvacc[db][i] = 0.f;

    wait_async_copies();
    __syncthreads();

    // One step: request the blocks of the next step into the other stage, then this wave's block from
    // stage ST (a compile-time constant, so that every LDS address is a register plus an immediate).
    auto step = [&](const bool more, auto stage_c) {
        constexpr int ST = decltype(stage_c)::value;
        constexpr uint32_t SO = ST * C::kStage;
        constexpr uint32_t VO = ST * C::kVecStage;
        const int q0 = (qb_top - 2 * nxt.i) * 32;
        if (more) {
            advance(nxt);
            request(nxt, IntC<1 - ST>{});
        }
        if (active && q0 + 31 >= wk0 && q0 < wq_lim) {
            // ---- S = Q K^T, dP = dO V^T for the pair's 32 keys, two contraction chunks at a time
            f32x16 sacc, pacc;
            {
                frag qa[DC], kf[DC];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    qa[t] = ld(ra[t] + SO);
                    kf[t] = ld(ka + t * C::kChunk);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
                for (int t = 0; t < DC; t += 2) {
                    if (t + 2 < DC) {
#pragma unroll
                        for (int u = t + 2; u < t + 4; ++u) {
                            qa[u] = ld(ra[u] + SO);
                            kf[u] = ld(ka + u * C::kChunk);
                        }
                    }
                    issue_fence();
                    sacc = mma(qa[t], kf[t], sacc);
                    sacc = mma(qa[t + 1], kf[t + 1], sacc);
                }
            }
            {
                frag ga[DC], vf[DC];
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    ga[t] = ld(ra[t] + SO + C::kBlk);
                    vf[t] = ld(ka + t * C::kChunk + (C::kVBase - C::kKBase));
                }
#pragma unroll
                for (int i = 0; i < 16; ++i) pacc[i] = 0.f;
#pragma unroll
                for (int t = 0; t < DC; t += 2) {
                    if (t + 2 < DC) {
#pragma unroll
                        for (int u = t + 2; u < t + 4; ++u) {
                            ga[u] = ld(ra[u] + SO + C::kBlk);
                            vf[u] = ld(ka + u * C::kChunk + (C::kVBase - C::kKBase));
                        }
                    }
                    issue_fence();
                    pacc = mma(ga[t], vf[t], pacc);
                    pacc = mma(ga[t + 1], vf[t + 1], pacc);
                }
            }
            // ---- P and dS.  Every row of the block sees every key of the pair iff the block lies at
            // or below the pair's last key, ends before that key's document does, and the pair's keys
            // are all in one document
            const bool need_mask = q0 < wk0 + 31 || q0 + 31 >= wq_end || wave_split;
            {
                f32x4 l4[4];
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) l4[i4] = ld_vec(VO, i4);
                if (need_mask) {
                    f32x4 s4[4];
#pragma unroll
                    for (int i4 = 0; i4 < 4; ++i4) s4[i4] = ld_vec(VO + 256, i4);
#pragma unroll
                    for (int x = 0; x < 16; ++x) {
                        const int q = q0 + acc_row(x, hh);
                        const float p = fast_exp2(fmaf(sacc[x], c, -l4[x / 4][x % 4]));
                        const bool see = (kvi <= q) & (q < wq_end) & (kvi >= __float_as_int(s4[x / 4][x % 4]));
                        sacc[x] = see ? p : 0.f;
                    }
                } else {
#pragma unroll
                    for (int x = 0; x < 16; ++x) sacc[x] = fast_exp2(fmaf(sacc[x], c, -l4[x / 4][x % 4]));
                }
            }
            issue_fence();
            frag tfr[NE];
#pragma unroll
            for (int x = 0; x < 2; ++x) tfr[x] = ld_tr(SO, 1 - (x & 1), (x >> 1) / DB, (x >> 1) % DB);
            {
                f32x4 d4[4];
#pragma unroll
                for (int i4 = 0; i4 < 4; ++i4) d4[i4] = ld_vec(VO + 128, i4);
#pragma unroll
                for (int x = 0; x < 16; ++x) pacc[x] = sacc[x] * (pacc[x] - d4[x / 4][x % 4]);
            }
            // ---- dV += P^T dO, dK += dS^T Q: the accumulator chunks are the A operands as they are
            frag pfr[2], sfr[2];
#pragma unroll
            for (int c2 = 0; c2 < 2; ++c2) {
                pfr[c2] = acc_chunk<T>(sacc, c2);
                sfr[c2] = acc_chunk<T>(pacc, c2);
            }
            // transposed fragment x = (c2 * DB + db) * 2 + (0: dO for dV, 1: Q for dK), two at a time
#pragma unroll
            for (int x = 0; x < NE; x += 2) {
                if (x + 2 < NE) {
#pragma unroll
                    for (int y = x + 2; y < x + 4; ++y) tfr[y] = ld_tr(SO, 1 - (y & 1), (y >> 1) / DB, (y >> 1) % DB);
                }
                issue_fence();
                const int c2 = (x >> 1) / DB, db = (x >> 1) % DB;
                dvacc[db] = mma(pfr[c2], tfr[x], dvacc[db]);
                dkacc[db] = mma(sfr[c2], tfr[x + 1], dkacc[db]);
            }
        }
        wait_async_copies();
        lds_barrier();   // the blocks of the next step are in LDS; everybody is done with those of this one
    };
    for (int s = 0; s < n_steps2; s += 2) {
        step(s + 1 < n_steps2, IntC<0>{});
        if (s + 1 < n_steps2) step(s + 2 < n_steps2, IntC<1>{});
    }
    // The two waves of a key range first add their sums in LDS (the last barrier of the loop has
    // freed all of it): half as many atomics.  Quad q of a lane's accumulators sits at
    // (q * 256 + pair * 64 + lane) * 16 bytes.
    static_assert(2 * DB * 4 * 256 * 16 <= C::kLds, "the sums of one wave group fit in LDS");
    typedef __attribute__((address_space(3))) f32x4 lds_f32x4;
    const uint32_t sum_addr = lds0 + (pair * 64 + lane) * 16;
    if (grp == 1) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i4 = 0; i4 < 4; ++i4) {
                *(lds_f32x4*)(uintptr_t)(sum_addr + ((db * 4 + i4) * 2 + 0) * 4096) =
                    f32x4{dkacc[db][4 * i4], dkacc[db][4 * i4 + 1], dkacc[db][4 * i4 + 2], dkacc[db][4 * i4 + 3]};
                *(lds_f32x4*)(uintptr_t)(sum_addr + ((db * 4 + i4) * 2 + 1) * 4096) =
                    f32x4{dvacc[db][4 * i4], dvacc[db][4 * i4 + 1], dvacc[db][4 * i4 + 2], dvacc[db][4 * i4 + 3]};
            }
    }
    __syncthreads();
    if (!active || grp == 1) return;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
            const f32x4 k4 = *(const lds_f32x4*)(uintptr_t)(sum_addr + ((db * 4 + i4) * 2 + 0) * 4096);
            const f32x4 v4 = *(const lds_f32x4*)(uintptr_t)(sum_addr + ((db * 4 + i4) * 2 + 1) * 4096);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = 4 * i4 + e;
                const int kv = wk0 + acc_row(i, hh);
                if (kv < Tn) {
                    const int64_t off = ((int64_t)kv * geo.hkv + g) * D + db * 32 + n;
                    atomicAdd(a.dk0_acc + off, dkacc[db][i] + k4[e]);
                    atomicAdd(a.dv0_acc + off, dvacc[db][i] + v4[e]);
                }
            }
        }
}

// One workgroup = one key tile x one chunk of `chunk_blocks` query blocks x one split of the
// (step, head) list of the kv head.  Units are numbered chunk by chunk, the tiles that a chunk can
// see (those that begin at or before its last row) side by side: workgroups with consecutive numbers
// stream the same Q / dO rows, (step, head) pair after pair, each pair costing all of them the same
// number of blocks -- except the few tiles on the chunk's diagonal -- so they stay together and the
// rows are read from HBM once per XCD, not once per workgroup.
template <typename T, int D>
__global__ __launch_bounds__(512) void ttt_bwd_dkv_p8_kernel(const BwdArgs a) {
    extern __shared__ __align__(16) char smem[];
    int g, rest;
    if (!decode_block(a.map, blockIdx.x, g, rest)) return;
    const int sp = rest / a.n_units;
    int r = rest % a.n_units;
    int chunk = 0;
    for (;; ++chunk) {
        const int tiles = min(a.n_tiles, (chunk + 1) * a.chunk_blocks / 4);   // 128-key tiles = 4 blocks
        if (r < tiles) break;
        r -= tiles;
    }
    dkv_p8_tile<T, D>(a, smem, g, sp, r, chunk);
}

// ------------------------------------------------------------------------------------------------
// small helpers: clear the block-0 accumulators; convert them to the output dtype
// ------------------------------------------------------------------------------------------------
__global__ void ttt_fill_zero_kernel(f32x4* __restrict__ p, int64_t n4) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) p[i] = f32x4{0.f, 0.f, 0.f, 0.f};
}

template <typename T, int D>
__global__ void ttt_bwd_finish_kernel(const BwdArgs a) {
    const Geometry& geo = a.geo;
    const int64_t n4 = (int64_t)geo.T * geo.hkv * (D / 4);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < n4; x += stride) {
        const int d4 = (int)(x % (D / 4));
        const int64_t tg = x / (D / 4);
        const int g = (int)(tg % geo.hkv);
        const int64_t t = tg / geo.hkv;
        const f32x4 k4 = reinterpret_cast<const f32x4*>(a.dk0_acc)[x];
        const f32x4 v4 = reinterpret_cast<const f32x4*>(a.dv0_acc)[x];
        const int64_t off = t * geo.kv_st + (int64_t)g * geo.kv_sh + d4 * 4;
        gstore_vec4<T>(static_cast<T*>(a.dk[0]) + off, k4[0] * geo.scale, k4[1] * geo.scale, k4[2] * geo.scale,
                       k4[3] * geo.scale);
        gstore_vec4<T>(static_cast<T*>(a.dv[0]) + off, v4[0], v4[1], v4[2], v4[3]);
    }
}

// ------------------------------------------------------------------------------------------------
// launch sequence
// ------------------------------------------------------------------------------------------------
static void set_head_map(HeadMap& m, int hkv, int rest_count, int64_t& grid) {
    m.hkv = hkv;
    m.rest_count = rest_count;
    if (hkv % 8 == 0) {
        m.mode = 1;
        grid = (int64_t)hkv * rest_count;
    } else if (8 % hkv == 0) {
        m.mode = 2;
        const int xp = 8 / hkv;
        grid = 8 * (int64_t)((rest_count + xp - 1) / xp);
    } else {
        m.mode = 0;
        grid = (int64_t)hkv * rest_count;
    }
}

// ------------------------------------------------------------------------------------------------
// Work split of the eight-wave dK/dV kernel: 32-row query blocks per chunk and ways to split the
// (step, head) list, chosen by a model of the launch.
//
// One workgroup fills a compute unit and handles one unit = (128-key tile, chunk, split).  Measured
// on MI355X (sweeps over chunk size and split at 2048 / 4096 / 16384 tokens, all steps and one step
// per call): a unit costs about 1.9 us per step (one 32-row query block per wave group and (step,
// head) pair) plus about 13 us of its own (workgroup launch, the K_0/V_0 tile and first query block
// arriving, the flush of its sums through LDS and fp32 atomics), and an empty unit (a tile that no
// row of the chunk sees) about 1 us.  The model deals one kv head's units, in launch order, to the
// head's share of the compute units (each to the one that frees up first) and takes the
// combination with the shortest finish time; it reproduces the sweeps within 10 % and their
// ranking.  Short (step, head) lists -- one step per call -- want long chunks (few units, little
// flushing).  Long lists keep the 512-row chunks: the model does not see HBM traffic, and with
// 2048-row chunks the units of one XCD no longer stream the same Q / dO rows together (measured at
// 4096 tokens, all steps: 2.6 GB fetched per launch against 0.9 GB, for 2 % of the kernel's time).
// ------------------------------------------------------------------------------------------------
struct DkvPlan {
    int chunk_blocks, n_split, n_units;
};

static int dkv_units_of(int T, int n_tiles, int chunk_blocks) {
    const int n_chunks = (T + chunk_blocks * 32 - 1) / (chunk_blocks * 32);
    int n = 0;
    for (int ch = 0; ch < n_chunks; ++ch) n += std::min(n_tiles, (ch + 1) * chunk_blocks / 4);
    return n;
}

static DkvPlan plan_dkv_split(const BwdArgs& a, int n_jh, int n_cu) {
    const Geometry& geo = a.geo;
    const int T = geo.T;
    const int n_tiles = (T + 127) / 128;
    constexpr double kStepUs = 1.9, kUnitUs = 13.0, kEmptyUs = 1.0;
    // one entry per distinct request: the plan depends on the document structure, the list length and the device
    struct Key {
        int T, n_docs, n_jh, hkv, n_cu;
        uint64_t cu_hash;
        bool operator==(const Key& o) const {
            return T == o.T && n_docs == o.n_docs && n_jh == o.n_jh && hkv == o.hkv && n_cu == o.n_cu && cu_hash == o.cu_hash;
        }
    };
    uint64_t h = 1469598103934665603ull;
    for (int r = 0; r <= a.n_docs; ++r) h = (h ^ (uint64_t)(uint32_t)(a.cu_host[r] - a.cu_base)) * 1099511628211ull;
    const Key key{T, a.n_docs, n_jh, geo.hkv, n_cu, h};
    static std::mutex mu;
    static std::vector<std::pair<Key, DkvPlan>> cache;
    {
        std::lock_guard<std::mutex> lock(mu);
        for (const auto& e : cache)
            if (e.first == key) return e.second;
    }
    // last query row (+1) that sees the last key of each tile: the end of that key's document
    std::vector<int> q_end(n_tiles);
    {
        int r = 0;
        for (int t = 0; t < n_tiles; ++t) {
            const int key_tok = std::min(t * 128 + 127, T - 1);
            while (r + 1 < a.n_docs && a.cu_host[r + 1] - a.cu_base <= key_tok) ++r;
            q_end[t] = a.cu_host[r + 1] - a.cu_base;
        }
    }
    const int cus = std::max(1, n_cu / geo.hkv);   // a kv head's share of the device
    DkvPlan best{16, 1, 0};
    double best_us = -1.;
    std::vector<int> nqb2;
    for (int cb : {16, 32, 64}) {
        if (cb > 16 && n_jh > 8) break;
        const int n_chunks = (T + cb * 32 - 1) / (cb * 32);
        nqb2.clear();
        for (int ch = 0; ch < n_chunks; ++ch) {
            const int tiles = std::min(n_tiles, (ch + 1) * cb / 4);
            for (int t = 0; t < tiles; ++t) {
                const int qb_lo = std::max(t * 4, ch * cb);
                const int nqb = std::min((q_end[t] - 1) / 32, (ch + 1) * cb - 1) - qb_lo + 1;
                nqb2.push_back(nqb > 0 ? (nqb + 1) / 2 : 0);
            }
        }
        for (int ns : {1, 2, 3, 4, 6, 8}) {
            if (ns > n_jh) break;
            double finish = 0.;
            if ((int64_t)nqb2.size() * ns <= 8192) {
                std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
                for (int c = 0; c < cus; ++c) free_at.push(0.);
                for (int sp = 0; sp < ns; ++sp) {
                    const int n_c = (n_jh - sp + ns - 1) / ns;
                    for (int u : nqb2) {
                        const double t0 = free_at.top();
                        free_at.pop();
                        const double t1 = t0 + (u > 0 ? (double)n_c * u * kStepUs + kUnitUs : kEmptyUs);
                        free_at.push(t1);
                        finish = std::max(finish, t1);
                    }
                }
            } else {   // very many units: the tail does not matter, the work and the per-unit cost do
                double work = 0., longest = 0.;
                for (int u : nqb2) {
                    work += u > 0 ? (double)n_jh * u * kStepUs + ns * kUnitUs : ns * kEmptyUs;
                    longest = std::max(longest, (double)((n_jh + ns - 1) / ns) * u * kStepUs + kUnitUs);
                }
                finish = work / cus + longest;
            }
            if (best_us < 0. || finish < best_us) {
                best_us = finish;
                best = DkvPlan{cb, ns, (int)nqb2.size()};
            }
        }
    }
    std::lock_guard<std::mutex> lock(mu);
    if (cache.size() >= 64) cache.erase(cache.begin());
    cache.emplace_back(key, best);
    return best;
}

template <typename T, int D, int QB_DQ, int NW_DQ, int NW_KV>
static hipError_t launch_bwd_t(BwdArgs& a, hipStream_t stream) {
    const Geometry& geo = a.geo;
    hipError_t e;
    const int64_t acc_n4 = (int64_t)geo.T * geo.hkv * (D / 4);

    // 1. clear the block-0 accumulators unless a carry from later steps is being continued
    if (!a.accumulate || a.carry_reset) {
        ProfileScope prof("ttt_fill_zero_kernel", stream);
        // the two accumulators follow each other in the workspace (the second one 256-byte aligned):
        // one launch clears both when nothing lies between them
        const bool adjacent = a.dv0_acc == a.dk0_acc + 4 * acc_n4;
        const int64_t n4 = adjacent ? 2 * acc_n4 : acc_n4;
        const int blocks = (int)((n4 + 255) / 256 < 8192 ? (n4 + 255) / 256 : 8192);
        hipLaunchKernelGGL(ttt_fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<f32x4*>(a.dk0_acc), n4);
        if (!adjacent)
            hipLaunchKernelGGL(ttt_fill_zero_kernel, dim3(blocks), dim3(256), 0, stream, reinterpret_cast<f32x4*>(a.dv0_acc), n4);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    // 2. D and the diagonal blocks
    {
        constexpr int UPB = 256 / (D / 8);
        const int64_t units = (int64_t)geo.T * geo.hkv;
        const int64_t grid = (units + UPB - 1) / UPB;
        const size_t lds = (size_t)UPB * geo.n_steps * geo.G * sizeof(float);
        if (grid > 0x7fffffffLL || lds > 160 * 1024) return hipErrorInvalidValue;
        constexpr int KREG = 8;   // steps whose diagonal rows and gradients fit the register file
        bool in_regs = false;
        if constexpr (sizeof(T) == 2) in_regs = geo.step_begin + geo.n_steps <= KREG;
        if (in_regs) {
            if constexpr (sizeof(T) == 2) {
                ProfileScope prof("ttt_bwd_pre_regs_kernel", stream);
                hipLaunchKernelGGL((ttt_bwd_pre_regs_kernel<T, D, KREG, 2>), dim3((unsigned)grid), dim3(256), 0, stream, a);
            }
        } else {
            auto kern = ttt_bwd_pre_kernel<T, D>;
            if (lds > 48 * 1024) {
                e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
                if (e != hipSuccess) return e;
            }
            ProfileScope prof("ttt_bwd_pre_kernel", stream);
            hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, stream, a);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    // 3. dQ
    {
        constexpr bool kPipe = sizeof(T) == 2;
        constexpr int NWQ = kPipe ? 8 : NW_DQ;
        constexpr int QT = NWQ * (kPipe ? 1 : QB_DQ) * 32;
        constexpr int LDS = kPipe ? 2 * (1 << 16) : 4 * 64 * D * (int)sizeof(T);
        const void* kern;
        if constexpr (kPipe) kern = (const void*)ttt_bwd_dq_pipe_kernel<T, D, NWQ>;
        else kern = (const void*)ttt_bwd_dq_kernel<T, D, QB_DQ, NW_DQ>;
        static LdsOptIn lds_opt_in;
        if ((e = lds_opt_in.ensure(kern, LDS)) != hipSuccess) return e;
        // the pipelined kernel addresses the pieces of up to 64 rows of K or V with 32-bit byte offsets
        if (kPipe && geo.kv_st * 64 * (int64_t)sizeof(T) >= (int64_t)1 << 32) return hipErrorInvalidValue;
        a.n_tiles = (geo.T + QT - 1) / QT;
        int64_t grid;
        set_head_map(a.map, geo.hkv, a.n_tiles * geo.n_steps * geo.G, grid);
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        {
            ProfileScope prof(kPipe ? "ttt_bwd_dq_pipe_kernel" : "ttt_bwd_dq_kernel", stream);
            if constexpr (kPipe)
                hipLaunchKernelGGL((ttt_bwd_dq_pipe_kernel<T, D, NWQ>), dim3((unsigned)grid), dim3(NWQ * 64), LDS, stream, a);
            else
                hipLaunchKernelGGL((ttt_bwd_dq_kernel<T, D, QB_DQ, NW_DQ>), dim3((unsigned)grid), dim3(NW_DQ * 64), LDS, stream, a);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    // 4. dK_0, dV_0
    {
        constexpr bool kWs = sizeof(T) == 2;      // the eight-equal-waves kernel is for 16-bit types
        constexpr int KVT = kWs ? 128 : NW_KV * 32;
        constexpr int P8_LDS = DkvP8<T, D>::kLds;
        constexpr int LDS = kWs ? P8_LDS : 2 * (2 * 64 * D * (int)sizeof(T) + 3 * 64 * 4);
        const void* kern;
        if constexpr (kWs) kern = (const void*)ttt_bwd_dkv_p8_kernel<T, D>;
        else kern = (const void*)ttt_bwd_dkv_kernel<T, D, NW_KV>;
        static LdsOptIn lds_opt_in;
        if ((e = lds_opt_in.ensure(kern, LDS)) != hipSuccess) return e;
        // that kernel addresses the rows of a 32-row block with 32-bit byte offsets
        if (kWs && geo.q_st * 32 * (int64_t)sizeof(T) >= (int64_t)1 << 32) return hipErrorInvalidValue;
        a.n_tiles = (geo.T + KVT - 1) / KVT;
        // split the (step, head) list of a unit so that the grid fills the device evenly
        const int n_jh = geo.n_steps * geo.G;
        int n_split = 1;
        int n_units = a.n_tiles;   // units per kv head and split: key tiles, or (key tile, query chunk) pairs
        if constexpr (kWs) {
            int n_cu = 0;
            if ((e = current_device_cu_count(n_cu)) != hipSuccess) return e;
            const DkvPlan plan = plan_dkv_split(a, n_jh, n_cu);
            a.chunk_blocks = plan.chunk_blocks;
            n_split = plan.n_split;
            n_units = dkv_units_of(geo.T, a.n_tiles, a.chunk_blocks);
            a.n_units = n_units;
        } else {
            while (n_split < n_jh && (int64_t)n_units * geo.hkv * n_split < 2048) ++n_split;
        }
        a.n_split = n_split;
        int64_t grid;
        set_head_map(a.map, geo.hkv, n_units * n_split, grid);
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        {
            ProfileScope prof(kWs ? "ttt_bwd_dkv_p8_kernel" : "ttt_bwd_dkv_kernel", stream);
            if constexpr (kWs)
                hipLaunchKernelGGL((ttt_bwd_dkv_p8_kernel<T, D>), dim3((unsigned)grid), dim3(512), LDS, stream, a);
            else
                hipLaunchKernelGGL((ttt_bwd_dkv_kernel<T, D, NW_KV>), dim3((unsigned)grid), dim3(NW_KV * 64), LDS, stream, a);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }

    // 5. block-0 sums -> output dtype, once the sweep has covered step 0
    if (!a.accumulate || geo.step_begin == 0) {
        const int blocks = (int)((acc_n4 + 255) / 256 < 4096 ? (acc_n4 + 255) / 256 : 4096);
        {
            ProfileScope prof("ttt_bwd_finish_kernel", stream);
            hipLaunchKernelGGL((ttt_bwd_finish_kernel<T, D>), dim3(blocks), dim3(256), 0, stream, a);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_bwd(int dtype, int head_dim, BwdArgs& a, hipStream_t stream) {
    if (dtype == 1 && head_dim == 128) return launch_bwd_t<__bf16, 128, 1, 8, 4>(a, stream);
    if (dtype == 1 && head_dim == 64) return launch_bwd_t<__bf16, 64, 1, 4, 4>(a, stream);
    if (dtype == 0 && head_dim == 128) return launch_bwd_t<float, 128, 1, 4, 4>(a, stream);
    if (dtype == 0 && head_dim == 64) return launch_bwd_t<float, 64, 1, 4, 4>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace ttt
