// Device-side building blocks shared by the TTT attention kernels (gfx950 only).
//
// One matrix "atom" is a 32x32 fp32 accumulator block updated by a contraction chunk of 16:
//   bf16:  one v_mfma_f32_32x32x16_bf16            (lane holds 8 consecutive k of its row/column)
//   fp32:  eight v_mfma_f32_32x32x2_f32            (lane holds 8 values; MFMA u contracts value u of
//                                                   both lane halves, i.e. k = u and k = 8+u)
// so for both element types an operand fragment is "8 values per lane, k = 8*(lane/32) + e" and the
// accumulator layout is the 32x32 one: lane (n = lane%32, hh = lane/32) holds column n and rows
// row(i) = 8*(i/4) + 4*hh + i%4, i = 0..15.
//
// An accumulator block is turned into an operand whose contraction index is the accumulator's ROW
// index without any data movement: the 16 values of a lane are split into two chunks of 8
// (chunk c = values 8c..8c+7 = rows 16c + {0..3, 8..11} + 4*hh), and the other operand is read
// "transposed" with exactly that row set per lane (frag_transposed below).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ttt {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

#define TTT_DEV __device__ __forceinline__

template <typename T> struct Elem;
template <> struct Elem<__bf16> {
    using frag = bf16x8;
    using vec4 = bf16x4;
    static constexpr int kBytes = 2;
};
template <> struct Elem<float> {
    using frag = f32x8;
    using vec4 = f32x4;
    static constexpr int kBytes = 4;
};

// ---- accumulate one contraction chunk of 16 into a 32x32 block
TTT_DEV f32x16 mma(const bf16x8& a, const bf16x8& b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
TTT_DEV f32x16 mma(const f32x8& a, const f32x8& b, f32x16 c) {
#pragma unroll
    for (int u = 0; u < 8; ++u) c = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], c, 0, 0, 0);
    return c;
}

// ---- accumulator chunk -> operand fragment (values 8c..8c+7 of the lane)
template <typename T> TTT_DEV typename Elem<T>::frag acc_chunk(const f32x16& acc, int c);
template <> TTT_DEV bf16x8 acc_chunk<__bf16>(const f32x16& acc, int c) {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (__bf16)acc[8 * c + e];
    return r;
}
template <> TTT_DEV f32x8 acc_chunk<float>(const f32x16& acc, int c) {
    f32x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = acc[8 * c + e];
    return r;
}

// row of accumulator value i for lane half hh
TTT_DEV constexpr int acc_row(int i, int hh) { return 8 * (i / 4) + 4 * hh + (i % 4); }

// ---- LDS tiles: ROWS x D elements, row-major, each row cut into 16-byte pieces; piece c of row r
// lives at piece position c ^ swz(r) so that both the row-wise 16-byte reads and the transposing
// reads spread over the banks.
template <typename T, int D> struct Tile {
    static constexpr int kRowBytes = D * Elem<T>::kBytes;
    static constexpr int kPieces = kRowBytes / 16;              // 8, 16 or 32
    static constexpr int kElemsPerPiece = 16 / Elem<T>::kBytes;
    // swz(r): the two low row bits go to the top of the piece index, the next two to the bottom.
    // LDS has 64 banks x 4 B (one 256-byte window).  A transposing 8-byte read serves 32 lanes per
    // cycle = 4 consecutive rows x 4 pieces x 2 halves: the low row bits move each row to a
    // different group of 4 pieces, so the 256 bytes are distinct.  A row-wise 16-byte read serves
    // 16 lanes = 16 consecutive rows per cycle: swz is a bijection of the low four row bits, so the
    // 16 pieces are distinct.  Measured with SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE on MI355X:
    // 4.0 cycles per 16-byte read and 2.0 per transposing read, no conflict cycles (a plain row & 15
    // gives 8 cycles per transposing read, a one-bit rotation 4).
    static constexpr int kBits = kPieces >= 16 ? 4 : 3;
    TTT_DEV static int swz(int r) {
        if constexpr (kBits == 4) return ((r & 3) << 2) | ((r >> 2) & 3);
        else return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);   // 128-byte rows: two rows per bank window
    }
    // byte offset of element (r, col) inside the tile
    TTT_DEV static int offset(int r, int col) {
        const int piece = col / kElemsPerPiece;
        const int within = col % kElemsPerPiece;
        return r * kRowBytes + ((piece ^ swz(r)) * 16) + within * Elem<T>::kBytes;
    }
};

// 8 consecutive elements (r, col..col+7), col a multiple of 8: the k-contiguous operand fragment.
template <typename T, int D> TTT_DEV typename Elem<T>::frag frag_rowwise(const char* tile, int r, int col);
template <> TTT_DEV bf16x8 frag_rowwise<__bf16, 128>(const char* tile, int r, int col) {
    return *reinterpret_cast<const bf16x8*>(tile + Tile<__bf16, 128>::offset(r, col));
}
template <> TTT_DEV bf16x8 frag_rowwise<__bf16, 64>(const char* tile, int r, int col) {
    return *reinterpret_cast<const bf16x8*>(tile + Tile<__bf16, 64>::offset(r, col));
}
template <> TTT_DEV f32x8 frag_rowwise<float, 128>(const char* tile, int r, int col) {
    const f32x4 lo = *reinterpret_cast<const f32x4*>(tile + Tile<float, 128>::offset(r, col));
    const f32x4 hi = *reinterpret_cast<const f32x4*>(tile + Tile<float, 128>::offset(r, col + 4));
    return f32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}
template <> TTT_DEV f32x8 frag_rowwise<float, 64>(const char* tile, int r, int col) {
    const f32x4 lo = *reinterpret_cast<const f32x4*>(tile + Tile<float, 64>::offset(r, col));
    const f32x4 hi = *reinterpret_cast<const f32x4*>(tile + Tile<float, 64>::offset(r, col + 4));
    return f32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}

// Transposed fragment for the 32-column block starting at col0: the lane's column is col0 + lane%32
// and its 8 values are rows row0 + {0,1,2,3, 8,9,10,11} + 4*(lane/32)  (row0 a multiple of 16).
// bf16 uses the gfx950 transposing LDS read: inside each group of 16 lanes, lane t supplies the
// address of 4 consecutive elements (row t/4, columns 4*(t%4)..+3 of the group's 16 columns) and
// receives the 4 rows of column t.
template <typename T, int D> TTT_DEV typename Elem<T>::frag frag_transposed(const char* tile, int row0, int col0, int lane);
template <int D> TTT_DEV bf16x8 frag_transposed_bf16(const char* tile, int row0, int col0, int lane) {
    const int t = lane & 15, grp = (lane >> 4) & 1, hh = lane >> 5;
    const int r = row0 + 4 * hh + (t >> 2);
    const int c = col0 + 16 * grp + 4 * (t & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4*)(uintptr_t)(tile + Tile<__bf16, D>::offset(r, c)));
    const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4*)(uintptr_t)(tile + Tile<__bf16, D>::offset(r + 8, c)));
    union { s16x4 s[2]; bf16x8 v; } u;
    u.s[0] = a;
    u.s[1] = b;
    return u.v;
}
template <> TTT_DEV bf16x8 frag_transposed<__bf16, 128>(const char* tile, int row0, int col0, int lane) {
    return frag_transposed_bf16<128>(tile, row0, col0, lane);
}
template <> TTT_DEV bf16x8 frag_transposed<__bf16, 64>(const char* tile, int row0, int col0, int lane) {
    return frag_transposed_bf16<64>(tile, row0, col0, lane);
}
template <int D> TTT_DEV f32x8 frag_transposed_f32(const char* tile, int row0, int col0, int lane) {
    const int n = lane & 31, hh = lane >> 5;
    f32x8 v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int r = row0 + 8 * (e / 4) + 4 * hh + (e % 4);
        v[e] = *reinterpret_cast<const float*>(tile + Tile<float, D>::offset(r, col0 + n));
    }
    return v;
}
template <> TTT_DEV f32x8 frag_transposed<float, 128>(const char* tile, int row0, int col0, int lane) {
    return frag_transposed_f32<128>(tile, row0, col0, lane);
}
template <> TTT_DEV f32x8 frag_transposed<float, 64>(const char* tile, int row0, int col0, int lane) {
    return frag_transposed_f32<64>(tile, row0, col0, lane);
}

// ---- per-lane fragment addressing, computed once per kernel.  The swizzle involves row bits 0..3
// only, so stepping by whole 16-row chunks (transposed reads) or 32-row blocks (row-wise reads) and
// switching tiles or pipeline stages adds compile-time constants, which the LDS instructions carry
// in their immediate offset field: no address arithmetic is left in the inner loops.
template <typename T, int D> struct LaneFrags {
    using frag = typename Elem<T>::frag;
    int lane;
    TTT_DEV void init(int lane_) { lane = lane_; }
    TTT_DEV frag rowwise(const char* tile, int rb, int t) const {
        return frag_rowwise<T, D>(tile, rb * 32 + (lane & 31), t * 16 + (lane >> 5) * 8);
    }
    TTT_DEV frag transposed(const char* tile, int c16, int db) const {
        return frag_transposed<T, D>(tile, c16 * 16, db * 32, lane);
    }
};
template <int D> struct LaneFrags<__bf16, D> {
    using TL = Tile<__bf16, D>;
    uint32_t row[D / 16];      // fragment t of row lane%32
    uint32_t tr[D / 32][2];    // 4-element piece this lane addresses in 32-column block db, rows +0 / +8
    TTT_DEV void init(int lane) {
        const int n = lane & 31, hh = lane >> 5;
#pragma unroll
        for (int t = 0; t < D / 16; ++t) row[t] = TL::offset(n, t * 16 + hh * 8);
        const int q = lane & 15, grp = (lane >> 4) & 1;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
            tr[db][0] = TL::offset(4 * hh + (q >> 2), db * 32 + 16 * grp + 4 * (q & 3));
            tr[db][1] = TL::offset(4 * hh + (q >> 2) + 8, db * 32 + 16 * grp + 4 * (q & 3));
        }
    }
    TTT_DEV bf16x8 rowwise(const char* tile, int rb, int t) const {
        return *reinterpret_cast<const bf16x8*>(tile + rb * 32 * TL::kRowBytes + row[t]);
    }
    TTT_DEV bf16x8 transposed(const char* tile, int c16, int db) const {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const char* base = tile + c16 * 16 * TL::kRowBytes;
        union { s16x4 s[2]; bf16x8 v; } u;
        u.s[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(base + tr[db][0]));
        u.s[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(base + tr[db][1]));
        return u.v;
    }
};

// Ordering fence for the compiler only (no instruction): memory operations -- in particular LDS
// reads requested ahead of their use -- stay on their side of it, and the instruction scheduler does
// not move anything across it.
TTT_DEV void issue_fence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// compile-time integer handed to generic lambdas (pipeline stage)
template <int V> struct IntC { static constexpr int value = V; };

// ---- global -> LDS copy requests (LDS-DMA loads), 16 or 4 bytes per lane: the wave's 64 pieces land
// at lds_dst + lane * size, lds_dst being wave-uniform (it travels in M0).  Written as inline
// assembly on purpose: for the builtin form the compiler cannot tell which LDS reads depend on a
// pending copy and makes every transposing LDS read wait for ALL outstanding copies of the wave,
// which serialises a copy with the work it was meant to overlap.  Here the program states the
// dependency itself: wait_async_copies() (or a partial vmcnt wait) plus a barrier before the first
// read of a stage.  The compiler keeps no value in M0 across statements (reserved register).
TTT_DEV uint32_t lds_addr(const void* p) {
    typedef __attribute__((address_space(3))) char lds_char;
    return (uint32_t)(uintptr_t)(lds_char*)p;
}
TTT_DEV void async_copy16(const void* gsrc, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_dst)), "v"(gsrc) : "memory");
}
TTT_DEV void async_copy4(const void* gsrc, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_dst)), "v"(gsrc) : "memory");
}

// the same with the source given as a wave-uniform 64-bit base plus a 32-bit byte offset per lane
TTT_DEV void async_copy16(const void* gbase, uint32_t lane_off, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_dst)), "v"(lane_off), "s"(gbase) : "memory");
}
TTT_DEV void async_copy4(const void* gbase, uint32_t lane_off, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :: "s"(__builtin_amdgcn_readfirstlane(lds_dst)), "v"(lane_off), "s"(gbase) : "memory");
}

// ---- global -> LDS tile copy without passing through registers (16 bytes per lane per
// instruction; one wave instruction fills 1024 contiguous LDS bytes).  ROWS*kRowBytes must be a
// multiple of NTHREADS*16.  Rows are clamped to [0, max_row] so the copy never leaves the tensor;
// clamped rows are hidden by the mask later.  `g` points at element (token 0, this head, 0).
template <typename T, int D, int ROWS, int NTHREADS>
TTT_DEV void tile_load_async(char* tile, const T* g, int64_t stride_token, int row_first, int max_row, int tid) {
    using TL = Tile<T, D>;
    constexpr int kTotalPieces = ROWS * TL::kPieces;
    static_assert(kTotalPieces % NTHREADS == 0, "tile does not divide over the workgroup");
    constexpr int kIters = kTotalPieces / NTHREADS;
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
        const int base = (it * (NTHREADS / 64) + wave) * 64;   // first piece of this wave instruction
        const int p = base + lane;
        const int r = p / TL::kPieces;
        const int pos = p % TL::kPieces;
        const int piece = pos ^ TL::swz(r);
        int gr = row_first + r;
        gr = gr > max_row ? max_row : gr;
        const T* src = g + (int64_t)gr * stride_token + piece * TL::kElemsPerPiece;
        async_copy16(src, lds_addr(tile + base * 16));
    }
}

// The same copy for a tile all of whose rows exist, with the per-lane part of the source address
// (row within the workgroup's pass, swizzled piece) worked out once.  One pass of the workgroup
// covers kRowsPerIter rows, a multiple of 16, so the swizzle -- and with it the lane's offset from
// the first row of the pass -- is the same in every pass: a tile costs kIters copy instructions and
// as many wave-uniform pointer additions.  kRowsPerIter * stride_token * sizeof(T) must stay
// below 2^32.
template <typename T, int D, int ROWS, int NTHREADS>
struct TileCopy {
    using TL = Tile<T, D>;
    static constexpr int kIters = ROWS * TL::kPieces / NTHREADS;
    static constexpr int kRowsPerIter = NTHREADS / TL::kPieces;
    static_assert(ROWS * TL::kPieces % NTHREADS == 0, "tile does not divide over the workgroup");
    static_assert(NTHREADS % TL::kPieces == 0 && kRowsPerIter % 16 == 0, "the swizzle must repeat from pass to pass");
    uint32_t off;           // bytes from the first element of a pass's first row to this lane's piece
    uint32_t wave_dst;      // bytes from the start of a pass in the LDS tile to this wave's first piece
    int64_t iter_stride;    // elements from one pass to the next
    TTT_DEV void init(int64_t stride_token, int tid) {
        const int wave = tid >> 6, lane = tid & 63;
        const int p = wave * 64 + lane;
        const int r = p / TL::kPieces, pos = p % TL::kPieces;
        off = (uint32_t)((r * stride_token + (pos ^ TL::swz(r)) * TL::kElemsPerPiece) * (int64_t)sizeof(T));
        wave_dst = __builtin_amdgcn_readfirstlane(wave * 1024);
        iter_stride = kRowsPerIter * stride_token;
    }
    TTT_DEV void copy(uint32_t tile_lds, const T* first_row) const {
#pragma unroll
        for (int it = 0; it < kIters; ++it)
            async_copy16(first_row + it * iter_stride, off, tile_lds + wave_dst + it * NTHREADS * 16);
    }
};

// Workgroup barrier for data handed over through LDS only: this wave's LDS accesses are complete,
// but its outstanding global-memory requests (copies into LDS stages that nobody reads yet) stay
// in flight -- __syncthreads() would wait for them too.
TTT_DEV void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The bare barrier, for a wave whose LDS traffic before it consists of reads that have already been
// consumed (so they are complete) plus reads of data that stays valid past the barrier.
TTT_DEV void bare_barrier() { asm volatile("s_barrier" ::: "memory"); }

// all outstanding global->LDS copies of this wave have landed
TTT_DEV void wait_async_copies() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// Waits until at most N of this wave's global-memory requests are outstanding.  Requests complete
// in order, so the N newest may stay in flight.  The count sits in bits 3:0 and 15:14 of the
// immediate; the other counters are left alone.
template <int N> TTT_DEV void wait_copies_but(IntC<N>) {
    static_assert(N >= 0 && N < 64, "6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// ---- small helpers
TTT_DEV float xor32(float v) { return __shfl_xor(v, 32, 64); }
// max / sum of a value with its partner in the other lane half (lane ^ 32), on the vector ALU:
// v_permlane32_swap exchanges the upper half of one register with the lower half of the other, so
// swapping a value with itself yields {lower-half copy, upper-half copy} in every lane.
TTT_DEV float half_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
TTT_DEV float half_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
TTT_DEV float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T> TTT_DEV float to_f32(T v);
template <> TTT_DEV float to_f32<float>(float v) { return v; }
template <> TTT_DEV float to_f32<__bf16>(__bf16 v) { return (float)v; }

// acc + <a, b> over the 8 elements of two fragments (fp32 accumulation; bf16 pairs go through the
// packed dot instruction, which needs no unpacking)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
TTT_DEV float dot8(const bf16x8& a, const bf16x8& b, float acc) {
#pragma unroll
    for (int e = 0; e < 8; e += 2)
        acc = __builtin_amdgcn_fdot2_f32_bf16(bf16x2{a[e], a[e + 1]}, bf16x2{b[e], b[e + 1]}, acc, false);
    return acc;
}
TTT_DEV float dot8(const f32x8& a, const f32x8& b, float acc) {
#pragma unroll
    for (int e = 0; e < 8; ++e) acc = fmaf(a[e], b[e], acc);
    return acc;
}

// Row-wise fragments of ONE row per lane pair (lane (n,hh) holds elements 16t + 8hh + e of row n)
// -> the accumulator-column order (lane (n,hh) holds elements 32db + 8*i4 + 4hh + x), as fp32.
// Each lane keeps half of its own values and takes the other half from its partner lane n +- 32;
// one v_permlane32_swap per register pair moves both directions at once.
template <typename T, int DC> TTT_DEV void frags_to_acc_order(const typename Elem<T>::frag (&f)[DC], float (&out)[DC / 2][16]) {
    constexpr int R = sizeof(typename Elem<T>::frag) / 4;   // 32-bit registers per fragment
    union U { typename Elem<T>::frag v; uint32_t r[R]; };
#pragma unroll
    for (int t = 0; t < DC; ++t) {
        U u;
        u.v = f[t];
        union { uint32_t r[R / 2]; T e[4]; } even, odd;
#pragma unroll
        for (int i = 0; i < R / 2; ++i) {
            const auto sw = __builtin_amdgcn_permlane32_swap(u.r[i], u.r[i + R / 2], false, false);
            even.r[i] = sw[0];   // half 0: own first half,       half 1: partner's second half
            odd.r[i] = sw[1];    // half 0: partner's first half, half 1: own second half
        }
        const int db = t / 2, i4 = 2 * (t % 2);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            out[db][i4 * 4 + x] = to_f32<T>(even.e[x]);
            out[db][(i4 + 1) * 4 + x] = to_f32<T>(odd.e[x]);
        }
    }
}

// The same reordering for 16-bit elements, left packed (two elements per register) so that the row
// costs half the registers until its values are used: out[t] = {even pair 0, even pair 1, odd pair 0,
// odd pair 1} of fragment t; acc_order_elem() unpacks accumulator element i of 32-column block db.
template <typename T, int DC> TTT_DEV void frags_to_acc_order_packed(const typename Elem<T>::frag (&f)[DC], uint32_t (&out)[DC][4]) {
    static_assert(sizeof(T) == 2, "packed form is for 16-bit elements");
    union U { typename Elem<T>::frag v; uint32_t r[4]; };
#pragma unroll
    for (int t = 0; t < DC; ++t) {
        U u;
        u.v = f[t];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const auto sw = __builtin_amdgcn_permlane32_swap(u.r[i], u.r[i + 2], false, false);
            out[t][i] = sw[0];
            out[t][2 + i] = sw[1];
        }
    }
}
template <int DC> TTT_DEV float acc_order_elem(const uint32_t (&p)[DC][4], int db, int i) {
    const int i4 = i / 4, x = i % 4;
    const uint32_t r = p[2 * db + i4 / 2][2 * (i4 % 2) + x / 2];
    return __uint_as_float((x % 2) ? (r & 0xffff0000u) : (r << 16));   // bf16 -> fp32 is a shift
}

// load 8 consecutive elements from global as a fragment
template <typename T> TTT_DEV typename Elem<T>::frag gload_frag(const T* p);
template <> TTT_DEV bf16x8 gload_frag<__bf16>(const __bf16* p) { return *reinterpret_cast<const bf16x8*>(p); }
template <> TTT_DEV f32x8 gload_frag<float>(const float* p) {
    const f32x4 lo = *reinterpret_cast<const f32x4*>(p);
    const f32x4 hi = *reinterpret_cast<const f32x4*>(p + 4);
    return f32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}
template <typename T> TTT_DEV typename Elem<T>::vec4 gload_vec4(const T* p) {
    return *reinterpret_cast<const typename Elem<T>::vec4*>(p);
}
template <typename T> TTT_DEV void gstore_vec4(T* p, float a, float b, float c, float d);
template <> TTT_DEV void gstore_vec4<float>(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<f32x4*>(p) = f32x4{a, b, c, d};
}
template <> TTT_DEV void gstore_vec4<__bf16>(__bf16* p, float a, float b, float c, float d) {
    *reinterpret_cast<bf16x4*>(p) = bf16x4{(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
}

// Workgroup index -> (kv head, remaining index) so that workgroups that share one kv head's K_0/V_0
// land on the same XCD (consecutive workgroup ids go round-robin over the 8 XCDs, each with its own
// L2).  `rest_count` items per kv head; returns false for padding workgroups.
struct HeadMap {
    int mode;        // 0: no remap, 1: hkv multiple of 8, 2: hkv divides 8
    int hkv;
    int rest_count;
};
TTT_DEV bool decode_block(const HeadMap& m, int id, int& g, int& rest) {
    if (m.mode == 1) {
        const int hp = m.hkv >> 3;
        const int xcd = id & 7, slot = id >> 3;
        g = xcd * hp + slot % hp;
        rest = slot / hp;
    } else if (m.mode == 2) {
        const int xp = 8 / m.hkv;
        const int xcd = id & 7, slot = id >> 3;
        g = xcd / xp;
        rest = slot * xp + xcd % xp;
    } else {
        g = id % m.hkv;
        rest = id / m.hkv;
    }
    return rest < m.rest_count;
}

}  // namespace ttt
