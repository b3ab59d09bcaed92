// Device-side building blocks shared by the MDN kernels (gfx950 / CDNA4, wave64).
//
// All dense contractions go through one 16x16 MFMA tile primitive:
//   bf16 storage -> v_mfma_f32_16x16x32_bf16 (8 bf16 per lane per operand, K step 32)
//   fp32 storage -> 4 x v_mfma_f32_16x16x4_f32 (4 floats per lane per operand, K step 16)
// Operand fragments are always read as ONE 16-byte vector of K-contiguous elements, so every
// operand matrix must be laid out with the contraction index fastest.
//
// Register layouts (lane = 0..63, r = lane % 16, kg = lane / 16):
//   A fragment: row r of the 16-row tile, K elements [kg*EPL, kg*EPL + EPL) of the K step
//   B fragment: column r of the 16-column tile, same K elements
//   accumulator f32x4: D[m = kg*4 + x][n = r], x = 0..3
// The K index inside a step is permuted identically for A and B in the fp32 variant (lane group
// kg feeds k = 4*kg + s to the s-th instruction); a contraction does not care.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace mdn {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16_t;

constexpr int kC = 64;        // chunk size
constexpr int kThreads = 256; // 4 waves per workgroup
constexpr int kCoefRows = 8;  // per-chunk coefficient block: [64 tokens][kCoefRows] floats (= kCoefBlockCols of mdn_kernels.h)

// the coefficients of token i of a chunk, as two 16-byte vectors {a_i, b_i, alpha_i b_{i-1}, a_C} and
// {Gamma_C eta_i, Rho_C eta_i, b_C, m_C}: the chunk scalars a_C, b_C, m_C are repeated in every row, so that a
// lane has everything about its token and its chunk after two loads (the scaling of Z is alpha_i b_{i-1}; that of
// Y, alpha_i a_{i-1}, is a_i itself)
enum { COEF_A = 0, COEF_B = 1, COEF_PB = 2, COEF_AC = 3, COEF_GC = 4, COEF_RC = 5, COEF_BC = 6, COEF_MC = 7 };

template <typename T> struct Op;

template <> struct Op<bf16_t> {
    static constexpr int EPL = 8;    // elements per lane per fragment
    static constexpr int KSTEP = 32; // contraction elements per mma()
    static constexpr int PAD = 8;    // LDS row padding (elements) that keeps 16-byte row alignment
    typedef bf16x8 Frag;
    static __device__ __forceinline__ Frag load(const bf16_t *p) { return *reinterpret_cast<const Frag *>(p); }
    static __device__ __forceinline__ f32x4 mma(Frag a, Frag b, f32x4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};

template <> struct Op<float> {
    static constexpr int EPL = 4;
    static constexpr int KSTEP = 16;
    static constexpr int PAD = 4;
    typedef f32x4 Frag;
    static __device__ __forceinline__ Frag load(const float *p) { return *reinterpret_cast<const Frag *>(p); }
    static __device__ __forceinline__ f32x4 mma(Frag a, Frag b, f32x4 c) {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[0], b[0], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[1], b[1], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[2], b[2], c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[3], b[3], c, 0, 0, 0);
        return c;
    }
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x) { return (T)x; }
// value of x after a round trip through the storage type
template <typename T> __device__ __forceinline__ float rounded(float x) { return to_f32(from_f32<T>(x)); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
// value held by lane `src` (a compile-time constant) as a wave-uniform scalar
__device__ __forceinline__ float lane_value(float v, int src) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src));
}
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// acc[nt] += A(16 x K) * B(K x 16*NT)
//   A(m, k)  = A[m * lda + k]          (16 rows starting at A)
//   B(k, n)  = Bt[n * ldb + k]         (16*NT columns starting at Bt)
template <typename T, int NT, int K>
__device__ __forceinline__ void mma_rows(f32x4 (&acc)[NT], const T *__restrict__ A, int lda,
                                         const T *__restrict__ Bt, int ldb) {
    typedef Op<T> O;
    const int r = lane_id() & 15, kg = lane_id() >> 4;
    const T *ap = A + r * lda + kg * O::EPL;
    const T *bp = Bt + r * ldb + kg * O::EPL;
#pragma unroll
    for (int k0 = 0; k0 < K; k0 += O::KSTEP) {
        typename O::Frag a = O::load(ap + k0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            typename O::Frag b = O::load(bp + nt * 16 * ldb + k0);
            acc[nt] = O::mma(a, b, acc[nt]);
        }
    }
}

// four consecutive storage elements from four floats, as one vector store / load
__device__ __forceinline__ void store4(bf16_t *p, f32x4 v) {
    bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
    *reinterpret_cast<bf16x4 *>(p) = o;
}
__device__ __forceinline__ void store4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
__device__ __forceinline__ f32x4 load4(const bf16_t *p) {
    const bf16x4 v = *reinterpret_cast<const bf16x4 *>(p);
    return f32x4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
}
__device__ __forceinline__ f32x4 load4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
// the same four elements kept in storage form (so that the conversion can sit at the use, not at the load)
template <typename T> struct Raw4;
template <> struct Raw4<bf16_t> { typedef bf16x4 type; };
template <> struct Raw4<float> { typedef f32x4 type; };
__device__ __forceinline__ bf16x4 load4_raw(const bf16_t *p) { return *reinterpret_cast<const bf16x4 *>(p); }
__device__ __forceinline__ f32x4 load4_raw(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
template <typename T> __device__ __forceinline__ typename Raw4<T>::type narrow4(f32x4 v);
template <> __device__ __forceinline__ bf16x4 narrow4<bf16_t>(f32x4 v) {
    return bf16x4{(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
}
template <> __device__ __forceinline__ f32x4 narrow4<float>(f32x4 v) { return v; }
__device__ __forceinline__ void store4_raw(bf16_t *p, bf16x4 v) { *reinterpret_cast<bf16x4 *>(p) = v; }
__device__ __forceinline__ void store4_raw(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
__device__ __forceinline__ f32x4 widen4(bf16x4 v) { return f32x4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]}; }
__device__ __forceinline__ f32x4 widen4(f32x4 v) { return v; }
// widen4 of a value that was narrowed a moment ago, by shifts and masks of the packed words (so that the compiler
// widens the PACKED value instead of rounding each fp32 source a second time, one conversion per element)
__device__ __forceinline__ f32x4 widen4_packed(bf16x4 v) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 w = __builtin_bit_cast(u32x2, v);
    return f32x4{__uint_as_float(w[0] << 16), __uint_as_float(w[0] & 0xffff0000u), __uint_as_float(w[1] << 16),
                 __uint_as_float(w[1] & 0xffff0000u)};
}
__device__ __forceinline__ f32x4 widen4_packed(f32x4 v) { return v; }

// A lane's MV accumulator vectors as MV*4 CONSECUTIVE storage elements at p (16-bit storage, MV = 2: one 16-byte
// access instead of two of 8 bytes).  Which columns of a [.., dv] tensor a lane's accumulator rows stand for is
// the kernel's choice when dv is a pure batch index of the computation; choosing them consecutive halves the
// number of vector-memory instructions for everything that is exchanged in accumulator layout.
template <int MV> __device__ __forceinline__ void load_cols_raw(const bf16_t *p, bf16x4 (&u)[MV]) {
    if constexpr (MV == 2) {
        const bf16x8 w = *reinterpret_cast<const bf16x8 *>(p);
        u[0] = __builtin_shufflevector(w, w, 0, 1, 2, 3);
        u[1] = __builtin_shufflevector(w, w, 4, 5, 6, 7);
    } else {
#pragma unroll
        for (int mv = 0; mv < MV; ++mv) u[mv] = load4_raw(p + mv * 4);
    }
}
template <int MV> __device__ __forceinline__ void load_cols_raw(const float *p, f32x4 (&u)[MV]) {
#pragma unroll
    for (int mv = 0; mv < MV; ++mv) u[mv] = load4_raw(p + mv * 4);
}
template <int MV> __device__ __forceinline__ void store_cols_raw(bf16_t *p, const bf16x4 (&u)[MV]) {
    if constexpr (MV == 2) {
        *reinterpret_cast<bf16x8 *>(p) = __builtin_shufflevector(u[0], u[1], 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
#pragma unroll
        for (int mv = 0; mv < MV; ++mv) store4_raw(p + mv * 4, u[mv]);
    }
}
template <int MV> __device__ __forceinline__ void store_cols_raw(float *p, const f32x4 (&u)[MV]) {
#pragma unroll
    for (int mv = 0; mv < MV; ++mv) store4_raw(p + mv * 4, u[mv]);
}
template <typename T, int MV> __device__ __forceinline__ void store_cols(T *p, const f32x4 (&v)[MV]) {
    typename Raw4<T>::type u[MV];
#pragma unroll
    for (int mv = 0; mv < MV; ++mv) u[mv] = narrow4<T>(v[mv]);
    store_cols_raw<MV>(p, u);
}

// 16 bytes of storage elements
template <typename T> struct Vec16 {
    T e[Op<T>::EPL];
};

// base + 32-bit element offset, formed as a 32-bit BYTE offset: a wave-uniform base plus a per-lane
// 32-bit offset is one address register (the hardware adds the scalar base) instead of a 64-bit pair
template <typename T> __device__ __forceinline__ const T *at32(const T *base, unsigned elem_off) {
    return reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + elem_off * (unsigned)sizeof(T));
}
template <typename T> __device__ __forceinline__ T *at32(T *base, unsigned elem_off) {
    return reinterpret_cast<T *>(reinterpret_cast<char *>(base) + elem_off * (unsigned)sizeof(T));
}

// An MFMA A operand [M rows][K] in LDS that a workgroup writes from accumulators (a lane holds 4 consecutive
// rows m of one column k) and reads back as fragments (row m, EPL consecutive k).
//   fp32 storage: kept [m][k]: four 4-byte writes per accumulator, one 16-byte read per fragment.
//   bf16 storage: kept [k][m], rows of M + 8 elements: ONE 8-byte write per accumulator, and a fragment is two
//     transposing reads (ds_read_b64_tr_b16: inside each group of 16 lanes, lane 4e + c addresses 4 consecutive
//     m of row k0 + e, e = 0..3, and lane l receives element m0 + l of those four rows).  Measured per CU with 4
//     waves: 1.7 ns per 8-byte write instruction against 4 x 3.7 ns for the four 2-byte writes of the [m][k]
//     form, and 2 x 1.8 ns for the two transposing reads against 6.9 ns for the 16-byte fragment read.
//     The row length M + 8 (M = 16, 32, 64) puts the 16 rows one write instruction touches, and the rows one
//     read touches, on different banks.
template <typename T, int M, int K> struct ATile;
template <int M, int K> struct ATile<float, M, K> {
    typedef Op<float> O;
    static constexpr int LD = K + O::PAD, SIZE = M * LD;
    // rows m0 .. m0+3 of column k
    static __device__ __forceinline__ void put4(float *t, int m0, int k, f32x4 v) {
#pragma unroll
        for (int x = 0; x < 4; ++x) t[(m0 + x) * LD + k] = v[x];
    }
    static __device__ __forceinline__ void put4_raw(float *t, int m0, int k, f32x4 v) { put4(t, m0, k, v); }
    // fragment of row 16 mt + r, k = k0 + kg*EPL .. (k0 a multiple of KSTEP)
    static __device__ __forceinline__ O::Frag frag(const float *t, int mt, int k0, int r, int kg) {
        return O::load(t + (mt * 16 + r) * LD + k0 + kg * O::EPL);
    }
};
// fragment (row or column 16*.. + r of the operand, k = k0 + kg*8 .. +7) of a bf16 matrix kept [k][n] with row
// length ld in LDS, n0 = first of the 16 n: two transposing reads (rows k0 + kg*8 + 0..3 and + 4..7)
// (the two reads given as addresses: for layouts whose rows are permuted piecewise)
__device__ __forceinline__ bf16x8 tr_pair(const bf16_t *p_lo, const bf16_t *p_hi) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p_lo));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)(p_hi));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ bf16x8 tr_frag(const bf16_t *t, int ld, int k0, int n0, int r, int kg) {
    const bf16_t *p = t + (k0 + kg * 8 + (r >> 2)) * ld + n0 + (r & 3) * 4;
    return tr_pair(p, p + 4 * ld);
}
template <int M, int K> struct ATile<bf16_t, M, K> {
    typedef Op<bf16_t> O;
    static constexpr int LD = M + 8, SIZE = K * LD;
    static __device__ __forceinline__ void put4(bf16_t *t, int m0, int k, f32x4 v) { store4(t + k * LD + m0, v); }
    // the same four rows, already in storage form
    static __device__ __forceinline__ void put4_raw(bf16_t *t, int m0, int k, bf16x4 v) { store4_raw(t + k * LD + m0, v); }
    static __device__ __forceinline__ O::Frag frag(const bf16_t *t, int mt, int k0, int r, int kg) {
        return tr_frag(t, LD, k0, mt * 16, r, kg);
    }
};

// one natural-layout [64][D] token tile, HBM -> LDS without registers: the 16-byte slot (row, position p)
// receives piece p ^ (row & XM) of that row (XM = min(pieces per row, 16) - 1).  Issued by NW waves
// (lw = 0 .. NW-1), each D / (EPL * NW) instructions of 64 consecutive slots (m0 = LDS address of the 64
// slots; lane l fills slot l).
// Written as inline assembly on purpose: the compiler then does not know of the transfer, and so neither makes
// the issuing wave (nor, through its path-insensitive bookkeeping, any other wave) drain its whole load queue
// at the next LDS instruction.  Waiting for the transfer is the caller's job (a vector-memory wait of the
// issuing wave that covers it, before the barrier that publishes the tile); the compiler's own waits for loads
// it knows of can only become longer through the extra entries in the queue, never shorter (loads return in
// order).
template <typename T, int D, int NW = 2>
__device__ __forceinline__ void dma_token_tile(T *ldst, const T *src, unsigned rs, int lw, int lane) {
    constexpr int E = Op<T>::EPL, CPR = D / E, XM = (CPR < 16 ? CPR : 16) - 1, NDMA = CPR / NW;
#pragma unroll
    for (int u = 0; u < NDMA; ++u) {
        const int blk64 = u * NW + lw, sl = blk64 * 64 + lane, row = sl / CPR, pc = (sl % CPR) ^ (row & XM);
        const T *g = at32(src, row * rs + pc * E);
        const unsigned l = (unsigned)(size_t)((__attribute__((address_space(3))) T *)(ldst + blk64 * 64 * E));
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(l) : "memory", "m0");
    }
}
// Fragments out of such a tile (bf16: the transposing read is a 16-bit instruction).
//   row fragment: row `row`, elements 32 st + 8 kg .. + 7 (the tile as [row][k] operand)
template <int D> __device__ __forceinline__ bf16x8 token_tile_row_frag(const bf16_t *tile, int row, int st, int kg) {
    constexpr int CPR = D / 8, XM = (CPR < 16 ? CPR : 16) - 1;
    return Op<bf16_t>::load(tile + row * D + (((st * 4 + kg) ^ (row & XM)) * 8));
}
//   column fragment: column 16 ct + r, rows 32 s + 8 kg .. + 7 (the transposed tile as [column][row] operand): two
//   transposing reads; lane 4e + c of a 16-lane group addresses rows 32 s + 8 kg (+ 4) + e, columns 16 ct + 4c .. 4c+3
template <int D> __device__ __forceinline__ bf16x8 token_tile_col_frag(const bf16_t *tile, int ct, int s, int r, int kg) {
    constexpr int CPR = D / 8, XM = (CPR < 16 ? CPR : 16) - 1;
    const int row = s * 32 + kg * 8 + (r >> 2), c = ct * 2 + ((r & 3) >> 1), sub = ((r & 3) * 4) & 7;
    return tr_pair(tile + row * D + ((c ^ (row & XM)) * 8) + sub, tile + (row + 4) * D + ((c ^ ((row + 4) & XM)) * 8) + sub);
}

// Blocked layouts of the chunk-local tensors that the library itself produces and consumes.
// kblk: a [R][K] MFMA operand (fragment = row, KSTEP consecutive k) is stored as [K/KSTEP][R][KSTEP],
//       so the 16 rows x KSTEP elements one wave-level fragment load touches are contiguous.
// vblk: a [R][dv] tensor exchanged in accumulator layout (a lane holds 4 consecutive dv of one row)
//       is stored as [dv/16][R][16], so the 16 rows x 16 dv of one accumulator tile are contiguous.
template <typename T> __device__ __forceinline__ size_t kblk(int R, int row, int k) {
    constexpr int S = Op<T>::KSTEP;
    return ((size_t)(k / S) * R + row) * S + (k % S);
}
__device__ __forceinline__ size_t vblk(int R, int row, int dv) {
    return ((size_t)(dv >> 4) * R + row) * 16 + (dv & 15);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>)
template <int N, int I = 0, typename F> __device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

template <int NT> __device__ __forceinline__ void zero_acc(f32x4 (&acc)[NT]) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
}

// dst[(m) * ld + n] = sgn * D(m, n) for the 16 x 16*NT block held in acc (row-major destination)
template <typename T, int NT>
__device__ __forceinline__ void store_rows(const f32x4 (&acc)[NT], T *dst, int ld, float sgn) {
    const int r = lane_id() & 15, kg = lane_id() >> 4;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int x = 0; x < 4; ++x) dst[(kg * 4 + x) * ld + nt * 16 + r] = from_f32<T>(sgn * acc[nt][x]);
}

// dst[(n) * ld + m] = sgn * D(m, n): transposed destination, 4 consecutive m per lane
template <typename T, int NT>
__device__ __forceinline__ void store_rows_t(const f32x4 (&acc)[NT], T *dst, int ld, float sgn) {
    const int r = lane_id() & 15, kg = lane_id() >> 4;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
        store4(dst + (nt * 16 + r) * ld + kg * 4, sgn * acc[nt]);
}

// as mma_rows, with B stored in the vblk layout of a [R][K] tensor: B(k, n) = Bv[vblk(R, n, k)]
template <typename T, int NT, int K>
__device__ __forceinline__ void mma_rows_vblk(f32x4 (&acc)[NT], const T *__restrict__ A, int lda,
                                              const T *__restrict__ Bv, int R) {
    typedef Op<T> O;
    const int r = lane_id() & 15, kg = lane_id() >> 4;
    const T *ap = A + r * lda + kg * O::EPL;
#pragma unroll
    for (int k0 = 0; k0 < K; k0 += O::KSTEP) {
        typename O::Frag a = O::load(ap + k0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            typename O::Frag b = O::load(Bv + vblk(R, nt * 16 + r, k0 + kg * O::EPL));
            acc[nt] = O::mma(a, b, acc[nt]);
        }
    }
}

// as mma_rows, with B stored in the kblk layout of a [R][K] operand
template <typename T, int NT, int K>
__device__ __forceinline__ void mma_rows_kblk(f32x4 (&acc)[NT], const T *__restrict__ A, int lda,
                                              const T *__restrict__ Bk, int R) {
    typedef Op<T> O;
    const int r = lane_id() & 15, kg = lane_id() >> 4;
    const T *ap = A + r * lda + kg * O::EPL;
#pragma unroll
    for (int k0 = 0; k0 < K; k0 += O::KSTEP) {
        typename O::Frag a = O::load(ap + k0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            typename O::Frag b = O::load(Bk + kblk<T>(R, nt * 16 + r, k0 + kg * O::EPL));
            acc[nt] = O::mma(a, b, acc[nt]);
        }
    }
}

// Cross-lane sums without the LDS crossbar (a shuffle compiles to ds_bpermute: an LDS instruction with LDS
// latency).  Inside a row of 16 lanes: DPP quad permutes and row rotations.  Across rows: the row / half swaps
// (v_permlane16_swap: odd rows of the first operand <-> even rows of the second; v_permlane32_swap: upper half of
// the first <-> lower half of the second): with the same value in both operands the two results are the value of
// the lane's own row (half) pair member and that of the other, in every lane.
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// v + (v of lane ^ 16), in every lane
__device__ __forceinline__ float add_xor16(float v) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 p = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}
// v + (v of lane ^ 32), in every lane
__device__ __forceinline__ float add_xor32(float v) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 p = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(p[0]) + __uint_as_float(p[1]);
}
// sum over the 16 lanes that share kg (i.e. over the column index r of an accumulator row)
__device__ __forceinline__ float reduce16(float v) {
    v += dpp_move<0xB1>(v);  // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);  // quad_perm [2,3,0,1]
    v += dpp_move<0x124>(v); // row_ror 4
    v += dpp_move<0x128>(v); // row_ror 8
    return v;
}

// sum over the whole wave
__device__ __forceinline__ float reduce64(float v) { return add_xor32(add_xor16(reduce16(v))); }

// Workgroup id -> (bh, sub) with all `nsub` workgroups of one bh on the same XCD (workgroups are
// dealt round-robin to the 8 XCDs, each with its own L2).  Grid must be 8 * ceil(BH/8) * nsub.
__device__ __forceinline__ void xcd_map(int bid, int nsub, int &bh, int &sub) {
    const int xcd = bid & 7, slot = bid >> 3;
    bh = (slot / nsub) * 8 + xcd;
    sub = slot % nsub;
}

} // namespace mdn
