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
constexpr int kCoefRows = 6;  // per-chunk coefficient block: [kCoefRows][64] floats

// rows of the coefficient block
enum { COEF_A = 0, COEF_B = 1, COEF_GC = 2, COEF_RC = 3, COEF_SCALAR = 4, COEF_PB = 5 };
// COEF_SCALAR row: [0] = a_C, [1] = b_C, [2] = m_C;  COEF_PB row: alpha_i b_{i-1} (the scaling of Z; that of Y,
// alpha_i a_{i-1}, is a_i itself)

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
__device__ __forceinline__ f32x4 tr_pair(const float *, const float *) { return f32x4{0.f, 0.f, 0.f, 0.f}; } // (never used)
__device__ __forceinline__ bf16x8 tr_frag(const bf16_t *t, int ld, int k0, int n0, int r, int kg) {
    const bf16_t *p = t + (k0 + kg * 8 + (r >> 2)) * ld + n0 + (r & 3) * 4;
    return tr_pair(p, p + 4 * ld);
}
template <int M, int K> struct ATile<bf16_t, M, K> {
    typedef Op<bf16_t> O;
    static constexpr int LD = M + 8, SIZE = K * LD;
    static __device__ __forceinline__ void put4(bf16_t *t, int m0, int k, f32x4 v) { store4(t + k * LD + m0, v); }
    static __device__ __forceinline__ O::Frag frag(const bf16_t *t, int mt, int k0, int r, int kg) {
        return tr_frag(t, LD, k0, mt * 16, r, kg);
    }
};

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

// sum over the 16 lanes that share kg (i.e. over the column index r of an accumulator row)
__device__ __forceinline__ float reduce16(float v) {
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 8);
    return v;
}

// sum over the whole wave
__device__ __forceinline__ float reduce64(float v) {
    v = reduce16(v);
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    return v;
}

// Workgroup id -> (bh, sub) with all `nsub` workgroups of one bh on the same XCD (workgroups are
// dealt round-robin to the 8 XCDs, each with its own L2).  Grid must be 8 * ceil(BH/8) * nsub.
__device__ __forceinline__ void xcd_map(int bid, int nsub, int &bh, int &sub) {
    const int xcd = bid & 7, slot = bid >> 3;
    bh = (slot / nsub) * 8 + xcd;
    sub = slot % nsub;
}

} // namespace mdn
