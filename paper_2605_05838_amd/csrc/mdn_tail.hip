// A sequence whose length is not a multiple of the chunk size (Algorithm 1 pads such a sequence): the
// full chunks run on the caller's tensors as they are; the last, partial chunk runs on a padded copy of its
// tokens.  A padding token has k = v = q = 0, alpha = mu = 1, beta = 0: by Eq. Mt.recurrent / St.recurrent it
// changes neither S nor M, so the states after the padded chunk are the exact final states, and with dO = 0 on
// the padding rows the reverse pass is exact as well.  These two kernels move the partial chunk's rows into
// and out of the padded [B, 64, H, *] copies.
#include "mdn_device.h"
#include "mdn_kernels.h"

namespace mdn {

namespace {

// one row = row_bytes (a multiple of 4) of tensor t; blockIdx.y = tensor, blockIdx.x = (b, i, h) row
__global__ __launch_bounds__(64) void tail_gather_kernel(TailCopy c) {
    const TailTensor t = c.t[blockIdx.y];
    const int row = blockIdx.x, h = row % c.H, i = (row / c.H) % 64, b = row / (c.H * 64);
    const int words = t.row_bytes / 4;
    uint32_t *dst = reinterpret_cast<uint32_t *>(static_cast<char *>(t.padded) + (size_t)row * t.row_bytes);
    if (i < c.r) {
        const size_t srow = ((size_t)b * c.T + (size_t)c.t0 + i) * c.H + h;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(static_cast<const char *>(t.full) + srow * t.row_bytes);
        for (int x = threadIdx.x; x < words; x += 64) dst[x] = src[x];
    } else {
        for (int x = threadIdx.x; x < words; x += 64) dst[x] = t.pad_word;
    }
}

__global__ __launch_bounds__(64) void tail_scatter_kernel(TailCopy c) {
    const TailTensor t = c.t[blockIdx.y];
    const int row = blockIdx.x, h = row % c.H, i = (row / c.H) % 64, b = row / (c.H * 64);
    if (i >= c.r) return;
    const int words = t.row_bytes / 4;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(static_cast<const char *>(t.padded) + (size_t)row * t.row_bytes);
    const size_t drow = ((size_t)b * c.T + (size_t)c.t0 + i) * c.H + h;
    uint32_t *dst = reinterpret_cast<uint32_t *>(static_cast<char *>(const_cast<void *>(t.full)) + drow * t.row_bytes);
    for (int x = threadIdx.x; x < words; x += 64) dst[x] = src[x];
}

// chunks of C < 64 tokens as 64-token tiles: blockIdx.y = tensor, blockIdx.x = (b, chunk, i, h) row of the padded tensor
template <bool EXPAND> __global__ __launch_bounds__(64) void chunk_copy_kernel(ChunkCopy c) {
    const TailTensor t = c.t[blockIdx.y];
    const int row = blockIdx.x, h = row % c.H, i = (row / c.H) % 64, nc = (row / (c.H * 64)) % c.NC, b = row / (c.H * 64 * c.NC);
    const int words = t.row_bytes / 4, tok = nc * c.C + i;
    const bool real = i < c.C && tok < c.T;
    uint32_t *pad = reinterpret_cast<uint32_t *>(static_cast<char *>(t.padded) + (size_t)row * t.row_bytes);
    uint32_t *full = reinterpret_cast<uint32_t *>(static_cast<char *>(const_cast<void *>(t.full)) +
                                                  (((size_t)b * c.T + (real ? tok : 0)) * c.H + h) * t.row_bytes);
    if (EXPAND) {
        for (int x = threadIdx.x; x < words; x += 64) pad[x] = real ? full[x] : t.pad_word;
    } else if (real) {
        for (int x = threadIdx.x; x < words; x += 64) full[x] = pad[x];
    }
}

// blockIdx.x = entry of the token list; threads over the heads
__global__ __launch_bounds__(64) void set_at_tokens_kernel(float *a, float *b, float value, SeqStarts st) {
    const size_t row = (size_t)st.t[blockIdx.x] * st.H;
    for (int h = threadIdx.x; h < st.H; h += 64) {
        a[row + h] = value;
        if (b) b[row + h] = value;
    }
}

// blockIdx.y = tensor, blockIdx.x = (entry, i, h) row of the padded batch
__global__ __launch_bounds__(64) void gather_seq_rows_kernel(SeqRows g) {
    const TailTensor t = g.t[blockIdx.y];
    const int row = blockIdx.x, h = row % g.H, i = (row / g.H) % 64, e = row / (g.H * 64);
    const int words = t.row_bytes / 4;
    uint32_t *dst = reinterpret_cast<uint32_t *>(static_cast<char *>(t.padded) + (size_t)row * t.row_bytes);
    if (i < g.r[e]) {
        const size_t srow = ((size_t)g.t0[e] + i) * g.H + h;
        const uint32_t *src = reinterpret_cast<const uint32_t *>(static_cast<const char *>(t.full) + srow * t.row_bytes);
        for (int x = threadIdx.x; x < words; x += 64) dst[x] = src[x];
    } else {
        for (int x = threadIdx.x; x < words; x += 64) dst[x] = t.pad_word;
    }
}

// blockIdx.x = entry, blockIdx.y = head, blockIdx.z = 0: S, 1: M
template <typename T> __global__ __launch_bounds__(256) void states_to_f32_kernel(const T *full, const T *tail, const T *lo_full,
                                                                                  const T *lo_tail, SeqChunks c, float *S, float *M) {
    const int e = blockIdx.x, h = blockIdx.y, which = blockIdx.z, n = c.chunk[e];
    const size_t blk = (size_t)c.dk * c.dv;
    const size_t off = n < c.N ? (((size_t)h * c.N + n) * 2 + which) * blk : ((size_t)h * 2 + which) * blk;
    const T *src = (n < c.N ? full : tail) + off;
    const T *lo = (n < c.N ? lo_full : lo_tail);
    float *dst = (which ? M : S) + ((size_t)e * c.H + h) * blk;
    for (int x = threadIdx.x; x < c.dk * c.dv; x += 256) {
        const int row = x / c.dv, col = x % c.dv;
        const size_t i = vblk(c.dk, row, col);
        dst[x] = to_f32(src[i]) + (lo ? to_f32(lo[off + i]) : 0.f);
    }
}

} // namespace

hipError_t launch_gather_seq_rows(const SeqRows &g, hipStream_t s) {
    if (g.n < 1 || g.ntens < 1) return hipSuccess;
    if (g.n > kSeqRowsPerLaunch || g.ntens > 8 || g.H < 1) return hipErrorInvalidValue;
    for (int e = 0; e < g.n; ++e)
        if (g.t0[e] < 0 || g.r[e] < 1 || g.r[e] > 64) return hipErrorInvalidValue;
    for (int k = 0; k < g.ntens; ++k)
        if (!g.t[k].full || !g.t[k].padded || g.t[k].row_bytes < 4 || g.t[k].row_bytes % 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(gather_seq_rows_kernel, dim3(g.n * 64 * g.H, g.ntens), dim3(64), 0, s, g);
    return hipGetLastError();
}

hipError_t launch_states_to_f32(const void *states_full, const void *states_tail, const void *lo_full, const void *lo_tail,
                                const SeqChunks &c, float *S, float *M, hipStream_t s) {
    if (c.n < 1) return hipSuccess;
    if (c.n > kSeqRowsPerLaunch || !S || !M || c.H < 1 || c.N < 0) return hipErrorInvalidValue;
    for (int e = 0; e < c.n; ++e) {
        if (c.chunk[e] < 0 || c.chunk[e] > c.N) return hipErrorInvalidValue;
        if (c.chunk[e] < c.N ? !states_full : !states_tail) return hipErrorInvalidValue;
    }
    const dim3 grid(c.n, c.H, 2), block(256);
    if (c.dtype == 1)
        hipLaunchKernelGGL(states_to_f32_kernel<float>, grid, block, 0, s, static_cast<const float *>(states_full),
                           static_cast<const float *>(states_tail), static_cast<const float *>(nullptr),
                           static_cast<const float *>(nullptr), c, S, M);
    else
        hipLaunchKernelGGL(states_to_f32_kernel<bf16_t>, grid, block, 0, s, static_cast<const bf16_t *>(states_full),
                           static_cast<const bf16_t *>(states_tail), static_cast<const bf16_t *>(lo_full),
                           static_cast<const bf16_t *>(lo_tail), c, S, M);
    return hipGetLastError();
}

hipError_t launch_set_at_tokens(float *a, float *b, float value, const SeqStarts &st, hipStream_t s) {
    if (st.n < 1) return hipSuccess;
    if (!a || st.n > kSeqStartsPerLaunch || st.H < 1) return hipErrorInvalidValue;
    hipLaunchKernelGGL(set_at_tokens_kernel, dim3(st.n), dim3(64), 0, s, a, b, value, st);
    return hipGetLastError();
}

hipError_t launch_chunk_copy(const ChunkCopy &c, bool expand, hipStream_t s) {
    if (c.n < 1) return hipSuccess;
    if (c.n > 12 || c.B < 1 || c.H < 1 || c.T < 1 || (c.C != 16 && c.C != 32) || c.NC != (c.T + c.C - 1) / c.C) return hipErrorInvalidValue;
    for (int k = 0; k < c.n; ++k)
        if (!c.t[k].full || !c.t[k].padded || c.t[k].row_bytes < 4 || c.t[k].row_bytes % 4) return hipErrorInvalidValue;
    const long long rows = (long long)c.B * c.NC * 64 * c.H;
    if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)rows, c.n), block(64);
    if (expand)
        hipLaunchKernelGGL(chunk_copy_kernel<true>, grid, block, 0, s, c);
    else
        hipLaunchKernelGGL(chunk_copy_kernel<false>, grid, block, 0, s, c);
    return hipGetLastError();
}

hipError_t launch_tail_copy(const TailCopy &c, bool gather, hipStream_t s) {
    if (c.n < 1) return hipSuccess;
    dim3 grid(c.B * 64 * c.H, c.n), block(64);
    if (gather)
        hipLaunchKernelGGL(tail_gather_kernel, grid, block, 0, s, c);
    else
        hipLaunchKernelGGL(tail_scatter_kernel, grid, block, 0, s, c);
    return hipGetLastError();
}

} // namespace mdn
