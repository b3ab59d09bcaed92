// Host-side launch interface between the C ABI (mdn_api.hip) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mdn {

struct Dims {
    int B, T, H, N, BH; // N = T / 64 chunks, BH = B * H
    int n0, n1;         // chunks [n0, n1) handled by this launch (0, N unless the call is split into segments)
    int dk, dv;
    int dtype; // MDN_DTYPE_*
    float scale;
};

// Chunk-parallel precompute ("intra") kernel arguments.  Workspace tensors are chunk-blocked,
// [BH][N][tile], in the storage dtype unless noted; inside a tile, an MFMA operand [rows][k] is in
// the kblk layout and a [rows][dv] tensor in the vblk layout of mdn_device.h.
constexpr int kCoefBlockCols = 8; // floats per token in the coefficient block

struct IntraArgs {
    const void *q, *k;                      // [B,T,H,dk]
    const float *alpha, *beta, *mu, *eta;   // [B,T,H]; eta may be null
    float *coef;                            // [BH][N][64][kCoefBlockCols] fp32 (one row of coefficients per token)
    void *KT;                               // kblk [dk][64]   raw k, transposed
    // forward mode
    void *Tm;                               // kblk [64][64]   T = (I + A)^-1: row i, contraction index j
    void *Bm;                               // kblk [64][64]   (Q~ K~^T) .* Gamma
    // backward mode
    void *QT;                               // kblk [dk][64]   raw q, transposed
    void *BmT;                              // kblk [64][64]   Bm transposed
    void *TmT;                              // kblk [64][64]   T transposed
};

struct ScanFwdArgs {
    const void *q, *k;                      // [B,T,H,dk]
    const void *v;                          // [B,T,H,dv]
    const float *coef;
    const void *KT, *Tm, *Bm;
    const float *S0, *M0;                   // [B,H,dk,dv] or null
    void *o;                                // [B,T,H,dv]
    void *vt_saved;                         // [B,T,H,dv] or null
    void *states_saved;                     // [BH][N][2] x vblk [dk][dv], or null
    void *states_lo;                        // same layout, or null: what the 16-bit rounding of states_saved dropped
                                            // (see GradArgs, and the packed prefill in mdn_api.hip)
    float *S_final, *M_final;               // or null
};

// State reconstruction from saved V~ (backward, when the forward did not keep the states).
struct RebuildArgs {
    const float *coef;
    const void *k;                          // [B,T,H,dk] (16-bit storage reads K^T out of the k rows)
    const void *KT;
    const void *vt_saved;                   // [B,T,H,dv]
    const float *S0, *M0;
    void *states;                           // [BH][N][2] x vblk [dk][dv]
    void *states_lo;                        // or null: the rounding remainders of `states` (16-bit storage)
    float *S_final, *M_final;               // states after the last chunk, or null
};

struct ScanBwdArgs {
    const void *k;                          // [B,T,H,dk]
    const void *dO;                         // [B,T,H,dv]
    const float *coef;
    const void *QT, *KT, *BmT, *TmT;
    const float *dS_final, *dM_final;       // or null
    void *dv;                               // [B,T,H,dv]  dV = T^T dV~
    void *dstates;                          // [BH][N][2] x vblk [dk][dv]: adjoints of the chunk-END states
    void *dstates_lo;                       // or null: the rounding remainders of `dstates` (16-bit storage)
    float *dS0, *dM0;                       // or null
};

struct GradArgs {
    const void *q, *k;                      // [B,T,H,dk]
    const float *alpha, *beta, *mu, *eta;
    const void *vt_saved, *dO, *dv;         // [B,T,H,dv]; dv (= dR, from the reverse scan) is read
    const void *KT, *QT;
    const void *states, *dstates;           // [BH][N][2] x vblk [dk][dv]
    // 16-bit storage, calls that bring adjoints of the final states in (both or neither): x - bf16(x) of the two
    // tensors above, again in bf16.  Adjoints that enter from outside can be large against everything dO puts into
    // the states; <dS', S>, <dS', M>, <dM', M> and the products of dS', dM' with V~ are then sums of dk dv terms
    // whose storage rounding alone would reach the tolerance, so those sums take hi + lo of both factors.
    const void *states_lo, *dstates_lo;
    void *dq, *dk;
    float *dalpha, *dbeta, *dmu, *deta;     // deta may be null
};

struct RecurrentArgs {
    const void *q, *k, *v;
    const float *alpha, *beta, *mu, *eta;
    float *S, *M;
    void *o;
};

// compute units of the current device (256 if it cannot be asked)
int num_cus();
// dv columns per workgroup of the scans for this shape: 32, unless that leaves a quarter of the CUs or more without
// a workgroup or (32-bit storage, d = 128) the prefetched fragments of 32 columns do not fit the registers: then 16
int scan_dvb(const Dims &d);
// workgroups of one scan launch: (batch*head rounded up to 8) x dv / scan_dvb
int scan_workgroups(const Dims &d);

// mode 0: forward operands, 1: reverse-pass operands, 2: both
hipError_t launch_intra(const Dims &d, int mode, const IntraArgs &a, hipStream_t s);
hipError_t launch_scan_fwd(const Dims &d, const ScanFwdArgs &a, hipStream_t s);
// Dynamic LDS bytes that keep a second workgroup of `kernel` off a CU (0 if one workgroup fills more than half of the
// 160 KB already).  For launches with fewer workgroups than CUs: the dispatcher otherwise puts two of them on one CU
// and leaves other CUs empty, and two scan workgroups that share a CU take turns at everything.
size_t lds_bytes_for_one_workgroup_per_cu(const void *kernel);

// whether that launch reads a.KT (32-bit storage; 16-bit storage forms K^T out of the k rows in LDS)
bool scan_fwd_reads_KT(const Dims &d);
hipError_t launch_rebuild(const Dims &d, const RebuildArgs &a, hipStream_t s);
hipError_t launch_scan_bwd(const Dims &d, const ScanBwdArgs &a, hipStream_t s);
hipError_t launch_grad(const Dims &d, const GradArgs &a, hipStream_t s);
hipError_t launch_recurrent(const Dims &d, const RecurrentArgs &a, hipStream_t s);

// Rows of a partial last chunk: tokens t0 .. t0+r-1 of every sequence of a [B,T,H,row] tensor <-> rows 0 .. r-1 of
// a padded [B,64,H,row] copy (gather fills the rows from r on with pad_word).
struct TailTensor {
    const void *full; // the caller's tensor (written by scatter)
    void *padded;     // the padded copy (written by gather)
    int row_bytes;    // a multiple of 4
    uint32_t pad_word;
};
struct TailCopy {
    int B, T, H, t0, r, n; // n tensors
    TailTensor t[12];
};
hipError_t launch_tail_copy(const TailCopy &c, bool gather, hipStream_t s);

// Chunk sizes below 64 (Algorithm 1 lists C in {16, 32, 64}): every chunk of C tokens becomes one 64-token tile whose
// rows from C on are padding (TailTensor::pad_word).  expand: [B,T,H,row] -> [B, ceil(T/C) * 64, H, row];
// collect: the real rows back.
struct ChunkCopy {
    int B, T, H, C, NC, n; // NC = ceil(T / C) chunks, n tensors
    TailTensor t[12];
};
hipError_t launch_chunk_copy(const ChunkCopy &c, bool expand, hipStream_t s);

// Packed variable-length batches run as one stream of tokens whose state is cut at the first token of every
// sequence but the first: x[t, h] = value for the listed tokens t of up to two [T, H] fp32 tensors (a, b; b may be
// null).  The token list travels in the kernel arguments, kSeqStartsPerLaunch at a time.
constexpr int kSeqStartsPerLaunch = 240;
struct SeqStarts {
    int n, H;
    int t[kSeqStartsPerLaunch];
};
hipError_t launch_set_at_tokens(float *a, float *b, float value, const SeqStarts &st, hipStream_t s);

// The last (possibly partial) chunk of each listed sequence of a token stream [T, H, *], as a batch of padded
// 64-token rows [n, 64, H, *]: entry i takes tokens [t0[i], t0[i] + r[i]) (1 <= r <= 64) and pads like TailCopy.
constexpr int kSeqRowsPerLaunch = 200;
struct SeqRows {
    int n, H, ntens;
    int t0[kSeqRowsPerLaunch], r[kSeqRowsPerLaunch];
    TailTensor t[8];
};
hipError_t launch_gather_seq_rows(const SeqRows &g, hipStream_t s);

// Chunk-start states out of the saved-states buffer of a single-batch call (blocks [H][N][2] in the vblk layout and
// the storage type, then one block pair per head for the partial chunk) as fp32 [n, H, dk, dv]: entry i takes chunk
// chunk[i] (== N: the partial chunk's block).
struct SeqChunks {
    int n, H, N, dk, dv, dtype;
    int chunk[kSeqRowsPerLaunch];
};
// (lo_full, lo_tail: the rounding remainders of the same blocks, or null)
hipError_t launch_states_to_f32(const void *states_full, const void *states_tail, const void *lo_full, const void *lo_tail,
                                const SeqChunks &c, float *S, float *M, hipStream_t s);

} // namespace mdn
