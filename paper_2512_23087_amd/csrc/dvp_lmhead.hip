// LM-head variant of the DVP hot path for gfx950: the logits z = H W^T are
// produced tile by tile on the matrix cores (MFMA, bf16 in, fp32 accumulate)
// and consumed in the tile epilogues; the [N, V] logits are never stored.
//
// Membership needs the final row maximum (Def. 5.1), so the logits of a side
// are produced twice:
//   pass A  z tiles -> running row max, and z_y where a tile holds column y
//   pass B  z tiles -> safe-set size and masked sum at tau = fl32(m + log_rho)
//           (Def. 5.1 / 5.2), per 256-column partials, reduced in fixed order
// When a gradient is asked for, the training side runs in blocks of 8192 token
// rows and pass B also leaves the block's masked exponentials
//   E_ik = [z_ik >= tau_i] exp(z_ik - m_i)          (bf16, [rows, V] in panels of 256 columns)
// behind, with the sampled token's own entry E_iy set to zero.  With S_i the
// row sum (sampled token included), c_i = grad_out_i (0 when y_i is pruned),
// s_i = -c_i / S_i and q_i = c_i (1 - p_iy) the sampled token's gradient entry,
// Prop. 5.4 reads dz_ik = q_i delta(k, y_i) + s_i E_ik, so
//   dH_i = q_i W_y + s_i (E W)_i,   dW = onehot^T diag(q) H + E^T (diag(s) H).
// The two E products run on the matrix cores (the row factor s is applied in
// fp32 when dH is written and folded into H for dW, which is accumulated over
// the row blocks); the sampled token's entry, the one that cancels when the
// distribution is peaked, is formed and added in fp32 and never rounded to bf16.
// The forward products are C = A B^T with both operands K-major.  The two E products are not of that form
// (dH contracts over W's rows, dW over the token rows of E and of diag(s) H): the GEMM kernel has builds that
// take an operand as it lies, [K, ld], and fetch its fragments with the transposing LDS read, so that no
// transposed copy of W or E is ever written (dW still takes a transposed copy of its small operand, the row
// block's diag(s) H).  E is stored in panels of 256 columns, each panel [rows, 256] contiguous: as dW's
// first operand (rows = k) a tile's K step is then one 32 KB run; with E row-major (rows 300 KB apart) that
// product was a quarter slower than from a transposed copy.
#include <math.h>

#include <atomic>
#include <utility>

#include "dvp_device.h"
#include "dvp_lmhead_internal.h"

namespace dvp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 256, BN = 256, BK = 64;      // workgroup tile
constexpr int WM = 4, WN = 2;                   // 8 wavefronts as 4 x 2, two per SIMD
constexpr int MI = BM / WM / 32, NI = BN / WN / 32;   // 32x32 accumulator blocks per wavefront: a 64x128 block
constexpr int kGemmWaves = WM * WN;
constexpr int kGemmThreads = kGemmWaves * kWave;
constexpr int kRowBytes = BK * 2;               // one tile row in LDS: 128 B, its eight 16-byte chunks XOR-swizzled by row
constexpr int kTileBytes = BM * kRowBytes;      // one operand tile in LDS: 32 KB
constexpr int kStageBytes = 2 * kTileBytes;     // A tile, then B tile
constexpr int kPipeLdsBytes = 2 * kStageBytes;  // two stages: 128 KB of the CU's 160 KB
constexpr int kSumScratchBytes = 6 * BM * 4;    // pass B's per-row partials of the two column halves
constexpr int kGemmLdsBytes = kPipeLdsBytes + kSumScratchBytes;
constexpr int kWaveStageBytes = kPipeLdsBytes / kGemmWaves;   // 16 KB: a wavefront's 64x128 block as bf16
static_assert(kWaveStageBytes == MI * 32 * NI * 32 * 2, "epilogue staging assumes one bf16 block per wavefront");
constexpr int kCopiesPerWave = BM * (BK / 8) / kWave / kGemmWaves;   // 1 KB wavefront copies per operand tile and wavefront
static_assert(BM == BN, "the operand tiles share one copy schedule");
constexpr int kRowBlock = 8192;                 // token rows whose logits are held at a time
constexpr int kDwBlocks = 2;                    // row blocks whose masked exponentials are held for one dW product
constexpr int kHstPad = 64;                     // elements added to the row pitch of (diag(s) H)^T: a tile's 256 rows, a power of
                                                // two apart otherwise, then start on different 128-byte lines

__device__ __forceinline__ int float_to_ordered(float f)
{
    const int b = __float_as_int(f);
    return b >= 0 ? b : b ^ 0x7fffffff;
}
__device__ __forceinline__ float ordered_to_float(int k)
{
    return __int_as_float(k >= 0 ? k : k ^ 0x7fffffff);
}

// per-row quantities of one side, device arrays in the workspace
struct RowStats {
    int *max_key;        // [n] ordered-int row maximum (pass A, atomicMax)
    float *zy;           // [n] logit of the sampled token (pass A)
    float *m;            // [n] row maximum (after pass A)
    float *tau;          // [n] threshold
    float *part_s;       // [col_tiles][n] masked exp sums per 256-column tile (pass B)
    float *part_f;       // [col_tiles][n] full exp sums, or null
    int *part_c;         // [col_tiles][n] safe counts per tile
    float *coef;         // [n] q = c (1 - p_y), c = grad_out where the sampled token is safe, else 0 (after pass B)
    float *scale;        // [n] s = -c / S (after pass B)
};

struct GemmArgs {
    const uint16_t *A;   // [M, lda] bf16, K-major
    const uint16_t *B;   // [N, ldb] bf16, K-major
    int64_t lda, ldb;
    int M, N, K;         // K a multiple of BK; rows beyond M / N are clamped on load and masked in the epilogue
    float scale;         // 8-bit operands only: the accumulators are multiplied by it before the epilogue
    // 8-bit (E4M3) operands are described in the same units: two bytes count as one element, so a K
    // step is still 128 bytes of every row and the copy schedule does not change.
    // A row count that only the device knows (a subset of rows chosen by an earlier kernel): n_dev
    // non-null says that the launch's rows are rows n_off .. of *n_dev rows in all.  dev_dim = 1: they
    // are the rows of A, M = clamp(*n_dev - n_off, 0, M) (the launch is sized for M; workgroups without a
    // tile leave at once); dev_dim = 2: they are the K dimension, K = that count rounded up to a whole row
    // tile (the operands are zero padded that far); none left: the launch does nothing.
    const int *n_dev = nullptr;
    int n_off = 0, dev_dim = 0;
    // Operands stored the other way round (the kernel's ATR / BTR builds): A is then [K, lda] with its M index
    // contiguous, B [K, ldb] with its N index contiguous (lda, ldb multiples of 8, at least a whole number of
    // 16-byte pieces per row).  kb_rows says how many of B's K rows exist in memory: rows past them are read from
    // the last one (the other operand carries zeros there); A's K rows all exist.  a_cols / b_cols: elements of a row that may be
    // read (a multiple of 8, at least 8; 0: the whole pitch): 16-byte pieces past them are read from the last piece.
    int kb_rows = 0, a_cols = 0, b_cols = 0;
    // A stored in panels (a_panel > 0, elements): the matrix [R, C] is cut into panels of 256 columns, each a
    // contiguous [R, 256] block, element (r, c) at (c / 256) * a_panel + r * 256 + c % 256; lda is 256.  As a K-major
    // operand its columns are k (a K step is a quarter of a panel row), as a [K, lda] operand its rows are k and a
    // tile of 256 m is one panel, 64 rows of k a contiguous 32 KB.  (Read by the ATR / BTR builds only.)
    int64_t a_panel = 0;
};

__device__ __forceinline__ int rows_on_device(const int *n_dev, int n_off, int rows_host)
{
    if (!n_dev) return rows_host;
    const int left = *n_dev - n_off;
    return left < 0 ? 0 : (left > rows_host ? rows_host : left);
}

// ---------------------------------------------------------------------------
// From a row per lane to whole lines per store.  In a swapped 32x32 block (see EpiMax) lane l holds, of token row
// l % 32, the columns 8 q + 4 (l / 32) .. + 3 in x[q]: a 16-byte store of x[q] puts 32 bytes on each of 32 rows.
// Afterwards lane l holds in x[q] the columns 16 (l / 32) + 4 (l % 4) .. + 3 of token row (l % 32 & ~3) + q: four
// neighbouring lanes then store 64 consecutive bytes, and the eight lanes l % 4, l / 32 a row's whole 128-byte line.
// Two steps: the two halves of the wavefront trade registers (v_permlane32_swap) so that a lane owns 16 consecutive
// columns of its row, then each group of four lanes transposes its 4 x 4 pieces of 16 bytes (two butterfly stages
// through the quad permutation of the data-parallel move).  Lane layout checked element by element on the device.
// ---------------------------------------------------------------------------
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
template <int QUAD_PERM>
__device__ __forceinline__ float quad_from(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), QUAD_PERM, 0xf, 0xf, true));
}
template <int QUAD_PERM>
__device__ __forceinline__ void trade_pieces(f32x4 &lo, f32x4 &hi, bool upper)
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const float sent = upper ? lo[c] : hi[c];
        const float got = quad_from<QUAD_PERM>(sent);
        lo[c] = upper ? got : lo[c];
        hi[c] = upper ? hi[c] : got;
    }
}
__device__ __forceinline__ void rows_to_lines(f32x4 (&x)[4], int lane)
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x[0][c]), __float_as_uint(x[2][c]), false, false);
        x[0][c] = __uint_as_float(r[0]); x[2][c] = __uint_as_float(r[1]);
        r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x[1][c]), __float_as_uint(x[3][c]), false, false);
        x[1][c] = __uint_as_float(r[0]); x[3][c] = __uint_as_float(r[1]);
    }
    const f32x4 t = x[1]; x[1] = x[2]; x[2] = t;     // x[s] now: columns 16 (l / 32) + 4 s .. + 3 of the lane's row
    constexpr int kXor1 = 0xB1, kXor2 = 0x4E;        // quad permutations [1, 0, 3, 2] and [2, 3, 0, 1]
    const bool odd = lane & 1, up = lane & 2;
    trade_pieces<kXor1>(x[0], x[1], odd); trade_pieces<kXor1>(x[2], x[3], odd);
    trade_pieces<kXor2>(x[0], x[2], up);  trade_pieces<kXor2>(x[1], x[3], up);
}

// ---------------------------------------------------------------------------
// epilogues: called once per wavefront with its 64x128 accumulator block.
// Every product is taken with the operands swapped (the B fragment is the matrix instruction's row operand): element
// (mi, ni, i) of lane l is row r0 + mi*32 + l%32, column c0 + ni*32 + (i/4)*8 + (l/32)*4 + i%4 of the launch's
// output, i.e. a lane owns one output row per mi and four consecutive columns per register quad (see EpiMax for
// what that buys).  `lds` is the workgroup's dynamic LDS: the operand tiles and, behind them, the scratch of pass
// B's sums.
// ---------------------------------------------------------------------------
// STORE_Z: the tile's logits are also stored as fp32, row-major in Z [rows of the launch, ldz]: the
// statistics at the threshold are then taken from them by a streaming kernel instead of a second
// pass of the product (re-reading a row block's logits costs a fraction of recomputing them).
template <bool STORE_Z>
struct EpiMax {
    static constexpr bool kRowMap = false;
    // A lane owns one token row per mi and four consecutive columns per register quad (in the matrix instruction's
    // natural order it would own a column of 16 rows): the row maximum is 63 in-lane maxima and one exchange
    // with lane l ^ 32 (the column-per-lane layout needs five exchanges for each of 32 rows and 32 atomic
    // instructions of two lanes each) and the sampled token's id is loaded once per lane.  Measured on the
    // forward product of configs[4] (9.44 ms per block of 8192 rows with the column-per-lane epilogue): 0.57 ms
    // of it were the maxima, 0.85 ms the 4-byte stores.  The logits leave as 16-byte stores after the lanes
    // have traded pieces so that a store covers whole lines (rows_to_lines): stored straight from the row-per-lane
    // layout (32 bytes on each of 32 rows per store) they cost 0.9 ms per block, two thirds of it spent issuing
    // them into the L2; with whole lines the block takes 8.15 ms instead of 8.45.  Whole lines can also leave as
    // nontemporal stores (0.3 ms per call less; as 32-byte pieces they had cost the call 11 ms).
    RowStats st;
    const int64_t *ids;
    float *Z;            // [rows padded to BM, ldz]; ldz covers whole column tiles, so every tile element has a place
    int64_t ldz;
    __device__ __forceinline__ void operator()(const GemmArgs &g, f32x16 (&acc)[MI][NI], int r0, int c0, int lane, uint8_t *, int, int) const
    {
        const int half = lane / 32;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = r0 + mi * 32 + (lane % 32);
            const bool row_ok = row < g.M;
            const int64_t y = row_ok ? ids[row] : -1;
            // the sampled token's column inside this wavefront's NI * 32 columns, or -1 (columns past N repeat
            // column N - 1 and are never the sampled one: y < N)
            const int yc = (y >= (int64_t)c0 && y < (int64_t)c0 + NI * 32) ? (int)(y - c0) : -1;
            float v = -INFINITY;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int colb = ni * 32 + q * 8 + half * 4;
                    const float z0 = acc[mi][ni][q * 4], z1 = acc[mi][ni][q * 4 + 1], z2 = acc[mi][ni][q * 4 + 2],
                                z3 = acc[mi][ni][q * 4 + 3];
                    v = fmaxf(fmaxf(v, fmaxf(z0, z1)), fmaxf(z2, z3));    // (repeated columns repeat a real logit)
                    if (yc >= colb && yc < colb + 4) st.zy[row] = yc == colb ? z0 : (yc == colb + 1 ? z1 : (yc == colb + 2 ? z2 : z3));
                }
                if constexpr (STORE_Z) {
                    f32x4 x[4];
#pragma unroll
                    for (int q = 0; q < 4; ++q) x[q] = (f32x4){acc[mi][ni][q * 4], acc[mi][ni][q * 4 + 1], acc[mi][ni][q * 4 + 2], acc[mi][ni][q * 4 + 3]};
                    rows_to_lines(x, lane);
                    const int row0 = r0 + mi * 32 + ((lane % 32) & ~3);
                    float *zline = Z + (int64_t)row0 * ldz + c0 + ni * 32 + 16 * half + 4 * (lane % 4);
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        if (row0 + q < g.M) __builtin_nontemporal_store(x[q], (f32x4 *)(zline + (int64_t)q * ldz));
                }
            }
            v = fmaxf(v, __shfl_xor(v, 32, kWave));
            if (half == 0 && row_ok) atomicMax(st.max_key + row, float_to_ordered(v));
        }
    }
};

// Pass A that also collects candidates for the safe set.  The threshold is m + log_rho with m the
// row maximum over the whole vocabulary, unknown here; any lower bound of m gives a lower threshold and
// so a superset of the safe set.  The bound used is the larger of the maximum over this wavefront's
// 128 columns and a value known to lie below the sampled token's logit (zy_low): both depend on the
// inputs only, not on the order in which tiles run, so a row's candidate set is the same in every run.
// Candidates (token, z) are appended in arrival order; at most cand_cap are kept.
struct EpiMaxCand {
    static constexpr bool kRowMap = false;
    // A lane owns a token row, so the maximum over the wavefront's 128 columns, the threshold and the test of the
    // row's 128 logits against it are all in-lane.  Candidates are rare where this
    // form is used (peaked rows): the lanes that have any are served one after the other, their hit mask and their
    // logits read through v_readlane, every register named statically.
    RowStats st;
    const int64_t *ids;
    const float *zy_low;     // [n] lower bound of the row maximum, -inf where there is none
    dvp_grad_entry *cand;    // [n, cand_cap]
    int *cursor;             // [n], zero before the launch
    int cand_cap;
    float log_rho;
    __device__ __forceinline__ void operator()(const GemmArgs &g, f32x16 (&acc)[MI][NI], int r0, int c0, int lane, uint8_t *, int, int) const
    {
        const int half = lane / 32;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = r0 + mi * 32 + (lane % 32);
            const bool row_ok = row < g.M;
            const int64_t y = row_ok ? ids[row] : -1;
            const int yc = (y >= (int64_t)c0 && y < (int64_t)c0 + NI * 32) ? (int)(y - c0) : -1;   // see EpiMax
            float v = -INFINITY;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int colb = ni * 32 + q * 8 + half * 4;
                    const float z0 = acc[mi][ni][q * 4], z1 = acc[mi][ni][q * 4 + 1], z2 = acc[mi][ni][q * 4 + 2],
                                z3 = acc[mi][ni][q * 4 + 3];
                    v = fmaxf(fmaxf(v, fmaxf(z0, z1)), fmaxf(z2, z3));    // (repeated columns repeat a real logit)
                    if (yc >= colb && yc < colb + 4) st.zy[row] = yc == colb ? z0 : (yc == colb + 1 ? z1 : (yc == colb + 2 ? z2 : z3));
                }
            }
            v = fmaxf(v, __shfl_xor(v, 32, kWave));
            if (half == 0 && row_ok) atomicMax(st.max_key + row, float_to_ordered(v));
            // <= the row's final threshold (fp32 addition is monotone)
            const float thr = row_ok ? fmaxf(v, zy_low[row]) + log_rho : INFINITY;
            // bit ni * 16 + q * 4 + e of the lane's mask: column c0 + ni * 32 + q * 8 + half * 4 + e is a candidate
            uint32_t m_lo = 0u, m_hi = 0u;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int col = c0 + ni * 32 + (i / 4) * 8 + half * 4 + (i % 4);
                    const uint32_t hit = (row_ok && col < g.N && acc[mi][ni][i] >= thr) ? 1u : 0u;   // (an infinite logit meets any threshold)
                    if (ni * 16 + i < 32) m_lo |= hit << (ni * 16 + i);
                    else                  m_hi |= hit << (ni * 16 + i - 32);
                }
            }
            static_assert(NI * 16 == 64, "the hit mask of a lane and row is two 32-bit words");
            bool mine = (m_lo | m_hi) != 0u;
            if (__builtin_amdgcn_ballot_w64(mine) == 0ull) continue;          // the same for the whole wavefront
            // one look per lane and row: a full buffer stops the appends (a stale value only costs appends)
            if (mine && __hip_atomic_load(cursor + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) > cand_cap) mine = false;
            unsigned long long todo = __builtin_amdgcn_ballot_w64(mine);
            while (todo != 0ull) {                                            // wavefront-uniform
                const int src = __builtin_ctzll(todo);
                todo &= todo - 1ull;
                const uint32_t s_lo = (uint32_t)__builtin_amdgcn_readlane((int)m_lo, src);
                const uint32_t s_hi = (uint32_t)__builtin_amdgcn_readlane((int)m_hi, src);
                const int s_row = r0 + mi * 32 + (src % 32), s_half = src / 32;
                int base = 0;
                if (lane == 0) base = atomicAdd(cursor + s_row, __builtin_popcount(s_lo) + __builtin_popcount(s_hi));
                base = __builtin_amdgcn_readfirstlane(base);
                dvp_grad_entry *out = cand + (int64_t)s_row * cand_cap;
                int pos = base;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const uint32_t word = ni * 16 + i < 32 ? s_lo : s_hi;
                        if (!((word >> ((ni * 16 + i) & 31)) & 1u)) continue;  // uniform
                        const float z = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(acc[mi][ni][i]), src));
                        if (lane == 0 && pos < cand_cap) {
                            out[pos].index = (uint32_t)(c0 + ni * 32 + (i / 4) * 8 + s_half * 4 + (i % 4));
                            out[pos].value = z;
                        }
                        ++pos;
                    }
                }
            }
        }
    }
};

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)   // hardware pack-convert, round to nearest even
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo, hi}, bf16x2));
}

// Sums at the threshold per column tile.
// WRITE_BITS: also store the side's membership bitmask.
// WRITE_LIST: also append every safe token of a row, with exp(z - m), to that row's list (arrival
// order; at most list_cap entries are kept, the cursor stops a little above that).  Meant for rows
// whose safe sets are short: the branch is then rarely taken.
// ROWMAP: the launch covers a subset of the token rows, gathered into consecutive rows of A: their
// number is read from device memory (*n_sub; zero: nothing to do), the per-row statistics and partials
// are indexed by position in the subset, and lists by the row's own index rowmap[position].
template <bool WRITE_BITS = false, bool WRITE_LIST = false, bool ROWMAP = false>
struct EpiSum {
    static constexpr bool kRowMap = ROWMAP;
    RowStats st;
    int n_rows;
    uint32_t *bits;          // membership bitmask [n_rows, bits_ld] of the side, or null
    int64_t bits_ld;
    dvp_grad_entry *entries; // WRITE_LIST: [n_rows, list_cap]
    int *cursor;             // WRITE_LIST: [n_rows] entries appended so far, zero before the launch
    int list_cap;
    const int *rowmap;       // ROWMAP
    const int *n_sub;        // ROWMAP
    __device__ __forceinline__ void operator()(const GemmArgs &g, f32x16 (&acc)[MI][NI], int r0, int c0, int lane, uint8_t *lds, int wave, int wn) const
    {
        const bool want_full = st.part_f != nullptr;
        float *ls = (float *)(lds + kPipeLdsBytes), *lf = ls + 2 * BM;
        int *lc = (int *)(ls + 4 * BM);
        const int tile_row0 = r0 - (r0 % BM);
        const int half = lane / 32;
        static_assert(NI * 16 == 64, "the safe mask of a lane and row is two 32-bit words");
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = r0 + mi * 32 + (lane % 32);
            const bool row_ok = row < g.M;
            const float m = row_ok ? st.m[row] : 0.0f;
            const float tau = row_ok ? st.tau[row] : INFINITY;
            float s = 0.0f, f = 0.0f;
            int c = 0;
            // bit ni * 16 + i of the lane's mask: column c0 + ni * 32 + (i / 4) * 8 + half * 4 + i % 4 is safe
            uint32_t safe_lo = 0u, safe_hi = 0u;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int col = c0 + ni * 32 + (i / 4) * 8 + half * 4 + (i % 4);
                    const float z = acc[mi][ni][i];
                    if (col < g.N && row_ok) {
                        const bool safe = z >= tau;
                        c += safe ? 1 : 0;
                        float kept = 0.0f;
                        if (want_full) {
                            const float e = __expf(z - m);
                            f += e;
                            kept = safe ? e : 0.0f;
                        } else if (safe) {
                            kept = __expf(z - m);
                        }
                        s += kept;
                        if constexpr (WRITE_BITS || WRITE_LIST) {
                            if (ni * 16 + i < 32) safe_lo |= (safe ? 1u : 0u) << (ni * 16 + i);
                            else                  safe_hi |= (safe ? 1u : 0u) << (ni * 16 + i - 32);
                        }
                    }
                }
            }
            if constexpr (WRITE_BITS) {
                // a 32-column word of the row: the 16 bits of this lane (4 i / 4 groups of 4 at 8 (i / 4) + 4 half)
                // and the 16 of the lane that holds the row's other columns
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const uint32_t mine16 = ((ni * 16 < 32 ? safe_lo : safe_hi) >> ((ni * 16) & 31)) & 0xffffu;
                    uint32_t word = 0u;
#pragma unroll
                    for (int q = 0; q < 4; ++q) word |= ((mine16 >> (4 * q)) & 0xfu) << (8 * q + 4 * half);
                    word |= (uint32_t)__shfl_xor((int)word, 32, kWave);
                    const int64_t w = (c0 + ni * 32) >> 5;
                    if (half == 0 && row_ok && w < bits_ld) bits[(int64_t)row * bits_ld + w] = word;
                }
            }
            if constexpr (WRITE_LIST) {
                // Lanes with safe tokens (few rows reach this pass, and their safe sets are short) are served one
                // after the other; the lane's mask, maximum and logits are read through v_readlane, so every
                // accumulator register is named statically.  One look at the cursor per lane and row: a full list
                // stops the appends.
                bool mine = (safe_lo | safe_hi) != 0u;
                int list_row = row;
                if (__builtin_amdgcn_ballot_w64(mine) != 0ull) {
                    if (mine) {
                        if constexpr (ROWMAP) list_row = rowmap[row];
                        if (__hip_atomic_load(cursor + list_row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) > list_cap) mine = false;
                    }
                    unsigned long long todo = __builtin_amdgcn_ballot_w64(mine);
                    while (todo != 0ull) {                                    // wavefront-uniform
                        const int src = __builtin_ctzll(todo);
                        todo &= todo - 1ull;
                        const uint32_t s_lo = (uint32_t)__builtin_amdgcn_readlane((int)safe_lo, src);
                        const uint32_t s_hi = (uint32_t)__builtin_amdgcn_readlane((int)safe_hi, src);
                        const int s_list_row = __builtin_amdgcn_readlane(list_row, src), s_half = src / 32;
                        const float s_m = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), src));
                        int base = 0;
                        if (lane == 0) base = atomicAdd(cursor + s_list_row, __builtin_popcount(s_lo) + __builtin_popcount(s_hi));
                        base = __builtin_amdgcn_readfirstlane(base);
                        dvp_grad_entry *out = entries + (int64_t)s_list_row * list_cap;
                        int pos = base;
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                            for (int i = 0; i < 16; ++i) {
                                const uint32_t word = ni * 16 + i < 32 ? s_lo : s_hi;
                                if (!((word >> ((ni * 16 + i) & 31)) & 1u)) continue;   // uniform
                                const float z = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(acc[mi][ni][i]), src));
                                if (lane == 0 && pos < list_cap) {
                                    out[pos].index = (uint32_t)(c0 + ni * 32 + (i / 4) * 8 + s_half * 4 + (i % 4));
                                    out[pos].value = __expf(z - s_m);
                                }
                                ++pos;
                            }
                        }
                    }
                }
            }
            s += __shfl_xor(s, 32, kWave);
            f += __shfl_xor(f, 32, kWave);
            c += __shfl_xor(c, 32, kWave);
            if (half == 0) {
                const int lr = row - tile_row0;           // 0..BM-1
                ls[wn * BM + lr] = s;
                lf[wn * BM + lr] = f;
                lc[wn * BM + lr] = c;
            }
        }
    }
    // after a barrier: one thread per tile row combines the two column halves in fixed order
    __device__ __forceinline__ void finish(const GemmArgs &g, int tile_row0, int tile_col, uint8_t *lds, int tid) const
    {
        if (tid >= BM) return;
        const int row = tile_row0 + tid;
        if (row >= g.M) return;
        const float *ls = (const float *)(lds + kPipeLdsBytes), *lf = ls + 2 * BM;
        const int *lc = (const int *)(ls + 4 * BM);
        const int64_t o = (int64_t)tile_col * n_rows + row;
        st.part_s[o] = ls[tid] + ls[BM + tid];
        st.part_c[o] = lc[tid] + lc[BM + tid];
        if (st.part_f) st.part_f[o] = lf[tid] + lf[BM + tid];
    }
};

struct EpiStore {
    static constexpr bool kRowMap = false;
    float *C;                // [M, ldc] fp32
    int64_t ldc;
    int accumulate;          // 0: C = v, 1: C += v
    const float *row_scale;  // v = row_scale[row] * acc (null: v = acc) ...
    const float *row_coef;   // ... + row_coef[row] * src[ids[row], col] where row_coef[row] != 0 (null: no such term)
    const int64_t *ids;
    const uint16_t *src;     // bf16 [*, ld_src]
    int64_t ld_src;
    __device__ __forceinline__ void operator()(const GemmArgs &g, f32x16 (&acc)[MI][NI], int r0, int c0, int lane, uint8_t *, int, int) const
    {
        const int half = lane / 32;
        // 16-byte accesses when the output rows allow them (the same for every lane), single elements otherwise
        const bool vec = ((((uintptr_t)C) | (uintptr_t)(ldc * 4)) & 15u) == 0 && (g.N & 3) == 0;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = r0 + mi * 32 + (lane % 32);
            const bool row_ok = row < g.M;
            float *crow = C + (int64_t)(row_ok ? row : 0) * ldc + c0;
            const float sc = (row_ok && row_scale) ? row_scale[row] : 1.0f;
            const float co = (row_ok && row_coef) ? row_coef[row] : 0.0f;
            const uint16_t *srow = co != 0.0f ? src + ids[row] * ld_src + c0 : nullptr;
            // accumulate: fetch the block's old values first, all loads in flight together
            f32x4 old[NI][4];
            if (accumulate) {
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int colb = ni * 32 + q * 8 + half * 4;
                        old[ni][q] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
                        if (!row_ok || c0 + colb >= g.N) continue;
                        if (vec) old[ni][q] = *(const f32x4 *)(crow + colb);
                        else {
#pragma unroll
                            for (int e = 0; e < 4; ++e) old[ni][q][e] = c0 + colb + e < g.N ? crow[colb + e] : 0.0f;
                        }
                    }
                }
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int colb = ni * 32 + q * 8 + half * 4;
                    if (!row_ok || c0 + colb >= g.N) continue;
                    f32x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        v[e] = sc * acc[mi][ni][q * 4 + e];
                        if (srow && c0 + colb + e < g.N) v[e] += co * __uint_as_float((uint32_t)srow[colb + e] << 16);
                        if (accumulate) v[e] += old[ni][q][e];
                    }
                    if (vec) *(f32x4 *)(crow + colb) = v;
                    else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (c0 + colb + e < g.N) crow[colb + e] = v[e];
                    }
                }
            }
        }
    }
};

// ---------------------------------------------------------------------------
// C = A B^T on MFMA.  256x256 tile per workgroup, K in steps of 64.
//
// Operand tiles go from global memory straight into LDS (16 bytes per lane,
// no register staging): a wavefront copy lands as 1 KB of consecutive LDS, so
// the lane -> global address map carries the row swizzle.  The copies are
// invisible to the compiler's wait-count bookkeeping; the loop waits for them
// explicitly, always together with the workgroup barrier.
//
// Two LDS stages.  The barrier of a K step sits between the LDS reads of the
// step's last 16-wide slice and that slice's MFMAs: past it, tile j+1 has
// landed and tile j is dead in every wavefront, so the copy of tile j+2 is
// issued into tile j's buffer and the first fragments of tile j+1 are fetched
// while the matrix cores still have the last slice of tile j to do.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void wait_copies_and_barrier()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// copy16_to_lds with the base address forced into scalar registers: it is wavefront-uniform by construction (tile
// bases and K steps), and saying so keeps it there in builds where the compiler's own analysis loses track of that
__device__ __forceinline__ void copy16_uniform(const void *gbase, uint32_t voff, uint32_t lds_addr)
{
    const uint64_t b = (uint64_t)(uintptr_t)gbase;
    const uint64_t ub = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                        (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
    copy16_to_lds((const void *)(uintptr_t)ub, voff, lds_addr);
}

// scheduling hint for a slice with more LDS reads than matrix instructions: after instruction i, its share of the reads
template <int NM, int NR, int... I>
__device__ __forceinline__ void spread_reads(std::integer_sequence<int, I...>)
{
    ((__builtin_amdgcn_sched_group_barrier(0x008, 1, 0),
      __builtin_amdgcn_sched_group_barrier(0x100, NR * (I + 1) / NM - NR * I / NM, 0)), ...);
}

// where a workgroup's tile sits and how its lanes address the operand rows
struct TilePlace {
    const uint8_t *baseA, *baseB;                        // first row of the A tile / B tile
    uint32_t off_a[kCopiesPerWave], off_b[kCopiesPerWave];   // per-lane byte offsets of the wavefront copies
    int tile_m, tile_n;
};

// Persistent: the grid has one workgroup per CU and each walks its share of the tiles.  The first two
// K steps of the next tile are copied under the last two K steps of the current one (no epilogue touches
// the tile buffers), so only the epilogue itself separates the MFMA streams of two tiles.
//
// F8: both operands are E4M3 bytes and the products run on the 64-deep 8-bit matrix instruction, whose
// operands are 32 bytes per lane: a K step (128 bytes of every row) is two instructions deep instead of
// four.  Lane l takes the 32 bytes (two swizzled 16-byte chunks) 4 * pair + 2 * (l / 32) of its row, of A
// and of B alike, so both operands present the same k to the same position of the instruction.
//
// ATR / BTR: the operand lies in memory as [K, ld], its M (N) index contiguous, and is NOT transposed beforehand:
// its tile goes into LDS as 64 rows of k, 512 bytes (256 m) each, and the fragments are fetched with the
// transposing LDS read of this chip (ds_read_b64_tr_b16: among 16 lanes, lane i receives element i % 4 of the 8
// bytes that lanes i / 4, 4 + i / 4, 8 + i / 4, 12 + i / 4 point at).  Lanes 4 e + j of a group of 16 point at row
// k0 + e, columns m0 + 4 j .. + 3, so lane i ends up with column m0 + i of rows k0 .. k0 + 3: two such reads are the
// eight consecutive k the matrix instruction wants from that lane.  A read touches 8 rows of k, 64 bytes each;
// rows are 512 bytes apart (the same banks), so the 16-byte chunks of row k sit at position chunk ^ 4 (k & 3):
// 165 B/clk per CU measured in this pattern against 63 unswizzled; a K step's fragments take 1200 cycles, under
// the 2048 of its matrix instructions.
template <class Epi, bool NEEDS_FINISH, bool F8, bool ATR = false, bool BTR = false>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_nt_kernel(const GemmArgs g_host, const Epi epi, int tiles_m, int tiles_n)
{
    static_assert(!(F8 && (ATR || BTR)), "8-bit operands are K-major");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];   // [stage][A | B][256 rows][128 B], then sums scratch

    GemmArgs g = g_host;
    if constexpr (Epi::kRowMap) {       // the row count comes from an earlier kernel; the grid was sized for g_host.M
        g.M = *epi.n_sub;
        tiles_m = (g.M + BM - 1) / BM;
        if ((int)blockIdx.x >= tiles_m * tiles_n) return;
    }
    if (g_host.dev_dim == 1) {
        g.M = rows_on_device(g_host.n_dev, g_host.n_off, g_host.M);
        tiles_m = (g.M + BM - 1) / BM;
        if ((int)blockIdx.x >= tiles_m * tiles_n) return;
    } else if (g_host.dev_dim == 2) {
        g.K = (rows_on_device(g_host.n_dev, g_host.n_off, g_host.K) + BM - 1) / BM * BM;
        if (g.K == 0) return;           // (only launched with an accumulating epilogue: nothing to add)
    }
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave), lane = tid % kWave;
    const int wm = wave / WN, wn = wave % WN;
    const int total = tiles_m * tiles_n;

    // Tile order.  Hardware deals workgroups round-robin to the 8 XCDs and the grid is a multiple of
    // 8 (or smaller than the tile count is not: then it equals it), so launch position t always runs
    // on XCD t % 8.  Each XCD gets a contiguous range of the walk below, so that the 32 workgroups
    // resident on it cover 4 row tiles x 8 column tiles and share operand tiles in its L2.
    // global -> LDS: copy c of a tile (c = i * 8 + wave) fills LDS chunks 64 c .. 64 c + 63, i.e. tile
    // rows 8 c .. 8 c + 7; the chunk at physical position p of row r holds logical chunk p ^ ((r >> 1) & 7).
    // (LDS has 64 four-byte banks here and a 16-byte read is served 16 lanes at a time: sixteen consecutive
    // rows of 128 bytes must put their chunks on 16 different bank groups, two rows per 256 bytes, hence the
    // key from r >> 1.  Measured with ds_read_b128 in this access pattern: 221 B/clk per CU with this key,
    // 125 B/clk with r & 7 (two-way conflicts), 32 B/clk with none.)
    auto place = [&](int t, TilePlace &tp) {
        const int per_xcd = total / 8;
        int pid = t;
        if (pid < per_xcd * 8) pid = (pid % 8) * per_xcd + pid / 8;
        constexpr int GROUP = 4;
        const int per_group = GROUP * tiles_n;
        const int group = pid / per_group;
        const int first_m = group * GROUP;
        const int group_rows = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
        const int in_group = pid - group * per_group;
        tp.tile_m = first_m + in_group % group_rows;
        tp.tile_n = in_group / group_rows;
        tp.baseA = (const uint8_t *)(ATR ? g.A + (int64_t)tp.tile_m * (g.a_panel > 0 ? g.a_panel : (int64_t)BM)
                                         : g.A + (int64_t)tp.tile_m * BM * g.lda);
        tp.baseB = (const uint8_t *)(BTR ? g.B + (int64_t)tp.tile_n * BN : g.B + (int64_t)tp.tile_n * BN * g.ldb);
        const int rows_a = g.M - tp.tile_m * BM, rows_b = g.N - tp.tile_n * BN;   // >= 1; rows past the end repeat the last one
        // [K, ld] operands: columns the row still has from the tile's first one (pieces past them repeat the last piece)
        const int cols_a = g.a_panel > 0 ? BM : (int)((g.a_cols > 0 ? g.a_cols : g.lda) - (int64_t)tp.tile_m * BM);
        const int cols_b = (int)((g.b_cols > 0 ? g.b_cols : g.ldb) - (int64_t)tp.tile_n * BN);
#pragma unroll
        for (int i = 0; i < kCopiesPerWave; ++i) {
            const int p = (i * kGemmWaves + wave) * kWave + lane;
            const int row = p >> 3, kc = (p & 7) ^ ((row >> 1) & 7);
            const int ra = row < rows_a ? row : rows_a - 1;
            const int rb = row < rows_b ? row : rows_b - 1;
            // [K, ld] operands: a wavefront copy is two rows of k; lane -> (k, physical chunk), logical chunk = physical ^ 4 (k & 3).
            // Copy i of a wavefront lies 16 i rows of k below its copy 0, same columns: only off[0] is used, the rest
            // of the way is a step of the wavefront's base address.
            const int tk = p >> 5, tc = ((p & 31) ^ (4 * (tk & 3))) * 8;
            const int ca = tc + 8 <= cols_a ? tc : cols_a - 8, cb = tc + 8 <= cols_b ? tc : cols_b - 8;
            tp.off_a[i] = ATR ? (uint32_t)(((int64_t)tk * g.lda + ca) * 2) : (uint32_t)(((int64_t)ra * g.lda + kc * 8) * 2);
            tp.off_b[i] = BTR ? (uint32_t)(((int64_t)tk * g.ldb + cb) * 2) : (uint32_t)(((int64_t)rb * g.ldb + kc * 8) * 2);
        }
    };
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;
    // rows of k a [K, ld] operand has in memory (K itself when the caller says nothing)
    const int kb_rows = g.kb_rows > 0 ? g.kb_rows : g.K;
    constexpr bool kPanels = ATR || BTR;             // only the gradient products take an A stored in panels
    constexpr int kTrCopyRows = 2 * kGemmWaves;      // rows of k between a wavefront's successive copies of a [K, ld] tile
    auto issue_copies = [&](const TilePlace &tp, int kt, int stage) {
        const uint8_t *pa = tp.baseA + (ATR ? (size_t)kt * BK * (size_t)g.lda * 2
                                            : kPanels && g.a_panel > 0 ? (size_t)(kt / (BM / BK)) * (size_t)g.a_panel * 2 + (size_t)(kt % (BM / BK)) * kRowBytes
                                                                       : (size_t)kt * kRowBytes);
        const uint8_t *pb = tp.baseB + (BTR ? (size_t)kt * BK * (size_t)g.ldb * 2 : (size_t)kt * kRowBytes);
        const uint32_t sa = lds_base + stage * kStageBytes;
#pragma unroll
        for (int i = 0; i < kCopiesPerWave; ++i) {
            if constexpr (ATR) copy16_uniform(pa + (size_t)i * kTrCopyRows * (size_t)g.lda * 2, tp.off_a[0], sa + (i * kGemmWaves + wave) * 1024);
            else               copy16_uniform(pa, tp.off_a[i], sa + (i * kGemmWaves + wave) * 1024);
        }
        // A [K, ld] B operand whose rows of k end inside or before this step: the rows past the end repeat the last one.
        // (`last` is that row relative to the step; when the whole step lies past it the base moves back to it, so that
        // the per-lane offsets, which are unsigned, never have to go below zero: a lane's row is 16 i + its row of copy 0,
        // it goes back by at most that.)
        if (BTR && (kt + 1) * BK > kb_rows) {
            const int last = kb_rows - 1 - kt * BK, lim = last < 0 ? 0 : last;
            const uint8_t *pb2 = last < 0 ? pb + (int64_t)last * g.ldb * 2 : pb;
            const int tk0 = (wave * kWave + lane) >> 5;
#pragma unroll
            for (int i = 0; i < kCopiesPerWave; ++i) {
                const int tk = tk0 + i * kTrCopyRows;
                const int row = tk > lim ? lim : tk;
                copy16_uniform(pb2, tp.off_b[0] + (uint32_t)(row - tk0) * (uint32_t)(g.ldb * 2), sa + kTileBytes + (i * kGemmWaves + wave) * 1024);
            }
        } else {
#pragma unroll
            for (int i = 0; i < kCopiesPerWave; ++i) {
                if constexpr (BTR) copy16_uniform(pb + (size_t)i * kTrCopyRows * (size_t)g.ldb * 2, tp.off_b[0], sa + kTileBytes + (i * kGemmWaves + wave) * 1024);
                else               copy16_uniform(pb, tp.off_b[i], sa + kTileBytes + (i * kGemmWaves + wave) * 1024);
            }
        }
    };

    // operand fetch: lane l reads row (l % 32), the 8 consecutive k of chunk 2 * ks + l / 32.
    // Rows 32 apart share (row >> 1) & 7, so one swizzle key serves all row blocks.
    const int frow = lane % 32, half = lane / 32, key = (frow >> 1) & 7;
    const int a_off = (wm * MI * 32 + frow) * kRowBytes;
    const int b_off = kTileBytes + (wn * NI * 32 + frow) * kRowBytes;
    // [K, ld] operands: this lane of its group of 16 points at row 8 (lane / 32) + (lane % 16) / 4 of a 16-deep slice,
    // columns 32 blk + 16 ((lane / 16) % 2) + 4 (lane % 4) .. + 3; the second read of a fragment is 4 rows further
    constexpr int kTrRowBytes = BM * 2;          // one row of k in LDS: 256 m
    int tr_a[MI], tr_b[NI];
    {
        const int e = (lane % 16) / 4, j = lane % 4, g2 = (lane / 16) % 2;
        const int row = 8 * half + e;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int chunk = (4 * (wm * MI + mi) + 2 * g2 + j / 2) ^ (4 * e);
            tr_a[mi] = row * kTrRowBytes + chunk * 16 + (j % 2) * 8;
        }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int chunk = (4 * (wn * NI + ni) + 2 * g2 + j / 2) ^ (4 * e);
            tr_b[ni] = row * kTrRowBytes + chunk * 16 + (j % 2) * 8;
        }
    }
    auto fetch_tr = [&](uint32_t lds_addr) {     // two transposing reads, 4 rows of k apart: eight consecutive k of this lane's column
        typedef short v4i16 __attribute__((ext_vector_type(4)));
        typedef short v8i16 __attribute__((ext_vector_type(8)));
        typedef v4i16 __attribute__((address_space(3))) *lds_v4;
        const v4i16 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)lds_addr);
        const v4i16 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(uintptr_t)(lds_addr + 4 * kTrRowBytes));
        const v8i16 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, both);
    };
    f32x16 acc[MI][NI];
    bf16x8 fa[2][MI], fb[2][NI];
    i32x8 fa8[2][MI], fb8[2][NI];       // F8 only
    auto fetch = [&](int buf, int stage, int ks) {
        const uint8_t *sb = lds + stage * kStageBytes;
        if constexpr (F8) {             // ks counts 64-deep pairs here: 0 or 1
            const int c0 = ((ks * 4 + half * 2) ^ key) * 16, c1 = ((ks * 4 + half * 2 + 1) ^ key) * 16;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const i32x4 lo = *(const i32x4 *)(sb + a_off + mi * 32 * kRowBytes + c0);
                const i32x4 hi = *(const i32x4 *)(sb + a_off + mi * 32 * kRowBytes + c1);
                fa8[buf][mi] = (i32x8){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const i32x4 lo = *(const i32x4 *)(sb + b_off + ni * 32 * kRowBytes + c0);
                const i32x4 hi = *(const i32x4 *)(sb + b_off + ni * 32 * kRowBytes + c1);
                fb8[buf][ni] = (i32x8){lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
            }
        } else {
            const int chunk = ((ks * 2 + half) ^ key) * 16;
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                if constexpr (ATR) fa[buf][mi] = fetch_tr(lds_base + stage * kStageBytes + tr_a[mi] + ks * 16 * kTrRowBytes);
                else               fa[buf][mi] = *(const bf16x8 *)(sb + a_off + mi * 32 * kRowBytes + chunk);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                if constexpr (BTR) fb[buf][ni] = fetch_tr(lds_base + stage * kStageBytes + kTileBytes + tr_b[ni] + ks * 16 * kTrRowBytes);
                else               fb[buf][ni] = *(const bf16x8 *)(sb + b_off + ni * 32 * kRowBytes + chunk);
            }
        }
    };
    auto multiply = [&](int buf) {
        if constexpr (F8) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)   // formats 0, 0: E4M3 x E4M3; zero scale operands: the unscaled instruction
                    acc[mi][ni] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb8[buf][ni], fa8[buf][mi], acc[mi][ni], 0, 0, 0, 0, 0, 0);
            // twelve 16-byte LDS reads of the next pair between these eight MFMAs
#pragma unroll
            for (int i = 0; i < MI * NI / 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
#pragma unroll
            for (int i = 0; i < MI * NI / 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            return;
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                // B first: the lane then owns an output row (both operands have the same lane layout, 32 rows x 8 k per half)
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][ni], fa[buf][mi], acc[mi][ni], 0, 0, 0);
        // scheduling hint: spread the LDS reads of the next slice between this slice's MFMAs
        constexpr int NM = MI * NI, NR = (ATR ? 2 : 1) * MI + (BTR ? 2 : 1) * NI;
        if constexpr (NR == NM) {      // two reads behind each of the first half of the instructions: every fragment is
#pragma unroll                          // asked for at least half a slice before it is used
            for (int i = 0; i < NM / 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, NM / 2, 0);
        } else if constexpr (NR < NM) {
            constexpr int PER = NM / NR;
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, PER, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            if constexpr (NM - PER * NR > 0) __builtin_amdgcn_sched_group_barrier(0x008, NM - PER * NR, 0);
        } else {
            spread_reads<NM, NR>(std::make_integer_sequence<int, NM>());
        }
    };

    const int nk = g.K / BK;
    const bool chain = nk >= 2;
    int t = blockIdx.x;                 // < total: the launcher never starts more workgroups than tiles
    int sp = 0;                         // LDS stage that holds K step 0 of the current tile
    TilePlace cur, nxt;
    place(t, cur);
    issue_copies(cur, 0, 0);
    wait_copies_and_barrier();
    if (nk > 1) issue_copies(cur, 1, 1);
    fetch(0, 0, 0);
    for (;;) {
        const int t_next = t + (int)gridDim.x;
        const bool has_next = t_next < total;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[mi][ni][i] = 0.0f;

        // one K step; `issue_next` starts the copies that may overwrite the stage this step has just finished with
        auto k_step = [&](int j, auto &&issue_next) {
            const int stage = (sp + j) & 1;
            if constexpr (F8) {
                fetch(1, stage, 1); multiply(0);
            } else {
                fetch(1, stage, 1); multiply(0);
                fetch(0, stage, 2); multiply(1);
                fetch(1, stage, 3); multiply(0);
            }
            // own reads of K step j are home, own copies of step j+1 have landed; past the
            // barrier that holds for every wavefront
            wait_copies_and_barrier();
            issue_next(stage);
            fetch(0, stage ^ 1, 0);         // step j+1, or step 0 of the next tile; unused (dead buffer) otherwise
            multiply(1);
        };
        int j = 0;
        for (; j + 2 < nk; ++j) k_step(j, [&](int stage) { issue_copies(cur, j + 2, stage); });
        // The last two steps copy the first two of the next tile.  Its placement is formed here and not before the
        // loop: its per-lane offsets would otherwise occupy registers through the whole loop (with them the builds
        // that take an operand as it lies spilled one and reloaded it inside the loop).
        if (has_next) place(t_next, nxt);
        for (; j < nk; ++j) k_step(j, [&](int stage) { if (chain && has_next) issue_copies(nxt, j + 2 - nk, stage); });

        if constexpr (F8) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[mi][ni][i] *= g.scale;
        }
        // every wavefront is past the tile's last barrier and its last useful fetch
        epi(g, acc, cur.tile_m * BM + wm * (MI * 32), cur.tile_n * BN + wn * (NI * 32), lane, lds, wave, wn);
        if constexpr (NEEDS_FINISH) {
            __syncthreads();
            epi.finish(g, cur.tile_m * BM, cur.tile_n, lds, tid);
        }
        if (!has_next) break;
        sp = (sp + nk) & 1;
        if (!chain) {
            __syncthreads();                // the tile buffers are free again in every wavefront
            issue_copies(nxt, 0, sp);
            wait_copies_and_barrier();
            if (nk > 1) issue_copies(nxt, 1, sp ^ 1);
            fetch(0, sp, 0);
        }
        cur = nxt;
        t = t_next;
    }
}

static std::atomic<int> g_gemm_cus{0};   // callers may come from several host threads
static hipError_t prepare_gemm_cu_count()
{
    int dev = 0, n = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess && n > 0) g_gemm_cus.store(n, std::memory_order_relaxed);
    return e;
}
static PrepareRegistrar g_gemm_cus_registrar(&prepare_gemm_cu_count);
static int gemm_cu_count()
{
    if (g_gemm_cus.load(std::memory_order_relaxed) == 0 && prepare_gemm_cu_count() != hipSuccess) return 256;
    const int n = g_gemm_cus.load(std::memory_order_relaxed);
    return n > 0 ? n : 256;
}

// More than 64 KB of LDS per workgroup has to be asked for, once per kernel and device (bit d of
// `configured`: device d has it).
template <class Epi, bool NEEDS_FINISH, bool F8, bool ATR = false, bool BTR = false>
struct GemmBuild {
    static inline std::atomic<uint64_t> configured{0};
    static hipError_t prepare()
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void *)gemm_nt_kernel<Epi, NEEDS_FINISH, F8, ATR, BTR>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLdsBytes);
        if (e == hipSuccess && dev < 64) configured.fetch_or(1ull << dev, std::memory_order_release);
        return e;
    }
    static inline PrepareRegistrar registrar{&prepare};
};

template <class Epi, bool NEEDS_FINISH, bool F8 = false, bool ATR = false, bool BTR = false>
static hipError_t launch_gemm(const GemmArgs &g, const Epi &epi, hipStream_t stream)
{
    typedef GemmBuild<Epi, NEEDS_FINISH, F8, ATR, BTR> Build;
    (void)&Build::registrar;             // instantiates the registration of this build
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev > 63 || !(Build::configured.load(std::memory_order_acquire) & (1ull << dev))) {
        e = Build::prepare();
        if (e != hipSuccess) return e;
    }
    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    const int total = tiles_m * tiles_n;
    int grid = gemm_cu_count() / 8 * 8;     // one workgroup per CU; a multiple of the XCD count
    if (grid < 8) grid = 8;
    if (grid > total) grid = total;
    if (g.a_panel > 0 && !(ATR || BTR)) return hipErrorInvalidValue;   // the other builds do not read a_panel
    hipLaunchKernelGGL((gemm_nt_kernel<Epi, NEEDS_FINISH, F8, ATR, BTR>), dim3((unsigned)grid), dim3(kGemmThreads),
                       kGemmLdsBytes, stream, g, epi, tiles_m, tiles_n);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// small helper kernels
// ---------------------------------------------------------------------------
__global__ void init_stats_kernel(RowStats st, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { st.max_key[i] = (int)0x80000000; st.zy[i] = 0.0f; }
}

__global__ void after_max_kernel(RowStats st, int n, float log_rho)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const float m = ordered_to_float(st.max_key[i]);
        st.m[i] = m;
        st.tau[i] = m + log_rho;                  // one fp32 rounding
    }
}

// A row's outputs and gradient factors from its sums over the safe set (s), over all tokens (f) and its
// safe-set size (c).  i indexes m and tau, w everything else (they differ for a gathered subset of rows).
__device__ __forceinline__ void finish_row(const RowStats &st, const SideOut &out, const int64_t *ids, const float *grad_out,
                                           uint8_t *row_flags, int i, int w, int vocab, int side, int unit_grad, float s,
                                           float f, int c)
{
    const float m = st.m[i], tau = st.tau[i];
    const float log_s = logf(s);
    const int64_t y = ids[w];
    const bool y_ok = y >= 0 && y < (int64_t)vocab;
    const float zy = st.zy[w];
    const bool y_safe = y_ok && zy >= tau;
    if (side == 0) {
        // unit_grad: the factors of a gradient still to come, q / g and s / g (Prop. 5.4 is linear in g)
        const float c_i = !y_safe ? 0.0f : (unit_grad ? 1.0f : (grad_out ? grad_out[w] : 0.0f));
        st.coef[w] = c_i != 0.0f ? c_i * (1.0f - __expf(zy - m) / s) : 0.0f;
        st.scale[w] = -c_i / s;
    }
    if (out.row_max) out.row_max[w] = m;
    if (out.lse_safe) out.lse_safe[w] = m + log_s;
    if (out.lse_full) out.lse_full[w] = m + logf(f);
    if (out.safe_count) out.safe_count[w] = c;
    if (out.logp)
        out.logp[w] = !y_ok ? __uint_as_float(0x7fc00000u) : (y_safe ? (zy - m) - log_s : -INFINITY);
    if (row_flags) {
        uint32_t fl = side == 0 ? (y_ok ? 0u : (uint32_t)DVP_ROW_ID_OUT_OF_RANGE) : row_flags[w];
        if (y_safe) fl |= side == 0 ? DVP_ROW_Y_IN_TRAIN_SAFE : DVP_ROW_Y_IN_INFER_SAFE;
        row_flags[w] = (uint8_t)fl;
    }
}

// The statistics at the threshold from a row block's stored logits (Def. 5.1 / 5.2), one workgroup per
// token row, one streaming pass: safe-set size, masked sum (and the full sum when lse_full is wanted),
// the side's outputs and the gradient factors; WRITE_E also stores the row's masked exponentials
// E_ik = [z_ik >= tau_i] exp(z_ik - m_i) as bf16 with a zero at the sampled token's column and zeros in
// the padding columns (they pad the K dimension of the dH product), in panels of 256 columns so that both
// gradient products find their tiles in compact memory (a row's 512 bytes of a panel are one run of a
// wavefront's store); WRITE_BITS the membership bitmask.
// Every thread owns fixed columns and the partial sums are combined in a fixed order: run-to-run identical.
constexpr int kZRowThreads = 512;
struct ZRowArgs {
    const float *Z;          // [rows, ldz] fp32 logits of the block
    int64_t ldz;
    RowStats st;             // m, tau, zy of the block's rows (index 0 = first row of the block)
    SideOut out;             // output pointers, already offset to the block's first row
    const int64_t *ids;
    const float *grad_out;
    uint8_t *row_flags;
    uint16_t *E;             // WRITE_E: bf16 [rows, v_pad] in panels of 256 columns, e_panel elements each (see GemmArgs)
    int64_t e_panel;
    uint32_t *bits;          // WRITE_BITS: [rows, bits_ld]
    int64_t bits_ld;
    int vocab, v_pad, side, unit_grad;
    const int *n_dev;        // see GemmArgs: the launch is sized for an upper bound of the rows
    int n_off, rows;
};

template <bool WRITE_E, bool WRITE_BITS>
__global__ __launch_bounds__(kZRowThreads) void lm_rows_from_z_kernel(const ZRowArgs a)
{
    constexpr int NW = kZRowThreads / kWave;
    __shared__ float lds_f[2 * NW];
    __shared__ int lds_i[NW];
    const int i = blockIdx.x, tid = threadIdx.x;
    const int rows = rows_on_device(a.n_dev, a.n_off, a.rows);
    if (i >= rows) {
        // WRITE_E launches cover the rows up to the next whole row tile: those rows of E are zeros (they pad the K
        // dimension of the dW product)
        if constexpr (WRITE_E) {
            if (i < (rows + BM - 1) / BM * BM) {
                const u32x4 zero = {0u, 0u, 0u, 0u};
                for (int u = tid; u < a.v_pad / 8; u += kZRowThreads)
                    __builtin_nontemporal_store(zero, (u32x4 *)(a.E + (int64_t)(u * 8 / BM) * a.e_panel + (int64_t)i * BM + u * 8 % BM));
            }
        }
        return;
    }
    const float m = a.st.m[i], tau = a.st.tau[i];
    const bool want_full = a.out.lse_full != nullptr;
    int64_t y = -1;
    if constexpr (WRITE_E) y = a.ids[i];
    const u32x4 *zrow = (const u32x4 *)(a.Z + (int64_t)i * a.ldz);
    const int units = a.v_pad / 8;              // 8 columns at a time: two 16-byte loads, one 16-byte store
    RowSums acc = {0.0f, 0.0f, 0};
#pragma unroll 2
    for (int u = tid; u < units; u += kZRowThreads) {
        const u32x4 lo = zrow[2 * u], hi = zrow[2 * u + 1];
        const float x[8] = {__uint_as_float(lo.x), __uint_as_float(lo.y), __uint_as_float(lo.z), __uint_as_float(lo.w),
                            __uint_as_float(hi.x), __uint_as_float(hi.y), __uint_as_float(hi.z), __uint_as_float(hi.w)};
        const int col0 = u * 8;
        float e[8];
        uint32_t mask = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const bool in = col0 + k < a.vocab;   // the padding columns of Z hold nothing
            const bool safe = in && x[k] >= tau;
            float kept = 0.0f;
            if (want_full) {
                const float ex = in ? __expf(x[k] - m) : 0.0f;
                acc.s_full += ex;
                kept = safe ? ex : 0.0f;
            } else if (safe) {
                kept = __expf(x[k] - m);
            }
            acc.s_safe += kept;
            acc.count += safe ? 1 : 0;
            mask |= (safe ? 1u : 0u) << k;
            e[k] = (int64_t)(col0 + k) == y ? 0.0f : kept;
        }
        if constexpr (WRITE_E) {
            const u32x4 v = {pack_bf16x2(e[0], e[1]), pack_bf16x2(e[2], e[3]), pack_bf16x2(e[4], e[5]), pack_bf16x2(e[6], e[7])};
            __builtin_nontemporal_store(v, (u32x4 *)(a.E + (int64_t)(col0 / BM) * a.e_panel + (int64_t)i * BM + col0 % BM));
        }
        if constexpr (WRITE_BITS) {
            if (u < 4 * a.bits_ld) ((uint8_t *)(a.bits + (int64_t)i * a.bits_ld))[u] = (uint8_t)mask;
        }
    }
    acc = block_sums<kZRowThreads>(acc, lds_f, lds_i);
    if (tid == 0)
        finish_row(a.st, a.out, a.ids, a.grad_out, a.row_flags, i, i, a.vocab, a.side, a.unit_grad, acc.s_safe, acc.s_full,
                   acc.count);
}

// Reduce the per-tile partials and write the side's outputs.  A workgroup takes 32 rows; the
// column tiles are cut into 8 contiguous segments, each summed in tile order by one thread per
// row, and the 8 segment sums are combined in segment order: a fixed order, run-to-run identical.
constexpr int kAfterRows = 32, kAfterSegs = 8;
__global__ __launch_bounds__(kAfterRows * kAfterSegs) void after_sum_kernel(RowStats st, SideOut out, const int64_t *ids,
                                                                            const float *grad_out, uint8_t *row_flags,
                                                                            int n, int vocab, int col_tiles, int side,
                                                                            int unit_grad, const int *rowmap, const int *n_sub)
{
    // rowmap / n_sub: see EpiSum's ROWMAP; n stays the stride of the partials
    const int n_rows = n_sub ? *n_sub : n;
    if ((int)blockIdx.x * kAfterRows >= n_rows) return;
    __shared__ float seg_s[kAfterSegs][kAfterRows], seg_f[kAfterSegs][kAfterRows];
    __shared__ int seg_c[kAfterSegs][kAfterRows];
    const int r = threadIdx.x % kAfterRows, seg = threadIdx.x / kAfterRows;
    const int i = blockIdx.x * kAfterRows + r;
    const int per = (col_tiles + kAfterSegs - 1) / kAfterSegs;
    const int t0 = seg * per, t1 = (t0 + per) < col_tiles ? (t0 + per) : col_tiles;
    float s = 0.0f, f = 0.0f;
    int c = 0;
    if (i < n_rows) {
        for (int t = t0; t < t1; ++t) {
            const int64_t o = (int64_t)t * n + i;
            s += st.part_s[o];
            c += st.part_c[o];
            if (st.part_f) f += st.part_f[o];
        }
    }
    seg_s[seg][r] = s; seg_f[seg][r] = f; seg_c[seg][r] = c;
    __syncthreads();
    if (seg != 0 || i >= n_rows) return;
#pragma unroll
    for (int q = 1; q < kAfterSegs; ++q) { s += seg_s[q][r]; f += seg_f[q][r]; c += seg_c[q][r]; }
    finish_row(st, out, ids, grad_out, row_flags, i, rowmap ? rowmap[i] : i, vocab, side, unit_grad, s, f, c);
}

// Sampled-token part of dW (Prop. 5.4): dW[y_i, :] += q_i H_i for the `rows` token rows of a block, in
// fp32 and in row order whatever the launch order (run-to-run identical).  One workgroup per token
// row; the first row of the launch that sampled a token adds the contributions of every row of the
// launch that sampled it; a block of rows is covered by successive launches of kOnehotRows rows.  Runs
// after the block's E^T product has been written to dW.
constexpr int kOnehotThreads = 256;
constexpr int kOnehotRows = 4096;       // rows per launch: every workgroup scans its launch's sampled tokens
// tokens[r] = the sampled token of row r as a 32-bit integer, -1 where the row contributes nothing (coef 0): what
// every workgroup of onehot_dw_kernel scans, a third of the bytes of the ids and factors themselves
__global__ void onehot_tokens_kernel(const int64_t *ids, const float *coef, int *tokens, int rows)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r < rows) tokens[r] = coef[r] != 0.0f ? (int)ids[r] : -1;
}

__global__ __launch_bounds__(kOnehotThreads) void onehot_dw_kernel(const int *tokens, const float *coef, const uint16_t *H,
                                                                   int64_t ld_h, float *dW, int64_t ld_w, int rows, int d,
                                                                   const int *n_dev = nullptr, int n_off = 0)
{
    rows = rows_on_device(n_dev, n_off, rows);
    if ((int)blockIdx.x >= rows) return;
    __shared__ int tok[kOnehotRows];    // sampled token per row, -1 where the row contributes nothing
    __shared__ uint16_t match[kOnehotRows];   // rows that sampled this workgroup's token, ascending
    __shared__ int n_match;
    const int i = blockIdx.x, tid = threadIdx.x;
    for (int r = tid; r < rows; r += kOnehotThreads) tok[r] = tokens[r];
    __syncthreads();
    const int y = tok[i];
    if (y < 0) return;
    int earlier = 0;
    for (int r = tid; r < i; r += kOnehotThreads) earlier |= tok[r] == y;
    if (__syncthreads_or(earlier)) return;
    if (tid < kWave) {                  // first wavefront: ordered list of the matching rows
        int count = 0;
        for (int base = i; base < rows; base += kWave) {
            const int r = base + tid;
            const bool hit = r < rows && tok[r] == y;
            const unsigned long long bal = __builtin_amdgcn_ballot_w64(hit);
            if (hit) match[count + (int)__builtin_popcountll(bal & ((1ull << tid) - 1ull))] = (uint16_t)r;
            count += (int)__builtin_popcountll(bal);
        }
        if (tid == 0) n_match = count;
    }
    __syncthreads();
    const int nm = n_match;
    float *wrow = dW + (int64_t)y * ld_w;
    // Four columns per thread where the rows of dW allow 16-byte accesses (the rows of H always allow 8-byte ones: the
    // entry points check its alignment and pitch): a few wide, independent accesses per thread instead of d / 256
    // narrow ones in a row, each waiting for the one before.  Per element the sums are formed in the same order.
    if (((((uintptr_t)dW) | (uintptr_t)(ld_w * 4)) & 15u) == 0 && (d & 3) == 0) {
#pragma unroll 4
        for (int u = tid; u < d / 4; u += kOnehotThreads) {
            f32x4 a = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int q = 0; q < nm; ++q) {
                const int r = match[q];
                const float c = coef[r];
                const uint2 h = *(const uint2 *)(H + (int64_t)r * ld_h + 4 * u);
                a[0] += c * __uint_as_float(h.x << 16);
                a[1] += c * __uint_as_float(h.x & 0xffff0000u);
                a[2] += c * __uint_as_float(h.y << 16);
                a[3] += c * __uint_as_float(h.y & 0xffff0000u);
            }
            f32x4 *p = (f32x4 *)(wrow + 4 * u);
            *p = *p + a;
        }
        return;
    }
    for (int j = tid; j < d; j += kOnehotThreads) {
        float a = 0.0f;
        for (int q = 0; q < nm; ++q) {
            const int r = match[q];
            a += coef[r] * __uint_as_float((uint32_t)H[(int64_t)r * ld_h + j] << 16);
        }
        wrow[j] += a;
    }
}

// out[c, r] = bf16(scale[r] * in[r, c]) (scale null: a plain copy) for r < rows, c < cols;
// out rows are ld_out long and zero padded up to rows_pad.  64 x 64 tiles, 16-byte accesses on both
// sides: cols and ld_in are multiples of 8 (cols of 64), rows_pad and ld_out multiples of 64.
// The tile is transposed on its way INTO LDS (two-byte writes, pitch 66 halfwords: two lanes per bank),
// so that on the way out eight neighbouring lanes hold the 128 bytes of one output row and a wavefront's
// store covers eight whole lines (written as 64 separate 16-byte pieces per store, the output ran at
// 3.2 TB/s for read plus write).
constexpr int kTrTile = 64, kTrThreads = 256, kTrPitch = kTrTile + 2;
// n_dev non-null: the rows are rows n_off .. of *n_dev in all (see GemmArgs); rows and rows_pad are then upper
// bounds and the padding ends at the next whole row tile.
__global__ __launch_bounds__(kTrThreads) void transpose_bf16_kernel(const uint16_t *in, int64_t ld_in, uint16_t *out,
                                                                    int64_t ld_out, int rows, int cols, int rows_pad,
                                                                    const float *scale, const int *n_dev = nullptr, int n_off = 0)
{
    if (n_dev) {
        rows = rows_on_device(n_dev, n_off, rows);
        rows_pad = (rows + BM - 1) / BM * BM;
    }
    __shared__ __attribute__((aligned(16))) uint16_t tile[kTrTile * kTrPitch];   // tile[c][r]
    const int r0 = blockIdx.y * kTrTile, c0 = blockIdx.x * kTrTile;
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < kTrTile * 8 / kTrThreads; ++k) {
        const int p = tid + k * kTrThreads, r = p >> 3, ch = p & 7;
        const int row = r0 + r;
        uint32_t w[4] = {0u, 0u, 0u, 0u};
        if (row < rows && c0 + ch * 8 < cols) {
            const u32x4 v = *(const u32x4 *)(in + (int64_t)row * ld_in + c0 + ch * 8);
            w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
            if (scale) {
                const float sc = scale[row];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float lo = sc * __uint_as_float(w[i] << 16), hi = sc * __uint_as_float(w[i] & 0xffff0000u);
                    w[i] = f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            tile[(ch * 8 + 2 * i) * kTrPitch + r] = (uint16_t)w[i];
            tile[(ch * 8 + 2 * i + 1) * kTrPitch + r] = (uint16_t)(w[i] >> 16);
        }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kTrTile * 8 / kTrThreads; ++k) {
        const int q = tid + k * kTrThreads, c = q >> 3, rc = q & 7;   // eight lanes: the 128 bytes of one output row
        if (c0 + c >= cols || r0 + rc * 8 >= rows_pad) continue;
        const uint32_t *src = (const uint32_t *)(tile + c * kTrPitch + rc * 8);   // 4-byte aligned
        *(u32x4 *)(out + (int64_t)(c0 + c) * ld_out + r0 + rc * 8) = (u32x4){src[0], src[1], src[2], src[3]};
    }
}

// ---------------------------------------------------------------------------
// workspace layout
// ---------------------------------------------------------------------------
static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct LmLayout {
    size_t total;
    size_t off_i32[2], off_zy[2], off_m[2], off_tau[2], off_coef, off_scale;
    size_t off_ps[2], off_pf[2], off_pc[2];
    size_t off_hst, off_e, off_z, off_tok;
    int block_pad, v_pad, col_tiles;
    int e_blocks;        // row blocks of E (and of the scaled H^T) the workspace holds: one dW product's worth
};

static LmLayout lm_layout(int64_t n, int64_t d, int64_t v, bool dense_buffers = true)
{
    LmLayout L;
    const int64_t block = n < kRowBlock ? n : kRowBlock;
    L.block_pad = (int)((block + BM - 1) / BM * BM);
    L.v_pad = (int)((v + BN - 1) / BN * BN);
    L.col_tiles = L.v_pad / BN;
    const int64_t n_blocks = (n + kRowBlock - 1) / kRowBlock;
    L.e_blocks = (int)(n_blocks < kDwBlocks ? (n_blocks < 1 ? 1 : n_blocks) : kDwBlocks);
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
    for (int s = 0; s < 2; ++s) {
        L.off_i32[s] = take(n * 4); L.off_zy[s] = take(n * 4); L.off_m[s] = take(n * 4);
        L.off_tau[s] = take(n * 4);
        L.off_ps[s] = take((size_t)L.col_tiles * n * 4);
        L.off_pf[s] = take((size_t)L.col_tiles * n * 4);
        L.off_pc[s] = take((size_t)L.col_tiles * n * 4);
    }
    L.off_coef = take(n * 4);
    L.off_scale = take(n * 4);
    L.off_hst = L.off_e = L.off_z = L.off_tok = 0;
    if (dense_buffers) {
        L.off_z = take((size_t)L.block_pad * L.v_pad * 4);      // fp32 logits of one row block
        L.off_tok = take(n * 4);                                // sampled tokens as 32-bit integers, for the sampled-token part of dW
        L.off_hst = take((size_t)d * (L.e_blocks * L.block_pad + kHstPad) * 2);   // (diag(s) H)^T of the blocks of one dW product
        L.off_e = take((size_t)L.e_blocks * L.block_pad * L.v_pad * 2);      // their masked exponentials
    }
    L.total = o;
    return L;
}

// The list form keeps no E: per-row statistics as above, then the list cursors, the safe-set sizes and
// the column-major copy of the lists.  Rows are cut into at most 256 blocks for the counting sort.
struct LmListLayout {
    LmLayout stats;
    size_t total, off_cursor, off_count, off_blk, off_colstart, off_grp, off_cscrow, off_cscval;
    size_t off_zylow, off_cand, off_candcur, off_need, off_ovf, off_rowmap, off_nsub, off_hc, off_msub, off_tausub;
    int n_blk, rows_per_blk;
};

static LmListLayout lm_list_layout(int64_t n, int64_t d, int64_t v, int64_t cap)
{
    LmListLayout L;
    L.stats = lm_layout(n, d, v, false);
    int64_t per = (n + 255) / 256;
    if (per < 64) per = 64;
    L.rows_per_blk = (int)per;
    L.n_blk = (int)((n + per - 1) / per);
    if (L.n_blk < 1) L.n_blk = 1;
    size_t o = L.stats.total;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
    L.off_cursor = take(n * 4);
    L.off_count = take(n * 4);
    L.off_blk = take((size_t)L.n_blk * v * 4);
    L.off_colstart = take((size_t)(v + 1) * 4);
    L.off_grp = take((size_t)((v + 255) / 256 + 1) * 4);
    L.off_cscrow = take((size_t)n * cap * 4);
    L.off_cscval = take((size_t)n * cap * 4);
    L.off_zylow = take(n * 4);
    L.off_cand = take((size_t)n * kLmCandMax * sizeof(dvp_grad_entry));
    L.off_candcur = take(n * 4);
    L.off_need = take(2 * 4);
    L.off_ovf = take(n * 4);
    L.off_rowmap = take(n * 4);
    L.off_nsub = take(4);
    L.off_hc = take((size_t)n * d * 2);
    L.off_msub = take(n * 4);
    L.off_tausub = take(n * 4);
    L.total = o;
    return L;
}

// What the forward leaves behind for a backward in a later call: per row block the masked exponentials,
// and per row the two factors the gradient multiplies (1 - p_y and -1 / S, zero for
// a row whose sampled token is pruned).
struct LmSaved {
    size_t total, off_ucoef, off_uscale, off_e, block_bytes;
    int n_blocks;
};

static LmSaved lm_saved_layout(int64_t n, int64_t v)
{
    LmSaved S;
    const int64_t block = n < kRowBlock ? n : kRowBlock;
    const int64_t block_pad = (block + BM - 1) / BM * BM, v_pad = (v + BN - 1) / BN * BN;
    S.n_blocks = (int)((n + kRowBlock - 1) / kRowBlock);
    if (S.n_blocks < 1) S.n_blocks = 1;
    S.block_bytes = align256((size_t)block_pad * v_pad * 2);
    size_t o = 0;
    S.off_ucoef = o; o += align256(n * 4);
    S.off_uscale = o; o += align256(n * 4);
    S.off_e = o; o += S.block_bytes * S.n_blocks;
    S.total = o;
    return S;
}

// coef[i] = g[i] * unit_coef[i], scale[i] = g[i] * unit_scale[i]
__global__ void apply_grad_kernel(float *coef, float *scale, const float *unit_coef, const float *unit_scale,
                                  const float *g, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { coef[i] = g[i] * unit_coef[i]; scale[i] = g[i] * unit_scale[i]; }
}

enum LmPhase { LM_FUSED = 0, LM_FORWARD_SAVE = 1, LM_BACKWARD_SAVED = 2 };

static bool lm_params_ok(const dvp_lmhead_params *p)
{
    if (!p) return false;
    if (p->n_rows < 0 || p->vocab < 1 || p->hidden < BK) return false;
    if (p->hidden % BK || p->ld_hidden < p->hidden || p->ld_w < p->hidden) return false;
    if (p->ld_hidden % 8 || p->ld_w % 8) return false;
    if (p->n_rows > (1 << 30) || p->vocab > (1 << 22) || p->hidden > (1 << 20)) return false;
    if (p->ld_hidden > (1 << 22) || p->ld_w > (1 << 22)) return false;   // tile-relative byte offsets stay in 32 bits
    if (p->log_rho != p->log_rho || p->log_rho > 0.0f) return false;
    return true;
}

// Both entry points.  The inference side is either a bf16 head applied to the same hidden states
// (w_infer) or an 8-bit engine with its own activations and head (f8), or absent (both null).
static dvp_status run_lmhead(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                             const void *w_infer, const dvp_lmhead_f8_side *f8, const int64_t *ids,
                             const float *grad_out, const dvp_side_out *out_train, const dvp_side_out *out_infer,
                             uint8_t *row_flags, float *d_hidden, float *d_w, void *workspace,
                             size_t workspace_bytes, void *stream_, LmPhase phase = LM_FUSED, void *saved = nullptr,
                             size_t saved_bytes = 0, bool dw_accumulate = false, bool stats_only_ws = false,
                             const int *n_dev = nullptr)
{
    // n_dev (device int32): the call's real row count, at most p->n_rows; every launch is sized for p->n_rows
    // and finds out on the device how far its rows go.  Training side with gradient, accumulated dW only.
    if (n_dev && (phase != LM_FUSED || !grad_out || !dw_accumulate || stats_only_ws || w_infer || f8)) return DVP_ERR_PARAM;
    if (!p) return DVP_ERR_NULL;
    if (p->log_rho != p->log_rho || p->log_rho > 0.0f) return DVP_ERR_PARAM;
    if (p->n_rows < 0 || p->vocab < 1 || p->hidden < 1 || p->ld_hidden < p->hidden || p->ld_w < p->hidden)
        return DVP_ERR_SHAPE;
    if (!lm_params_ok(p)) return DVP_ERR_UNSUPPORTED;
    if (p->n_rows == 0) return DVP_OK;
    if (!hidden || !w_train || !ids || (!out_train && phase != LM_BACKWARD_SAVED)) return DVP_ERR_NULL;
    if (grad_out && (!d_hidden || !d_w)) return DVP_ERR_NULL;
    if (phase == LM_BACKWARD_SAVED && !grad_out) return DVP_ERR_NULL;
    if ((out_train && out_train->entropy) || ((w_infer || f8) && out_infer && out_infer->entropy))
        return DVP_ERR_UNSUPPORTED;
    if (((uintptr_t)hidden | (uintptr_t)w_train | (uintptr_t)w_infer) % 16) return DVP_ERR_ALIGN;
    if (f8) {
        if (!f8->hidden || !f8->w) return DVP_ERR_NULL;
        if (f8->ld_hidden < p->hidden || f8->ld_w < p->hidden) return DVP_ERR_SHAPE;
        if (!(f8->scale == f8->scale) || f8->scale <= 0.0f || isinf(f8->scale)) return DVP_ERR_PARAM;
        // a K step is 128 bytes of every row; tile-relative byte offsets stay in 32 bits
        if (p->hidden % (2 * BK) || f8->ld_hidden % 16 || f8->ld_w % 16 || f8->ld_hidden > (1 << 23) ||
            f8->ld_w > (1 << 23))
            return DVP_ERR_UNSUPPORTED;
        if (((uintptr_t)f8->hidden | (uintptr_t)f8->w) % 16) return DVP_ERR_ALIGN;
    }
    const bool infer_side = w_infer != nullptr || f8 != nullptr;
    // stats_only_ws: a forward-only call uses the per-row statistics and partials only, which come first in
    // the layout; the caller vouches for a workspace of that size
    if (stats_only_ws && (phase != LM_FUSED || grad_out)) return DVP_ERR_PARAM;
    const LmLayout L = lm_layout(p->n_rows, p->hidden, p->vocab, !stats_only_ws);
    if (!workspace || ((uintptr_t)workspace % 256) || workspace_bytes < L.total) return DVP_ERR_WORKSPACE;
    const LmSaved SV = lm_saved_layout(p->n_rows, p->vocab);
    if (phase != LM_FUSED && (!saved || ((uintptr_t)saved % 256) || saved_bytes < SV.total)) return DVP_ERR_WORKSPACE;

    hipStream_t stream = (hipStream_t)stream_;
    const int n = (int)p->n_rows, d = (int)p->hidden, v = (int)p->vocab;
    char *ws = (char *)workspace;
    const void *w_side[2] = {w_train, w_infer};
    SideOut outs[2];
    uint32_t *side_bits[2];
    for (int s = 0; s < 2; ++s) {
        const dvp_side_out *o = s == 0 ? out_train : (infer_side ? out_infer : nullptr);
        outs[s] = SideOut{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        side_bits[s] = nullptr;
        if (o) {
            outs[s] = SideOut{o->logp, o->row_max, o->lse_safe, o->lse_full, o->safe_count, nullptr};
            side_bits[s] = o->safe_bits;
        }
    }
    uint16_t *hst = (uint16_t *)(ws + L.off_hst);
    float *unit_coef = saved ? (float *)((char *)saved + SV.off_ucoef) : nullptr;
    float *unit_scale = saved ? (float *)((char *)saved + SV.off_uscale) : nullptr;
    // Where the masked exponentials of the row block at r0 lie.  Up to kDwBlocks consecutive row blocks form a
    // group with one panelled E (panels of 256 columns over the group's rows, a block's rows following the
    // previous block's: every block but the call's last is full) and one dW product.  The fused call reuses one
    // group's room in the workspace; the saved phases keep every group, one after the other.
    struct EPlace {
        uint16_t *group;     // E of the group
        int64_t panel;       // elements per panel
        int64_t ld_t;        // row pitch of the group's (diag(s) H)^T
        int first_row;       // of the block within the group
    };
    const int n_blocks = (n + kRowBlock - 1) / kRowBlock;
    auto e_place = [&](int r0) {
        const int b = r0 / kRowBlock, grp = b / kDwBlocks;
        const int in_group = (n_blocks - grp * kDwBlocks) < kDwBlocks ? (n_blocks - grp * kDwBlocks) : kDwBlocks;
        char *base = phase == LM_FUSED ? ws + L.off_e : (char *)saved + SV.off_e + (size_t)grp * kDwBlocks * SV.block_bytes;
        return EPlace{(uint16_t *)base, (int64_t)in_group * L.block_pad * BM, (int64_t)in_group * L.block_pad + kHstPad,
                      (b % kDwBlocks) * L.block_pad};
    };
    const int tb = 256;
#define DVP_CHECK_LAUNCH() do { if (hipGetLastError() != hipSuccess) return DVP_ERR_HIP; } while (0)

    // Forward of `rows` token rows starting at r0 on side s: pass A, pass B, outputs.  The per-row
    // statistics and the partials are indexed from 0 within the call.
    auto forward = [&](int s, int r0, int rows, bool write_e, RowStats &st) -> dvp_status {
        st.max_key = (int *)(ws + L.off_i32[s]); st.zy = (float *)(ws + L.off_zy[s]);
        st.m = (float *)(ws + L.off_m[s]); st.tau = (float *)(ws + L.off_tau[s]);
        // (the gradient factors are kept for every row of the call: a group's dW product comes after its last block)
        st.coef = (float *)(ws + L.off_coef) + r0; st.scale = (float *)(ws + L.off_scale) + r0;
        if (phase == LM_FORWARD_SAVE) { st.coef = unit_coef + r0; st.scale = unit_scale + r0; }
        st.part_s = (float *)(ws + L.off_ps[s]); st.part_c = (int *)(ws + L.off_pc[s]);
        st.part_f = outs[s].lse_full ? (float *)(ws + L.off_pf[s]) : nullptr;
        SideOut o = outs[s];
        if (o.logp) o.logp += r0;
        if (o.row_max) o.row_max += r0;
        if (o.lse_safe) o.lse_safe += r0;
        if (o.lse_full) o.lse_full += r0;
        if (o.safe_count) o.safe_count += r0;
        const int nb = (rows + tb - 1) / tb;
        const bool bytes = s == 1 && f8 != nullptr;
        const int64_t bits_ld = (v + 31) / 32;
        uint32_t *bits = side_bits[s] ? side_bits[s] + (int64_t)r0 * bits_ld : nullptr;
        GemmArgs g;
        g.A = (const uint16_t *)hidden + (int64_t)r0 * p->ld_hidden; g.lda = p->ld_hidden;
        g.B = (const uint16_t *)w_side[s]; g.ldb = p->ld_w;
        g.M = rows; g.N = v; g.K = d; g.scale = 1.0f;
        if (n_dev) { g.n_dev = n_dev; g.n_off = r0; g.dev_dim = 1; }
        if (bytes) {   // two bytes count as one element
            g.A = (const uint16_t *)((const uint8_t *)f8->hidden + (int64_t)r0 * f8->ld_hidden); g.lda = f8->ld_hidden / 2;
            g.B = (const uint16_t *)f8->w; g.ldb = f8->ld_w / 2;
            g.K = d / 2; g.scale = f8->scale;
        }
        hipLaunchKernelGGL(init_stats_kernel, dim3(nb), dim3(tb), 0, stream, st, rows);
        DVP_CHECK_LAUNCH();
        const EPlace ep = e_place(r0);
        if (!stats_only_ws) {
            // One pass of the product: row maxima, and the block's logits kept as fp32; the sums at the
            // threshold (and E) are then read off the stored logits.  Re-reading them costs a few percent
            // of what producing them a second time would.
            float *Z = (float *)(ws + L.off_z);
            const EpiMax<true> em{st, ids + r0, Z, (int64_t)L.v_pad};
            if ((bytes ? launch_gemm<EpiMax<true>, false, true>(g, em, stream) : launch_gemm<EpiMax<true>, false>(g, em, stream)) !=
                hipSuccess)
                return DVP_ERR_HIP;
            hipLaunchKernelGGL(after_max_kernel, dim3(nb), dim3(tb), 0, stream, st, rows, p->log_rho);
            DVP_CHECK_LAUNCH();
            ZRowArgs za;
            za.Z = Z; za.ldz = L.v_pad; za.st = st; za.out = o; za.ids = ids + r0;
            za.grad_out = grad_out ? grad_out + r0 : nullptr; za.row_flags = row_flags ? row_flags + r0 : nullptr;
            za.E = ep.group + (int64_t)ep.first_row * BM; za.e_panel = ep.panel; za.bits = bits; za.bits_ld = bits_ld;
            za.vocab = v; za.v_pad = L.v_pad; za.side = s; za.unit_grad = phase == LM_FORWARD_SAVE ? 1 : 0;
            za.n_dev = n_dev; za.n_off = r0; za.rows = rows;
            const dim3 zg((unsigned)rows), zb(kZRowThreads);
            if (write_e) {
                const dim3 zge((unsigned)((rows + BM - 1) / BM * BM));   // E's rows up to the row tile: zeros past `rows`
                if (bits) hipLaunchKernelGGL((lm_rows_from_z_kernel<true, true>), zge, zb, 0, stream, za);
                else      hipLaunchKernelGGL((lm_rows_from_z_kernel<true, false>), zge, zb, 0, stream, za);
            } else {
                if (bits) hipLaunchKernelGGL((lm_rows_from_z_kernel<false, true>), zg, zb, 0, stream, za);
                else      hipLaunchKernelGGL((lm_rows_from_z_kernel<false, false>), zg, zb, 0, stream, za);
            }
            DVP_CHECK_LAUNCH();
            return DVP_OK;
        }
        // No room for a block's logits (the caller vouched for the statistics part of the workspace only):
        // the logits are produced twice, row maxima first, then the sums at the threshold per column tile.
        if (bytes) {
            if (launch_gemm<EpiMax<false>, false, true>(g, EpiMax<false>{st, ids + r0, nullptr, 0}, stream) != hipSuccess) return DVP_ERR_HIP;
        } else {
            if (launch_gemm<EpiMax<false>, false>(g, EpiMax<false>{st, ids + r0, nullptr, 0}, stream) != hipSuccess) return DVP_ERR_HIP;
        }
        hipLaunchKernelGGL(after_max_kernel, dim3(nb), dim3(tb), 0, stream, st, rows, p->log_rho);
        DVP_CHECK_LAUNCH();
        hipError_t eb;
        if (bytes) {
            eb = bits ? launch_gemm<EpiSum<true>, true, true>(g, EpiSum<true>{st, rows, bits, bits_ld}, stream)
                      : launch_gemm<EpiSum<>, true, true>(g, EpiSum<>{st, rows, nullptr, 0}, stream);
        } else {
            eb = bits ? launch_gemm<EpiSum<true>, true>(g, EpiSum<true>{st, rows, bits, bits_ld}, stream)
                      : launch_gemm<EpiSum<>, true>(g, EpiSum<>{st, rows, nullptr, 0}, stream);
        }
        if (eb != hipSuccess) return DVP_ERR_HIP;
        hipLaunchKernelGGL(after_sum_kernel, dim3((rows + kAfterRows - 1) / kAfterRows),
                           dim3(kAfterRows * kAfterSegs), 0, stream, st, o, ids + r0,
                           grad_out ? grad_out + r0 : nullptr, row_flags ? row_flags + r0 : nullptr, rows, v,
                           L.col_tiles, s, phase == LM_FORWARD_SAVE ? 1 : 0, (const int *)nullptr, (const int *)nullptr);
        DVP_CHECK_LAUNCH();
        return DVP_OK;
    };

    RowStats st;
    dvp_status rc;
    // dH of the row block at r0 from its E and the per-row factors coef (q) and scale (s), and the block's part of
    // the second operand of its group's dW product
    auto backward_dh = [&](int r0, int rows, const float *coef, const float *scale) -> dvp_status {
        const EPlace ep = e_place(r0);
        const int rows_pad = (rows + BM - 1) / BM * BM;
        const uint16_t *hblock = (const uint16_t *)hidden + (int64_t)r0 * p->ld_hidden;
        // (diag(s) H)^T of the block, zero columns up to the row tile (they pad the K dimension of the dW product)
        hipLaunchKernelGGL(transpose_bf16_kernel, dim3((d + kTrTile - 1) / kTrTile, (rows_pad + kTrTile - 1) / kTrTile),
                           dim3(kTrThreads), 0, stream,
                           hblock, p->ld_hidden, hst + ep.first_row, ep.ld_t, rows, d, rows_pad, scale, n_dev, r0);
        DVP_CHECK_LAUNCH();
        // dH[r0 : r0 + rows, :] = diag(s) . E [rows, v_pad] . W [v, d] + diag(q) . W[y, :]; W is read as it lies, its rows
        // are the product's k (E's columns from v to v_pad are zero)
        GemmArgs gh;
        gh.A = ep.group + (int64_t)ep.first_row * BM; gh.lda = BM; gh.a_panel = ep.panel;
        gh.B = (const uint16_t *)w_train; gh.ldb = p->ld_w;
        gh.M = rows; gh.N = d; gh.K = L.v_pad; gh.kb_rows = (int)v; gh.b_cols = (int)d; gh.scale = 1.0f;
        if (n_dev) { gh.n_dev = n_dev; gh.n_off = r0; gh.dev_dim = 1; }
        const EpiStore eh{d_hidden + (int64_t)r0 * p->ld_hidden, p->ld_hidden, 0, scale, coef, ids + r0,
                          (const uint16_t *)w_train, p->ld_w};
        if (launch_gemm<EpiStore, false, false, false, true>(gh, eh, stream) != hipSuccess) return DVP_ERR_HIP;
        return DVP_OK;
    };
    // dW (+)= E^T . diag(s) H over the `rows` token rows of the group that starts at r0, then the sampled tokens' rows:
    // E as it lies (the group's rows are the product's k, zero rows from the last one to the row tile), against the
    // small transposed copy of diag(s) H
    auto backward_dw = [&](int r0, int rows, const float *coef) -> dvp_status {
        const EPlace ep = e_place(r0);
        GemmArgs gw;
        gw.A = ep.group; gw.lda = BM; gw.a_panel = ep.panel; gw.B = hst; gw.ldb = ep.ld_t;
        gw.M = v; gw.N = d; gw.K = (rows + BM - 1) / BM * BM; gw.scale = 1.0f;
        if (n_dev) { gw.n_dev = n_dev; gw.n_off = r0; gw.dev_dim = 2; }
        const EpiStore ew{d_w, p->ld_w, r0 > 0 || dw_accumulate, nullptr, nullptr, nullptr, nullptr, 0};
        if (launch_gemm<EpiStore, false, false, true, false>(gw, ew, stream) != hipSuccess) return DVP_ERR_HIP;
        int *tokens = (int *)(ws + L.off_tok) + r0;
        hipLaunchKernelGGL(onehot_tokens_kernel, dim3((rows + tb - 1) / tb), dim3(tb), 0, stream, ids + r0, coef, tokens, rows);
        DVP_CHECK_LAUNCH();
        for (int q0 = 0; q0 < rows; q0 += kOnehotRows) {   // in row order: launches on one stream run in order
            const int qrows = (rows - q0) < kOnehotRows ? (rows - q0) : kOnehotRows;
            hipLaunchKernelGGL(onehot_dw_kernel, dim3(qrows), dim3(kOnehotThreads), 0, stream, tokens + q0,
                               coef + q0, (const uint16_t *)hidden + (int64_t)(r0 + q0) * p->ld_hidden, p->ld_hidden, d_w,
                               p->ld_w, qrows, d, n_dev, r0 + q0);
            DVP_CHECK_LAUNCH();
        }
        return DVP_OK;
    };
    // the training side with gradient: per group of row blocks, `block` for each of its blocks, then the group's dW
    auto by_groups = [&](auto &&block) -> dvp_status {
        constexpr int kGroupRows = kDwBlocks * kRowBlock;
        const float *coef = (const float *)(ws + L.off_coef);
        for (int g0 = 0; g0 < n; g0 += kGroupRows) {
            const int g_rows = (n - g0) < kGroupRows ? (n - g0) : kGroupRows;
            for (int r0 = g0; r0 < g0 + g_rows; r0 += kRowBlock) {
                const int rows = (g0 + g_rows - r0) < kRowBlock ? (g0 + g_rows - r0) : kRowBlock;
                const dvp_status rs = block(r0, rows);
                if (rs != DVP_OK) return rs;
            }
            const dvp_status rs = backward_dw(g0, g_rows, coef + g0);
            if (rs != DVP_OK) return rs;
        }
        return DVP_OK;
    };
    // a side's forward without E: row block by row block where the logits are stored (one block's worth of
    // room), all rows at once where they are produced twice
    auto forward_all = [&](int side) -> dvp_status {
        if (stats_only_ws) return forward(side, 0, n, false, st);
        for (int r0 = 0; r0 < n; r0 += kRowBlock) {
            const int rows = (n - r0) < kRowBlock ? (n - r0) : kRowBlock;
            const dvp_status rs = forward(side, r0, rows, false, st);
            if (rs != DVP_OK) return rs;
        }
        return DVP_OK;
    };

    if (phase == LM_BACKWARD_SAVED) {
        float *coef = (float *)(ws + L.off_coef), *scale = (float *)(ws + L.off_scale);
        return by_groups([&](int r0, int rows) -> dvp_status {
            hipLaunchKernelGGL(apply_grad_kernel, dim3((rows + tb - 1) / tb), dim3(tb), 0, stream, coef + r0, scale + r0,
                               (const float *)unit_coef + r0, (const float *)unit_scale + r0, grad_out + r0, rows);
            DVP_CHECK_LAUNCH();
            return backward_dh(r0, rows, coef + r0, scale + r0);
        });
    }
    if (phase == LM_FORWARD_SAVE) {
        for (int r0 = 0; r0 < n; r0 += kRowBlock) {
            const int rows = (n - r0) < kRowBlock ? (n - r0) : kRowBlock;
            if ((rc = forward(0, r0, rows, true, st)) != DVP_OK) return rc;
        }
    } else if (!grad_out) {
        if ((rc = forward_all(0)) != DVP_OK) return rc;
    } else {
        rc = by_groups([&](int r0, int rows) -> dvp_status {
            const dvp_status rs = forward(0, r0, rows, true, st);
            return rs != DVP_OK ? rs : backward_dh(r0, rows, st.coef, st.scale);
        });
        if (rc != DVP_OK) return rc;
    }
    if (infer_side) {
        if ((rc = forward_all(1)) != DVP_OK) return rc;
    }
#undef DVP_CHECK_LAUNCH
    return DVP_OK;
}

static bool lm_list_cap_ok(const dvp_lmhead_params *p, int32_t cap)
{
    return cap >= 1 && cap <= kLmListMax && p->n_rows * (int64_t)cap < ((int64_t)1 << 31);
}

__global__ void zero_cursor_kernel(int *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// List form of the call.  No row blocks: nothing of size N x V is kept.  A side's forward is one pass over
// the logits where that is enough: pass A collects, next to the row maxima, every token that can still
// be safe (EpiMaxCand), and the safe set, its sum and the list are then read off the candidates.  Where a
// row has more candidates than are kept (flat rows), and where lse_full is asked for, the side's second
// pass runs as in the dense call, appending to the lists on the training side.  Which of the two
// happens depends on the inputs only.  Then the list kernels form dH and dW.
static dvp_status run_lmhead_lists(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                   const void *w_infer, const dvp_lmhead_f8_side *f8, const int64_t *ids,
                                   const float *grad_out,
                                   const dvp_side_out *out_train, const dvp_side_out *out_infer, uint8_t *row_flags,
                                   dvp_grad_entry *entries, int32_t *grad_len, int32_t list_cap, float *d_hidden,
                                   float *d_w, void *workspace, size_t workspace_bytes, void *stream_)
{
    if (!p) return DVP_ERR_NULL;
    if (p->log_rho != p->log_rho || p->log_rho > 0.0f) return DVP_ERR_PARAM;
    if (p->n_rows < 0 || p->vocab < 1 || p->hidden < 1 || p->ld_hidden < p->hidden || p->ld_w < p->hidden)
        return DVP_ERR_SHAPE;
    if (list_cap < 1) return DVP_ERR_PARAM;
    if (!lm_params_ok(p) || !lm_list_cap_ok(p, list_cap)) return DVP_ERR_UNSUPPORTED;
    if (p->n_rows == 0) return DVP_OK;
    if (!hidden || !w_train || !ids || !out_train) return DVP_ERR_NULL;
    const bool lists = grad_out != nullptr;        // without grad_out: the forward of both sides only
    if (lists && (!row_flags || !entries || !grad_len || !d_hidden || !d_w)) return DVP_ERR_NULL;
    const bool infer_side = w_infer != nullptr || f8 != nullptr;
    if (out_train->entropy || (infer_side && out_infer && out_infer->entropy)) return DVP_ERR_UNSUPPORTED;
    if (out_train->safe_bits || (infer_side && out_infer && out_infer->safe_bits)) return DVP_ERR_UNSUPPORTED;
    if (f8) {   // as in run_lmhead
        if (!f8->hidden || !f8->w) return DVP_ERR_NULL;
        if (f8->ld_hidden < p->hidden || f8->ld_w < p->hidden) return DVP_ERR_SHAPE;
        if (!(f8->scale == f8->scale) || f8->scale <= 0.0f || isinf(f8->scale)) return DVP_ERR_PARAM;
        if (p->hidden % (2 * BK) || f8->ld_hidden % 16 || f8->ld_w % 16 || f8->ld_hidden > (1 << 23) ||
            f8->ld_w > (1 << 23))
            return DVP_ERR_UNSUPPORTED;
        if (((uintptr_t)f8->hidden | (uintptr_t)f8->w) % 16) return DVP_ERR_ALIGN;
    }
    if (((uintptr_t)hidden | (uintptr_t)w_train | (uintptr_t)w_infer) % 16) return DVP_ERR_ALIGN;
    if (lists && (((uintptr_t)d_hidden | (uintptr_t)d_w) % 16 || ((uintptr_t)entries % 8) || ((uintptr_t)grad_len % 4)))
        return DVP_ERR_ALIGN;
    const LmListLayout LL = lm_list_layout(p->n_rows, p->hidden, p->vocab, list_cap);
    const LmLayout &L = LL.stats;
    if (!workspace || ((uintptr_t)workspace % 256) || workspace_bytes < LL.total) return DVP_ERR_WORKSPACE;

    hipStream_t stream = (hipStream_t)stream_;
    const int n = (int)p->n_rows, d = (int)p->hidden, v = (int)p->vocab;
    char *ws = (char *)workspace;
    int *cursor = (int *)(ws + LL.off_cursor);
    const int tb = 256, nb = (n + tb - 1) / tb;
#define DVP_CHECK_LAUNCH() do { if (hipGetLastError() != hipSuccess) return DVP_ERR_HIP; } while (0)
    hipLaunchKernelGGL(zero_cursor_kernel, dim3(nb), dim3(tb), 0, stream, cursor, n);
    DVP_CHECK_LAUNCH();
    int *need = (int *)(ws + LL.off_need), *cand_cur = (int *)(ws + LL.off_candcur);
    float *zy_low = (float *)(ws + LL.off_zylow);
    dvp_grad_entry *cand = (dvp_grad_entry *)(ws + LL.off_cand);
    hipLaunchKernelGGL(zero_cursor_kernel, dim3(1), dim3(tb), 0, stream, need, 2);
    DVP_CHECK_LAUNCH();
    RowStats st0;
    int32_t *count0 = nullptr;
    for (int s = 0; s < (infer_side ? 2 : 1); ++s) {
        RowStats st;
        st.max_key = (int *)(ws + L.off_i32[s]); st.zy = (float *)(ws + L.off_zy[s]);
        st.m = (float *)(ws + L.off_m[s]); st.tau = (float *)(ws + L.off_tau[s]);
        st.coef = (float *)(ws + L.off_coef); st.scale = (float *)(ws + L.off_scale);
        st.part_s = (float *)(ws + L.off_ps[s]); st.part_c = (int *)(ws + L.off_pc[s]);
        const dvp_side_out *so = s == 0 ? out_train : out_infer;
        SideOut o = SideOut{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
        if (so) o = SideOut{so->logp, so->row_max, so->lse_safe, so->lse_full, so->safe_count, nullptr};
        if (s == 0) {
            if (!o.safe_count) o.safe_count = (int32_t *)(ws + LL.off_count);   // the list kernels need the sizes
            count0 = o.safe_count;
            st0 = st;
        }
        st.part_f = o.lse_full ? (float *)(ws + L.off_pf[s]) : nullptr;
        GemmArgs g;
        g.A = (const uint16_t *)hidden; g.lda = p->ld_hidden;
        g.B = (const uint16_t *)(s == 0 ? w_train : w_infer); g.ldb = p->ld_w;
        g.M = n; g.N = v; g.K = d; g.scale = 1.0f;
        const bool bytes = s == 1 && f8 != nullptr;
        if (bytes) {   // two bytes count as one element
            g.A = (const uint16_t *)f8->hidden; g.lda = f8->ld_hidden / 2;
            g.B = (const uint16_t *)f8->w; g.ldb = f8->ld_w / 2;
            g.K = d / 2; g.scale = f8->scale;
        }
        hipLaunchKernelGGL(init_stats_kernel, dim3(nb), dim3(tb), 0, stream, st, n);
        DVP_CHECK_LAUNCH();
        const bool one_pass = o.lse_full == nullptr;   // the full sum needs every token's exponential
        if (one_pass) {
            if (launch_lmhead_zy_low(g.A, g.lda, g.B, g.ldb, ids, zy_low, n, g.K, v, bytes ? g.scale : 0.0f, stream) != hipSuccess)
                return DVP_ERR_HIP;
            hipLaunchKernelGGL(zero_cursor_kernel, dim3(nb), dim3(tb), 0, stream, cand_cur, n);
            DVP_CHECK_LAUNCH();
            const EpiMaxCand ec{st, ids, zy_low, cand, cand_cur, kLmCandMax, p->log_rho};
            if ((bytes ? launch_gemm<EpiMaxCand, false, true>(g, ec, stream) : launch_gemm<EpiMaxCand, false>(g, ec, stream)) !=
                hipSuccess)
                return DVP_ERR_HIP;
        } else {
            if ((bytes ? launch_gemm<EpiMax<false>, false, true>(g, EpiMax<false>{st, ids, nullptr, 0}, stream)
                       : launch_gemm<EpiMax<false>, false>(g, EpiMax<false>{st, ids, nullptr, 0}, stream)) != hipSuccess)
                return DVP_ERR_HIP;
        }
        hipLaunchKernelGGL(after_max_kernel, dim3(nb), dim3(tb), 0, stream, st, n, p->log_rho);
        DVP_CHECK_LAUNCH();
        if (one_pass) {
            LmCandArgs c;
            c.cand = cand; c.cand_count = cand_cur; c.m = st.m; c.tau = st.tau; c.zy = st.zy; c.zy_low = zy_low;
            c.ids = ids; c.grad_out = grad_out; c.out = o; c.row_flags = row_flags;
            c.coef = st.coef; c.scale = st.scale;
            c.entries = (s == 0 && lists) ? entries : nullptr; c.list_cap = list_cap;
            c.overflow = (int32_t *)(ws + LL.off_ovf); c.n = n; c.v = v; c.side = s;
            if (launch_lmhead_candidates_finish(c, stream) != hipSuccess) return DVP_ERR_HIP;
        }
        // Second pass: over every row where lse_full is wanted; else over the rows whose candidates did
        // not fit, gathered into consecutive rows (their number is only known on the device: the launches
        // are sized for all rows and find out there; none: they exit at once).
        hipError_t eb;
        if (one_pass) {
            int *rowmap = (int *)(ws + LL.off_rowmap), *n_sub = (int *)(ws + LL.off_nsub);
            LmSubsetArgs sa;
            sa.overflow = (const int32_t *)(ws + LL.off_ovf); sa.rowmap = rowmap; sa.n_sub = n_sub; sa.n_report = need + s;
            sa.H = g.A; sa.ld_h = g.lda; sa.Hc = (uint16_t *)(ws + LL.off_hc);
            sa.m = st.m; sa.tau = st.tau; sa.m_sub = (float *)(ws + LL.off_msub); sa.tau_sub = (float *)(ws + LL.off_tausub);
            sa.n = n; sa.d = g.K;
            if (launch_lmhead_subset(sa, stream) != hipSuccess) return DVP_ERR_HIP;
            GemmArgs gs = g;
            gs.A = sa.Hc; gs.lda = g.K;
            RowStats sub = st;                    // m, tau and the partials by position in the subset
            sub.m = sa.m_sub; sub.tau = sa.tau_sub;
            if (s == 0 && lists)
                eb = launch_gemm<EpiSum<false, true, true>, true>(
                    gs, EpiSum<false, true, true>{sub, n, nullptr, 0, entries, cursor, list_cap,
                                                         rowmap, n_sub}, stream);
            else {
                const EpiSum<false, false, true> es{sub, n, nullptr, 0, nullptr, nullptr, 0,
                                                           rowmap, n_sub};
                eb = bytes ? launch_gemm<EpiSum<false, false, true>, true, true>(gs, es, stream)
                           : launch_gemm<EpiSum<false, false, true>, true>(gs, es, stream);
            }
            if (eb != hipSuccess) return DVP_ERR_HIP;
            hipLaunchKernelGGL(after_sum_kernel, dim3((n + kAfterRows - 1) / kAfterRows), dim3(kAfterRows * kAfterSegs), 0,
                               stream, sub, o, ids, grad_out, row_flags, n, v, L.col_tiles, s, 0, (const int *)rowmap,
                               (const int *)n_sub);
            DVP_CHECK_LAUNCH();
        } else {
            if (s == 0 && lists)
                eb = launch_gemm<EpiSum<false, true>, true>(
                    g, EpiSum<false, true>{st, n, nullptr, 0, entries, cursor, list_cap,
                                                  nullptr, nullptr}, stream);
            else if (bytes)
                eb = launch_gemm<EpiSum<>, true, true>(g, EpiSum<>{st, n, nullptr, 0}, stream);
            else
                eb = launch_gemm<EpiSum<>, true>(g, EpiSum<>{st, n, nullptr, 0}, stream);
            if (eb != hipSuccess) return DVP_ERR_HIP;
            hipLaunchKernelGGL(after_sum_kernel, dim3((n + kAfterRows - 1) / kAfterRows), dim3(kAfterRows * kAfterSegs), 0,
                               stream, st, o, ids, grad_out, row_flags, n, v, L.col_tiles, s, 0, (const int *)nullptr,
                               (const int *)nullptr);
            DVP_CHECK_LAUNCH();
        }
        if (s == 0 && lists) {   // before the inference side adds its bit to row_flags: the list kernels only add theirs
            LmListArgs a;
            a.entries = entries; a.grad_len = grad_len; a.row_flags = row_flags; a.safe_count = count0;
            a.ids = ids; a.coef = st0.coef; a.scale = st0.scale;
            a.W = (const uint16_t *)w_train; a.H = (const uint16_t *)hidden; a.ld_w = p->ld_w; a.ld_h = p->ld_hidden;
            a.d_hidden = d_hidden; a.d_w = d_w;
            a.n = n; a.d = d; a.v = v; a.list_cap = list_cap;
            a.blk_cnt = (int32_t *)(ws + LL.off_blk); a.col_start = (int32_t *)(ws + LL.off_colstart);
            a.grp_total = (int32_t *)(ws + LL.off_grp);
            a.csc_row = (int32_t *)(ws + LL.off_cscrow); a.csc_val = (float *)(ws + LL.off_cscval);
            a.n_blk = LL.n_blk; a.rows_per_blk = LL.rows_per_blk;
            if (launch_lmhead_lists_backward(a, stream) != hipSuccess) return DVP_ERR_HIP;
        }
    }
#undef DVP_CHECK_LAUNCH
    return DVP_OK;
}

// Dense gradient of a subset of the token rows (the rows a list-form call left out): their hidden
// states, ids and upstream gradients are gathered into consecutive rows, the dense call runs on those
// (training side only, dW accumulated), and the rows of dH go back to their places.
struct LmRowsLayout {
    size_t total, off_h, off_ids, off_g, off_dh, off_dense;
};

static LmRowsLayout lm_rows_layout(int64_t n_sub, int64_t d, int64_t v)
{
    LmRowsLayout R;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o += align256(bytes); return at; };
    R.off_h = take((size_t)n_sub * d * 2);
    R.off_ids = take((size_t)n_sub * 8);
    R.off_g = take((size_t)n_sub * 4);
    R.off_dh = take((size_t)n_sub * d * 4);
    R.off_dense = o;
    R.total = o + lm_layout(n_sub, d, v).total;
    return R;
}

// n_dev (device int32, nullable): the number of rows[] entries in use; n_sub is then the host's upper bound
// that sizes the workspace and the launches.
static dvp_status run_lmhead_rows(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                  const int64_t *ids, const float *grad_out, const int32_t *rows, int64_t n_sub,
                                  float *d_hidden, float *d_w, void *workspace, size_t workspace_bytes, void *stream_,
                                  const int32_t *n_dev = nullptr)
{
    if (!p) return DVP_ERR_NULL;
    if (p->log_rho != p->log_rho || p->log_rho > 0.0f) return DVP_ERR_PARAM;
    if (p->n_rows < 0 || p->vocab < 1 || p->hidden < 1 || p->ld_hidden < p->hidden || p->ld_w < p->hidden || n_sub < 0 ||
        n_sub > p->n_rows)
        return DVP_ERR_SHAPE;
    if (!lm_params_ok(p)) return DVP_ERR_UNSUPPORTED;
    if (n_sub == 0) return DVP_OK;
    if (!hidden || !w_train || !ids || !grad_out || !rows || !d_hidden || !d_w) return DVP_ERR_NULL;
    if (((uintptr_t)hidden | (uintptr_t)w_train | (uintptr_t)d_hidden | (uintptr_t)d_w) % 16 || (uintptr_t)rows % 4)
        return DVP_ERR_ALIGN;
    const LmRowsLayout R = lm_rows_layout(n_sub, p->hidden, p->vocab);
    if (!workspace || ((uintptr_t)workspace % 256) || workspace_bytes < R.total) return DVP_ERR_WORKSPACE;
    hipStream_t stream = (hipStream_t)stream_;
    char *ws = (char *)workspace;
    LmRowsArgs a;
    a.rows = rows; a.n_sub = (int32_t)n_sub; a.n = (int32_t)p->n_rows; a.d = (int32_t)p->hidden;
    a.H = (const uint16_t *)hidden; a.ld_h = p->ld_hidden; a.ids = ids; a.grad_out = grad_out;
    a.Hc = (uint16_t *)(ws + R.off_h); a.ids_c = (int64_t *)(ws + R.off_ids); a.g_c = (float *)(ws + R.off_g);
    a.dHc = (float *)(ws + R.off_dh); a.d_hidden = d_hidden; a.n_dev = n_dev;
    if (launch_lmhead_rows_gather(a, stream) != hipSuccess) return DVP_ERR_HIP;
    dvp_lmhead_params sub = *p;
    sub.n_rows = n_sub; sub.ld_hidden = p->hidden;
    const dvp_side_out none = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    const dvp_status st = run_lmhead(&sub, a.Hc, w_train, nullptr, nullptr, a.ids_c, a.g_c, &none, nullptr, nullptr, a.dHc,
                                     d_w, ws + R.off_dense, workspace_bytes - R.off_dense, stream_, LM_FUSED, nullptr, 0,
                                     true, false, (const int *)n_dev);
    if (st != DVP_OK) return st;
    if (launch_lmhead_rows_scatter(a, stream) != hipSuccess) return DVP_ERR_HIP;
    return DVP_OK;
}

// The forward-only call for callers that cannot allocate: its per-row statistics and per-tile partials
// live in this array instead of a caller's workspace.  In host code the array's name is only a handle:
// the address kernels and launchers use is asked for once per device (each device holds its own copy).
static __device__ __align__(256) unsigned char scratch[DVP_NOALLOC_SCRATCH_BYTES];
constexpr int kScratchDevices = 64;
static std::atomic<void *> g_scratch_ptr[kScratchDevices];

static hipError_t prepare_scratch()
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kScratchDevices) return hipErrorInvalidDevice;
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    return hipSuccess;
}
static PrepareRegistrar g_scratch_registrar(&prepare_scratch);

static dvp_status run_lmhead_forward_noalloc(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                             const void *w_infer, const int64_t *ids, const dvp_side_out *out_train,
                                             const dvp_side_out *out_infer, uint8_t *row_flags, void *stream)
{
    if (p && lm_params_ok(p) && p->n_rows > 0 &&
        lm_layout(p->n_rows, p->hidden, p->vocab, false).total > (size_t)DVP_NOALLOC_SCRATCH_BYTES)
        return DVP_ERR_SCRATCH;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kScratchDevices) return DVP_ERR_HIP;
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {                       // first call on this device and dvp_prepare() has not run there
        if (prepare_scratch() != hipSuccess) return DVP_ERR_HIP;
        ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    }
    // every per-row statistic is initialised and every partial overwritten by the call's own kernels:
    // what the previous call left in the array is never read
    return run_lmhead(p, hidden, w_train, w_infer, nullptr, ids, nullptr, out_train, out_infer, row_flags, nullptr,
                      nullptr, ptr, (size_t)DVP_NOALLOC_SCRATCH_BYTES, stream, LM_FUSED, nullptr, 0, false, true);
}

}  // namespace dvp

extern "C" {

dvp_status dvp_fused_lmhead_forward_noalloc(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                            const void *w_infer, const int64_t *ids, const dvp_side_out *out_train,
                                            const dvp_side_out *out_infer, uint8_t *row_flags, void *stream)
{
    return dvp::run_lmhead_forward_noalloc(p, hidden, w_train, w_infer, ids, out_train, out_infer, row_flags, stream);
}

size_t dvp_fused_lmhead_rows_workspace_bytes(const dvp_lmhead_params *p, int64_t n_sub)
{
    if (!dvp::lm_params_ok(p) || n_sub < 0 || n_sub > p->n_rows) return 0;
    return dvp::lm_rows_layout(n_sub, p->hidden, p->vocab).total;
}

dvp_status dvp_fused_lmhead_rows(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                 const int64_t *ids, const float *grad_out, const int32_t *rows, int64_t n_sub,
                                 float *d_hidden, float *d_w, void *workspace, size_t workspace_bytes, void *stream)
{
    return dvp::run_lmhead_rows(p, hidden, w_train, ids, grad_out, rows, n_sub, d_hidden, d_w, workspace, workspace_bytes,
                                stream);
}

dvp_status dvp_fused_lmhead_select_rows(int64_t n_rows, const uint8_t *row_flags, uint32_t mask, int32_t *rows,
                                        int64_t max_rows, int32_t *n_sub, int32_t *n_flagged, void *stream)
{
    if (n_rows < 0 || n_rows > (1 << 30) || max_rows < 0 || max_rows > (1 << 30)) return DVP_ERR_SHAPE;
    if (!n_sub || (n_rows > 0 && !row_flags) || (max_rows > 0 && !rows)) return DVP_ERR_NULL;
    if (((uintptr_t)rows | (uintptr_t)n_sub | (uintptr_t)n_flagged) % 4) return DVP_ERR_ALIGN;
    return dvp::launch_lmhead_select_rows(row_flags, mask, n_rows, rows, max_rows, n_sub, n_flagged, (hipStream_t)stream) ==
                   hipSuccess ? DVP_OK : DVP_ERR_HIP;
}

dvp_status dvp_fused_lmhead_rows_counted(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                         const int64_t *ids, const float *grad_out, const int32_t *rows,
                                         const int32_t *n_sub, int64_t max_rows, float *d_hidden, float *d_w,
                                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (!n_sub) return DVP_ERR_NULL;
    if ((uintptr_t)n_sub % 4) return DVP_ERR_ALIGN;
    return dvp::run_lmhead_rows(p, hidden, w_train, ids, grad_out, rows, max_rows, d_hidden, d_w, workspace, workspace_bytes,
                                stream, n_sub);
}

size_t dvp_fused_lmhead_lists_workspace_bytes(const dvp_lmhead_params *p, int32_t list_cap)
{
    if (!dvp::lm_params_ok(p) || !dvp::lm_list_cap_ok(p, list_cap)) return 0;
    return dvp::lm_list_layout(p->n_rows, p->hidden, p->vocab, list_cap).total;
}

size_t dvp_fused_lmhead_lists_second_pass_rows(const dvp_lmhead_params *p, int32_t list_cap)
{
    if (!dvp::lm_params_ok(p) || !dvp::lm_list_cap_ok(p, list_cap)) return 0;
    return dvp::lm_list_layout(p->n_rows, p->hidden, p->vocab, list_cap).off_need;
}

dvp_status dvp_fused_lmhead_lists(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                  const void *w_infer, const int64_t *ids, const float *grad_out,
                                  const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                  uint8_t *row_flags, dvp_grad_entry *entries, int32_t *grad_len,
                                  int32_t list_cap, float *d_hidden, float *d_w, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    return dvp::run_lmhead_lists(p, hidden, w_train, w_infer, nullptr, ids, grad_out, out_train, out_infer, row_flags,
                                 entries, grad_len, list_cap, d_hidden, d_w, workspace, workspace_bytes, stream);
}

dvp_status dvp_fused_lmhead_lists_f8infer(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                          const dvp_lmhead_f8_side *infer, const int64_t *ids, const float *grad_out,
                                          const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                          uint8_t *row_flags, dvp_grad_entry *entries, int32_t *grad_len,
                                          int32_t list_cap, float *d_hidden, float *d_w, void *workspace,
                                          size_t workspace_bytes, void *stream)
{
    if (!infer) return DVP_ERR_NULL;
    return dvp::run_lmhead_lists(p, hidden, w_train, nullptr, infer, ids, grad_out, out_train, out_infer, row_flags,
                                 entries, grad_len, list_cap, d_hidden, d_w, workspace, workspace_bytes, stream);
}

size_t dvp_fused_lmhead_workspace_bytes(const dvp_lmhead_params *p)
{
    if (!dvp::lm_params_ok(p)) return 0;
    return dvp::lm_layout(p->n_rows, p->hidden, p->vocab).total;
}

dvp_status dvp_fused_lmhead(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                            const void *w_infer, const int64_t *ids, const float *grad_out,
                            const dvp_side_out *out_train, const dvp_side_out *out_infer,
                            uint8_t *row_flags, float *d_hidden, float *d_w, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    return dvp::run_lmhead(p, hidden, w_train, w_infer, nullptr, ids, grad_out, out_train, out_infer, row_flags,
                           d_hidden, d_w, workspace, workspace_bytes, stream);
}

size_t dvp_fused_lmhead_saved_bytes(const dvp_lmhead_params *p)
{
    if (!dvp::lm_params_ok(p)) return 0;
    return dvp::lm_saved_layout(p->n_rows, p->vocab).total;
}

dvp_status dvp_fused_lmhead_forward(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                    const void *w_infer, const dvp_lmhead_f8_side *infer8, const int64_t *ids,
                                    const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                    uint8_t *row_flags, void *saved, size_t saved_bytes, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (w_infer && infer8) return DVP_ERR_PARAM;
    return dvp::run_lmhead(p, hidden, w_train, w_infer, infer8, ids, nullptr, out_train, out_infer, row_flags,
                           nullptr, nullptr, workspace, workspace_bytes, stream, dvp::LM_FORWARD_SAVE, saved,
                           saved_bytes);
}

dvp_status dvp_fused_lmhead_backward(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                     const int64_t *ids, const float *grad_out, const void *saved,
                                     size_t saved_bytes, float *d_hidden, float *d_w, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    if (!grad_out || !d_hidden || !d_w) return p ? DVP_ERR_NULL : DVP_ERR_NULL;
    return dvp::run_lmhead(p, hidden, w_train, nullptr, nullptr, ids, grad_out, nullptr, nullptr, nullptr, d_hidden,
                           d_w, workspace, workspace_bytes, stream, dvp::LM_BACKWARD_SAVED, (void *)saved,
                           saved_bytes);
}

dvp_status dvp_fused_lmhead_f8infer(const dvp_lmhead_params *p, const void *hidden, const void *w_train,
                                    const dvp_lmhead_f8_side *infer, const int64_t *ids, const float *grad_out,
                                    const dvp_side_out *out_train, const dvp_side_out *out_infer,
                                    uint8_t *row_flags, float *d_hidden, float *d_w, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (!infer) return DVP_ERR_NULL;
    return dvp::run_lmhead(p, hidden, w_train, nullptr, infer, ids, grad_out, out_train, out_infer, row_flags,
                           d_hidden, d_w, workspace, workspace_bytes, stream);
}

}  // extern "C"
