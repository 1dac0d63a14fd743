// Matrix products of the convolution (Eq.2/3, Eq.7, Eq.8) for bfloat16 inputs on the bf16 matrix
// instruction of gfx950 (v_mfma_f32_16x16x32_bf16: products exact, sums in fp32).  Same roles and
// operand modes as gemm_f32_kernel; the difference is what sits in LDS: bf16 bit patterns, with
// the reduction index fastest for BOTH operands, because a lane feeds the instruction 8
// consecutive reduction indices of its row (A) or column (B) as one 16-byte read.  Operands whose
// reduction index is the slow one in memory (the weights in the forward product, both operands
// of the weight gradient) are transposed on their way from registers to LDS.
//
// Included by hch_api.hip after kernels.hip.hpp.
#pragma once

namespace hch {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int BF16_BK = 64;   // reduction indices per tile = granularity of split reductions

// two 16-bit halves into one word with v_perm_b32 (the selector names, from the low byte up, bytes of
// the second operand as 0..3 and of the first as 4..7): {a.lo, b.lo} and {a.hi, b.hi}
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }

// C[M x N] (+ slices) = A[M x K] . B[K x N], fp32 out.
//   AMODE  A_ROWS      A(i,k) = A[i*lda + k]
//          A_COLS      A(i,k) = A[k*lda + i]
//          A_GATHER    A(i,k) = X[idx(i, k/c)][k%c]      (c = lda; rows of X have c elements)
//          A_GATHER_T  A(i,k) = X[idx(k, i/c)][i%c]
//          with idx(voxel, tap) = nbr[voxel*idx_row_stride + tap*idx_tap_stride]: strides (taps, 1)
//          for index rows [voxel][tap], (1, number of voxels) for the tap-major copy [tap][voxel],
//          in which the indices a tile needs for one tap lie side by side (a few cache accesses
//          instead of one per voxel)
//   B_KC   true: B(k,j) = B[j*ldb + k] (optionally cut into runs, see gemm_f32_kernel);
//          false: B(k,j) = B[k*ldb + j]
// Requirements, checked by the host: every 8-element unit along an operand's fast axis is
// 16-byte aligned and wholly inside or outside its matrix (lda, ldb, c multiples of 8; K, M or N
// multiples of 8 where they bound a fast axis); k_per_split and b_wrap multiples of 64.
// Units outside read a constant block of zeros; an absent neighbour (-1) likewise.
template <int BM, int BN, int WM, int AMODE, bool B_KC, bool LEAN = false>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ B, float *__restrict__ C,
    const int32_t *__restrict__ nbr, int M, int N, int K, int64_t lda, int64_t ldb, int64_t ldc,
    int k_per_split, int64_t c_split_stride, int c_vec_ok, unsigned m_tiles,
    int64_t idx_row_stride, int64_t idx_tap_stride, int b_wrap, int64_t b_tap_stride, int flat_slices)
{
    constexpr int BK = BF16_BK;
    // An LDS row holds the 64 reduction offsets of one row (A) or column (B) of the tile: 128
    // bytes, no padding.  Its eight 16-byte pieces are stored permuted, piece p of row r at
    // position p ^ (r % 8), so that the 8 lanes that read or write the same piece of 8
    // consecutive rows at once touch 8 different groups of banks.  Kernels that transpose an
    // operand on its way in (the weight gradient: both) permute by r / 8 as well: a transposing
    // store writes the same 8 bytes of rows that lie 8 apart, which otherwise all fall on the
    // same banks -- 54 % of that kernel's LDS cycles were bank conflicts, the LDS active 75 % of
    // the time; with the second permutation 1.42 -> 1.17 ms.  The kernels without a transposing
    // store keep the simpler form (the second permutation changes nothing for them).
    constexpr int LS = BK;
    constexpr bool SWZ2 = !(AMODE == A_ROWS || AMODE == A_GATHER) || !B_KC;
    auto lds_at = [](int row, int k) {
        const int perm = SWZ2 ? (row ^ ((row >> 3) << 1)) : row;
        return row * LS + ((((k >> 3) ^ perm) & 7) << 3) + (k & 7);
    };
    constexpr int WN = 4 / WM;
    constexpr int WTM = BM / WM, WTN = BN / WN;
    constexpr int MT = WTM / 16, NT = WTN / 16;
    static_assert(WTM % 16 == 0 && WTN % 16 == 0, "wave tile must be a multiple of 16x16");
    static_assert((MT == 1 || MT == 2 || MT == 4) && (NT == 1 || NT == 2 || NT == 4), "1, 2 or 4 tiles");
    constexpr bool A_K_FAST = (AMODE == A_ROWS || AMODE == A_GATHER);
    constexpr bool GATHER = (AMODE == A_GATHER || AMODE == A_GATHER_T);
    static_assert(A_K_FAST || BM == 128, "transposed A: 128-row tiles only");
    constexpr int A_UNITS = BM / 32;                  // 16-byte units of an A tile per thread
    constexpr int B_UNITS = B_KC ? (BN >= 32 ? BN / 32 : 1) : 2;

    __shared__ __attribute__((aligned(16))) uint16_t As2[2 * BM * LS];
    __shared__ __attribute__((aligned(16))) uint16_t Bs2[2 * BN * LS];

    // Which tile and which slice of the reduction this workgroup computes.
    // Grid (x, y, z) = (row tiles, column tiles, slices); with more row tiles than gridDim.x ==
    // m_tiles says, x is remapped so that each XCD owns a contiguous range of row tiles.
    // flat_slices > 0 (a multiple of 8): a one-dimensional grid in which workgroup b belongs to
    // XCD b % 8 (workgroups are handed to the XCDs in turn) and slice s is computed, all tiles of
    // it, by XCD s % 8.  The tiles of a slice of the weight gradient walk through the same voxels
    // at the same time -- each gathers them for its own taps -- and so meet the rows in one L2
    // instead of fetching them from memory once per tile.
    unsigned mtile, ntile, slice;
    if (flat_slices > 0) {
        const unsigned n_tiles = (unsigned)((N + BN - 1) / BN), tiles = m_tiles * n_tiles;
        const unsigned q = blockIdx.x / NUM_XCD, t = q % tiles;
        slice = (q / tiles) * NUM_XCD + blockIdx.x % NUM_XCD;
        mtile = t % m_tiles; ntile = t / m_tiles;
    } else {
        mtile = gridDim.x == m_tiles ? blockIdx.x : xcd_tile(blockIdx.x, gridDim.x / NUM_XCD);
        if (mtile >= m_tiles) return;
        ntile = blockIdx.y; slice = blockIdx.z;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int li = lane & 15, lk = lane >> 4;
    const int m0 = (int)mtile * BM, n0 = (int)ntile * BN;
    const int kbeg = (int)slice * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    const int c = (int)lda;
    C += (int64_t)slice * c_split_stride;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint16_t *zsrc = reinterpret_cast<const uint16_t *>(g_zero16);

    // ---- A: which units of a tile this thread moves.
    // k fast in memory: unit uu = row a_r + 32*uu, reduction offsets a_c .. a_c+7.
    // i fast in memory: rows (i) a_c .. a_c+7 at A_UNITS consecutive reduction offsets
    // a_r .. a_r + A_UNITS-1, which leave for LDS together as one write per row.  Four
    // neighbouring lanes take 64 contiguous bytes of one row of the operand in memory (the
    // address unit merges accesses of neighbouring lanes only; with the lanes of a row 16 apart
    // every lane cost its own cache access and the kernel was bound by their number).
    const int a_c = A_K_FAST ? (tid % 8) * 8 : ((tid & 3) + 4 * (tid >> 6)) * 8;
    const int a_r = A_K_FAST ? tid / 8 : ((tid >> 2) & 15) * A_UNITS;
    const uint16_t *pa[A_UNITS];
    const int32_t *pn[A_UNITS];
    bool a_ok[A_UNITS];
    int ka = kbeg, kn = kbeg;
    int tap_n = 0, cc_n = 0, cc_a = 0, dtap = 0, dcc = 0;
    if (AMODE == A_GATHER) {
        const int gk = kbeg + a_c;
        tap_n = gk / c; cc_n = gk - tap_n * c; cc_a = cc_n;
        dtap = BK / c; dcc = BK - dtap * c;
    }
#pragma unroll
    for (int uu = 0; uu < A_UNITS; ++uu) {
        pa[uu] = nullptr; pn[uu] = nullptr;
        if (AMODE == A_ROWS) { const int r = a_r + 32 * uu; a_ok[uu] = m0 + r < M; pa[uu] = A + (int64_t)(m0 + r) * lda + kbeg + a_c; }
        if (AMODE == A_COLS) { a_ok[uu] = m0 + a_c < M; pa[uu] = A + (int64_t)(kbeg + a_r + uu) * lda + m0 + a_c; }
        if (AMODE == A_GATHER) { const int r = a_r + 32 * uu; a_ok[uu] = m0 + r < M; pn[uu] = nbr + (int64_t)(m0 + r) * idx_row_stride; }
        if (AMODE == A_GATHER_T) {
            const int gi = m0 + a_c;
            const int tap = gi / c;
            cc_a = gi - tap * c;
            a_ok[uu] = gi < M; pn[uu] = nbr + (int64_t)(kbeg + a_r + uu) * idx_row_stride + tap * idx_tap_stride;
        }
    }

    // ---- B.  k fast in memory: unit uu = column b_r + 32*uu, reduction offsets b_c .. b_c+7.
    // j fast: columns b_c .. b_c+7 at the two reduction offsets b_r, b_r+1 (8 lanes side by side
    // along a row of B in memory).
    const int b_c = (tid % 8) * 8;
    const int b_r = B_KC ? tid / 8 : (tid / 8) * 2;
    const uint16_t *pb[B_UNITS];
    bool b_ok[B_UNITS];
    int kb = kbeg;
    int b_pos = b_wrap ? kbeg % b_wrap : 0;
#pragma unroll
    for (int uu = 0; uu < B_UNITS; ++uu) {
        if (B_KC) {
            const int r = b_r + 32 * uu;
            b_ok[uu] = r < BN && n0 + r < N;
            pb[uu] = B + (int64_t)(n0 + r) * ldb + b_c +
                     (b_wrap ? (int64_t)(kbeg / b_wrap) * b_tap_stride + kbeg % b_wrap : (int64_t)kbeg);
        } else {
            b_ok[uu] = b_c < BN && n0 + b_c < N;
            pb[uu] = B + (int64_t)(kbeg + b_r + uu) * ldb + n0 + b_c;
        }
    }
    // ---- LEAN (gather modes; A_GATHER: c a multiple of 64, a tile lies within one tap): as in
    // gemm_f32_kernel, loads through buffer descriptors with scalar offsets for what a tile
    // changes and one multiply-add per gathered row and lane.  Here a matrix instruction takes 16
    // cycles, so every vector instruction in the loop costs a quarter of one.
    [[maybe_unused]] __amdgpu_buffer_rsrc_t rs_idx, rs_a, rs_b;
    [[maybe_unused]] int lv_idx[A_UNITS], lv_b[B_UNITS], lv_a = 0;
    [[maybe_unused]] int tap_i = 0, tap_bb = 0, cc_i = 0, cc_r = 0, cc_b = 0;
    [[maybe_unused]] int64_t b_tap_lo = 0;
    constexpr int LEAN_TAPS = 27;
    constexpr uint32_t LEAN_OUT = 0x80000000u;
    if constexpr (LEAN) {
        static_assert(GATHER, "lean loop: gather modes");
        constexpr int SRD3 = 0x00020000;
        rs_a = __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (int)0x80000000u, SRD3);
        if (AMODE == A_GATHER) {
            tap_i = tap_bb = kbeg / c;
            cc_i = cc_r = cc_b = kbeg - tap_i * c;
            rs_idx = __builtin_amdgcn_make_buffer_rsrc((void *)nbr, 0, M * LEAN_TAPS * 4, SRD3);
            lv_a = a_c * 2;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                const int r = m0 + a_r + 32 * uu;
                lv_idx[uu] = r < M ? (int)((int64_t)r * idx_row_stride * 4) : (int)LEAN_OUT;
            }
            if (B_KC) {
                b_tap_lo = b_tap_stride < 0 ? (int64_t)(LEAN_TAPS - 1) * b_tap_stride : 0;
                rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)(B + b_tap_lo), 0,
                                                         (int)(((int64_t)(LEAN_TAPS - 1) * (b_tap_stride < 0 ? -b_tap_stride : b_tap_stride) + (int64_t)N * ldb) * 2), SRD3);
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) {
                    const int r = b_r + 32 * uu;
                    lv_b[uu] = (r < BN && n0 + r < N) ? (int)(((int64_t)(n0 + r) * ldb + b_c) * 2) : (int)LEAN_OUT;
                }
            } else {
                rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)B, 0, (int)((int64_t)LEAN_TAPS * c * ldb * 2), SRD3);
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu)
                    lv_b[uu] = (b_c < BN && n0 + b_c < N) ? (int)(((int64_t)(b_r + uu) * ldb + n0 + b_c) * 2) : (int)LEAN_OUT;
            }
        } else {
            // A_GATHER_T: reduction over the voxels kbeg .. kend of this slice.  B is described from
            // the slice's first row to its last: past the end it reads zeros, which is what makes
            // the tail of the last tile vanish (the rows gathered there are real, finite data).
            const int len = max(kend - kbeg, 0);
            rs_idx = __builtin_amdgcn_make_buffer_rsrc((void *)nbr, 0, K * LEAN_TAPS * 4, SRD3);
            rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)(B + (int64_t)kbeg * ldb), 0, (int)((int64_t)len * ldb * 2), SRD3);
            const int gi = m0 + a_c;
            const int tap = min(gi / c, LEAN_TAPS - 1);
            lv_a = (gi - (gi / c) * c) * 2;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu)
                lv_idx[uu] = (int)(((int64_t)(kbeg + a_r + uu) * idx_row_stride + (int64_t)tap * idx_tap_stride) * 4);
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu)
                lv_b[uu] = (b_c < BN && n0 + b_c < N) ? (int)(((int64_t)(b_r + uu) * ldb + n0 + b_c) * 2) : (int)LEAN_OUT;
        }
    }
    auto lean_fetch_idx = [&](int32_t *out) {
        if constexpr (LEAN) {
            const int soff = AMODE == A_GATHER ? __builtin_amdgcn_readfirstlane((int)((int64_t)min(tap_i, LEAN_TAPS - 1) * idx_tap_stride * 4)) : 0;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                out[uu] = (int32_t)__builtin_amdgcn_raw_buffer_load_b32(rs_idx, lv_idx[uu], soff, 0);
                if (AMODE == A_GATHER_T) lv_idx[uu] += (int)(BK * idx_row_stride * 4);
            }
            if (AMODE == A_GATHER) { cc_i += BK; if (cc_i >= c) { cc_i = 0; ++tap_i; } }
        }
    };
    auto lean_fetch = [&](const int32_t *rows, u32x4 *ra, u32x4 *rb) {
        if constexpr (LEAN) {
            const int rowbytes = c * 2;
            const int soff_a = AMODE == A_GATHER ? __builtin_amdgcn_readfirstlane(cc_r * 2) : 0;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu)
                ra[uu] = __builtin_amdgcn_raw_buffer_load_b128(rs_a, __mul24(rows[uu], rowbytes) + lv_a, soff_a, 0);
            int soff_b = 0;
            if (AMODE == A_GATHER) {
                const int tap = min(tap_bb, LEAN_TAPS - 1);
                if (B_KC) soff_b = (int)(((int64_t)tap * b_tap_stride - b_tap_lo + cc_b) * 2);
                else soff_b = (tap * c + cc_b) * (int)ldb * 2;
                soff_b = __builtin_amdgcn_readfirstlane(soff_b);
            }
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                rb[uu] = __builtin_amdgcn_raw_buffer_load_b128(rs_b, lv_b[uu], soff_b, 0);
                if (AMODE == A_GATHER_T) lv_b[uu] += BK * (int)ldb * 2;
            }
            if (AMODE == A_GATHER) {
                cc_r += BK; if (cc_r >= c) cc_r = 0;
                cc_b += BK; if (cc_b >= c) { cc_b = 0; ++tap_bb; }
            }
        }
    };

    // LDS row of column j of the tile: the NT MFMA tiles of a wave take interleaved columns
    // (tile nt: columns li*NT + nt of the wave's stretch, so that a lane ends up with NT
    // neighbouring outputs), stored tile after tile so that 16 lanes read 16 consecutive rows
    auto b_lds_row = [&](int j) {
        const int w = j / WTN, q = j - w * WTN;
        return w * WTN + (q % NT) * 16 + q / NT;
    };

    auto fetch_idx = [&](int32_t *out) {
        if (!GATHER) return;
        if constexpr (LEAN) { lean_fetch_idx(out); return; }
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu) {
            bool ok;
            if (AMODE == A_GATHER) ok = a_ok[uu] && kn + a_c < kend;
            else ok = a_ok[uu] && kn + a_r + uu < kend;
            out[uu] = *(ok ? pn[uu] + (AMODE == A_GATHER ? tap_n * idx_tap_stride : 0) : &g_minus1);
            if (AMODE == A_GATHER_T) pn[uu] += BK * idx_row_stride;
        }
        if (AMODE == A_GATHER) {
            tap_n += dtap; cc_n += dcc;
            if (cc_n >= c) { cc_n -= c; ++tap_n; }
        }
        kn += BK;
    };

    auto fetch = [&](const int32_t *rows, u32x4 *ra, u32x4 *rb) {
        if constexpr (LEAN) { lean_fetch(rows, ra, rb); return; }
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu) {
            const uint16_t *src;
            if (AMODE == A_ROWS) {
                src = (a_ok[uu] && ka + a_c < kend) ? pa[uu] : zsrc;
                pa[uu] += BK;
            } else if (AMODE == A_COLS) {
                src = (a_ok[uu] && ka + a_r + uu < kend) ? pa[uu] : zsrc;
                pa[uu] += (int64_t)BK * lda;
            } else {
                const int32_t j = rows[uu];
                src = j >= 0 ? A + (uint32_t)(j * c + cc_a) : zsrc;
            }
            ra[uu] = *reinterpret_cast<const u32x4 *>(src);
        }
        if (AMODE == A_GATHER) { cc_a += dcc; if (cc_a >= c) cc_a -= c; }
        ka += BK;
#pragma unroll
        for (int uu = 0; uu < B_UNITS; ++uu) {
            bool ok;
            if (B_KC) ok = b_ok[uu] && kb + b_c < kend;
            else ok = b_ok[uu] && kb + b_r + uu < kend;
            rb[uu] = *reinterpret_cast<const u32x4 *>(ok ? pb[uu] : zsrc);
            pb[uu] += B_KC ? (int64_t)BK : (int64_t)BK * ldb;
        }
        if (B_KC && b_wrap) {
            b_pos += BK;
            if (b_pos >= b_wrap) {
                b_pos -= b_wrap;
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) pb[uu] += b_tap_stride - b_wrap;
            }
        }
        kb += BK;
    };

    // registers -> LDS (both tiles end up with the reduction index fastest)
    auto stash = [&](int stage, const u32x4 *ra, const u32x4 *rb) {
        uint16_t *As = As2 + stage * BM * LS, *Bs = Bs2 + stage * BN * LS;
        if constexpr (A_K_FAST) {
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu)
                *reinterpret_cast<u32x4 *>(&As[lds_at(a_r + 32 * uu, a_c)]) = ra[uu];
        } else {
            // 4 reduction offsets x 8 rows in registers -> per row its 4 values, 8 bytes
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // one byte-permute instruction per output word: low halves of two words side by
                // side, or their high halves
                const u32x2 lo = {pack_lo(ra[0][q], ra[1][q]), pack_lo(ra[2][q], ra[3][q])};
                const u32x2 hi = {pack_hi(ra[0][q], ra[1][q]), pack_hi(ra[2][q], ra[3][q])};
                *reinterpret_cast<u32x2 *>(&As[lds_at(a_c + 2 * q, a_r)]) = lo;
                *reinterpret_cast<u32x2 *>(&As[lds_at(a_c + 2 * q + 1, a_r)]) = hi;
            }
        }
        if constexpr (B_KC) {
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                const int r = b_r + 32 * uu;
                if (r < BN) *reinterpret_cast<u32x4 *>(&Bs[lds_at(b_lds_row(r), b_c)]) = rb[uu];
            }
        } else if (b_c < BN) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                *reinterpret_cast<uint32_t *>(&Bs[lds_at(b_lds_row(b_c + 2 * q), b_r)]) = pack_lo(rb[0][q], rb[1][q]);
                *reinterpret_cast<uint32_t *>(&Bs[lds_at(b_lds_row(b_c + 2 * q + 1), b_r)]) = pack_hi(rb[0][q], rb[1][q]);
            }
        }
    };

    // A lane's operands of one instruction: 8 consecutive reduction offsets (32*ks + 8*lk ...) of
    // row li of an A tile and of column li of a B tile.  Both sides use the same offsets, which
    // is all the sum over the reduction index needs.
    u32x4 oa[2][MT], ob[2][NT];
    auto load_operands = [&](int stage) {
        const uint16_t *As = As2 + stage * BM * LS, *Bs = Bs2 + stage * BN * LS;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                oa[ks][mt] = *reinterpret_cast<const u32x4 *>(&As[lds_at(wm * WTM + mt * 16 + li, ks * 32 + lk * 8)]);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                ob[ks][nt] = *reinterpret_cast<const u32x4 *>(&Bs[lds_at(wn * WTN + nt * 16 + li, ks * 32 + lk * 8)]);
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, oa[ks][mt]), __builtin_bit_cast(bf16x8, ob[ks][nt]), acc[mt][nt], 0, 0, 0);
    };

    // software pipeline as in gemm_f32_kernel: one barrier per tile; loads two tiles ahead of the
    // store to LDS that needs them (two register sets and two index sets that alternate); nothing
    // in the loop body is conditional -- every load is guarded on its own and reads zeros past the
    // end of the range -- so that the compiler's wait before a store to LDS covers the loads of
    // that register set only.  Tiles go in pairs; an odd last tile follows the loop.
    u32x4 ra0[A_UNITS], rb0[B_UNITS], ra1[A_UNITS], rb1[B_UNITS];
    int32_t rx[A_UNITS] = {}, ry[A_UNITS] = {};
    auto iteration = [&](int stage, u32x4 *sa, u32x4 *sb, int32_t *use, int32_t *load) {
        load_operands(stage);
        multiply();
        stash(stage ^ 1, sa, sb);
        fetch_idx(load);
        fetch(use, sa, sb);
        __syncthreads();
    };
    if (kbeg < kend) {
        int32_t rz[A_UNITS] = {};
        fetch_idx(rx);
        fetch_idx(ry);
        fetch_idx(rz);
        fetch(rx, ra0, rb0);
        fetch(ry, ra1, rb1);
        stash(0, ra0, rb0);
        fetch_idx(ry);
        fetch(rz, ra0, rb0);
        __syncthreads();
        int k0 = kbeg;
        for (; k0 + BK < kend; k0 += 2 * BK) {
            iteration(0, ra1, rb1, ry, rx);
            iteration(1, ra0, rb0, rx, ry);
        }
        if (k0 < kend) {
            load_operands(0);
            multiply();
        }
    }

    // D layout (as for every 16x16 fp32 result): register e of lane l holds D[4*(l/16) + e][l%16];
    // column l%16 of tile nt is column li*NT + nt of the wave's stretch
    const int gj = n0 + wn * WTN + li * NT;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int gi = m0 + wm * WTM + mt * 16 + 4 * lk + e;
            if (gi >= M) continue;
            float *dst = C + (int64_t)gi * ldc + gj;
            if (NT == 4 && c_vec_ok && gj + 4 <= N) {
                *reinterpret_cast<f32x4 *>(dst) = f32x4{acc[mt][0][e], acc[mt][1 % NT][e], acc[mt][2 % NT][e], acc[mt][3 % NT][e]};
            } else if (NT == 2 && c_vec_ok && gj + 2 <= N) {
                typedef float f32x2 __attribute__((ext_vector_type(2)));
                *reinterpret_cast<f32x2 *>(dst) = f32x2{acc[mt][0][e], acc[mt][1 % NT][e]};
            } else {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    if (gj + nt < N) dst[nt] = acc[mt][nt][e];
            }
        }
}


}  // namespace hch
