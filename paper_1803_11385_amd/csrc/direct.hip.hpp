// Gathered products without a staging pass through LDS: every wavefront loads its matrix-core
// operands from memory straight into registers and runs on its own, with no workgroup barrier.
//
// The MFMA 16x16x4 instruction takes, from lane l, one element of each operand for reduction
// index l/16.  The reduction dimension of the gathered product (Eq.3 with the column matrix of
// Algorithm 1 never formed) is cut into 16-byte units: unit u = tap*(c/4) + q holds channels
// 4q..4q+3 of neighbour `tap`.  In reduction block j, lane group g = l/16 loads unit 4j+g of
// its voxel (ONE 16-byte load: a quarter of a neighbour row when c = 16, the whole row of one
// of four taps when c = 4) and the four instructions of the block take elements 0..3 of it, so
// the reduction runs in a permuted order that costs nothing.
#pragma once
#include "kernels.hip.hpp"

namespace hch {

template <int NT> struct FragOf;
template <> struct FragOf<1> { typedef float type; };
template <> struct FragOf<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct FragOf<4> { typedef f32x4 type; };

template <int NT> __device__ __forceinline__ float frag_get(const typename FragOf<NT>::type &f, int i)
{
    if constexpr (NT == 1) return f; else return f[i];
}

// Y[i][n] (+ split slices) = sum over taps and channels of X[nbr[i][tap]][ch] * Wm[tap*c + ch][n]
//   X    [M][c] rows, c % 4 == 0, 16-byte aligned
//   nbr  [M][27]
//   Wm   [27*c][N] row-major, 16-byte aligned, N % 4 == 0; or, with `flipped` (NT = 1 only), the
//        weights W[27][N][c] of the convolution whose data gradient this is, read as
//        Wm[t*c + ch][n] = W[26-t][n][ch] (Eq.8 through the symmetry of the 3x3x3 neighbourhood)
//   Y    [M][N] (slice z of a split reduction at Y + z*split_stride)
// A wavefront owns 16*RT voxels and 16*NT output columns; a workgroup is four independent
// wavefronts on consecutive voxel tiles.  Output column nb + NT*i + t belongs to column tile t
// (row i of the instruction's weight operand), so a lane loads its NT weights of one reduction
// row as one vector and ends up holding 4*NT consecutive outputs of one voxel.
// S register sets form a ring: the loads of block j+S-1 are issued before the products of
// block j.  CHECK: the last block may have units past the 27 taps (c % 16 != 0) or the column
// group may reach past N; without it c % 16 == 0 and N % (16*NT) == 0.
// SKIP (RT = 4: a wavefront's 64 voxels are one tile of the pattern order): row i of the
// wavefront is voxel rowmap[tile*64 + i] and tilemask[tile] has the taps those voxels have; the
// reduction runs over the units of the present taps only (tap t' of the compacted list is tap
// tmap[t']), tiles are dealt round-robin (neighbouring tiles have the same amount of work).
template <int RT, int NT, int S, bool CHECK, bool SKIP = false>
__global__ __launch_bounds__(256) void conv_direct_kernel(
    const float *__restrict__ X, const int32_t *__restrict__ nbr, const float *__restrict__ Wm,
    float *__restrict__ Y, int M, int c, int N, int J, int j_per_split, int upt, int step_t, int step_q,
    unsigned wave_tiles, int64_t split_stride, int flipped, const int32_t *__restrict__ rowmap,
    const uint32_t *__restrict__ tilemask)
{
    typedef typename FragOf<NT>::type wfrag;
    constexpr int ROWS = 16 * RT;
    constexpr int IDX = ROWS * 27;
    static_assert(!SKIP || ROWS == PATTERN_TILE, "a wavefront's rows are one tile of the pattern order");
    __shared__ int32_t sidx[4 * IDX];
    __shared__ int32_t srow[SKIP ? 4 * ROWS : 1];
    __shared__ uint8_t stap[SKIP ? 4 * 32 : 1];

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const unsigned tile = (SKIP ? xcd_chunk_tile(blockIdx.x, skip_chunk(wave_tiles, 4)) : xcd_tile(blockIdx.x, gridDim.x / NUM_XCD)) * 4 + wv;
    if (tile >= wave_tiles) return;                    // no barrier below: a wave may leave alone
    const int nb = blockIdx.y * (16 * NT);
    int jb = blockIdx.z * j_per_split;
    int je = min(J, jb + j_per_split);
    int n_taps = 27;                                   // taps of the reduction (present ones with SKIP)
    int32_t *rv = srow + (SKIP ? wv * ROWS : 0);
    uint8_t *tmap = stap + (SKIP ? wv * 32 : 0);
    if constexpr (SKIP) {
        const uint32_t present = tilemask[tile];
        n_taps = __popc(present);
        if (lane < 27 && ((present >> lane) & 1u)) tmap[__popc(present & ((1u << lane) - 1u))] = (uint8_t)lane;
        const int64_t row = (int64_t)tile * ROWS + lane;
        rv[lane] = row < M ? rowmap[row] : -1;
        const int Jp = (n_taps * upt + 3) / 4;
        const int per = ((Jp + (int)gridDim.z - 1) / (int)gridDim.z + S - 1) / S * S;
        jb = blockIdx.z * per;
        je = min(Jp, jb + per);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }

    // this wave's 16*RT x 27 neighbour indices: one contiguous piece of the list, kept in LDS
    // (written and read by this wave only)
    int32_t *my = sidx + wv * IDX;
    {
        const int64_t pos0 = (int64_t)tile * IDX, lim = (int64_t)M * 27;
        constexpr int PER = (IDX + 63) / 64;
        int32_t v[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {                 // all loads first, then all stores
            if constexpr (SKIP) {
                // element e of the tile: column e % 27 of the index row of voxel rv[e / 27]
                const int e = i * 64 + lane, row = e / 27, vox = rv[min(row, ROWS - 1)];
                v[i] = *((e < IDX && vox >= 0) ? nbr + ((int64_t)vox * 27 + (e - row * 27)) : &g_minus1);
            } else {
                const int64_t o = pos0 + i * 64 + lane;
                v[i] = *(o < lim ? nbr + o : &g_minus1);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < PER; ++i)
            if (IDX % 64 == 0 || i * 64 + lane < IDX) my[i * 64 + lane] = v[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    // (t, q): tap and unit-in-tap of the block whose indices are read next, for this lane group
    int jn = jb;
    int t = (4 * jb + g) / upt;
    int q = (4 * jb + g) - t * upt;
    int32_t nidx[RT];
    int cur_q4 = 0, cur_k = 0, cur_t = 0;
    auto fetch_idx = [&]() {
        const bool ok = (jn < je) & (t < n_taps);
        int tt = t < 27 ? t : 26;
        if constexpr (SKIP) tt = tmap[min(t, 31)] % 27;     // the tap behind entry t of the compacted list
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const int32_t v = my[(16 * i + r) * 27 + tt];
            nidx[i] = ok ? v : -1;
        }
        cur_q4 = 4 * q; cur_k = tt * c + 4 * q; cur_t = tt;
        t += step_t; q += step_q;
        if (q >= upt) { q -= upt; ++t; }
        ++jn;
    };
    // Weight loads never leave the matrix: past its last reduction row (blocks beyond this
    // slice, units beyond the 27 taps) the row is clamped, which is harmless because the
    // gathered operand is zero there; past its last column the column is clamped, and the
    // outputs of such a lane are never stored.
    const int wcol = CHECK ? min(nb + NT * r, N - NT) : nb + NT * r;
    const int k_last = 27 * c - 4;
    auto issue = [&](f32x4 (&a)[RT], wfrag (&b)[4]) {
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            const float *p = nidx[i] >= 0 ? X + (uint32_t)(nidx[i] * c + cur_q4) : zsrc;
            a[i] = *reinterpret_cast<const f32x4 *>(p);
        }
        bool plain = true;
        if constexpr (NT == 1) {
            if (flipped) {
                // the four reduction rows of this unit are four neighbouring channels of one weight row
                const f32x4 v = *reinterpret_cast<const f32x4 *>(Wm + ((uint32_t)(((26 - cur_t) * N + wcol) * c) + cur_q4));
#pragma unroll
                for (int e = 0; e < 4; ++e) b[e] = v[e];
                plain = false;
            }
        }
        if (plain) {
            const float *wp = Wm + ((uint32_t)(min(cur_k, k_last) * N) + wcol);
#pragma unroll
            for (int e = 0; e < 4; ++e) b[e] = *reinterpret_cast<const wfrag *>(wp + e * N);
        }
    };

    f32x4 acc[RT][NT];
#pragma unroll
    for (int i = 0; i < RT; ++i)
#pragma unroll
        for (int n = 0; n < NT; ++n) acc[i][n] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto multiply = [&](const f32x4 (&a)[RT], const wfrag (&b)[4]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int n = 0; n < NT; ++n)
                    acc[i][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(frag_get<NT>(b[e], n), a[i][e], acc[i][n], 0, 0, 0);
    };

    f32x4 ra[S][RT];
    wfrag rb[S][4];
    fetch_idx();
#pragma unroll
    for (int s = 0; s < S - 1; ++s) { issue(ra[s], rb[s]); fetch_idx(); }
    __builtin_amdgcn_sched_barrier(0);
    for (int j0 = jb; j0 < je; j0 += S) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            // the scheduler must not sink these loads down to their use two steps later
            issue(ra[(s + S - 1) % S], rb[(s + S - 1) % S]);
            __builtin_amdgcn_sched_barrier(0);
            fetch_idx();
            multiply(ra[s], rb[s]);      // blocks past je were gathered as zeros
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // accumulator register e of column tile n, lane (r, g): voxel r, output column
    // nb + NT*(4g + e) + n, i.e. element NT*e + n of this lane's 4*NT consecutive columns
    float *out = Y + (int64_t)blockIdx.z * split_stride;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        int64_t row = (int64_t)tile * ROWS + 16 * i + r;
        if (row >= M) continue;
        if constexpr (SKIP) row = rv[16 * i + r];
#pragma unroll
        for (int f = 0; f < NT; ++f) {
            const int col = nb + 4 * NT * g + 4 * f;
            if (CHECK && col >= N) continue;
            f32x4 v;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int m = 4 * f + x;
                v[x] = acc[i][m % NT][m / NT];
            }
            *reinterpret_cast<f32x4 *>(out + row * N + col) = v;
        }
    }
}

}  // namespace hch

namespace hch {

// Gathered product into FOUR output columns (the data gradient of a first layer with 4 input
// channels):  Y[i][0..3] = sum over taps t and channels ch of X[nbr[i][t]][ch] * Wm[t*C + ch][0..3],
// C = 16*CC.  With 4 columns a 16x16x4 instruction would carry 12 rows of padding, so this kernel
// uses v_mfma_f32_4x4x1 (16 independent 4x4 outer products per instruction): the 16 blocks take
// 16 different reduction indices and the 4 rows of a block 4 voxels,
//   lane l = 4*b + i,  b = 4*tq + cq:  tap 4*T + tq of voxel i, channels 4*cq .. 4*cq+3 of the
//   current 16-channel chunk (ONE 16-byte load feeds four instructions, element e = channel
//   4*cq + e); the same lane holds, as j = l % 4, the weights of output column j for those
//   reduction indices (kept in registers for the whole kernel).
// A block's accumulator is D[b][i][j] in register i of lane 4*b + j; the 16 blocks are summed
// through LDS once per group of 4 voxels.  A wavefront owns 64 voxels (their 27 indices each in
// LDS, as in conv_direct_kernel) and works on 16 of them at a time: all 28*1 loads of a chunk
// are issued before its 112 instructions.
//   X [M][C] rows, nbr [M][27], Wm [27*C][4], Y [M][4]; all 16-byte aligned.  With `flipped`, Wm is
//   the weight tensor W[27][4][C] of the convolution whose data gradient this is:
//   Wm[t*C + ch][j] = W[26-t][j][ch].
// SKIP: as in conv_direct_kernel: the wavefront's 64 voxels are tile `tile` of the pattern order
// (voxel rowmap[tile*64 + i]), and only the taps of tilemask[tile] are multiplied, four at a
// time: TA = ceil(present taps / 4) groups instead of 7 (one instantiation of the loop body per
// TA, so that the loads of a chunk stay in one straight run).
template <int CC, int TA>
__device__ __forceinline__ void narrow4_tile(const float *__restrict__ X, const float *__restrict__ Wm,
                                             float *__restrict__ Y, const int32_t *my, float *red,
                                             const int32_t *rv, const uint8_t *tmap, int n_taps, int M,
                                             unsigned tile, int lane, int flipped, bool skip)
{
    constexpr int C = 16 * CC;
    const int i = lane & 3, b = lane >> 2, tq = b >> 2, cq = b & 3, j = i;
    // this lane's taps: entry 4T + tq of the (compacted) tap list
    int tap[TA];
#pragma unroll
    for (int T = 0; T < TA; ++T) {
        const int t = 4 * T + tq;
        tap[T] = t < n_taps ? (skip ? (int)tmap[t] : t) : -1;
    }
    // this lane's weights: reduction row tap*C + 16*cc + 4*cq + e, column j
    float w[TA][CC][4];
#pragma unroll
    for (int T = 0; T < TA; ++T)
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int t = tap[T];
                const int ch = 16 * cc + 4 * cq + e;
                const float *src = t < 0 ? reinterpret_cast<const float *>(g_zero16)
                                         : (flipped ? Wm + (((26 - t) * 4 + j) * C + ch) : Wm + ((t * C + ch) * 4 + j));
                w[T][cc][e] = *src;
            }
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    for (int it = 0; it < 4; ++it) {                   // 16 voxels = 4 groups of 4 per pass
        f32x4 acc[4];
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) acc[gq] = f32x4{0.f, 0.f, 0.f, 0.f};
        int32_t idx[TA][4];
#pragma unroll
        for (int T = 0; T < TA; ++T)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int32_t v = my[(16 * it + 4 * gq + i) * 27 + max(tap[T], 0)];
                idx[T][gq] = tap[T] >= 0 ? v : -1;
            }
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) {
            f32x4 a[TA][4];
#pragma unroll
            for (int T = 0; T < TA; ++T)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const float *p = idx[T][gq] >= 0 ? X + (uint32_t)(idx[T][gq] * C + 16 * cc + 4 * cq) : zsrc;
                    a[T][gq] = *reinterpret_cast<const f32x4 *>(p);
                }
            __builtin_amdgcn_sched_barrier(0);         // all loads of the chunk before its products
#pragma unroll
            for (int T = 0; T < TA; ++T)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq)
                        acc[gq] = __builtin_amdgcn_mfma_f32_4x4x1f32(a[T][gq][e], w[T][cc][e], acc[gq], 0, 0, 0);
        }
        // sum of the 16 blocks: red[((gq*4 + i)*4 + j)*16 + b], then lane (gq, i, j) adds its 16
#pragma unroll
        for (int gq = 0; gq < 4; ++gq)
#pragma unroll
            for (int r = 0; r < 4; ++r) red[((gq * 4 + r) * 4 + j) * 16 + b] = acc[gq][r];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(red + lane * 16 + 4 * q);
            s += (v[0] + v[1]) + (v[2] + v[3]);
        }
        // lane = (gq*4 + i)*4 + j: voxel 16*it + lane/4 of the tile, column lane%4
        const int local = 16 * it + (lane >> 2);
        int64_t row = (int64_t)tile * 64 + local;
        if (row < M) {
            if (skip) row = rv[local];
            Y[row * 4 + (lane & 3)] = s;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();               // red is reused by the next pass
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

template <int CC, bool SKIP = false>
__global__ __launch_bounds__(256) void conv_narrow4_kernel(
    const float *__restrict__ X, const int32_t *__restrict__ nbr, const float *__restrict__ Wm,
    float *__restrict__ Y, int M, unsigned wave_tiles, int flipped, const int32_t *__restrict__ rowmap,
    const uint32_t *__restrict__ tilemask)
{
    constexpr int IDX = 64 * 27;
    __shared__ int32_t sidx[4 * IDX];
    __shared__ float sred[4 * 1024];
    __shared__ int32_t srow[SKIP ? 4 * 64 : 1];
    __shared__ uint8_t stap[SKIP ? 4 * 32 : 1];

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const unsigned tile = (SKIP ? xcd_chunk_tile(blockIdx.x, skip_chunk(wave_tiles, 4)) : xcd_tile(blockIdx.x, gridDim.x / NUM_XCD)) * 4 + wv;
    if (tile >= wave_tiles) return;                    // no workgroup barrier below

    int32_t *my = sidx + wv * IDX;
    float *red = sred + wv * 1024;
    int32_t *rv = srow + (SKIP ? wv * 64 : 0);
    uint8_t *tmap = stap + (SKIP ? wv * 32 : 0);
    int n_taps = 27;
    if constexpr (SKIP) {
        const uint32_t present = tilemask[tile];
        n_taps = __popc(present);
        if (lane < 27 && ((present >> lane) & 1u)) tmap[__popc(present & ((1u << lane) - 1u))] = (uint8_t)lane;
        const int64_t row = (int64_t)tile * 64 + lane;
        rv[lane] = row < M ? rowmap[row] : -1;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    {
        const int64_t pos0 = (int64_t)tile * IDX, lim = (int64_t)M * 27;
        int32_t v[27];
#pragma unroll
        for (int q = 0; q < 27; ++q) {
            if constexpr (SKIP) {
                const int e = q * 64 + lane, row = e / 27, vox = rv[row];
                v[q] = *(vox >= 0 ? nbr + ((int64_t)vox * 27 + (e - row * 27)) : &g_minus1);
            } else {
                const int64_t o = pos0 + q * 64 + lane;
                v[q] = *(o < lim ? nbr + o : &g_minus1);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 27; ++q) my[q * 64 + lane] = v[q];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    if constexpr (SKIP) {
        switch ((n_taps + 3) / 4) {
        case 1: narrow4_tile<CC, 1>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        case 2: narrow4_tile<CC, 2>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        case 3: narrow4_tile<CC, 3>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        case 4: narrow4_tile<CC, 4>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        case 5: narrow4_tile<CC, 5>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        case 6: narrow4_tile<CC, 6>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        default: narrow4_tile<CC, 7>(X, Wm, Y, my, red, rv, tmap, n_taps, M, tile, lane, flipped, true); break;
        }
    } else {
        narrow4_tile<CC, 7>(X, Wm, Y, my, red, rv, tmap, 27, M, tile, lane, flipped, false);
    }
}

}  // namespace hch
