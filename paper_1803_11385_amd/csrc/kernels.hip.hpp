// Device kernels of the H-CNN hot path for gfx950 (wave64, MFMA).
//
// Everything here works on the voxel-major layout: feature rows X[N][c], neighbour index
// rows nbr[N][27], column matrix col[N][27*c].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hch {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------
// PSH lookup (paper Section 3.1, Eq.1; super tables Eq.4-6)
// ---------------------------------------------------------------------------------------

// Device view of one level of the mini-batch super-PSH.  Prefix arrays are 32-bit on the
// device (the host checks that they fit).
struct PshView {
    const int32_t *H;      // [M_total]     local data index or -1
    const uint16_t *T;     // [M_total][3]  position tag
    const uint8_t *Phi;    // [R_total][3]  offsets
    const int32_t *mbar;   // [b]
    const int32_t *rbar;   // [b]
    const int32_t *M;      // [b+1]
    const int32_t *R;      // [b+1]
    const int32_t *N;      // [b+1]
    int32_t ubar;
};

// Global data index of position (x,y,z) of model v, or -1 if it is outside the grid, lands
// on a redundant slot, or lands on a slot tagged with another position.
__device__ __forceinline__ int32_t psh_lookup(const PshView &L, int v, int x, int y, int z)
{
    const unsigned u = (unsigned)L.ubar;
    if ((unsigned)x >= u || (unsigned)y >= u || (unsigned)z >= u) return -1;
    const unsigned m = (unsigned)L.mbar[v], r = (unsigned)L.rbar[v];
    const unsigned ux = (unsigned)x, uy = (unsigned)y, uz = (unsigned)z;
    const unsigned iphi = (unsigned)L.R[v] + ((ux % r) * r + (uy % r)) * r + (uz % r);   // Eq.4
    const uint8_t *ph = L.Phi + 3u * (size_t)iphi;
    const unsigned hx = (ux % m + ph[0]) % m;                                            // Eq.1
    const unsigned hy = (uy % m + ph[1]) % m;
    const unsigned hz = (uz % m + ph[2]) % m;
    const unsigned s = (unsigned)L.M[v] + (hx * m + hy) * m + hz;                        // Eq.5
    const int32_t h = L.H[s];
    if (h < 0) return -1;
    const uint16_t *t = L.T + 3u * (size_t)s;
    if (t[0] != ux || t[1] != uy || t[2] != uz) return -1;
    return L.N[v] + h;                                                                   // Eq.6
}

// Index side of the traversal of Algorithm 1: for every output voxel i of model
// v = blockIdx.y and every position `row` of its F^3 receptive field (x slowest, z fastest),
// the global input data index or -1.  out[(No[v] + i) * F^3 + row].
//   Ss == 1:  field = [p - (F-1)/2, p + (F-1)/2]^3        (same level)
//   Ss  > 1:  field = [p*Ss - Sp, p*Ss - Sp + F - 1]^3    (input level is finer)
__global__ __launch_bounds__(256) void field_index_kernel(
    PshView Li, const int32_t *__restrict__ out_coords, const int32_t *__restrict__ No,
    int F, int Ss, int Sp, int32_t *__restrict__ out)
{
    const int v = blockIdx.y;
    const int F3 = F * F * F;
    const int32_t base = No[v];
    const int64_t n_items = (int64_t)(No[v + 1] - base) * F3;
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_items) return;
    const int32_t i = (int32_t)(t / F3);
    const int row = (int)(t - (int64_t)i * F3);
    const int fx = row / (F * F), fy = (row / F) % F, fz = row % F;
    const int32_t *p = out_coords + 3 * (int64_t)(base + i);
    int lx, ly, lz;
    if (Ss == 1) {
        const int h = (F - 1) / 2;
        lx = p[0] - h; ly = p[1] - h; lz = p[2] - h;
    } else {
        lx = p[0] * Ss - Sp; ly = p[1] * Ss - Sp; lz = p[2] * Ss - Sp;
    }
    out[(int64_t)(base + i) * F3 + row] = psh_lookup(Li, v, lx + fx, ly + fy, lz + fz);
}

// ---------------------------------------------------------------------------------------
// hash2col (Algorithm 1) through the pre-stored neighbour indices
// ---------------------------------------------------------------------------------------

// 16-byte units: cv = c_in * sizeof(element) / 16.  One thread moves one unit:
// col[r][k][u] = X[nbr[row_begin + r][k]][u] or 0.
__global__ __launch_bounds__(256) void hash2col_vec_kernel(
    const uint4 *__restrict__ X, const int32_t *__restrict__ nbr, uint4 *__restrict__ col,
    int64_t row_begin, int64_t rows, int cv)
{
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int per_row = 27 * cv;
    if (item >= rows * per_row) return;
    const int64_t r = item / per_row;
    const int rem = (int)(item - r * per_row);
    const int k = rem / cv, u = rem - k * cv;
    const int32_t j = nbr[(row_begin + r) * 27 + k];
    uint4 val = make_uint4(0u, 0u, 0u, 0u);
    if (j >= 0) val = X[(int64_t)j * cv + u];
    col[item] = val;
}

// any channel count, one element per thread
template <typename E>
__global__ __launch_bounds__(256) void hash2col_elem_kernel(
    const E *__restrict__ X, const int32_t *__restrict__ nbr, E *__restrict__ col,
    int64_t row_begin, int64_t rows, int c)
{
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int per_row = 27 * c;
    if (item >= rows * per_row) return;
    const int64_t r = item / per_row;
    const int rem = (int)(item - r * per_row);
    const int k = rem / c, ch = rem - k * c;
    const int32_t j = nbr[(row_begin + r) * 27 + k];
    E val = (E)0;
    if (j >= 0) val = X[(int64_t)j * c + ch];
    col[item] = val;
}

// ---------------------------------------------------------------------------------------
// col2hash (Algorithm 2) as a gather: the 3x3x3 stride-1 neighbourhood is symmetric, so the
// voxels that hold row j as their neighbour k are exactly nbr[j][26-k].  Summing per
// destination row in tap order needs no atomics and is bit-reproducible.
// ---------------------------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(256) void col2hash_kernel(
    const float *__restrict__ dcol, const int32_t *__restrict__ nbr, float *__restrict__ dX,
    int64_t n, int c)
{
    const int cv = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n * cv) return;
    const int64_t j = item / cv;
    const int u = (int)(item - j * cv);
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    const int32_t *nb = nbr + j * 27;
    for (int k = 0; k < 27; ++k) {
        const int32_t i = nb[26 - k];
        if (i < 0) continue;
        const float *src = dcol + ((int64_t)i * 27 + k) * c + u * VEC;
        if constexpr (VEC == 4) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(src);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] += v[e];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += src[e];
        }
    }
    float *dst = dX + j * c + u * VEC;
#pragma unroll
    for (int e = 0; e < VEC; ++e) dst[e] = acc[e];
}

// ---------------------------------------------------------------------------------------
// fp32 GEMM on the matrix cores:  C[M x N] (+split) = A[M x K] * B[K x N]
//
//   A_KC : A(i,k) = A[i*lda + k]  (k contiguous)   else  A(i,k) = A[k*lda + i]
//   B_KC : B(k,j) = B[j*ldb + k]  (k contiguous)   else  B(k,j) = B[k*ldb + j]
//
// Block = 256 threads = 4 waves, tile 128 x BN x 32.  Operands are staged in LDS k-major
// (As[k][i], Bs[k][j]) so that the 16 lanes of an MFMA operand row read consecutive words.
// Wave w owns rows [32w, 32w+32) of the tile as 2 x (BN/16) tiles of v_mfma_f32_16x16x4_f32.
// blockIdx.z selects a slice of the reduction dimension (split-K): slice z covers
// k in [z*k_per_split, (z+1)*k_per_split) and writes to C + z*c_split_stride.
// The next tile's global loads are issued before the current tile's MFMAs.
// ---------------------------------------------------------------------------------------
constexpr int GEMM_BM = 128;
constexpr int GEMM_BK = 32;

template <int BN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const float *__restrict__ A, const float *__restrict__ B, float *__restrict__ C,
    int M, int N, int K, int64_t lda, int64_t ldb, int64_t ldc,
    int k_per_split, int64_t c_split_stride, int vec_ok)
{
    constexpr int BM = GEMM_BM, BK = GEMM_BK;
    constexpr int AS = BM + 16;                       // row strides chosen so that the four
    constexpr int BS = (BN == 16) ? 16 : BN + 16;     // k-rows of an operand hit distinct banks
    constexpr int A_UNITS = BM * BK / 4 / 256;        // float4 units per thread (= 4)
    constexpr int B_TOTAL = BK * BN / 4;              // float4 units in a B tile
    constexpr int B_UNITS = (B_TOTAL + 255) / 256;
    constexpr int NT = BN / 16;

    __shared__ __attribute__((aligned(16))) float As[BK * AS];
    __shared__ __attribute__((aligned(16))) float Bs[BK * BS];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    const int kbeg = blockIdx.z * k_per_split;
    const int kend = min(K, kbeg + k_per_split);
    C += (int64_t)blockIdx.z * c_split_stride;

    f32x4 acc[2][NT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    f32x4 ra[A_UNITS], rb[B_UNITS];

    // fetch the tile starting at reduction index k0 into registers (zero outside the matrices)
    auto fetch = [&](int k0) {
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu) {
            const int f = tid + 256 * uu;
            f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
            if (A_KC) {
                const int i = f / (BK / 4), kq = f % (BK / 4);
                const int gi = m0 + i, gk = k0 + kq * 4;
                if (gi < M && gk < kend) {
                    const float *src = A + (int64_t)gi * lda + gk;
                    if (vec_ok && gk + 3 < kend) v = *reinterpret_cast<const f32x4 *>(src);
                    else {
                        v[0] = src[0];
                        if (gk + 1 < kend) v[1] = src[1];
                        if (gk + 2 < kend) v[2] = src[2];
                        if (gk + 3 < kend) v[3] = src[3];
                    }
                }
            } else {
                const int k = f / (BM / 4), iq = f % (BM / 4);
                const int gk = k0 + k, gi = m0 + iq * 4;
                if (gk < kend && gi < M) {
                    const float *src = A + (int64_t)gk * lda + gi;
                    if (vec_ok && gi + 3 < M) v = *reinterpret_cast<const f32x4 *>(src);
                    else {
                        v[0] = src[0];
                        if (gi + 1 < M) v[1] = src[1];
                        if (gi + 2 < M) v[2] = src[2];
                        if (gi + 3 < M) v[3] = src[3];
                    }
                }
            }
            ra[uu] = v;
        }
#pragma unroll
        for (int uu = 0; uu < B_UNITS; ++uu) {
            const int f = tid + 256 * uu;
            f32x4 v = f32x4{0.f, 0.f, 0.f, 0.f};
            if (f < B_TOTAL) {
                if (B_KC) {
                    const int j = f / (BK / 4), kq = f % (BK / 4);
                    const int gj = n0 + j, gk = k0 + kq * 4;
                    if (gj < N && gk < kend) {
                        const float *src = B + (int64_t)gj * ldb + gk;
                        if (vec_ok && gk + 3 < kend) v = *reinterpret_cast<const f32x4 *>(src);
                        else {
                            v[0] = src[0];
                            if (gk + 1 < kend) v[1] = src[1];
                            if (gk + 2 < kend) v[2] = src[2];
                            if (gk + 3 < kend) v[3] = src[3];
                        }
                    }
                } else {
                    const int k = f / (BN / 4), jq = f % (BN / 4);
                    const int gk = k0 + k, gj = n0 + jq * 4;
                    if (gk < kend && gj < N) {
                        const float *src = B + (int64_t)gk * ldb + gj;
                        if (vec_ok && gj + 3 < N) v = *reinterpret_cast<const f32x4 *>(src);
                        else {
                            v[0] = src[0];
                            if (gj + 1 < N) v[1] = src[1];
                            if (gj + 2 < N) v[2] = src[2];
                            if (gj + 3 < N) v[3] = src[3];
                        }
                    }
                }
            }
            rb[uu] = v;
        }
    };

    // registers -> LDS (k-major)
    auto stash = [&]() {
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu) {
            const int f = tid + 256 * uu;
            if (A_KC) {
                const int i = f / (BK / 4), kq = f % (BK / 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) As[(kq * 4 + e) * AS + i] = ra[uu][e];
            } else {
                const int k = f / (BM / 4), iq = f % (BM / 4);
                *reinterpret_cast<f32x4 *>(&As[k * AS + iq * 4]) = ra[uu];
            }
        }
#pragma unroll
        for (int uu = 0; uu < B_UNITS; ++uu) {
            const int f = tid + 256 * uu;
            if (f < B_TOTAL) {
                if (B_KC) {
                    const int j = f / (BK / 4), kq = f % (BK / 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) Bs[(kq * 4 + e) * BS + j] = rb[uu][e];
                } else {
                    const int k = f / (BN / 4), jq = f % (BN / 4);
                    *reinterpret_cast<f32x4 *>(&Bs[k * BS + jq * 4]) = rb[uu];
                }
            }
        }
    };

    const int li = lane & 15, lk = lane >> 4;

    if (kbeg < kend) fetch(kbeg);
    for (int k0 = kbeg; k0 < kend; k0 += BK) {
        stash();
        __syncthreads();
        if (k0 + BK < kend) fetch(k0 + BK);
#pragma unroll
        for (int kk = 0; kk < BK / 4; ++kk) {
            float a[2], b[NT];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) a[mt] = As[(kk * 4 + lk) * AS + wave * 32 + mt * 16 + li];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b[nt] = Bs[(kk * 4 + lk) * BS + nt * 16 + li];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
        }
        __syncthreads();
    }

    // D layout of v_mfma_f32_16x16x4_f32: register e of lane l holds D[4*(l/16) + e][l%16]
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int gi = m0 + wave * 32 + mt * 16 + 4 * lk + e;
                const int gj = n0 + nt * 16 + li;
                if (gi < M && gj < N) C[(int64_t)gi * ldc + gj] = acc[mt][nt][e];
            }
}

// out[i] = sum_z part[z*stride + i], z ascending inside four interleaved groups that are then
// added in group order: the same order on every run.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(
    const float *__restrict__ part, float *__restrict__ out, int64_t n, int splits, int64_t stride)
{
    __shared__ float sh[4][64];
    const int ex = threadIdx.x & 63, zg = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + ex;
    float s = 0.f;
    if (i < n)
        for (int z = zg; z < splits; z += 4) s += part[(int64_t)z * stride + i];
    sh[zg][ex] = s;
    __syncthreads();
    if (zg == 0 && i < n) out[i] = ((sh[0][ex] + sh[1][ex]) + sh[2][ex]) + sh[3][ex];
}

// ---------------------------------------------------------------------------------------
// 2x2x2 max-pooling through the child index rows
// ---------------------------------------------------------------------------------------

// one thread per (coarse voxel, channel); the first occupied child seeds the maximum and a
// later child replaces it only when strictly greater
__global__ __launch_bounds__(256) void pool_fwd_kernel(
    const float *__restrict__ X, const int32_t *__restrict__ child8, float *__restrict__ Y,
    int32_t *__restrict__ argmax, int64_t n_coarse, int c)
{
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * c) return;
    const int64_t o = item / c;
    const int ch = (int)(item - o * c);
    const int32_t *kids = child8 + o * 8;
    float best = 0.f;
    int32_t arg = -1;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int32_t j = kids[k];
        if (j < 0) continue;
        const float v = X[(int64_t)j * c + ch];
        if (arg < 0 || v > best) { best = v; arg = j; }
    }
    Y[item] = best;
    argmax[item] = arg;
}

// one thread per (coarse voxel, child, channel): every fine row is the child of exactly one
// coarse voxel, so this writes all of dX exactly once (the zero fill is part of it)
__global__ __launch_bounds__(256) void pool_bwd_kernel(
    const float *__restrict__ dY, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ child8, float *__restrict__ dX, int64_t n_coarse, int c)
{
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * 8 * c) return;
    const int64_t ok = item / c;            // coarse voxel * 8 + child
    const int ch = (int)(item - ok * c);
    const int32_t j = child8[ok];
    if (j < 0) return;
    const int64_t o = ok >> 3;
    const float g = dY[o * c + ch];
    dX[(int64_t)j * c + ch] = (argmax[o * c + ch] == j) ? g : 0.f;
}

__global__ __launch_bounds__(256) void relu_fwd_kernel(const float *__restrict__ x,
                                                       float *__restrict__ y, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) { const float v = x[i]; y[i] = v > 0.f ? v : 0.f; }
}

__global__ __launch_bounds__(256) void relu_bwd_kernel(const float *__restrict__ y,
                                                       const float *__restrict__ dy,
                                                       float *__restrict__ dx, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) dx[i] = y[i] > 0.f ? dy[i] : 0.f;
}

}  // namespace hch
