// Construction of the perfect spatial hash tables on the device (the paper leaves this as
// future work, Section 5.2 and the conclusion; its tables are built offline on the host).
//
// The structure and the sizes are the paper's (Section 3.1, 5.2): hash table side m with
// m^3 > n, offset table side r starting from 6 r^3 >= n and growing when an attempt fails,
// h(p) = (p mod m + Phi[p mod r]) mod m per axis, H holding data indices, T the position tags.
// The assignment of offsets is a parallel greedy one, made for thousands of threads instead
// of the one-bucket-at-a-time order of the host construction:
//   * every (level, model) pair of the batch is built in the same launches;
//   * buckets (voxels sharing p mod r) are placed in classes of decreasing size (9 and more,
//     8, 7, ..., 2, 1), one launch per class, all buckets of a class at once;
//   * before each class the free slots of every table are listed; a bucket's candidates are the
//     free slots (its first voxel goes there, which fixes the offset), starting at a hashed
//     position of the list;
//   * one wavefront per bucket: 64 candidates are examined at once (a lane looks whether the
//     slots of all the bucket's voxels are free), then the first lane that found room claims the
//     slots with compare-and-swap on H and, if another bucket was faster on one of them, gives
//     the claimed ones back and the next lane tries;
//   * buckets of one voxel need no search: the i-th of them takes the i-th free slot;
//   * a bucket that runs out of candidates fails its pair; failed pairs are cleared and repeated
//     with the next r.
// Which of two racing buckets gets a slot depends on timing, so the tables are valid but not
// reproducible bit for bit; everything computed THROUGH them (lookups, neighbour and child
// lists, convolutions) is the same for every valid table.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hch {

struct PairDesc {
    const int32_t *coords;   // [n][3] positions of this model at this level, data order
    int32_t *H;              // [m^3] this pair's part of H*, -1 = free
    uint16_t *T;             // [m^3][3]
    int32_t n, m, r;
    int32_t cell_base;       // first offset cell of the pair in this attempt's cell arrays
    int32_t vox_base;        // first entry of the pair in this attempt's member arrays
    int32_t slot_base;       // first entry of the pair in this attempt's free-slot list
    int32_t pair_id;         // index into the failure flags
};

constexpr int PSH_CLASSES = 10;      // class k holds the buckets of k voxels, class 9 those of 9 and more

// bucket number of every voxel, bucket sizes
__global__ __launch_bounds__(256) void psh_count_kernel(const PairDesc *__restrict__ pairs,
                                                        int32_t *__restrict__ cnt, int32_t *__restrict__ bucket_of)
{
    const PairDesc P = pairs[blockIdx.y];
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= P.n) return;
    const int32_t *p = P.coords + 3 * (int64_t)i;
    const int r = P.r;
    const int g = ((p[0] % r) * r + (p[1] % r)) * r + (p[2] % r);
    bucket_of[P.vox_base + i] = g;
    atomicAdd(&cnt[P.cell_base + g], 1);
}

// exclusive prefix sum of `n` counts, one workgroup of 1024 threads (the arrays here have at most
// a few million entries)
__global__ __launch_bounds__(1024) void psh_scan_kernel(const int32_t *__restrict__ in, int32_t *__restrict__ out, int n)
{
    __shared__ int32_t part[1024];
    const int t = threadIdx.x;
    const int per = (n + 1023) / 1024;
    const int a = min(n, t * per), b = min(n, a + per);
    int32_t s = 0;
    for (int i = a; i < b; ++i) s += in[i];
    part[t] = s;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {            // inclusive scan of the 1024 partial sums
        const int32_t v = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int32_t run = part[t] - s;
    for (int i = a; i < b; ++i) { const int32_t v = in[i]; out[i] = run; run += v; }
}

// member lists: the voxels of every bucket (order inside a bucket is arbitrary) with their
// residues modulo m, packed x | y << 8 | z << 16
__global__ __launch_bounds__(256) void psh_fill_kernel(const PairDesc *__restrict__ pairs,
                                                       const int32_t *__restrict__ bucket_of,
                                                       const int32_t *__restrict__ first,
                                                       int32_t *__restrict__ fill, int32_t *__restrict__ members,
                                                       uint32_t *__restrict__ residues)
{
    const PairDesc P = pairs[blockIdx.y];
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= P.n) return;
    const int cell = P.cell_base + bucket_of[P.vox_base + i];
    const int pos = first[cell] + atomicAdd(&fill[cell], 1);
    const int32_t *p = P.coords + 3 * (int64_t)i;
    const int m = P.m;
    members[pos] = i;
    residues[pos] = (uint32_t)(p[0] % m) | ((uint32_t)(p[1] % m) << 8) | ((uint32_t)(p[2] % m) << 16);
}

// position of this lane among the lanes of its wavefront for which `flag` is set, after a
// counter has been advanced once for all of them (one atomic per wavefront instead of per lane)
__device__ __forceinline__ int psh_wave_append(bool flag, int32_t *counter)
{
    const unsigned long long mask = __ballot(flag);
    if (mask == 0) return 0;
    const int lane = threadIdx.x & 63;
    const int leader = __builtin_ctzll(mask);
    int base = 0;
    if (lane == leader) base = atomicAdd(counter, __builtin_popcountll(mask));
    base = __shfl(base, leader);
    return base + __builtin_popcountll(mask & ((1ull << lane) - 1ull));
}

// the buckets of 2 and more voxels, listed by class: entry = (active pair, bucket number)
__global__ __launch_bounds__(256) void psh_classify_kernel(const PairDesc *__restrict__ pairs,
                                                           const int32_t *__restrict__ cnt,
                                                           int32_t *__restrict__ class_count,
                                                           int2 *__restrict__ class_cells, int64_t class_stride)
{
    const PairDesc P = pairs[blockIdx.y];
    const int g = blockIdx.x * 256 + threadIdx.x;
    const int c = g < P.r * P.r * P.r ? cnt[P.cell_base + g] : 0;
    const int mine = c < 2 ? 0 : (c < PSH_CLASSES - 1 ? c : PSH_CLASSES - 1);
#pragma unroll
    for (int k = 2; k < PSH_CLASSES; ++k) {           // no lane leaves before the last ballot
        const int pos = psh_wave_append(mine == k, &class_count[k]);
        if (mine == k) class_cells[k * class_stride + pos] = make_int2((int)blockIdx.y, g);
    }
}

// the free slots of every table (any order)
__global__ __launch_bounds__(256) void psh_free_list_kernel(const PairDesc *__restrict__ pairs,
                                                            int32_t *__restrict__ n_free, int32_t *__restrict__ free_list)
{
    const PairDesc P = pairs[blockIdx.y];
    const int e = blockIdx.x * 256 + threadIdx.x;
    const bool is_free = e < P.m * P.m * P.m && P.H[e] == -1;
    const int pos = psh_wave_append(is_free, &n_free[blockIdx.y]);
    if (is_free) free_list[P.slot_base + pos] = e;
}

__device__ __forceinline__ int32_t psh_peek(const int32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// slot of a voxel with packed residues h under the offset (ox, oy, oz)
__device__ __forceinline__ int psh_slot_of(uint32_t h, int ox, int oy, int oz, int m)
{
    int x = (int)(h & 255u) + ox; if (x >= m) x -= m;
    int y = (int)((h >> 8) & 255u) + oy; if (y >= m) y -= m;
    int z = (int)(h >> 16) + oz; if (z >= m) z -= m;
    return (x * m + y) * m + z;
}

// Place the buckets of one class (2 voxels and more): one wavefront per bucket, 4 per workgroup.
// phi4[cell] receives the offset, packed x | y << 8 | z << 16.
__global__ __launch_bounds__(256) void psh_place_kernel(
    const PairDesc *__restrict__ pairs, const int2 *__restrict__ cells, int n_buckets,
    const int32_t *__restrict__ cnt, const int32_t *__restrict__ first, const int32_t *__restrict__ members,
    const uint32_t *__restrict__ residues, const int32_t *__restrict__ n_free,
    const int32_t *__restrict__ free_list, uint32_t *__restrict__ phi4, int32_t *__restrict__ fail)
{
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b >= n_buckets) return;                       // whole wavefronts leave together
    const int2 ag = cells[b];
    const PairDesc P = pairs[ag.x];
    const int g = ag.y, cell = P.cell_base + g;
    const int c = cnt[cell], base = first[cell];
    const int m = P.m;
    const int nf = n_free[ag.x];
    int32_t *H = P.H;
    const int32_t *list = free_list + P.slot_base;
    const uint32_t h_first = residues[base];
    const int ax = h_first & 255u, ay = (h_first >> 8) & 255u, az = h_first >> 16;
    const int start = nf > 0 ? (int)(((uint32_t)g * 2654435761u) % (uint32_t)nf) : 0;

    for (int i0 = 0; i0 < nf; i0 += 64) {
        if (psh_peek(&fail[P.pair_id])) return;       // the pair is lost anyway
        const int i = i0 + lane;
        bool room = i < nf;
        int ox = 0, oy = 0, oz = 0;
        if (room) {
            int w = start + i; if (w >= nf) w -= nf;
            const int e = list[w];
            room = psh_peek(H + e) == -1;
            if (room) {
                const int sx = e / (m * m), sy = (e / m) % m, sz = e % m;
                ox = sx - ax; if (ox < 0) ox += m;
                oy = sy - ay; if (oy < 0) oy += m;
                oz = sz - az; if (oz < 0) oz += m;
                for (int k = 1; k < c && room; ++k)
                    room = psh_peek(H + psh_slot_of(residues[base + k], ox, oy, oz, m)) == -1;
            }
        }
        unsigned long long cand = __ballot(room);
        while (cand) {                                // wave-uniform loop
            const int j = __builtin_ctzll(cand);
            cand &= cand - 1;
            int won = 0;
            if (lane == j) {
                int got = 0;
                bool twice = false;     // two voxels of the bucket on one slot: no offset can separate them
                for (int k = 0; k < c && got == k; ++k) {
                    const int32_t old = atomicCAS(H + psh_slot_of(residues[base + k], ox, oy, oz, m), -1, members[base + k]);
                    if (old == -1) got = k + 1;
                    else for (int kk = 0; kk < k; ++kk) twice |= old == members[base + kk];
                }
                if (twice) { fail[P.pair_id] = 1; won = 1; }
                if (got == c) {
                    for (int k = 0; k < c; ++k) {
                        const int32_t *p = P.coords + 3 * (int64_t)members[base + k];
                        uint16_t *tag = P.T + 3 * (int64_t)psh_slot_of(residues[base + k], ox, oy, oz, m);
                        tag[0] = (uint16_t)p[0]; tag[1] = (uint16_t)p[1]; tag[2] = (uint16_t)p[2];
                    }
                    phi4[cell] = (uint32_t)ox | ((uint32_t)oy << 8) | ((uint32_t)oz << 16);
                    won = 1;
                } else {
                    for (int k = 0; k < got; ++k)     // give the claimed slots back
                        atomicExch(H + psh_slot_of(residues[base + k], ox, oy, oz, m), -1);
                }
            }
            if (__ballot(won)) return;
        }
    }
    if (lane == 0) fail[P.pair_id] = 1;
}

// Buckets of one voxel: the i-th of a table takes the i-th entry of its (fresh) free-slot list.
// Nothing else writes H during this launch.  One thread per offset cell.
__global__ __launch_bounds__(256) void psh_place_single_kernel(
    const PairDesc *__restrict__ pairs, const int32_t *__restrict__ cnt, const int32_t *__restrict__ first,
    const int32_t *__restrict__ members, const uint32_t *__restrict__ residues, const int32_t *__restrict__ n_free,
    const int32_t *__restrict__ free_list, int32_t *__restrict__ rank, uint32_t *__restrict__ phi4,
    int32_t *__restrict__ fail)
{
    const PairDesc P = pairs[blockIdx.y];
    const int g = blockIdx.x * 256 + threadIdx.x;
    if (g >= P.r * P.r * P.r) return;
    const int cell = P.cell_base + g;
    if (cnt[cell] != 1) return;
    const int i = atomicAdd(&rank[blockIdx.y], 1);
    if (i >= n_free[blockIdx.y]) { fail[P.pair_id] = 1; return; }   // cannot happen while m^3 > n
    const int e = free_list[P.slot_base + i];
    const int m = P.m;
    const uint32_t h = residues[first[cell]];
    const int32_t v = members[first[cell]];
    int ox = e / (m * m) - (int)(h & 255u); if (ox < 0) ox += m;
    int oy = (e / m) % m - (int)((h >> 8) & 255u); if (oy < 0) oy += m;
    int oz = e % m - (int)(h >> 16); if (oz < 0) oz += m;
    P.H[e] = v;
    const int32_t *p = P.coords + 3 * (int64_t)v;
    uint16_t *tag = P.T + 3 * (int64_t)e;
    tag[0] = (uint16_t)p[0]; tag[1] = (uint16_t)p[1]; tag[2] = (uint16_t)p[2];
    phi4[cell] = (uint32_t)ox | ((uint32_t)oy << 8) | ((uint32_t)oz << 16);
}

// One level's packed lookup records, model indices and byte offset table from H*, T* and the
// per-pair offset words.  grid.y = model.
struct PackDesc {
    const uint32_t *phi_src;  // this pair's offset words of its successful attempt
    int32_t m3, r3, M, R;     // sizes and bases inside the level's super tables
};

__global__ __launch_bounds__(256) void psh_pack_kernel(const PackDesc *__restrict__ desc, const int32_t *__restrict__ H,
                                                       const uint16_t *__restrict__ T, uint32_t *__restrict__ slot3,
                                                       int32_t *__restrict__ V, uint32_t *__restrict__ phi4,
                                                       uint8_t *__restrict__ Phi)
{
    const PackDesc D = desc[blockIdx.y];
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < D.m3) {
        const int64_t q = (int64_t)D.M + i;
        slot3[SLOT_WORDS * q + 0] = (uint32_t)H[q];
        slot3[SLOT_WORDS * q + 1] = (uint32_t)T[3 * q] | ((uint32_t)T[3 * q + 1] << 16);
        slot3[SLOT_WORDS * q + 2] = (uint32_t)T[3 * q + 2];
        if (SLOT_WORDS > 3) slot3[SLOT_WORDS * q + 3] = 0u;
        V[q] = (int32_t)blockIdx.y;
    }
    if (i < D.r3) {
        const uint32_t w = D.phi_src[i];
        const int64_t q = (int64_t)D.R + i;
        phi4[q] = w;
        Phi[3 * q + 0] = (uint8_t)(w & 255u); Phi[3 * q + 1] = (uint8_t)((w >> 8) & 255u); Phi[3 * q + 2] = (uint8_t)((w >> 16) & 255u);
    }
}

}  // namespace hch
