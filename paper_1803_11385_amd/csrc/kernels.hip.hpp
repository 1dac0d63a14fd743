// Device kernels of the H-CNN hot path for gfx950 (wave64, MFMA).
//
// Everything here works on the voxel-major layout: feature rows X[N][c], neighbour index
// rows nbr[N][27], column matrix col[N][27*c].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hch {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte unit of anything

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin.  Kernels whose
// neighbouring tiles touch the same memory launch 8*per_xcd workgroups and use this mapping
// so that every XCD works on one contiguous range of tiles.
constexpr unsigned NUM_XCD = 8;
__device__ __forceinline__ unsigned xcd_tile(unsigned bid, unsigned per_xcd)
{
    return (bid % NUM_XCD) * per_xcd + bid / NUM_XCD;
}

// Kernels that leave out taps walk the tiles of the pattern order, in which equal neighbour
// patterns lie together: contiguous ranges per XCD would give one XCD all the dense patterns, plain
// round-robin makes every XCD fetch every row.  In between: chunks of `chunk` consecutive tiles
// (neighbours in space as far as the order allows) go to the XCDs in turn.  The grid holds a
// multiple of 8*chunk workgroups; tiles past the last one are skipped by the caller.
__device__ __forceinline__ unsigned xcd_chunk_tile(unsigned bid, unsigned chunk)
{
    const unsigned x = bid % NUM_XCD, q = bid / NUM_XCD;
    return ((q / chunk) * NUM_XCD + x) * chunk + q % chunk;
}
// Tiles per chunk when a workgroup computes `group` of `tiles64` 64-row tiles: 16 tiles' worth of
// rows; on small levels 1, which is plain round-robin (few chunks per XCD would leave some XCDs
// with a chunk more than others).  Host and kernels derive the chunk, and the host the grid from
// it, with this one function.
__host__ __device__ __forceinline__ unsigned skip_chunk(unsigned tiles64, unsigned group)
{
    return tiles64 >= 512u ? 16u / group : 1u;
}
// workgroups to launch for `blocks` workgroups' worth of tiles: whole rounds of chunks
__host__ __device__ __forceinline__ unsigned skip_grid(unsigned blocks, unsigned chunk)
{
    const unsigned round = NUM_XCD * chunk;
    return chunk > 1u ? (blocks + round - 1) / round * round : blocks;
}

// Where there is nothing to load (an empty neighbour, a unit of a tile outside its matrix) the
// kernels load from these constants instead (16 bytes of zeros, an index of -1): loads stay
// unconditional, so a thread issues all of them back to back and nothing waits on a branch.
__device__ __attribute__((aligned(16))) uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};   // never written
__device__ int32_t g_minus1 = -1;                                                   // never written

// ---------------------------------------------------------------------------------------
// PSH lookup (paper Section 3.1, Eq.1; super tables Eq.4-6)
// ---------------------------------------------------------------------------------------

// Device view of one level of the mini-batch super-PSH.  The lookup kernels read packed
// copies of the paper's tables: one 16-byte record per hash slot (a record never straddles a
// cache line, so a probe is exactly one cache access)
//   slot3[4s] = H*[s],  slot3[4s+1] = T*[s].x | T*[s].y << 16,  slot3[4s+2] = T*[s].z,  slot3[4s+3] = 0
// and one 32-bit word per offset cell, phi4[c] = Phi*[c].x | .y << 8 | .z << 16.
// Prefix arrays are 32-bit on the device (the host checks that they fit).
constexpr int SLOT_WORDS = 4;
struct PshView {
    const uint32_t *slot3;  // [M_total][SLOT_WORDS]
    const uint32_t *phi4;   // [R_total]
    const int32_t *mbar;    // [b]
    const int32_t *rbar;    // [b]
    const int32_t *M;       // [b+1]
    const int32_t *R;       // [b+1]
    const int32_t *N;       // [b+1]
    int32_t ubar;
};

// residues of q-1, q, q+1 modulo d, given q mod d
__device__ __forceinline__ void residues3(unsigned q_mod, unsigned d, unsigned out[3])
{
    out[0] = q_mod == 0 ? d - 1 : q_mod - 1;
    out[1] = q_mod;
    out[2] = q_mod + 1 == d ? 0 : q_mod + 1;
}

// A probe in two steps, so that a thread can have the loads of many probes in flight at once.
// Step 1: the offset cell of a position with residues (xr,yr,zr) mod r (Eq.4).
__device__ __forceinline__ uint32_t psh_offset(const PshView &L, unsigned Rv, unsigned r,
                                               unsigned xr, unsigned yr, unsigned zr)
{
    return L.phi4[Rv + (xr * r + yr) * r + zr];
}
// Step 2: the slot record of a position with residues (xm,ym,zm) mod m, given its offset cell
// (Eq.1, Eq.5).
__device__ __forceinline__ unsigned psh_slot_index(unsigned Mv, unsigned m, uint32_t ph,
                                                   unsigned xm, unsigned ym, unsigned zm)
{
    unsigned hx = xm + (ph & 255u);         if (hx >= m) hx -= m;
    unsigned hy = ym + ((ph >> 8) & 255u);  if (hy >= m) hy -= m;
    unsigned hz = zm + ((ph >> 16) & 255u); if (hz >= m) hz -= m;
    return Mv + (hx * m + hy) * m + hz;
}
__device__ __forceinline__ const uint32_t *psh_slot(const PshView &L, unsigned Mv, unsigned m, uint32_t ph,
                                                    unsigned xm, unsigned ym, unsigned zm)
{
    return L.slot3 + (size_t)SLOT_WORDS * (size_t)psh_slot_index(Mv, m, ph, xm, ym, zm);
}
// the record itself: one aligned 16-byte load
// (the three words in use, as a 12-byte load of the 16-byte aligned record: a register that a load
// fills and nothing reads is handed out again at once, and whoever gets it must wait for the load)
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
__device__ __forceinline__ u32x3 psh_record(const uint32_t *rec) { return *reinterpret_cast<const u32x3 *>(rec); }
// Step 3: the local data index if the record is occupied and tagged with (x,y,z), else -1
// (Section 3.1: redundant slot, or a slot that belongs to another position).
__device__ __forceinline__ int32_t psh_match(uint32_t h, uint32_t xy, uint32_t zz,
                                             unsigned x, unsigned y, unsigned z)
{
    const bool hit = ((int32_t)h >= 0) & (xy == (x | (y << 16))) & (zz == z);
    return hit ? (int32_t)h : -1;
}

// All levels of a hierarchy, as one kernel argument: the index-list kernels cover every
// (level, model) in a single launch.  Work is cut into tiles of 256 voxels of one model at one
// level; tile_prefix[e] = number of tiles before entry e = level*batch + model (level-major),
// so a workgroup finds its entry by a short binary search with wave-uniform loads.
constexpr int MAX_LEVELS = 16;
struct LevelSet {
    PshView view[MAX_LEVELS];
    const int32_t *coords[MAX_LEVELS];
    int32_t *nbr[MAX_LEVELS];
    int32_t *child[MAX_LEVELS];      // children (at level l-1) of level l's voxels; null for l = 0
    uint32_t *mask27[MAX_LEVELS];    // per voxel: bit k set iff neighbour k exists
    // inputs of the counting sort that puts every level's voxels into pattern order (see
    // pattern_key): one key per voxel (level l's voxels at sort_off[l] ...) and one histogram of
    // the keys per 256-voxel tile of the index-list kernels
    uint8_t *sort_key;
    int32_t *tile_hist;              // level l at hist_off[l]: [PATTERN_BINS][tiles of the level], key-major
    int32_t sort_off[MAX_LEVELS];
    int32_t hist_off[MAX_LEVELS];
    int32_t level_tiles[MAX_LEVELS]; // 256-voxel tiles of the index-list kernels at level l
    int32_t level_tile0[MAX_LEVELS]; // flat number of the level's first tile
    int32_t batch;
};

// Which neighbours a surface voxel has depends on the local orientation of the surface.  The key
// has one bit for each of the 6 pairs of opposite edge-adjacent neighbours (two coordinates
// differ; taps k and 26-k): set if either of the pair exists.  Voxels ordered by this key come in
// runs with similar neighbour patterns, and a tile of consecutive rows of that order lacks most
// of the taps its voxels lack: the fused products work on such tiles and skip those taps.
constexpr int PATTERN_BINS = 64;
__device__ __forceinline__ uint32_t pattern_key(uint32_t mask27)
{
    uint32_t key = 0;
    // edge-adjacent taps below the centre: 1, 3, 5, 7, 9, 11
#pragma unroll
    for (int k = 1; k < 13; k += 2) key = (key << 1) | (((mask27 >> k) | (mask27 >> (26 - k))) & 1u);
    return key;
}

__device__ __forceinline__ int find_entry(const int32_t *__restrict__ prefix, int n_entries, int tile)
{
    int lo = 0, hi = n_entries;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

// "Pre-stored neighbour information": for every voxel the global data indices of its 27
// neighbours p + (dx,dy,dz), tap k = (dx+1)*9 + (dy+1)*3 + (dz+1), or -1 (empty, or outside
// the grid).  This is the index side of the stride-1 traversal of Algorithm 1.
// One thread per voxel: the six residues are computed once and stepped to the neighbours.  Tiles
// [tile_first, tile_first + n_tiles) are processed, numbered XCD-contiguously: the tiles of one
// model (whose tables are a few hundred KB) then stay in one XCD's L2.
//
// A probe is two dependent loads, the offset cell (Eq.4) and the slot record (Eq.5), and the
// kernel is bound by the number of such cache accesses, not by bytes.  The offset cells a tile
// needs are the planes x' mod r of Phi for x' in [xmin - 1, xmax + 1] over the tile's voxels; when
// these fit (a tile of voxels that lie close together in x: always the case for data ordered by
// position, and for small tables) they are copied to LDS once, with coalesced loads, and the
// offset reads of every voxel come from there; otherwise the cells are read from memory as the
// slot records are.  The centre tap is the voxel itself; lanes whose voxels are z-neighbours hand
// each other results (below), so a voxel makes 8 to 26 probes.  Results are kept in registers until
// all probes of the workgroup are done, then go through the same LDS space so that the rows are
// written coalesced.
constexpr int NBR_LDS_WORDS = 256 * 27;
__global__ __launch_bounds__(256) void neighbour_kernel(
    LevelSet S, const int32_t *__restrict__ tile_prefix, int n_entries, int tile_first, unsigned n_tiles)
{
    __shared__ uint32_t lds[NBR_LDS_WORDS];          // offset planes first, the 256 x 27 result tile afterwards
    __shared__ int32_t xrange[8];
    __shared__ int32_t hist[PATTERN_BINS];
    const unsigned t = xcd_tile(blockIdx.x, gridDim.x / NUM_XCD);
    if (t >= n_tiles) return;
    const int flat = tile_first + (int)t;
    const int e = find_entry(tile_prefix, n_entries, flat);
    const int lev = e / S.batch, v = e - lev * S.batch;
    const PshView &L = S.view[lev];
    const int32_t base = L.N[v];
    const int32_t n = L.N[v + 1] - base;
    const int32_t blk0 = (flat - tile_prefix[e]) * 256;
    const int32_t i = blk0 + threadIdx.x;
    const bool live = i < n;
    const unsigned m = (unsigned)L.mbar[v], r = (unsigned)L.rbar[v];
    const unsigned Mv = (unsigned)L.M[v], Rv = (unsigned)L.R[v], u = (unsigned)L.ubar;
    unsigned x = 0, y = 0, z = 0;
    if (live) {
        const int32_t *p = S.coords[lev] + 3 * (int64_t)(base + i);
        x = (unsigned)p[0]; y = (unsigned)p[1]; z = (unsigned)p[2];
    }
    // smallest and largest x of the tile
    int xlo = live ? (int)x : 0x7fffffff, xhi = live ? (int)x : -1;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        xlo = min(xlo, __shfl_xor(xlo, d));
        xhi = max(xhi, __shfl_xor(xhi, d));
    }
    if ((threadIdx.x & 63) == 0) { xrange[threadIdx.x >> 6] = xlo; xrange[4 + (threadIdx.x >> 6)] = xhi; }
    if (threadIdx.x < PATTERN_BINS) hist[threadIdx.x] = 0;
    __syncthreads();
    xlo = min(min(xrange[0], xrange[1]), min(xrange[2], xrange[3]));
    xhi = max(max(xrange[4], xrange[5]), max(xrange[6], xrange[7]));
    if (!live) x = (unsigned)xlo;                      // lanes past the end: a position whose offset plane is staged
    // planes of Phi to stage: residues res0, res0 + 1, ... (mod r) of x' = xlo - 1 .. xhi + 1
    const unsigned r2 = r * r;
    const unsigned planes = min((unsigned)(xhi - xlo + 3), r);
    const bool staged = planes * r2 <= (unsigned)NBR_LDS_WORDS;
    const unsigned xlo_r = (unsigned)xlo % r;
    const unsigned res0 = xlo_r == 0 ? r - 1 : xlo_r - 1;
    if (staged) {
        unsigned res = res0;
        for (unsigned pl = 0; pl < planes; ++pl) {
            const uint32_t *src = L.phi4 + Rv + res * r2;
            for (unsigned q = threadIdx.x; q < r2; q += 256) lds[pl * r2 + q] = src[q];
            if (++res == r) res = 0;
        }
    }
    __syncthreads();

    // Probes run in three rounds of 9 (dx, dy) columns each: dz = 0 first, then dz = -1 and dz = +1.
    // Between them neighbouring lanes exchange results: when the voxel of the next lane sits at
    // (x, y, z+1) -- the usual case for data ordered by position, checked on the coordinates, not
    // assumed -- its dz = 0 results ARE this voxel's dz = +1 results (and the other way round for
    // the lane before), every one of them the outcome of a hash probe.  A lane that got a round's
    // results this way points its loads of that round at the first record of the model's table
    // instead: same instructions, one cache line for all such lanes of a wavefront (the number of
    // requests is what bounds this kernel).  Lanes past the end of the model do so in every round.
    int32_t out[27];
    {
        unsigned xm[3], ym[3], zm[3], xr[3], yr[3], zr[3];
        residues3(x % m, m, xm); residues3(y % m, m, ym); residues3(z % m, m, zm);
        residues3(x % r, r, xr); residues3(y % r, r, yr); residues3(z % r, r, zr);
        unsigned plane[3];                               // where the staged plane of x-1, x, x+1 starts in LDS
#pragma unroll
        for (int a = 0; a < 3; ++a) plane[a] = (xr[a] >= res0 ? xr[a] - res0 : xr[a] + r - res0) * r2;
        // Positions outside the grid are probed too (their residues are valid table coordinates)
        // and discarded afterwards, so there is no branch between the loads of a round.
        // step 2 and 3 of a round: 9 record loads back to back, then the comparisons
        auto records = [&](const int dzi, const bool need, const uint32_t *ph) {
            uint32_t rh[9], rxy[9], rz[9];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                if (dzi == 1 && q == 4) continue;        // the voxel itself
                unsigned slot = psh_slot_index(Mv, m, ph[q], xm[q / 3], ym[q % 3], zm[dzi]);
                asm("" : "+v"(slot));                    // computed by every lane: the choice below stays a select
                // a lane that does not need the record reads the table's first one (one line for all such lanes)
                const u32x3 rec = psh_record(L.slot3 + (size_t)SLOT_WORDS * (size_t)(need ? slot : Mv));
                rh[q] = rec[0]; rxy[q] = rec[1]; rz[q] = rec[2];
            }
            __builtin_amdgcn_sched_barrier(0);           // all loads of the round issued before anything uses one
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                if (dzi == 1 && q == 4) { out[13] = base + i; continue; }
                const unsigned qx = x + q / 3 - 1, qy = y + q % 3 - 1, qz = z + dzi - 1;   // wrap below 0
                const int32_t h = psh_match(rh[q], rxy[q], rz[q], qx, qy, qz);
                const bool inside = (qx < u) & (qy < u) & (qz < u);
                if (need) out[q * 3 + dzi] = (inside & (h >= 0)) ? base + h : -1;       // Eq.6
            }
        };
        // step 1, the offset cells: from the staged planes, or from memory
        auto round_staged = [&](const int dzi, const bool need) {
            uint32_t ph[9];
#pragma unroll
            for (int q = 0; q < 9; ++q) ph[q] = lds[plane[q / 3] + yr[q % 3] * r + zr[dzi]];
            records(dzi, need, ph);
        };
        auto round_memory = [&](const int dzi, const bool need) {
            uint32_t ph[9];
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                unsigned cell = Rv + (xr[q / 3] * r + yr[q % 3]) * r + zr[dzi];
                asm("" : "+v"(cell));
                ph[q] = L.phi4[need ? cell : Rv];
            }
            records(dzi, need, ph);
        };
        bool above = false, below = false;
        auto exchange = [&]() {
            const int ln = threadIdx.x & 63;
            const unsigned nx = (unsigned)__shfl_down((int)x, 1), ny = (unsigned)__shfl_down((int)y, 1), nz = (unsigned)__shfl_down((int)z, 1);
            above = live & (ln < 63) & (i + 1 < n) & (nx == x) & (ny == y) & (nz == z + 1u);
            below = (__shfl_up((int)above, 1) != 0) & (ln > 0);
#pragma unroll
            for (int q = 0; q < 9; ++q) {
                const int32_t mid = out[q * 3 + 1];
                const int32_t up = __shfl_down(mid, 1), dn = __shfl_up(mid, 1);
                if (above) out[q * 3 + 2] = up;
                if (below) out[q * 3 + 0] = dn;
            }
        };
#pragma unroll
        for (int k = 0; k < 27; ++k) out[k] = -1;
        // the two ways to read the offset cells never share a basic block: the waits of the one
        // with loads from memory would otherwise land between the record loads of the other
        if (staged) {
            round_staged(1, live);
            exchange();
            round_staged(0, live & !below);
            round_staged(2, live & !above);
        } else {
            round_memory(1, live);
            exchange();
            round_memory(0, live & !below);
            round_memory(2, live & !above);
        }
    }
    __syncthreads();                                  // every thread is done with the offset planes
    if (live) {
        int32_t *row = reinterpret_cast<int32_t *>(lds) + threadIdx.x * 27;
        uint32_t mask = 0;
#pragma unroll
        for (int k = 0; k < 27; ++k) { row[k] = out[k]; mask |= (uint32_t)(out[k] >= 0) << k; }
        S.mask27[lev][base + i] = mask;
        const uint32_t key = pattern_key(mask);
        S.sort_key[S.sort_off[lev] + base + i] = (uint8_t)key;
        atomicAdd(&hist[key], 1);
    }
    __syncthreads();
    const int32_t cnt = min(256, n - blk0) * 27;
    int32_t *dst = S.nbr[lev] + (int64_t)(base + blk0) * 27;
    const int32_t *tile = reinterpret_cast<const int32_t *>(lds);
    for (int q = threadIdx.x; q < cnt; q += 256) dst[q] = tile[q];
    if (threadIdx.x < PATTERN_BINS)
        S.tile_hist[S.hist_off[lev] + (int64_t)threadIdx.x * S.level_tiles[lev] + (flat - S.level_tile0[lev])] = hist[threadIdx.x];
}

// Counting sort of every level's voxels by pattern key, stable (voxels with equal keys keep
// their data order, so the order is the same from run to run), in two steps after the
// index-list kernel has left one key per voxel and one histogram per tile.
//
// Step 1, one workgroup per (key, level): turns the tile histograms into offsets.  Sorted position
// of a voxel = sort_off[level] + (voxels of the level with a smaller key) + (voxels with the same
// key in earlier tiles) + (voxels with the same key earlier in its tile).  The histograms are
// stored key-major, so the third term is an exclusive prefix sum along one row, which this
// kernel computes in place; the row's total goes to key_total[level][key], from which step 2
// takes the second term.
__global__ __launch_bounds__(256) void pattern_scan_kernel(LevelSet S, int32_t *__restrict__ key_total, int level_first)
{
    __shared__ int32_t sums[256];
    const int lev = level_first + blockIdx.y, key = blockIdx.x;
    const int T = S.level_tiles[lev];
    int32_t *row = S.tile_hist + S.hist_off[lev] + (int64_t)key * T;
    const int per = (T + 255) / 256;
    const int a = min(T, (int)threadIdx.x * per), b = min(T, a + per);
    int32_t sum = 0;
    for (int t = a; t < b; ++t) sum += row[t];
    sums[threadIdx.x] = sum;
    __syncthreads();
    // exclusive prefix of the 256 stretch sums (Hillis-Steele in LDS)
    for (int o = 1; o < 256; o <<= 1) {
        const int32_t add = (int)threadIdx.x >= o ? sums[threadIdx.x - o] : 0;
        __syncthreads();
        sums[threadIdx.x] += add;
        __syncthreads();
    }
    int32_t run = sums[threadIdx.x] - sum;
    for (int t = a; t < b; ++t) {
        const int32_t c = row[t];
        row[t] = run;
        run += c;
    }
    if (threadIdx.x == 255) key_total[lev * PATTERN_BINS + key] = sums[255];
}

// Step 2, one workgroup per tile of the index-list kernels: every voxel finds its rank among the
// voxels of its tile with the same key (lanes with the same key through six ballots, earlier
// wavefronts through LDS) and writes its data index to its sorted position.
__global__ __launch_bounds__(256) void pattern_scatter_kernel(
    LevelSet S, const int32_t *__restrict__ tile_prefix, int n_entries, int tile_first, unsigned n_tiles,
    const int32_t *__restrict__ key_total, int32_t *__restrict__ order)
{
    __shared__ int32_t wcnt[4][PATTERN_BINS];
    __shared__ int32_t below[PATTERN_BINS];
    const unsigned t = blockIdx.x;
    if (t >= n_tiles) return;
    const int flat = tile_first + (int)t;
    const int e = find_entry(tile_prefix, n_entries, flat);
    const int lev = e / S.batch, v = e - lev * S.batch;
    const int32_t base = S.view[lev].N[v];
    const int32_t n = S.view[lev].N[v + 1] - base;
    const int32_t i = (flat - tile_prefix[e]) * 256 + threadIdx.x;
    const bool live = i < n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t key = live ? S.sort_key[S.sort_off[lev] + base + i] : 0u;
    wcnt[wave][lane] = 0;
    if (wave == 0) {                       // voxels of the level with a smaller key
        const int32_t total = key_total[lev * PATTERN_BINS + lane];
        int32_t incl = total;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int32_t up = __shfl_up(incl, o);
            if (lane >= o) incl += up;
        }
        below[lane] = incl - total;
    }
    // lanes of this wavefront with the same key (dead lanes match nobody)
    unsigned long long same = __ballot(live);
#pragma unroll
    for (int b = 0; b < 6; ++b) {
        const unsigned long long bal = __ballot((key >> b) & 1u);
        same &= ((key >> b) & 1u) ? bal : ~bal;
    }
    const int before = __builtin_amdgcn_mbcnt_hi((unsigned)(same >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)same, 0u));
    if (live && before == 0) wcnt[wave][key] = __popcll(same);        // one lane per key present
    __syncthreads();
    if (live) {
        int32_t pos = S.sort_off[lev] + below[key] + before +
                      S.tile_hist[S.hist_off[lev] + (int64_t)key * S.level_tiles[lev] + (flat - S.level_tile0[lev])];
        for (int w = 0; w < wave; ++w) pos += wcnt[w][key];
        order[pos] = base + i;
    }
}


// dst[t][i] = src[i][t] for an index list src[n][taps] (taps <= 27 here): the tap-major copy of
// the neighbour lists.  256 rows per workgroup through LDS, both sides coalesced.
__global__ __launch_bounds__(256) void index_transpose_kernel(
    const int32_t *__restrict__ src, int32_t *__restrict__ dst, int64_t n, int taps)
{
    __shared__ int32_t tile[256 * 27];
    const int64_t r0 = (int64_t)blockIdx.x * 256;
    const int rows = (int)min((int64_t)256, n - r0);
    for (int q = threadIdx.x; q < rows * taps; q += 256) tile[q] = src[r0 * taps + q];
    __syncthreads();
    if ((int)threadIdx.x < rows)
        for (int t = 0; t < taps; ++t) dst[(int64_t)t * n + r0 + threadIdx.x] = tile[threadIdx.x * taps + t];
}

// Tap masks of the tiles of the pattern order: tile b of level l covers rows 64b .. 64b+63 of the
// level's sorted voxel list `order`, and bit k of its mask says whether any of them has
// neighbour k.  One wavefront per tile; tiles of all levels of the range in one launch
// (tile_prefix[l - l0] = tiles before level l).
struct TileMaskArgs {
    const uint32_t *mask27[MAX_LEVELS];
    uint32_t *tile_mask[MAX_LEVELS];
    const int32_t *order[MAX_LEVELS];
    int32_t n[MAX_LEVELS];
    int32_t tile_prefix[MAX_LEVELS + 1];
    int32_t n_levels;
};
constexpr int PATTERN_TILE = 64;
__global__ __launch_bounds__(256) void tile_mask_kernel(TileMaskArgs A)
{
    const int flat = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (flat >= A.tile_prefix[A.n_levels]) return;
    int l = 0;
    while (l + 1 < A.n_levels && A.tile_prefix[l + 1] <= flat) ++l;
    const int b = flat - A.tile_prefix[l];
    const int r = b * PATTERN_TILE + lane;
    uint32_t m = r < A.n[l] ? A.mask27[l][A.order[l][r]] : 0u;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m |= (uint32_t)__shfl_xor((int)m, d);
    if (lane == 0) A.tile_mask[l][b] = m;
}

// For every coarse voxel the global data indices, at the next finer level, of its 8 children
// 2p + (dx,dy,dz), k = dx*4 + dy*2 + dz, or -1: the stride-2, F = 2, no-padding traversal of
// Algorithm 1 (receptive field [2p, 2p+1]^3).  Same tiling as above; entries of level 0 have no
// tiles in this kernel's prefix.
__global__ __launch_bounds__(256) void child_kernel(
    LevelSet S, const int32_t *__restrict__ tile_prefix, int n_entries, int tile_first, unsigned n_tiles)
{
    const unsigned t = xcd_tile(blockIdx.x, gridDim.x / NUM_XCD);
    if (t >= n_tiles) return;
    const int flat = tile_first + (int)t;
    const int e = find_entry(tile_prefix, n_entries, flat);
    const int lev = e / S.batch, v = e - lev * S.batch;      // lev >= 1
    const PshView &Lf = S.view[lev - 1];
    const int32_t *Nc = S.view[lev].N;
    const int32_t cbase = Nc[v];
    const int32_t n = Nc[v + 1] - cbase;
    const int32_t i = (flat - tile_prefix[e]) * 256 + threadIdx.x;
    if (i >= n) return;
    const unsigned m = (unsigned)Lf.mbar[v], r = (unsigned)Lf.rbar[v];
    const unsigned Mv = (unsigned)Lf.M[v], Rv = (unsigned)Lf.R[v];
    const int32_t fbase = Lf.N[v];
    const int32_t *p = S.coords[lev] + 3 * (int64_t)(cbase + i);
    const unsigned x = 2u * (unsigned)p[0], y = 2u * (unsigned)p[1], z = 2u * (unsigned)p[2];
    unsigned xm[2], ym[2], zm[2], xr[2], yr[2], zr[2];
    xm[0] = x % m; xm[1] = xm[0] + 1 == m ? 0 : xm[0] + 1;
    ym[0] = y % m; ym[1] = ym[0] + 1 == m ? 0 : ym[0] + 1;
    zm[0] = z % m; zm[1] = zm[0] + 1 == m ? 0 : zm[0] + 1;
    xr[0] = x % r; xr[1] = xr[0] + 1 == r ? 0 : xr[0] + 1;
    yr[0] = y % r; yr[1] = yr[0] + 1 == r ? 0 : yr[0] + 1;
    zr[0] = z % r; zr[1] = zr[0] + 1 == r ? 0 : zr[0] + 1;
    int32_t out[8];
    uint32_t ph[8], rh[8], rxy[8], rz[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) ph[q] = psh_offset(Lf, Rv, r, xr[q >> 2], yr[(q >> 1) & 1], zr[q & 1]);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const u32x3 rec = psh_record(psh_slot(Lf, Mv, m, ph[q], xm[q >> 2], ym[(q >> 1) & 1], zm[q & 1]));
        rh[q] = rec[0]; rxy[q] = rec[1]; rz[q] = rec[2];
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        // 2p + 1 < 2 * (coarse side) = fine side: always inside the grid
        const int32_t h = psh_match(rh[q], rxy[q], rz[q], x + (q >> 2), y + ((q >> 1) & 1), z + (q & 1));
        out[q] = h >= 0 ? fbase + h : -1;
    }
    int4 *dst = reinterpret_cast<int4 *>(S.child[lev] + (int64_t)(cbase + i) * 8);
    dst[0] = make_int4(out[0], out[1], out[2], out[3]);
    dst[1] = make_int4(out[4], out[5], out[6], out[7]);
}

// One probe at an arbitrary position (Eq.1, Eq.4-6 and the tag test): global data index or -1.
// The position must be inside the grid.
__device__ __forceinline__ int32_t psh_lookup(const PshView &L, int v, unsigned x, unsigned y, unsigned z)
{
    const unsigned m = (unsigned)L.mbar[v], r = (unsigned)L.rbar[v];
    const uint32_t ph = psh_offset(L, (unsigned)L.R[v], r, x % r, y % r, z % r);
    const u32x3 rec = psh_record(psh_slot(L, (unsigned)L.M[v], m, ph, x % m, y % m, z % m));
    const int32_t h = psh_match(rec[0], rec[1], rec[2], x, y, z);
    return h >= 0 ? L.N[v] + h : -1;
}

// Receptive fields of the general traversal of Algorithm 1 (kernel side F, stride S, padding P)
// between an input level and an output level S times coarser (the same level when S = 1):
// output voxel p covers the input positions lo(p) + (fx,fy,fz), 0 <= f < F, with lo(p) =
// p - (F-1)/2 per axis when S = 1 and p*S - P otherwise; row = (fx*F + fy)*F + fz.
//   TRANSPOSED = false:  out[o][row] = input data index at that position, or -1
//                        (rows owned by the output voxels; probes go to the input level's tables)
//   TRANSPOSED = true :  out[i][row] = data index of the output voxel o whose field holds input
//                        voxel i at this row, or -1 (rows owned by the input voxels; probes go to
//                        the output level's tables): the index rows of Algorithm 2 turned into
//                        a gather.
// One thread per (voxel, row); grid.y = model.  `owner` = coordinates and N* prefix of the level
// that owns the rows, `probe` = tables of the other level.
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void field_kernel(
    PshView probe, const int32_t *__restrict__ owner_coords, const int32_t *__restrict__ owner_N,
    int32_t *__restrict__ out, int F, int S, int P)
{
    const int v = blockIdx.y;
    const int F3 = F * F * F;
    const int32_t base = owner_N[v], n = owner_N[v + 1] - base;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= (int64_t)n * F3) return;
    const int i = (int)(item / F3), row = (int)(item - (int64_t)i * F3);
    const int f[3] = {row / (F * F), (row / F) % F, row % F};
    const int32_t *p = owner_coords + 3 * (int64_t)(base + i);
    int q[3];
    bool ok = true;
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        if (!TRANSPOSED) q[a] = (S == 1 ? p[a] - (F - 1) / 2 : p[a] * S - P) + f[a];
        else if (S == 1) q[a] = p[a] - f[a] + (F - 1) / 2;
        else {
            const int t = p[a] + P - f[a];
            ok &= t >= 0 && t % S == 0;
            q[a] = t / S;
        }
        ok &= q[a] >= 0 && q[a] < probe.ubar;
    }
    out[(int64_t)(base + i) * F3 + row] = ok ? psh_lookup(probe, v, (unsigned)q[0], (unsigned)q[1], (unsigned)q[2]) : -1;
}

// ---------------------------------------------------------------------------------------
// hash2col (Algorithm 1) through the pre-stored neighbour indices
// ---------------------------------------------------------------------------------------

// Tile of `tv` voxels per workgroup (tv * 27 indices staged in LDS, small enough for 8 workgroups
// per CU).  A unit is `UB`
// bytes (16: uint4, or one element); a voxel row has cu units.  Threads are split into groups
// of g = min(cu, 256) lanes; group q moves the units of one (voxel, tap) pair per step, so a
// step of the whole workgroup writes one contiguous stretch of col.
template <typename U>
__global__ __launch_bounds__(256) void hash2col_kernel(
    const U *__restrict__ X, const int32_t *__restrict__ nbr, U *__restrict__ col,
    int64_t row_begin, int64_t rows, int cu, int tv, unsigned n_tiles)
{
    extern __shared__ int32_t idx[];                  // tv * 27 indices (sized at launch)
    const unsigned tile = xcd_tile(blockIdx.x, gridDim.x / NUM_XCD);
    if (tile >= n_tiles) return;
    const int64_t r0 = (int64_t)tile * tv;
    const int nv = (int)min((int64_t)tv, rows - r0);
    const int32_t *src = nbr + (row_begin + r0) * 27;
    for (int t = threadIdx.x; t < nv * 27; t += 256) idx[t] = src[t];
    __syncthreads();
    const int g = min(cu, 256);
    const int groups = 256 / g;
    const int grp = threadIdx.x / g, lane = threadIdx.x - grp * g;
    if (grp >= groups) return;
    U *dst = col + r0 * 27 * cu;
    const U *zsrc = reinterpret_cast<const U *>(g_zero16);
    // four (voxel, tap) pairs per pass: their loads are independent and issued together
    const int total = nv * 27;
    for (int q = grp; q < total; q += 4 * groups) {
        int32_t j[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) j[t] = q + t * groups < total ? idx[q + t * groups] : -1;
        for (int u = lane; u < cu; u += g) {
            U v[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] = *(j[t] >= 0 ? X + (int64_t)j[t] * cu + u : zsrc);
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (q + t * groups < total) __builtin_nontemporal_store(v[t], &dst[(int64_t)(q + t * groups) * cu + u]);
        }
    }
}

// ---------------------------------------------------------------------------------------
// col2hash (Algorithm 2) as a gather: the 3x3x3 stride-1 neighbourhood is symmetric, so the
// voxels that hold row j as their neighbour k are exactly nbr[j][26-k].  Summing per
// destination row in tap order needs no atomics and is bit-reproducible.
// Tile of tv destination voxels per workgroup, their index rows staged in LDS; a thread owns
// (voxel, VEC-float unit) pairs.  The sources of neighbouring destinations share cache lines
// of dcol, hence the XCD-contiguous tile order.
// ---------------------------------------------------------------------------------------
template <int VEC, bool PLANES>
__global__ __launch_bounds__(256) void col2hash_kernel(
    const float *__restrict__ dcol, const int32_t *__restrict__ nbr, float *__restrict__ dX,
    int64_t n, int c, int tv, unsigned n_tiles)   // PLANES: dcol is [27][n][c] instead of [n][27*c]
{
    extern __shared__ int32_t idx[];                  // tv * 27 indices (sized at launch)
    const unsigned tile = xcd_tile(blockIdx.x, gridDim.x / NUM_XCD);
    if (tile >= n_tiles) return;
    const int64_t j0 = (int64_t)tile * tv;
    const int nv = (int)min((int64_t)tv, n - j0);
    const int32_t *src = nbr + j0 * 27;
    for (int t = threadIdx.x; t < nv * 27; t += 256) idx[t] = src[t];
    __syncthreads();
    const int cu = c / VEC;
    for (int item = threadIdx.x; item < nv * cu; item += 256) {
        const int jl = item / cu, u = item - jl * cu;
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
        const int32_t *nb = idx + jl * 27;
        const float *zsrc = reinterpret_cast<const float *>(g_zero16);
#pragma unroll 9
        for (int k = 0; k < 27; ++k) {
            const int32_t i = nb[26 - k];
            const float *s = i >= 0 ? dcol + (PLANES ? (int64_t)k * n + i : (int64_t)i * 27 + k) * c + u * VEC : zsrc;
            if constexpr (VEC == 4) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(s);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += v[e];
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] += s[e];
            }
        }
        float *d = dX + (j0 + jl) * c + u * VEC;
        if constexpr (VEC == 4) {
            *reinterpret_cast<f32x4 *>(d) = f32x4{acc[0], acc[1], acc[2], acc[3]};
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) d[e] = acc[e];
        }
    }
}

// ---------------------------------------------------------------------------------------
// fp32 GEMM on the matrix cores:  C[M x N] (+split) = A[M x K] * B[K x N]
//
// A and B hold TIN elements (float, or bf16 bit patterns widened exactly to fp32 on load); all
// arithmetic is fp32.
// A operand (AMODE):
//   A_ROWS    A(i,k) = A[i*lda + k]                       plain, k contiguous
//   A_COLS    A(i,k) = A[k*lda + i]                       plain, i contiguous
//   A_GATHER  A(i,k) = X[nbr[i][k / c]][k % c] or 0       (nbr rows of `taps` entries) row i of the column matrix of
//             hash2col (Algorithm 1) read straight from the feature rows: i = voxel,
//             k = tap*c + channel.  `A` = X, `lda` = c, `nbr` = the level's index rows.
//   A_GATHER_T  A(i,k) = X[nbr[k][i / c]][i % c] or 0     the transpose of the above:
//             i = tap*c + channel, k = voxel (reduction over the voxels, Eq.7).
// B operand:  B_KC : B(k,j) = B[j*ldb + k]   else   B(k,j) = B[k*ldb + j]
//
// Block = 256 threads = 4 waves arranged WM x (4/WM); tile BM x BN x BK, staged in LDS.  Each
// wave owns a (BM/WM) x (BN*WM/4) sub-tile as MT x NT tiles of v_mfma_f32_16x16x4_f32 and reads
// its operands from LDS with 64/128-bit accesses.  blockIdx.z selects a slice of the reduction dimension (split-K):
// slice z covers k in [z*k_per_split, (z+1)*k_per_split) and writes to C + z*c_split_stride.
// The next tile's global loads are issued before the current tile's MFMAs.
// When the rows are voxels and there are many row tiles, the host launches a multiple of 8 of
// them and blockIdx.x is remapped so that each XCD owns a contiguous range: gathered rows of
// neighbouring voxels then meet in one L2.
// ---------------------------------------------------------------------------------------
constexpr int GEMM_BK = 32;   // granularity of reduction slices (split-K)
enum { A_ROWS = 0, A_COLS = 1, A_GATHER = 2, A_GATHER_T = 3 };

// Input element types of the GEMM: float, or bfloat16 bit patterns (uint16_t) that are widened
// to fp32 on load (exact), so that all products and sums are fp32.
template <typename T> struct InElem;
template <> struct InElem<float> {
    static __device__ __forceinline__ float one(const float *p) { return *p; }
    static __device__ __forceinline__ f32x4 four(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
};
template <> struct InElem<uint16_t> {
    static __device__ __forceinline__ float one(const uint16_t *p) { return __uint_as_float((uint32_t)*p << 16); }
    static __device__ __forceinline__ f32x4 four(const uint16_t *p)
    {
        const uint2 r = *reinterpret_cast<const uint2 *>(p);
        return f32x4{__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xFFFF0000u),
                     __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xFFFF0000u)};
    }
};

template <int N> struct FVec;
template <> struct FVec<1> { typedef float type; };
template <> struct FVec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct FVec<4> { typedef float type __attribute__((ext_vector_type(4))); };
template <int N> __device__ __forceinline__ float vget(const typename FVec<N>::type &v, int i) { return v[i]; }
template <> __device__ __forceinline__ float vget<1>(const float &v, int) { return v; }

template <typename TIN, int BM, int BN, int BK, int WM, int AMODE, bool B_KC, bool VEC, bool C_PLANES, bool SKIP = false, bool LEAN = false>
__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const TIN *__restrict__ A, const TIN *__restrict__ B, float *__restrict__ C,
    const int32_t *__restrict__ nbr, int M, int N, int K, int64_t lda, int64_t ldb, int64_t ldc,
    int k_per_split, int64_t c_split_stride, int c_vec_ok, unsigned m_tiles, int c_planes, int taps,
    int b_wrap, int64_t b_tap_stride, const int32_t *__restrict__ rowmap, const uint32_t *__restrict__ tilemask,
    int flat_slices, const uint32_t *__restrict__ rowmask, int mask_c)
{
    constexpr int WN = 4 / WM;
    constexpr int WTM = BM / WM, WTN = BN / WN;       // wave tile
    constexpr int MT = WTM / 16, NT = WTN / 16;       // MFMA tiles per wave
    static_assert(WTM % 16 == 0 && WTN % 16 == 0, "wave tile must be a multiple of 16x16");
    static_assert((MT == 1 || MT == 2 || MT == 4) && (NT == 1 || NT == 2 || NT == 4), "1, 2 or 4 tiles");
    static_assert(BK % 16 == 0, "BK must be a multiple of 16");
    constexpr bool A_K_FAST = (AMODE == A_ROWS || AMODE == A_GATHER);   // k contiguous in memory
    constexpr bool GATHER = (AMODE == A_GATHER || AMODE == A_GATHER_T);
    // LDS layouts.  A with k fast in memory is kept row-major As[i][k] (a lane reads 4
    // consecutive k of its row at once); A with i fast is kept k-major As[k][i] and the MT MFMA
    // tiles of a wave take interleaved rows (tile mt: rows r*MT + mt) so that a lane reads its MT
    // operands at once.  B is always k-major Bs[k][j], tile nt taking columns r*NT + nt.
    // The +4 padding keeps rows 16-byte aligned and spreads consecutive rows over the banks.
    constexpr int AS = A_K_FAST ? BK + 4 : BM + 4;
    // B rows: +4 floats; +2 where B is transposed on its way in (B_KC) and a lane reads at most two
    // floats of a row at once: the 8 lanes that store the same column to rows 4 apart then fall
    // on 4 different banks instead of 2
    constexpr int BS = (B_KC && NT <= 2) ? BN + 2 : BN + 4;
    constexpr int A_ROWLEN = A_K_FAST ? BK : BM;      // floats per LDS row that are loaded
    constexpr int A_TOTAL = BM * BK / 4;              // float4 units in an A tile
    constexpr int A_UNITS = A_TOTAL / 256;
    constexpr int A_UPR = A_ROWLEN / 4;               // units per LDS row
    constexpr int A_RSTEP = 256 / A_UPR;              // unit uu sits in row a_row0 + uu*A_RSTEP
    constexpr int B_TOTAL = BK * BN / 4;
    constexpr int B_UNITS = (B_TOTAL + 255) / 256;
    constexpr int B_UPR = B_KC ? BK / 4 : BN / 4;
    static_assert(A_TOTAL % 256 == 0 && 256 % A_UPR == 0, "A tile must split evenly over the threads");
    typedef typename FVec<NT>::type bvec_t;

    // two LDS stages: while the MFMAs read one, the next tile is written into the other
    constexpr int A_LDS = A_K_FAST ? BM * AS : BK * AS;
    constexpr int B_LDS = BK * BS;
    __shared__ __attribute__((aligned(16))) float As2[2 * A_LDS];
    __shared__ __attribute__((aligned(16))) float Bs2[2 * B_LDS];

    // gridDim.x == m_tiles: plain order; gridDim.x > m_tiles (a multiple of 8): XCD-contiguous.
    // flat_slices > 0 (a multiple of 8): a one-dimensional grid in which workgroup b belongs to XCD
    // b % 8 (workgroups are handed to the XCDs in turn) and slice s of the reduction is computed,
    // all tiles of it, by XCD s % 8.  The tiles of a slice of the weight gradient walk through the
    // same voxels at the same time -- each gathers them for its own taps -- and so meet the rows
    // in one L2 instead of fetching them from memory once per tile.
    unsigned mtile, ntile = blockIdx.y, slice = blockIdx.z, n_slices = gridDim.z;
    if (flat_slices > 0) {
        const unsigned n_tiles = (unsigned)((N + BN - 1) / BN), tiles = m_tiles * n_tiles;
        const unsigned q = blockIdx.x / NUM_XCD, t = q % tiles;
        slice = (q / tiles) * NUM_XCD + blockIdx.x % NUM_XCD;
        mtile = t % m_tiles; ntile = t / m_tiles;
        n_slices = (unsigned)flat_slices;
    } else {
        if constexpr (SKIP) mtile = xcd_chunk_tile(blockIdx.x, skip_chunk(m_tiles * (BM / 64), BM / 64));
        else mtile = gridDim.x == m_tiles ? blockIdx.x : xcd_tile(blockIdx.x, gridDim.x / NUM_XCD);
        if (mtile >= m_tiles) return;
    }

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int li = lane & 15, lk = lane >> 4;
    const int m0 = (int)mtile * BM, n0 = (int)ntile * BN;
    const int c = (int)lda;                           // channels per tap in the gather modes
    // Tap skipping (gather along k, rows in pattern order): `rowmap` gives the voxel behind each
    // row of this product and `tilemask` the taps that the voxels of each 64-row tile have.  The
    // reduction then runs over the present taps only, k' = position in the compacted list of taps
    // * c + channel, and tapmap translates back wherever the real tap is needed: the column of the
    // index rows and the rows of the weights.
    // (SKIP: instantiated for the vector path of the gather along k only.)
    static_assert(!SKIP || (AMODE == A_GATHER && VEC), "tap skipping belongs to the gathered, vectorised product");
    constexpr bool skipping = SKIP;
    __shared__ uint8_t tapmap[SKIP ? 32 : 1];
    __shared__ int32_t rowtile[SKIP ? BM : 1];        // the voxels behind this tile's rows
    int kbeg = (int)slice * k_per_split;
    int kend = min(K, kbeg + k_per_split);
    uint32_t present = taps >= 32 ? 0xFFFFFFFFu : (1u << taps) - 1u;     // taps of the reduction, as a bit set
    if constexpr (SKIP) {
        const unsigned t64 = mtile * (BM / 64), n64 = (unsigned)((M + 63) / 64);
        present = tilemask[t64];
        if (BM == 128 && t64 + 1 < n64) present |= tilemask[t64 + 1];
        present = (uint32_t)__builtin_amdgcn_readfirstlane((int)present);    // the same for every lane: keep it scalar
        if (tid < 32) {
            // entry j: the j-th present tap; entries past the last one name tap 0, so that an
            // index load for a reduction offset past the end still reads inside the index rows
            uint32_t m = present;
            for (int q = 0; q < tid && m; ++q) m &= m - 1u;
            tapmap[tid] = m ? (uint8_t)(__ffs(m) - 1) : (uint8_t)0;
        }
        if (tid < BM) rowtile[tid] = m0 + tid < M ? rowmap[m0 + tid] : 0;
        const int Kp = __popc(present) * c;
        const int per = ((Kp + (int)n_slices - 1) / (int)n_slices + BK - 1) / BK * BK;
        kbeg = (int)slice * per;
        kend = min(Kp, kbeg + per);
        __syncthreads();
    }
    C += (int64_t)slice * c_split_stride;

    f32x4 acc[MT][NT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    // position of this thread's units inside a tile: the same column of units in every row
    const int a_col = (tid % A_UPR) * 4;              // first of 4 elements along the fast axis
    const int a_row0 = tid / A_UPR;
    const int b_col = (tid % B_UPR) * 4;
    const int b_row0 = tid / B_UPR;
    constexpr int B_RSTEP = 256 / B_UPR;
    const f32x4 zero4 = f32x4{0.f, 0.f, 0.f, 0.f};
    const TIN *zsrc = reinterpret_cast<const TIN *>(g_zero16);

    // ---- VEC: every unit is one aligned 4-element load that is either wholly inside its matrix
    // or wholly outside (the host checks that the fast dimensions are multiples of 4).  Loads
    // are unconditional -- an outside unit reads a constant block of zeros -- so that a tile's
    // loads are issued back to back, without branches and without anything waiting on them.
    // Addresses are carried from tile to tile (pointers advanced by one tile per fetch), so the
    // loop has no multiplications or divisions.
    //
    // A side.  pa[uu]: where unit uu of the next tile starts (plain modes), or the position in
    // the index rows its feature-row index is read from (gather modes).
    const TIN *pa[A_UNITS];
    const int32_t *pn[A_UNITS];
    bool a_ok[A_UNITS];                               // the unit's row (k-fast) / column (i-fast) exists
    int ka = kbeg;                                    // reduction index of the next tile's row loads
    int kn = kbeg;                                    // ... of the next tile's index loads
    // gather along k (A_GATHER): tap and channel of this thread's column, for both streams
    int tap_n = 0, cc_n = 0, cc_a = 0;
    int dtap = 0, dcc = 0;                            // one tile further along k: BK = dtap*c + dcc
    if (VEC) {
        if (AMODE == A_GATHER) {
            const int gk = kbeg + a_col;
            tap_n = gk / c; cc_n = gk - tap_n * c; cc_a = cc_n;
            dtap = BK / c; dcc = BK - dtap * c;
        }
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu) {
            const int r = a_row0 + uu * A_RSTEP;
            if (AMODE == A_ROWS) { a_ok[uu] = m0 + r < M; pa[uu] = A + (int64_t)(m0 + r) * lda + kbeg + a_col; }
            if (AMODE == A_COLS) { a_ok[uu] = m0 + a_col < M; pa[uu] = A + (int64_t)(kbeg + r) * lda + m0 + a_col; }
            if (AMODE == A_GATHER) {
                a_ok[uu] = m0 + r < M;
                int64_t vox = min(m0 + r, M - 1);     // index loads are unconditional: stay inside
                if constexpr (SKIP) vox = rowtile[r];
                pn[uu] = nbr + vox * taps;
            }
            if (AMODE == A_GATHER_T) {
                const int gi = m0 + a_col;
                const int tap = min(gi / c, taps - 1);
                cc_a = gi - (gi / c) * c;
                a_ok[uu] = gi < M; pn[uu] = nbr + tap;
            }
        }
    }
    // B side
    // b_wrap > 0 (B_KC only): the reduction axis of B is cut into runs of b_wrap elements (a
    // multiple of BK) that lie b_tap_stride apart instead of back to back: B(k, j) =
    // B[(k / b_wrap)*b_tap_stride + j*ldb + k % b_wrap].  This reads the weight tensor
    // W[27][c_in][c_out] of a convolution as the flipped, transposed matrix of its data gradient.
    const TIN *pb[B_UNITS];
    bool b_ok[B_UNITS];
    int kb = kbeg;
    int b_pos = b_wrap ? kbeg % b_wrap : 0;
    // with tap skipping the weights' rows are addressed anew for every tile: B_KC: this unit's
    // column start (pb0) plus the tap's offset; else per unit the (compacted tap, channel) of its row
    const TIN *pb0[B_UNITS];
    int b_tap = b_wrap ? kbeg / b_wrap : 0;
    int tapb[B_UNITS], ccb[B_UNITS];
    if (VEC) {
#pragma unroll
        for (int uu = 0; uu < B_UNITS; ++uu) {
            const int r = b_row0 + uu * B_RSTEP;
            if (B_KC) {
                b_ok[uu] = r < BN && n0 + r < N;
                pb0[uu] = B + (int64_t)(n0 + r) * ldb + b_col;
                pb[uu] = pb0[uu] + (b_wrap ? (int64_t)(kbeg / b_wrap) * b_tap_stride + kbeg % b_wrap : (int64_t)kbeg);
            }
            else {
                b_ok[uu] = r < BK && n0 + b_col < N;
                pb0[uu] = B + n0 + b_col;
                pb[uu] = B + (int64_t)(kbeg + r) * ldb + n0 + b_col;
                tapb[uu] = (kbeg + r) / c; ccb[uu] = (kbeg + r) - tapb[uu] * c;
            }
        }
    }

    // ---- LEAN (float operands, vector path, gather modes; A_GATHER: c a multiple of BK, so that a
    // tile lies within one tap).  A vector-ALU instruction and a matrix instruction of the same
    // SIMD do not overlap on this chip: every address computation in the loop costs matrix time,
    // 4 cycles of the 32 one instruction takes.  Here the loop computes next to nothing per lane:
    // loads go through buffer descriptors, whose range check returns zeros for anything outside
    // (no guards, no 64-bit pointers); what a tile changes is a scalar offset kept by the scalar
    // unit (the tap, the channel block, the row of the weights); per lane there remains one
    // multiply-add per gathered row -- its index times the row length.
    // Rules kept below: a scalar offset never leaves its buffer (taps are clamped to present
    // ones), so only the per-lane offset decides inside/outside; an absent neighbour (-1) gives a
    // negative, i.e. huge unsigned, per-lane offset.  Values a load past the end of a reduction
    // slice brings in are multiplied by zeros of the other operand or never multiplied.
    [[maybe_unused]] __amdgpu_buffer_rsrc_t rs_idx, rs_a, rs_b;
    [[maybe_unused]] int lv_idx[A_UNITS], lv_b[B_UNITS], lv_a = 0;     // per-lane byte offsets
    [[maybe_unused]] uint32_t rem_i = 0, rem_b = 0;                    // taps still ahead: index / B stream
    [[maybe_unused]] int cc_i = 0, cc_r = 0, cc_b = 0;                 // channel block within the tap, per stream
    [[maybe_unused]] int64_t b_tap_lo = 0;
    [[maybe_unused]] int lv_au[A_UNITS];                               // per-lane byte offsets of A without a gather
    [[maybe_unused]] int k_lean = 0, k_last = 0;                       // A_ROWS: next tile's first k, the last real tile's
    constexpr uint32_t LEAN_OUT = 0x80000000u;                          // a per-lane offset outside every buffer
    if constexpr (LEAN) {
        static_assert(VEC && !C_PLANES && sizeof(TIN) == 4, "lean loop: float operands on the vector path");
        constexpr int SRD3 = 0x00020000;                               // raw buffer of dwords, gfx9 family
        const int rowbytes = c * 4;
        rs_a = __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (int)0x80000000u, SRD3);
        if (AMODE == A_GATHER) {
            // skip the taps before this slice's first tile
            const int t0 = kbeg / c;
            uint32_t m = present;
            for (int q = 0; q < t0 && m; ++q) m &= m - 1u;
            rem_i = rem_b = m;
            cc_i = cc_r = cc_b = kbeg - t0 * c;
            rs_idx = __builtin_amdgcn_make_buffer_rsrc((void *)nbr, 0, M * taps * 4, SRD3);
            lv_a = a_col * 4;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                const int r = a_row0 + uu * A_RSTEP;
                int vox = m0 + r;
                if constexpr (SKIP) vox = rowtile[r];
                lv_idx[uu] = m0 + r < M ? vox * taps * 4 : (int)LEAN_OUT;
            }
            if (B_KC) {
                // B(k, j) = B[(k / c)*b_tap_stride + j*ldb + k % c]; with a negative tap stride the
                // buffer starts at the last tap
                b_tap_lo = b_tap_stride < 0 ? (int64_t)(taps - 1) * b_tap_stride : 0;
                rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)(B + b_tap_lo), 0,
                                                         (int)(((int64_t)(taps - 1) * (b_tap_stride < 0 ? -b_tap_stride : b_tap_stride) + (int64_t)N * ldb) * 4), SRD3);
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) {
                    const int r = b_row0 + uu * B_RSTEP;
                    lv_b[uu] = (r < BN && n0 + r < N) ? (int)(((int64_t)(n0 + r) * ldb + b_col) * 4) : (int)LEAN_OUT;
                }
            } else {
                rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)B, 0, (int)((int64_t)taps * c * ldb * 4), SRD3);
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) {
                    const int r = b_row0 + uu * B_RSTEP;
                    lv_b[uu] = (r < BK && n0 + b_col < N) ? (int)(((int64_t)r * ldb + n0 + b_col) * 4) : (int)LEAN_OUT;
                }
            }
        } else if (AMODE == A_ROWS) {
            // plain row-major A (the column matrix, or dY): the reduction offset is a scalar.  The
            // host guarantees whole tiles (K and the slices multiples of BK); a tile past the end
            // of the range, which the pipeline requests and never multiplies, re-reads the last one.
            rs_a = __builtin_amdgcn_make_buffer_rsrc((void *)A, 0, (int)((int64_t)M * lda * 4), SRD3);
            k_lean = kbeg;
            k_last = kbeg + max(0, (kend - kbeg - 1) / BK) * BK;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                const int r = a_row0 + uu * A_RSTEP;
                lv_au[uu] = m0 + r < M ? (int)(((int64_t)(m0 + r) * lda + a_col) * 4) : (int)LEAN_OUT;
            }
            rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)B, 0, (int)((int64_t)(B_KC ? N : K) * ldb * 4), SRD3);
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                const int r = b_row0 + uu * B_RSTEP;
                if (B_KC) lv_b[uu] = (r < BN && n0 + r < N) ? (int)(((int64_t)(n0 + r) * ldb + b_col) * 4) : (int)LEAN_OUT;
                else lv_b[uu] = (r < BK && n0 + b_col < N) ? (int)(((int64_t)r * ldb + n0 + b_col) * 4) : (int)LEAN_OUT;
            }
        } else if (AMODE == A_COLS) {
            // A(i, k) = A[k*lda + i], B(k, j) = B[k*ldb + j]: both described from the first to the
            // last reduction index of this slice, so the tail of the last tile reads zeros; the
            // tile's position advances in the per-lane offsets (the range check sees all of it)
            const int len = max(kend - kbeg, 0);
            rs_a = __builtin_amdgcn_make_buffer_rsrc((void *)(A + (int64_t)kbeg * lda), 0, (int)((int64_t)len * lda * 4), SRD3);
            rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)(B + (int64_t)kbeg * ldb), 0, (int)((int64_t)len * ldb * 4), SRD3);
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu)
                lv_au[uu] = m0 + a_col < M ? (int)(((int64_t)(a_row0 + uu * A_RSTEP) * lda + m0 + a_col) * 4) : (int)LEAN_OUT;
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                const int r = b_row0 + uu * B_RSTEP;
                lv_b[uu] = (r < BK && n0 + b_col < N) ? (int)(((int64_t)r * ldb + n0 + b_col) * 4) : (int)LEAN_OUT;
            }
        } else {
            // A_GATHER_T: the reduction runs over the voxels of this slice; both the index rows and
            // B are described from the slice's first voxel to its last, so the tail reads zeros
            const int len = max(kend - kbeg, 0);
            rs_idx = __builtin_amdgcn_make_buffer_rsrc((void *)(nbr + (int64_t)kbeg * taps), 0, len * taps * 4, SRD3);
            rs_b = __builtin_amdgcn_make_buffer_rsrc((void *)(B + (int64_t)kbeg * ldb), 0, (int)((int64_t)len * ldb * 4), SRD3);
            const int gi = m0 + a_col;
            const int tap = min(gi / c, taps - 1);
            lv_a = (gi - (gi / c) * c) * 4;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) lv_idx[uu] = ((a_row0 + uu * A_RSTEP) * taps + tap) * 4;
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                const int r = b_row0 + uu * B_RSTEP;
                lv_b[uu] = (r < BK && n0 + b_col < N) ? (int)(((int64_t)r * ldb + n0 + b_col) * 4) : (int)LEAN_OUT;
            }
        }
        (void)rowbytes;
    }
    auto lean_tap = [&](uint32_t rem) { return rem ? __builtin_ctz(rem) : 0; };   // clamped: never outside
    auto lean_fetch_idx = [&](int32_t *out) {
        if constexpr (LEAN) {
            const int soff = AMODE == A_GATHER ? __builtin_amdgcn_readfirstlane(lean_tap(rem_i) * 4) : 0;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                out[uu] = (int32_t)__builtin_amdgcn_raw_buffer_load_b32(rs_idx, lv_idx[uu], soff, 0);
                if (AMODE == A_GATHER_T) lv_idx[uu] += BK * taps * 4;
            }
            if (AMODE == A_GATHER) {
                cc_i += BK;
                if (cc_i >= c) { cc_i = 0; rem_i &= rem_i - 1u; }
            }
        }
    };
    auto lean_fetch = [&](const int32_t *rows, f32x4 *ra, f32x4 *rb) {
        if constexpr (LEAN && !GATHER) {
            if (AMODE == A_ROWS) {
                const int kc = min(k_lean, k_last);
                const int soff = __builtin_amdgcn_readfirstlane(kc * 4);
                const int soff_b = __builtin_amdgcn_readfirstlane(B_KC ? kc * 4 : kc * (int)ldb * 4);
#pragma unroll
                for (int uu = 0; uu < A_UNITS; ++uu)
                    ra[uu] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs_a, lv_au[uu], soff, 0));
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu)
                    rb[uu] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs_b, lv_b[uu], soff_b, 0));
                k_lean += BK;
            } else {
#pragma unroll
                for (int uu = 0; uu < A_UNITS; ++uu) {
                    ra[uu] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs_a, lv_au[uu], 0, 0));
                    lv_au[uu] += BK * (int)lda * 4;
                }
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) {
                    rb[uu] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs_b, lv_b[uu], 0, 0));
                    lv_b[uu] += BK * (int)ldb * 4;
                }
            }
        }
        if constexpr (LEAN && GATHER) {
            const int rowbytes = c * 4;
            const int soff_a = AMODE == A_GATHER ? __builtin_amdgcn_readfirstlane(cc_r * 4) : 0;
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                // index -1: a negative offset, outside the buffer, zeros
                const int off = __mul24(rows[uu], rowbytes) + lv_a;
                ra[uu] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs_a, off, soff_a, 0));
            }
            int soff_b = 0;
            if (AMODE == A_GATHER) {
                const int tap = lean_tap(rem_b);
                if (B_KC) soff_b = (int)(((int64_t)tap * b_tap_stride - b_tap_lo + cc_b) * 4);
                else soff_b = (tap * c + cc_b) * (int)ldb * 4;
                soff_b = __builtin_amdgcn_readfirstlane(soff_b);
            }
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                rb[uu] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs_b, lv_b[uu], soff_b, 0));
                if (AMODE == A_GATHER_T) lv_b[uu] += BK * (int)ldb * 4;
            }
            if (AMODE == A_GATHER) {
                cc_r += BK; if (cc_r >= c) cc_r = 0;
                cc_b += BK; if (cc_b >= c) { cc_b = 0; rem_b &= rem_b - 1u; }
            }
        }
    };

    // Gather modes, stage 1: the index of the feature row behind each unit of the next tile
    // (-1 = nothing to load).  Issued ahead of the dependent row loads of stage 2.
    auto fetch_idx = [&](int32_t *out) {
        if (!GATHER || !VEC) return;
        if constexpr (LEAN) { lean_fetch_idx(out); return; }
        // The load itself is unconditional and always inside the index rows (rows and voxels
        // clamped, tap columns valid); what lies outside the product becomes -1 afterwards.  With
        // the choice made on the address instead, the compiler put each load behind a branch.
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu) {
            if (AMODE == A_GATHER) {
                const bool ok = a_ok[uu] && kn + a_col < kend;
                int tap_col = min(tap_n, taps - 1);
                if constexpr (SKIP) tap_col = tapmap[min(tap_n, 31)];
                const int32_t j = pn[uu][tap_col];
                out[uu] = ok ? j : -1;
            } else {
                const int kv = kn + a_row0 + uu * A_RSTEP;
                const bool ok = a_ok[uu] && kv < kend;
                const int32_t j = pn[uu][(int64_t)min(kv, K - 1) * taps];
                out[uu] = ok ? j : -1;
            }
        }
        if (AMODE == A_GATHER) {
            tap_n += dtap; cc_n += dcc;
            if (cc_n >= c) { cc_n -= c; ++tap_n; }
        }
        kn += BK;
    };

    auto one = [&](const TIN *base, int64_t off, bool ok) { return ok ? InElem<TIN>::one(base + off) : 0.f; };

    // stage 2: the next tile into registers (zero outside the matrices); `rows` = the indices
    // stage 1 produced for this tile.  The generic path takes the tile's reduction index k0.
    auto fetch = [&](int k0, const int32_t *rows, f32x4 *ra, f32x4 *rb) {
        if constexpr (LEAN) { lean_fetch(rows, ra, rb); return; }
        if (VEC) {
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                if (AMODE == A_ROWS) {
                    const bool ok = a_ok[uu] && ka + a_col < kend;
                    ra[uu] = InElem<TIN>::four(ok ? pa[uu] : zsrc);
                    pa[uu] += BK;
                } else if (AMODE == A_COLS) {
                    const bool ok = a_ok[uu] && ka + a_row0 + uu * A_RSTEP < kend;
                    ra[uu] = InElem<TIN>::four(ok ? pa[uu] : zsrc);
                    pa[uu] += (int64_t)BK * lda;
                } else {
                    const int32_t j = rows[uu];
                    ra[uu] = InElem<TIN>::four(j >= 0 ? A + (uint32_t)(j * c + cc_a) : zsrc);
                }
            }
            if (AMODE == A_GATHER) { cc_a += dcc; if (cc_a >= c) cc_a -= c; }
            ka += BK;
            if constexpr (skipping) {
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) {
                    bool ok;
                    const TIN *src;
                    if (B_KC) {
                        ok = b_ok[uu] && kb + b_col < kend;
                        src = pb0[uu] + ((int64_t)tapmap[min(b_tap, 31)] * b_tap_stride + b_pos);
                    } else {
                        ok = b_ok[uu] && kb + b_row0 + uu * B_RSTEP < kend;
                        src = pb0[uu] + (int64_t)((int)tapmap[min(tapb[uu], 31)] * c + ccb[uu]) * ldb;
                        tapb[uu] += dtap; ccb[uu] += dcc;
                        if (ccb[uu] >= c) { ccb[uu] -= c; ++tapb[uu]; }
                    }
                    rb[uu] = InElem<TIN>::four(ok ? src : zsrc);
                }
                if (B_KC) { b_pos += BK; if (b_pos >= b_wrap) { b_pos -= b_wrap; ++b_tap; } }
            } else {
#pragma unroll
                for (int uu = 0; uu < B_UNITS; ++uu) {
                    bool ok;
                    if (B_KC) ok = b_ok[uu] && kb + b_col < kend;
                    else ok = b_ok[uu] && kb + b_row0 + uu * B_RSTEP < kend;
                    rb[uu] = InElem<TIN>::four(ok ? pb[uu] : zsrc);
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
            }
            kb += BK;
        } else {
            // any shape and alignment: element by element with every guard
#pragma unroll
            for (int uu = 0; uu < A_UNITS; ++uu) {
                f32x4 v = zero4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int gi, gk;
                    if (A_K_FAST) { gi = m0 + a_row0 + uu * A_RSTEP; gk = k0 + a_col + e; }
                    else { gk = k0 + a_row0 + uu * A_RSTEP; gi = m0 + a_col + e; }
                    const bool in = gi < M && gk < kend;
                    if (AMODE == A_ROWS) v[e] = one(A, (int64_t)gi * lda + gk, in);
                    else if (AMODE == A_COLS) v[e] = one(A, (int64_t)gk * lda + gi, in);
                    else if (in) {
                        const int kk = (AMODE == A_GATHER) ? gk : gi;      // column-matrix column
                        const int64_t vox = (AMODE == A_GATHER) ? gi : gk; // voxel
                        const int tap = kk / c;
                        const int32_t j = nbr[vox * taps + tap];
                        v[e] = one(A, (int64_t)j * c + (kk - tap * c), j >= 0);
                    }
                }
                ra[uu] = v;
            }
#pragma unroll
            for (int uu = 0; uu < B_UNITS; ++uu) {
                const int r = b_row0 + uu * B_RSTEP;
                f32x4 v = zero4;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (B_KC) { const int gj = n0 + r, gk = k0 + b_col + e; v[e] = one(B, (int64_t)gj * ldb + gk, r < BN && gj < N && gk < kend); }
                    else { const int gk = k0 + r, gj = n0 + b_col + e; v[e] = one(B, (int64_t)gk * ldb + gj, r < BK && gk < kend && gj < N); }
                }
                rb[uu] = v;
            }
        }
    };

    // registers -> LDS
    auto stash = [&](int stage, const f32x4 *ra, const f32x4 *rb) {
        float *As = As2 + stage * A_LDS, *Bs = Bs2 + stage * B_LDS;
#pragma unroll
        for (int uu = 0; uu < A_UNITS; ++uu)
            *reinterpret_cast<f32x4 *>(&As[(a_row0 + uu * A_RSTEP) * AS + a_col]) = ra[uu];
        constexpr bool B_EVEN = (B_TOTAL % 256 == 0);     // every thread holds B_UNITS units of the tile
#pragma unroll
        for (int uu = 0; uu < B_UNITS; ++uu) {
            const int r = b_row0 + uu * B_RSTEP;
            if (B_KC) {
                if (B_EVEN || r < BN) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) Bs[(b_col + e) * BS + r] = rb[uu][e];
                }
            } else if (B_EVEN || r < BK) {
                *reinterpret_cast<f32x4 *>(&Bs[r * BS + b_col]) = rb[uu];
            }
        }
    };

    // The wave's operands of the tile in LDS, all of them, into registers: one LDS latency per
    // tile instead of one per slab, and LDS is free again (second barrier) before the MFMAs run.
    constexpr int A_REGS = A_K_FAST ? (BK / 16) * MT : BK / 4;
    constexpr int B_REGS = A_K_FAST ? BK / 4 : BK / 4;
    typedef typename FVec<A_K_FAST ? 4 : MT>::type areg_t;
    areg_t oa[A_REGS];
    bvec_t ob[B_REGS];
    auto load_operands = [&](int stage) {
        const float *As = As2 + stage * A_LDS, *Bs = Bs2 + stage * B_LDS;
        if constexpr (A_K_FAST) {
#pragma unroll
            for (int slab = 0; slab < BK / 16; ++slab) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    oa[slab * MT + mt] = *reinterpret_cast<const areg_t *>(&As[(wm * WTM + mt * 16 + li) * AS + slab * 16 + lk * 4]);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    ob[slab * 4 + e] = *reinterpret_cast<const bvec_t *>(&Bs[(slab * 16 + lk * 4 + e) * BS + wn * WTN + li * NT]);
            }
        } else {
#pragma unroll
            for (int kk = 0; kk < BK / 4; ++kk) {
                oa[kk] = *reinterpret_cast<const areg_t *>(&As[(kk * 4 + lk) * AS + wm * WTM + li * MT]);
                ob[kk] = *reinterpret_cast<const bvec_t *>(&Bs[(kk * 4 + lk) * BS + wn * WTN + li * NT]);
            }
        }
    };
    auto multiply = [&]() {
        if constexpr (A_K_FAST) {
#pragma unroll
            for (int slab = 0; slab < BK / 16; ++slab)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            // plane-wise output: the operands change places, which transposes the
                            // 16x16 result in the registers (see the stores below)
                            if constexpr (C_PLANES)
                                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                                    vget<NT>(ob[slab * 4 + e], nt), vget<4>(oa[slab * MT + mt], e), acc[mt][nt], 0, 0, 0);
                            else
                                acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                                    vget<4>(oa[slab * MT + mt], e), vget<NT>(ob[slab * 4 + e], nt), acc[mt][nt], 0, 0, 0);
                        }
        } else {
#pragma unroll
            for (int kk = 0; kk < BK / 4; ++kk)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(
                            vget<A_K_FAST ? 4 : MT>(oa[kk], mt), vget<NT>(ob[kk], nt), acc[mt][nt], 0, 0, 0);
        }
    };

    // Software pipeline over the tiles t = 0, 1, ... of this workgroup's reduction range, one
    // barrier per tile:
    //   iteration t:  operands of t: LDS stage t%2 -> registers;  MFMAs of t;
    //                 registers(t+1) -> LDS stage (t+1)%2;  issue index loads of t+4, row loads of
    //                 t+3 into the register set just emptied;  barrier.
    // Loads are two tiles ahead of their use: a gathered row takes about as long to arrive as one
    // iteration lasts, and with one tile of lead the store to LDS kept waiting for it.  The two
    // register sets and the two index sets alternate (no copies).
    // Nothing in the loop body is conditional: every load is guarded on its own (zeros past the
    // end of the range), and with a fetch that some path skips the compiler must assume the
    // registers it stores to LDS were loaded last, and waits for ALL outstanding loads there --
    // which undoes the lead.  Tiles go in pairs (one per stage); an odd last tile follows the loop.
    f32x4 ra0[A_UNITS], rb0[B_UNITS], ra1[A_UNITS], rb1[B_UNITS];
    int32_t rx[A_UNITS] = {}, ry[A_UNITS] = {};
    auto iteration = [&](int k0, int stage, f32x4 *sa, f32x4 *sb, int32_t *use, int32_t *load) {
        load_operands(stage);
        multiply();
        stash(stage ^ 1, sa, sb);
        fetch_idx(load);
        fetch(k0 + 3 * BK, use, sa, sb);
        __syncthreads();
    };
    if (kbeg < kend) {
        // start-up: the indices of tiles 0, 1, 2 are requested together and the rows of the three
        // tiles after them, two memory latencies instead of one per tile; the order of the last
        // requests (indices of tile 3, then rows of tile 2) is the loop's, whose waits count the
        // loads issued after the one they need
        int32_t rz[A_UNITS] = {};
        fetch_idx(rx);
        fetch_idx(ry);
        fetch_idx(rz);
        fetch(kbeg, rx, ra0, rb0);
        fetch(kbeg + BK, ry, ra1, rb1);
        stash(0, ra0, rb0);
        fetch_idx(ry);
        fetch(kbeg + 2 * BK, rz, ra0, rb0);
        __syncthreads();
        int k0 = kbeg;
        for (; k0 + BK < kend; k0 += 2 * BK) {
            iteration(k0, 0, ra1, rb1, ry, rx);
            iteration(k0 + BK, 1, ra0, rb0, rx, ry);
        }
        if (k0 < kend) {
            load_operands(0);
            multiply();
        }
    }

    // D layout of v_mfma_f32_16x16x4_f32: register e of lane l holds D[4*(l/16) + e][l%16].
    // Lane li fed columns li*NT + nt of the wave's stretch to tile nt, so for one row it holds NT
    // neighbouring columns.  Rows: tile mt covers mt*16 + r (row-major A) or r*MT + mt (k-major A).
    // C_PLANES: the output is stored plane by plane, C[j / c_planes][i][j % c_planes] (a
    // lane's NT <= 4 columns start at a multiple of NT and c_planes is a multiple of 4, so they
    // share a plane); else row-major with leading dimension ldc
    // C_PLANES (row-major A only): the product was computed transposed, register e of lane l holds
    // D[l%16][4*(l/16) + e]: the 16 lanes of a group hold 16 consecutive rows of the same NT
    // columns, and a store instruction writes 16 rows x 16 bytes = 256 contiguous bytes of a plane
    // (untransposed, the rows of one instruction lie 4 apart and every 16-byte piece is a request
    // of its own: 112 -> see the measurements).
    static_assert(!C_PLANES || A_K_FAST, "plane-wise output: row-major A");
    int gj = n0 + wn * WTN + li * NT;
    int64_t row_stride = ldc, col_off = gj;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r = C_PLANES ? li : 4 * lk + e;
            const int gi = m0 + wm * WTM + (A_K_FAST ? mt * 16 + r : r * MT + mt);
            if constexpr (C_PLANES) {
                gj = n0 + wn * WTN + (4 * lk + e) * NT;
                const int pl = gj / c_planes;
                row_stride = c_planes;
                col_off = (int64_t)pl * M * c_planes + (gj - pl * c_planes);
            }
            if (gi >= M) continue;
            int64_t orow = gi;
            if constexpr (SKIP) orow = rowtile[gi - m0];
            // rowmask (the data-gradient product of the columns algorithm): columns come in groups
            // of mask_c, one group per tap, and bit t of rowmask[row] says whether the row has
            // neighbour t.  The group of a row without it would be added to nothing (Algorithm 2
            // drops it), so it is not stored either.
            if (rowmask != nullptr && !((rowmask[orow] >> (gj / mask_c)) & 1u)) continue;
            float *dst = C + orow * row_stride + col_off;
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

// Wt[k][co][ci] = W[flip ? taps-1-k : k][ci][co]: the weights of the convolution that maps
// output gradients back to the input (Eq.8).  For the 3x3x3 stride-1 neighbourhood, which is
// symmetric, the gradient is gathered through the same index rows with the taps flipped; a
// general receptive field uses its transposed index rows and the taps as they are.
template <typename T>
__global__ __launch_bounds__(256) void flip_transpose_weights_kernel(
    const T *__restrict__ W, T *__restrict__ Wt, int c_in, int c_out, int taps, int flip)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t per = (int64_t)c_in * c_out;
    if (t >= taps * per) return;
    const int k = (int)(t / per);
    const int r = (int)(t - k * per);
    const int co = r / c_in, ci = r - co * c_in;
    Wt[t] = W[((int64_t)(flip ? taps - 1 - k : k) * c_in + ci) * c_out + co];
}

// out[i] = sum_z part[z*stride + i], the slices of a split reduction, always added in the same
// order.  LANES lanes share one output: lane q adds slices q, q+LANES, ... (ascending), then the
// LANES partial sums are added in lane order.  LANES = 1: one thread per output, plain loop.
template <int LANES>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(
    const float *__restrict__ part, float *__restrict__ out, int64_t n, int splits, int64_t stride)
{
    constexpr int OUTS = 256 / LANES;
    __shared__ float sh[LANES == 1 ? 1 : LANES][OUTS + 1];
    const int ex = threadIdx.x % OUTS, zg = threadIdx.x / OUTS;
    const int64_t i = (int64_t)blockIdx.x * OUTS + ex;
    float s = 0.f;
    if (i < n)
        for (int z = zg; z < splits; z += LANES) s += part[(int64_t)z * stride + i];
    if (LANES == 1) {
        if (i < n) out[i] = s;
        return;
    }
    sh[zg][ex] = s;
    __syncthreads();
    if (zg == 0 && i < n) {
        float t = sh[0][ex];
#pragma unroll
        for (int q = 1; q < LANES; ++q) t += sh[q][ex];
        out[i] = t;
    }
}

// A loop of independent matrix instructions with nothing else in it: what the matrix pipes of
// the chip deliver at their best, measured next to the kernels that use them.  BF16 = false:
// v_mfma_f32_16x16x4_f32 (2048 flops each), true: v_mfma_f32_16x16x32_bf16 (16384 flops each);
// 8 instructions per iteration and wavefront.
typedef __bf16 bf16x8_probe __attribute__((ext_vector_type(8)));
template <bool BF16>
__global__ __launch_bounds__(256) void mfma_probe_kernel(float *__restrict__ sink, int iters)
{
    f32x4 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    const float a = threadIdx.x * 1e-3f, b = threadIdx.x * 2e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (BF16) {
                bf16x8_probe va, vb;
#pragma unroll
                for (int e = 0; e < 8; ++e) { va[e] = (__bf16)a; vb[e] = (__bf16)b; }
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, vb, acc[i], 0, 0, 0);
            } else {
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// number of entries >= 0 in an index list (the occupied neighbours of a level: the nnz of the
// traffic model); count must be zero before the launch
__global__ __launch_bounds__(256) void count_valid_kernel(const int32_t *__restrict__ idx, int64_t n,
                                                          unsigned long long *__restrict__ count)
{
    int local = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) local += idx[i] >= 0;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) local += __shfl_xor(local, d);
    if ((threadIdx.x & 63) == 0 && local) atomicAdd(count, (unsigned long long)local);
}

// ---------------------------------------------------------------------------------------
// 2x2x2 max-pooling through the child index rows.  VEC channels per thread (4 when the
// channel count allows 16-byte accesses).
// ---------------------------------------------------------------------------------------

// one thread per (coarse voxel, channel unit); the first occupied child seeds the maximum and
// a later child replaces it only when strictly greater
template <int VEC>
__global__ __launch_bounds__(256) void pool_fwd_kernel(
    const float *__restrict__ X, const int32_t *__restrict__ child8, float *__restrict__ Y,
    int32_t *__restrict__ argmax, int64_t n_coarse, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    const int32_t *kids = child8 + o * 8;
    float best[VEC];
    int32_t arg[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { best[e] = 0.f; arg[e] = -1; }
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int32_t j = kids[k];
        float v[VEC];
        const float *s = j >= 0 ? X + (int64_t)j * c + u * VEC : zsrc;
        if constexpr (VEC == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4 *>(s);
            v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = s[e];
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool take = (j >= 0) & ((arg[e] < 0) | (v[e] > best[e]));
            best[e] = take ? v[e] : best[e];
            arg[e] = take ? j : arg[e];
        }
    }
    float *dy = Y + o * c + u * VEC;
    int32_t *da = argmax + o * c + u * VEC;
    if constexpr (VEC == 4) {
        *reinterpret_cast<f32x4 *>(dy) = f32x4{best[0], best[1], best[2], best[3]};
        *reinterpret_cast<int4 *>(da) = make_int4(arg[0], arg[1], arg[2], arg[3]);
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { dy[e] = best[e]; da[e] = arg[e]; }
    }
}

// one thread per (coarse voxel, child, channel unit): every fine row is the child of exactly
// one coarse voxel, so this writes all of dX exactly once (the zero fill is part of it)
template <int VEC>
__global__ __launch_bounds__(256) void pool_bwd_kernel(
    const float *__restrict__ dY, const int32_t *__restrict__ argmax,
    const int32_t *__restrict__ child8, float *__restrict__ dX, int64_t n_coarse, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * 8 * cu) return;
    const int64_t ok = item / cu;            // coarse voxel * 8 + child
    const int u = (int)(item - ok * cu);
    const int32_t j = child8[ok];
    if (j < 0) return;
    const int64_t o = ok >> 3;
    const float *g = dY + o * c + u * VEC;
    const int32_t *a = argmax + o * c + u * VEC;
    float *d = dX + (int64_t)j * c + u * VEC;
    if constexpr (VEC == 4) {
        const f32x4 gv = *reinterpret_cast<const f32x4 *>(g);
        const int4 av = *reinterpret_cast<const int4 *>(a);
        *reinterpret_cast<f32x4 *>(d) = f32x4{av.x == j ? gv[0] : 0.f, av.y == j ? gv[1] : 0.f,
                                             av.z == j ? gv[2] : 0.f, av.w == j ? gv[3] : 0.f};
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) d[e] = (a[e] == j) ? g[e] : 0.f;
    }
}

// Max-pooling over general receptive fields (Section 4: pooling is the strided traversal of
// Algorithm 1 with the maximum taken instead of the inner product): field[o][0..taps) holds the
// input indices of output voxel o's field in traversal order (-1 = empty).  Same rules as
// pool_fwd_kernel: the first occupied entry seeds the maximum, a later one replaces it only
// when strictly greater; an output voxel whose field is empty gets 0 and the switch -1.
template <int VEC>
__global__ __launch_bounds__(256) void field_pool_fwd_kernel(
    const float *__restrict__ X, const int32_t *__restrict__ field, float *__restrict__ Y,
    int32_t *__restrict__ argmax, int64_t n_out, int taps, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_out * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    const int32_t *rows = field + o * taps;
    float best[VEC];
    int32_t arg[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { best[e] = 0.f; arg[e] = -1; }
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    for (int k = 0; k < taps; ++k) {
        const int32_t j = rows[k];
        float v[VEC];
        const float *s = j >= 0 ? X + (int64_t)j * c + u * VEC : zsrc;
        if constexpr (VEC == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4 *>(s);
            v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[e] = s[e];
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const bool take = (j >= 0) & ((arg[e] < 0) | (v[e] > best[e]));
            best[e] = take ? v[e] : best[e];
            arg[e] = take ? j : arg[e];
        }
    }
    float *dy = Y + o * c + u * VEC;
    int32_t *da = argmax + o * c + u * VEC;
    if constexpr (VEC == 4) {
        *reinterpret_cast<f32x4 *>(dy) = f32x4{best[0], best[1], best[2], best[3]};
        *reinterpret_cast<int4 *>(da) = make_int4(arg[0], arg[1], arg[2], arg[3]);
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { dy[e] = best[e]; da[e] = arg[e]; }
    }
}

// Its backward pass as a gather: field_t[q][0..taps) holds, per field row, the output voxel
// whose field contains input voxel q at that row (-1 = none).  dX[q][ch] = sum of dY[o][ch]
// over those o whose switch for channel ch is q, added in row order (with fields that do not
// overlap there is at most one such o).  Every element of dX is written.
template <int VEC>
__global__ __launch_bounds__(256) void field_pool_bwd_kernel(
    const float *__restrict__ dY, const int32_t *__restrict__ argmax, const int32_t *__restrict__ field_t,
    float *__restrict__ dX, int64_t n_in, int taps, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_in * cu) return;
    const int64_t q = item / cu;
    const int u = (int)(item - q * cu);
    const int32_t *rows = field_t + q * taps;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    // nine rows at a time: their owners, then the owners' switches and gradients (row 0 stands in
    // where a row has no owner; its values are not used), with no branch between the loads
    for (int r0 = 0; r0 < taps; r0 += 9) {
        int32_t o[9];
#pragma unroll
        for (int j = 0; j < 9; ++j) o[j] = *(r0 + j < taps ? rows + r0 + j : &g_minus1);
        float g[9][VEC];
        int32_t a[9][VEC];
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const int64_t at = (int64_t)max(o[j], 0) * c + u * VEC;
            if constexpr (VEC == 4) {
                const f32x4 gv = *reinterpret_cast<const f32x4 *>(dY + at);
                const int4 av = *reinterpret_cast<const int4 *>(argmax + at);
                g[j][0] = gv[0]; g[j][1] = gv[1]; g[j][2] = gv[2]; g[j][3] = gv[3];
                a[j][0] = av.x; a[j][1] = av.y; a[j][2] = av.z; a[j][3] = av.w;
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) { g[j][e] = dY[at + e]; a[j][e] = argmax[at + e]; }
            }
        }
#pragma unroll
        for (int j = 0; j < 9; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += (o[j] >= 0 && a[j][e] == (int32_t)q) ? g[j][e] : 0.f;
    }
    float *d = dX + q * c + u * VEC;
    if constexpr (VEC == 4) {
        *reinterpret_cast<f32x4 *>(d) = f32x4{acc[0], acc[1], acc[2], acc[3]};
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) d[e] = acc[e];
    }
}

// The backward passes of pooling when the fields PARTITION the input level (kernel side =
// stride, no padding: every input voxel lies in exactly one field): one thread per (output
// voxel, field row, channel unit) writes the row of the input voxel at that place, so all of
// dX is written exactly once.  MAXPOOL: the gradient where the switch points here, else 0;
// otherwise the average's scale * dY.
template <int VEC, bool MAXPOOL>
__global__ __launch_bounds__(256) void field_unpool_kernel(
    const float *__restrict__ dY, const int32_t *__restrict__ argmax, const int32_t *__restrict__ field,
    float *__restrict__ dX, int64_t n_out, int taps, int c, float scale)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_out * taps * cu) return;
    const int64_t ok = item / cu;            // output voxel * taps + row
    const int u = (int)(item - ok * cu);
    const int32_t j = field[ok];
    if (j < 0) return;
    const int64_t o = ok / taps;
    const float *g = dY + o * c + u * VEC;
    float *d = dX + (int64_t)j * c + u * VEC;
    float v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = g[e];
    if constexpr (MAXPOOL) {
        const int32_t *a = argmax + o * c + u * VEC;
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = (a[e] == j) ? v[e] : 0.f;
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] *= scale;
    }
    if constexpr (VEC == 4) {
        *reinterpret_cast<f32x4 *>(d) = f32x4{v[0], v[1], v[2], v[3]};
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) d[e] = v[e];
    }
}

// col2hash for a general receptive field (Algorithm 2), as a gather: dX[q][:] = sum over the
// field rows r with o = field_t[q][r] >= 0 of dcol[o][r*c + :], added in row order (no atomics,
// reproducible).  dcol is [N_out][taps*c]; every element of dX is written.
template <int VEC>
__global__ __launch_bounds__(256) void field_col2hash_kernel(
    const float *__restrict__ dcol, const int32_t *__restrict__ field_t, float *__restrict__ dX,
    int64_t n_in, int taps, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_in * cu) return;
    const int64_t q = item / cu;
    const int u = (int)(item - q * cu);
    const int32_t *rows = field_t + q * taps;
    const int64_t ld = (int64_t)taps * c;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    // nine rows at a time: their indices, then their pieces (a constant block of zeros where a
    // row has no owner), with no branch between the loads
    for (int r0 = 0; r0 < taps; r0 += 9) {
        int32_t o[9];
#pragma unroll
        for (int j = 0; j < 9; ++j) o[j] = *(r0 + j < taps ? rows + r0 + j : &g_minus1);
        float v[9][VEC];
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const float *p = o[j] >= 0 ? dcol + o[j] * ld + (r0 + j) * c + u * VEC : zsrc;
            if constexpr (VEC == 4) {
                const f32x4 t = *reinterpret_cast<const f32x4 *>(p);
                v[j][0] = t[0]; v[j][1] = t[1]; v[j][2] = t[2]; v[j][3] = t[3];
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[j][e] = p[e];
            }
        }
#pragma unroll
        for (int j = 0; j < 9; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += v[j][e];
    }
    float *d = dX + q * c + u * VEC;
    if constexpr (VEC == 4) {
        *reinterpret_cast<f32x4 *>(d) = f32x4{acc[0], acc[1], acc[2], acc[3]};
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) d[e] = acc[e];
    }
}

// Average pooling over general receptive fields (Section 4: the convolution whose weights all
// equal 1/F^3, channel by channel; empty entries add nothing): Y[o] = sum of the occupied
// entries' rows, in row order, times `scale` = 1/taps.  TRANSPOSED = false: idx = field (rows of
// the outputs, gathering X); true: idx = field_t (rows of the inputs, gathering dY) -- the
// backward pass spreads scale * dY[o] over o's field, here summed per input voxel.
template <int VEC>
__global__ __launch_bounds__(256) void field_avg_kernel(
    const float *__restrict__ src, const int32_t *__restrict__ idx, float *__restrict__ dst,
    int64_t n_dst, int taps, int c, float scale)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_dst * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    const int32_t *rows = idx + o * taps;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    for (int r0 = 0; r0 < taps; r0 += 9) {          // nine rows at a time, no branch between the loads
        int32_t jj[9];
#pragma unroll
        for (int j = 0; j < 9; ++j) jj[j] = *(r0 + j < taps ? rows + r0 + j : &g_minus1);
        float v[9][VEC];
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const float *p = jj[j] >= 0 ? src + (int64_t)jj[j] * c + u * VEC : zsrc;
            if constexpr (VEC == 4) {
                const f32x4 t = *reinterpret_cast<const f32x4 *>(p);
                v[j][0] = t[0]; v[j][1] = t[1]; v[j][2] = t[2]; v[j][3] = t[3];
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) v[j][e] = p[e];
            }
        }
#pragma unroll
        for (int j = 0; j < 9; ++j)
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] += v[j][e];
    }
    float *d = dst + o * c + u * VEC;
#pragma unroll
    for (int e = 0; e < VEC; ++e) d[e] = acc[e] * scale;
}

// ReLU followed by 2x2x2 max-pooling in one pass: A = max(Y, 0) is written for every child row
// (each fine voxel is the child of exactly one coarse voxel, so all of A is covered) unless A is
// null, and the maximum / switch are taken over the rectified values with the rules of
// pool_fwd_kernel.
template <int VEC>
__global__ __launch_bounds__(256) void relu_pool_fwd_kernel(
    const float *__restrict__ Y, const int32_t *__restrict__ child8, float *__restrict__ A,
    float *__restrict__ P, int32_t *__restrict__ argmax, int64_t n_coarse, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    const int32_t *kids = child8 + o * 8;
    float best[VEC];
    int32_t arg[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { best[e] = 0.f; arg[e] = -1; }
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    int32_t j[8];
    float v[8][VEC];
#pragma unroll
    for (int k = 0; k < 8; ++k) j[k] = kids[k];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float *s = j[k] >= 0 ? Y + (int64_t)j[k] * c + u * VEC : zsrc;
        if constexpr (VEC == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4 *>(s);
            v[k][0] = t[0]; v[k][1] = t[1]; v[k][2] = t[2]; v[k][3] = t[3];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[k][e] = s[e];
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            v[k][e] = v[k][e] > 0.f ? v[k][e] : 0.f;
            const bool take = (j[k] >= 0) & ((arg[e] < 0) | (v[k][e] > best[e]));
            best[e] = take ? v[k][e] : best[e];
            arg[e] = take ? j[k] : arg[e];
        }
        if (A != nullptr && j[k] >= 0) {
            float *d = A + (int64_t)j[k] * c + u * VEC;
            if constexpr (VEC == 4) *reinterpret_cast<f32x4 *>(d) = f32x4{v[k][0], v[k][1], v[k][2], v[k][3]};
            else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) d[e] = v[k][e];
            }
        }
    }
    float *dy = P + o * c + u * VEC;
    int32_t *da = argmax + o * c + u * VEC;
    if constexpr (VEC == 4) {
        *reinterpret_cast<f32x4 *>(dy) = f32x4{best[0], best[1], best[2], best[3]};
        *reinterpret_cast<int4 *>(da) = make_int4(arg[0], arg[1], arg[2], arg[3]);
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { dy[e] = best[e]; da[e] = arg[e]; }
    }
}

// Max-pool backward followed by ReLU backward in one pass:
// dY[j][ch] = (argmax[o][ch] == j and A[j][ch] > 0) ? dP[o][ch] : 0 for child j of coarse voxel o.
// Only the sign of A is used, so the values before the ReLU serve as well.
// POOLED: `A` holds the pooled rows P[o][ch] of the forward pass instead ([n_coarse][c]): the child
// the switch names carries the maximum, A[argmax[o][ch]][ch] = P[o][ch], so its sign is P's and
// the fine rows need not be read (nor kept) at all.
template <int VEC, bool POOLED = false>
__global__ __launch_bounds__(256) void pool_relu_bwd_kernel(
    const float *__restrict__ dP, const int32_t *__restrict__ argmax, const int32_t *__restrict__ child8,
    const float *__restrict__ A, float *__restrict__ dY, int64_t n_coarse, int c)
{
    // one thread per (coarse voxel, channel unit): the coarse gradient and switches are read once
    // and dealt to the up to 8 child rows
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    const int32_t *kids = child8 + o * 8;
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    int32_t j[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) j[k] = kids[k];
    float g[VEC], x[8][VEC];
    int32_t a[VEC];
    if constexpr (VEC == 4) {
        const f32x4 gv = *reinterpret_cast<const f32x4 *>(dP + o * c + u * 4);
        const int4 av = *reinterpret_cast<const int4 *>(argmax + o * c + u * 4);
        g[0] = gv[0]; g[1] = gv[1]; g[2] = gv[2]; g[3] = gv[3];
        a[0] = av.x; a[1] = av.y; a[2] = av.z; a[3] = av.w;
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) { g[e] = dP[o * c + u * VEC + e]; a[e] = argmax[o * c + u * VEC + e]; }
    }
    if constexpr (POOLED) {
        // the pooled row decides once for all children: a channel whose maximum is not positive passes nothing
        float pv[VEC];
        if constexpr (VEC == 4) {
            const f32x4 t = *reinterpret_cast<const f32x4 *>(A + o * c + u * 4);
            pv[0] = t[0]; pv[1] = t[1]; pv[2] = t[2]; pv[3] = t[3];
        } else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) pv[e] = A[o * c + u * VEC + e];
        }
#pragma unroll
        for (int e = 0; e < VEC; ++e) g[e] = pv[e] > 0.f ? g[e] : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int e = 0; e < VEC; ++e) x[k][e] = 1.f;
    } else {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float *s = j[k] >= 0 ? A + (int64_t)j[k] * c + u * VEC : zsrc;
            if constexpr (VEC == 4) {
                const f32x4 t = *reinterpret_cast<const f32x4 *>(s);
                x[k][0] = t[0]; x[k][1] = t[1]; x[k][2] = t[2]; x[k][3] = t[3];
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) x[k][e] = s[e];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (j[k] < 0) continue;
        float r[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) r[e] = ((a[e] == j[k]) & (x[k][e] > 0.f)) ? g[e] : 0.f;
        float *d = dY + (int64_t)j[k] * c + u * VEC;
        if constexpr (VEC == 4) *reinterpret_cast<f32x4 *>(d) = f32x4{r[0], r[1], r[2], r[3]};
        else {
#pragma unroll
            for (int e = 0; e < VEC; ++e) d[e] = r[e];
        }
    }
}

// 2x2x2 average pooling as the paper defines it (Section 4): a stride-2 convolution whose
// weights all equal 1/F^3, so an empty child counts as zero and the divisor is always 8.
// One thread per (coarse voxel, channel unit).
template <int VEC>
__global__ __launch_bounds__(256) void avgpool_fwd_kernel(
    const float *__restrict__ X, const int32_t *__restrict__ child8, float *__restrict__ Y, int64_t n_coarse, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    const float *zsrc = reinterpret_cast<const float *>(g_zero16);
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int32_t j = child8[o * 8 + k];
        const float *s = j >= 0 ? X + (int64_t)j * c + u * VEC : zsrc;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += s[e];
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) Y[o * c + u * VEC + e] = acc[e] * 0.125f;
}

// its adjoint, the average-unpooling of Section 4: every occupied child receives an eighth of
// the coarse value; all fine rows are written (each has exactly one parent)
template <int VEC>
__global__ __launch_bounds__(256) void avgpool_bwd_kernel(
    const float *__restrict__ dY, const int32_t *__restrict__ child8, float *__restrict__ dX, int64_t n_coarse, int c)
{
    const int cu = c / VEC;
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * cu) return;
    const int64_t o = item / cu;
    const int u = (int)(item - o * cu);
    float g[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) g[e] = dY[o * c + u * VEC + e] * 0.125f;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int32_t j = child8[o * 8 + k];
        if (j < 0) continue;
#pragma unroll
        for (int e = 0; e < VEC; ++e) dX[(int64_t)j * c + u * VEC + e] = g[e];
    }
}

// backward of max-unpooling: the coarse gradient reads the fine gradient back at its switch,
// dXc[o][ch] = dY[argmax[o][ch]][ch]
__global__ __launch_bounds__(256) void unpool_bwd_kernel(
    const float *__restrict__ dY, const int32_t *__restrict__ argmax, float *__restrict__ dXc,
    int64_t n_coarse, int c)
{
    const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (item >= n_coarse * c) return;
    const int ch = (int)(item % c);
    const int32_t j = argmax[item];
    dXc[item] = j >= 0 ? dY[(int64_t)j * c + ch] : 0.f;
}

// element-wise ReLU; n4 = number of float4 units, the remaining n - 4*n4 floats are done one
// per thread by the first threads (n4 = 0 when the pointers are not 16-byte aligned)
__global__ __launch_bounds__(256) void relu_fwd_kernel(const float *__restrict__ x,
                                                       float *__restrict__ y, int64_t n, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        f32x4 v = reinterpret_cast<const f32x4 *>(x)[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
        reinterpret_cast<f32x4 *>(y)[i] = v;
    }
    const int64_t t = 4 * n4 + i;
    if (t < n) { const float v = x[t]; y[t] = v > 0.f ? v : 0.f; }
}

__global__ __launch_bounds__(256) void relu_bwd_kernel(const float *__restrict__ y,
                                                       const float *__restrict__ dy,
                                                       float *__restrict__ dx, int64_t n, int64_t n4)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) {
        const f32x4 a = reinterpret_cast<const f32x4 *>(y)[i];
        f32x4 g = reinterpret_cast<const f32x4 *>(dy)[i];
#pragma unroll
        for (int e = 0; e < 4; ++e) g[e] = a[e] > 0.f ? g[e] : 0.f;
        reinterpret_cast<f32x4 *>(dx)[i] = g;
    }
    const int64_t t = 4 * n4 + i;
    if (t < n) dx[t] = y[t] > 0.f ? dy[t] : 0.f;
}

}  // namespace hch
