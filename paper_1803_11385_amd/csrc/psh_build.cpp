// Host-side construction of perfect spatial hash tables.
//
// Paper Section 3.1 defines the structure (hash table H holding data indices, offset
// table Phi, position tags T, and h(p) = (p mod m + Phi[p mod r]) mod m per axis);
// Section 5.2 fixes the sizes (m smallest with m^3 > n, r from sigma = 1/(2d) growing by
// the cube root of two on failure) and defers the assignment of offsets to the original
// PSH paper.  The assignment used here is a deterministic greedy one:
//   * a bucket is the set of voxels sharing p mod r, numbered g = lin_r(p mod r);
//   * buckets are placed largest first (ties: smaller g first), their voxels kept in data
//     order;
//   * for a bucket whose first voxel is q0 the candidates t = 0, 1, ... put q0 on slot
//     number (s0 + t) mod m^3, s0 = ((g * 2654435761) mod 2^32) mod m^3, which fixes the
//     offset; the first candidate sending all voxels of the bucket to free, distinct slots
//     is kept;
//   * a bucket without a candidate fails the attempt, and r grows.
// r is kept coprime to m so that no two positions of the grid share both residues unless
// they are m*r apart.
#include "psh_build.hpp"

#include <algorithm>
#include <numeric>

namespace hch {

int hash_side(int64_t n)
{
    int64_t m = 1;
    while (m * m * m <= n) ++m;
    return (int)m;
}

static int coprime_up(int64_t r, int m)
{
    while (std::gcd((int64_t)m, r) != 1) ++r;
    return (int)r;
}

int offset_side_first(int64_t n, int m)
{
    int64_t r = 1;
    while (6 * r * r * r < n) ++r;
    return coprime_up(r, m);
}

int offset_side_next(int r, int m)
{
    const int64_t need = 2 * (int64_t)r * r * r;
    int64_t k = (int64_t)r + 1;
    while (k * k * k < need) ++k;
    return coprime_up(k, m);
}

namespace {

struct Cell { uint8_t x, y, z; };   // residues modulo m (m <= 256)

struct Bucket {
    int64_t id;
    uint32_t first;   // range in the bucket-sorted voxel list
    uint32_t count;
};

// One attempt with a fixed offset table side.  Returns false if some bucket cannot be placed.
bool attempt(const int32_t *xyz, int64_t n, int m, int r, ModelTables &tb)
{
    const int64_t m3 = (int64_t)m * m * m;
    const int64_t r3 = (int64_t)r * r * r;

    tb.H.assign((size_t)m3, -1);
    tb.T.assign((size_t)m3 * 3, (uint16_t)0xFFFF);
    tb.Phi.assign((size_t)r3 * 3, (uint8_t)0);

    // residues and bucket number of every voxel
    std::vector<Cell> h0((size_t)n);
    std::vector<int64_t> bucket_of((size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        const int32_t *p = xyz + 3 * i;
        h0[i] = Cell{(uint8_t)(p[0] % m), (uint8_t)(p[1] % m), (uint8_t)(p[2] % m)};
        bucket_of[i] = ((int64_t)(p[0] % r) * r + (p[1] % r)) * r + (p[2] % r);
    }

    // voxels grouped by bucket, data order preserved inside a group
    std::vector<uint32_t> by_bucket((size_t)n);
    std::iota(by_bucket.begin(), by_bucket.end(), 0u);
    std::stable_sort(by_bucket.begin(), by_bucket.end(),
                     [&](uint32_t a, uint32_t b) { return bucket_of[a] < bucket_of[b]; });

    std::vector<Bucket> buckets;
    for (int64_t i = 0; i < n;) {
        int64_t j = i;
        while (j < n && bucket_of[by_bucket[j]] == bucket_of[by_bucket[i]]) ++j;
        buckets.push_back(Bucket{bucket_of[by_bucket[i]], (uint32_t)i, (uint32_t)(j - i)});
        i = j;
    }
    std::sort(buckets.begin(), buckets.end(), [](const Bucket &a, const Bucket &b) {
        return a.count != b.count ? a.count > b.count : a.id < b.id;
    });

    std::vector<uint8_t> taken((size_t)m3, 0);
    std::vector<uint32_t> stamp((size_t)m3, 0);   // last candidate that touched a slot
    uint32_t serial = 0;
    std::vector<int64_t> where;

    for (const Bucket &bk : buckets) {
        const uint32_t *mem = by_bucket.data() + bk.first;
        const Cell a = h0[mem[0]];
        const int64_t s0 = (int64_t)((uint32_t)((uint64_t)bk.id * 2654435761ULL)) % m3;
        int64_t e = s0;
        int sx = (int)(e / ((int64_t)m * m)), sy = (int)((e / m) % m), sz = (int)(e % m);
        bool placed = false;
        int ox = 0, oy = 0, oz = 0;
        where.assign(bk.count, 0);

        for (int64_t t = 0; t < m3; ++t) {
            // a lone voxel goes on slot e itself: only free slots can work
            if (!taken[e]) {
                ox = sx - a.x; if (ox < 0) ox += m;
                oy = sy - a.y; if (oy < 0) oy += m;
                oz = sz - a.z; if (oz < 0) oz += m;
                bool fits = true;
                if (++serial == 0) { std::fill(stamp.begin(), stamp.end(), 0u); serial = 1; }
                for (uint32_t k = 0; k < bk.count; ++k) {
                    const Cell c = h0[mem[k]];
                    int x = c.x + ox; if (x >= m) x -= m;
                    int y = c.y + oy; if (y >= m) y -= m;
                    int z = c.z + oz; if (z >= m) z -= m;
                    const int64_t s = ((int64_t)x * m + y) * m + z;
                    if (taken[s] || stamp[s] == serial) { fits = false; break; }
                    stamp[s] = serial;
                    where[k] = s;
                }
                if (fits) { placed = true; break; }
            }
            // next slot number, wrapping around the table
            ++e; ++sz;
            if (sz == m) { sz = 0; ++sy; if (sy == m) { sy = 0; ++sx; } }
            if (e == m3) { e = 0; sx = sy = sz = 0; }
        }
        if (!placed) return false;

        tb.Phi[3 * bk.id + 0] = (uint8_t)ox;
        tb.Phi[3 * bk.id + 1] = (uint8_t)oy;
        tb.Phi[3 * bk.id + 2] = (uint8_t)oz;
        for (uint32_t k = 0; k < bk.count; ++k) {
            const int64_t s = where[k];
            const int32_t *p = xyz + 3 * (int64_t)mem[k];
            taken[s] = 1;
            tb.H[s] = (int32_t)mem[k];
            tb.T[3 * s + 0] = (uint16_t)p[0];
            tb.T[3 * s + 1] = (uint16_t)p[1];
            tb.T[3 * s + 2] = (uint16_t)p[2];
        }
    }
    return true;
}

}  // namespace

BuildResult build_model_tables(const int32_t *xyz, int64_t n, int ubar, ModelTables &out)
{
    out.m = hash_side(n);
    if (out.m > 256) return BUILD_UNSUPPORTED;   // an 8-bit offset must reach every slot
    int r = offset_side_first(n, out.m);
    out.attempts = 0;
    for (;;) {
        ++out.attempts;
        if (attempt(xyz, n, out.m, r, out)) break;
        if (r >= ubar) return BUILD_FAILED;      // singleton buckets cannot fail
        r = offset_side_next(r, out.m);
        // an offset table beyond what the super tables can index (32 bits, 3 bytes per cell) is
        // refused before anything of that size is allocated
        if ((int64_t)r * r * r >= ((int64_t)1 << 31) / 3) return BUILD_UNSUPPORTED;
    }
    out.r = r;
    return BUILD_OK;
}

void coarsen_model(const int32_t *xyz, int64_t n, int ubar_fine, int ratio, std::vector<int32_t> &out_xyz)
{
    const int64_t uc = (ubar_fine + ratio - 1) / ratio;
    std::vector<int64_t> lin((size_t)n);
    for (int64_t i = 0; i < n; ++i)
        lin[i] = ((int64_t)(xyz[3 * i] / ratio) * uc + (xyz[3 * i + 1] / ratio)) * uc + (xyz[3 * i + 2] / ratio);
    std::sort(lin.begin(), lin.end());
    lin.erase(std::unique(lin.begin(), lin.end()), lin.end());
    out_xyz.resize(lin.size() * 3);
    for (size_t i = 0; i < lin.size(); ++i) {
        out_xyz[3 * i + 0] = (int32_t)(lin[i] / (uc * uc));
        out_xyz[3 * i + 1] = (int32_t)((lin[i] / uc) % uc);
        out_xyz[3 * i + 2] = (int32_t)(lin[i] % uc);
    }
}

}  // namespace hch
