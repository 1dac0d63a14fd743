// C ABI of the hch library: host logic, table upload and kernel launches.
#include "../../include/hch.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "kernels.hip.hpp"
#include "direct.hip.hpp"
#include "gemm_bf16.hip.hpp"
#include "psh_device.hip.hpp"
#include "profile.hpp"
#include "psh_build.hpp"

// Every kernel launch of the library: carries the two timing events of the enclosing LaunchTimer,
// if there is one and timing is on; an ordinary launch otherwise.
#define HCH_LAUNCH(kernel, grid, block, lds, stream, ...)                                          \
    do {                                                                                           \
        hipEvent_t ev_a_ = hch::tls_start_event, ev_b_ = hch::tls_stop_event;                      \
        hch::tls_start_event = hch::tls_stop_event = nullptr;                                      \
        if (ev_a_) hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ev_a_, ev_b_, 0, __VA_ARGS__); \
        else hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                    \
    } while (0)

namespace {

thread_local std::string g_err;

hch_status fail(hch_status st, const std::string &msg)
{
    g_err = msg;
    return st;
}

#define HCH_HIP(call)                                                                      \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail(HCH_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));      \
    } while (0)

#define HCH_LAUNCH_CHECK(name)                                                             \
    do {                                                                                   \
        hipError_t e_ = hipGetLastError();                                                 \
        if (e_ != hipSuccess)                                                              \
            return fail(HCH_EHIP, std::string("launch ") + name + ": " + hipGetErrorString(e_)); \
    } while (0)

// One level of the super-PSH, host and device side.
struct Level {
    int32_t ubar = 0, b = 0;
    int32_t ratio = 1;                         // side of the next finer level / side of this one (1 at level 0)
    int64_t n_total = 0, m_total = 0, r_total = 0;
    int32_t max_n = 0;                         // largest model of the level
    int64_t nbr_valid = 0;                     // occupied entries of nbr27 (incl. the centre)
    std::vector<int32_t> mbar, rbar, attempts, coords;
    std::vector<int64_t> M, R, N;
    std::vector<int32_t> H, V;                 // host copies of the super tables
    std::vector<uint16_t> T;
    std::vector<uint8_t> Phi;
    // device
    int32_t *dH = nullptr, *dV = nullptr, *dcoords = nullptr, *dnbr = nullptr, *dchild = nullptr;
    int32_t *dnbr_t = nullptr;                 // tap-major copy of dnbr ([27][n_total]), built on request
    uint32_t *dmask27 = nullptr;               // [n_total] bit k: neighbour k exists
    uint32_t *dtilemask = nullptr;             // [ceil(n_total/64)] taps present in each tile of the pattern order
    const int32_t *dorder = nullptr;           // [n_total] the level's voxels in pattern order (into hch_levels' sort output)
    uint16_t *dT = nullptr;
    uint8_t *dPhi = nullptr;
    uint32_t *dslot3 = nullptr, *dphi4 = nullptr;   // packed copies of H*,T* and Phi* for the lookups
    int32_t *dmeta = nullptr;                  // mbar[b] rbar[b] M[b+1] R[b+1] N[b+1] as int32

    hch::PshView view() const
    {
        hch::PshView v;
        v.slot3 = dslot3; v.phi4 = dphi4;
        v.mbar = dmeta; v.rbar = dmeta + b; v.M = dmeta + 2 * b; v.R = dmeta + 3 * b + 1;
        v.N = dmeta + 4 * b + 2; v.ubar = ubar;
        return v;
    }
    const int32_t *dN() const { return dmeta + 4 * b + 2; }
};

void free_level(Level &L)
{
    void *ptrs[] = {L.dH, L.dV, L.dcoords, L.dnbr, L.dchild, L.dT, L.dPhi, L.dmeta, L.dslot3, L.dphi4, L.dnbr_t, L.dmask27, L.dtilemask};
    for (void *p : ptrs) if (p) (void)hipFree(p);
    L.dH = L.dV = L.dcoords = L.dnbr = L.dchild = L.dmeta = L.dnbr_t = nullptr;
    L.dmask27 = L.dtilemask = nullptr; L.dorder = nullptr;
    L.dT = nullptr; L.dPhi = nullptr; L.dslot3 = L.dphi4 = nullptr;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline unsigned blocks_for(int64_t items) { return (unsigned)((items + 255) / 256); }

constexpr int64_t MAX_GRID_ITEMS = (int64_t)2147483647 * 256;   // grid.x limit * block size

}  // namespace

struct hch_levels {
    std::vector<Level> lv;
    // one-launch index-list kernels: all levels as a kernel argument, and the tile prefix
    // arrays (host copy + device) of the neighbour and child kernels
    hch::LevelSet set{};
    std::vector<int32_t> nbr_prefix, child_prefix;
    int32_t *d_nbr_prefix = nullptr, *d_child_prefix = nullptr;
    // pattern order of every level's voxels (level l at sort_off[l]): keys and tile histograms
    // written by the neighbour kernel, the sorted data indices
    std::vector<int32_t> sort_off;
    uint8_t *d_sort_key = nullptr;
    int32_t *d_tile_hist = nullptr, *d_key_total = nullptr, *d_order = nullptr;
};

extern "C" const char *hch_last_error(void) { return g_err.c_str(); }

extern "C" void hch_free_levels(hch_levels *levels)
{
    if (!levels) return;
    for (Level &L : levels->lv) free_level(L);
    if (levels->d_nbr_prefix) (void)hipFree(levels->d_nbr_prefix);
    if (levels->d_child_prefix) (void)hipFree(levels->d_child_prefix);
    void *sort_ptrs[] = {levels->d_sort_key, levels->d_tile_hist, levels->d_key_total, levels->d_order};
    for (void *p : sort_ptrs) if (p) (void)hipFree(p);
    delete levels;
}

extern "C" int32_t hch_num_levels(const hch_levels *levels)
{
    return levels ? (int32_t)levels->lv.size() : 0;
}

// ---------------------------------------------------------------------------------------
// build
// ---------------------------------------------------------------------------------------

static hch_status upload(void **dst, const void *src, size_t bytes, hipStream_t s)
{
    *dst = nullptr;
    hipError_t e = hipMalloc(dst, bytes ? bytes : 16);
    if (e != hipSuccess) { *dst = nullptr; return fail(HCH_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e)); }
    if (bytes) HCH_HIP(hipMemcpyAsync(*dst, src, bytes, hipMemcpyHostToDevice, s));
    return HCH_OK;
}

// dnbr_t[t][i] = dnbr[i][t], if the level has the copy
static hch_status transpose_neighbours(const Level &L, hipStream_t s)
{
    if (!L.dnbr_t || L.n_total == 0) return HCH_OK;
    hch::LaunchTimer lt(HCH_KERNEL_ID("index_transpose_kernel"), s, 216.0 * (double)L.n_total, 0.0);
    HCH_LAUNCH(hch::index_transpose_kernel, dim3(blocks_for(L.n_total)), dim3(256), 0, s, L.dnbr, L.dnbr_t, L.n_total, 27);
    HCH_LAUNCH_CHECK("index_transpose_kernel");
    return HCH_OK;
}

// index lists of levels [l0, l1) in one launch each
static hch_status launch_index_lists(const hch_levels *hl, int l0, int l1, hipStream_t s)
{
    const int b = hl->lv[0].b;
    const int n_entries = (int)hl->lv.size() * b;
    {
        const int first = hl->nbr_prefix[(size_t)l0 * b], last = hl->nbr_prefix[(size_t)l1 * b];
        if (last > first) {
            double bytes = 0.0;   // per voxel: its position in, 27 indices out; the level's tables once
            for (int l = l0; l < l1; ++l)
                bytes += (double)hl->lv[l].n_total * 120.0 + (double)hl->lv[l].m_total * 10.0 + (double)hl->lv[l].r_total * 3.0;
            const unsigned n_tiles = (unsigned)(last - first);
            const unsigned grid = (n_tiles + hch::NUM_XCD - 1) / hch::NUM_XCD * hch::NUM_XCD;
            hch::LaunchTimer lt(HCH_KERNEL_ID("neighbour_kernel"), s, bytes, 0.0);
            HCH_LAUNCH(hch::neighbour_kernel, dim3(grid), dim3(256), 0, s, hl->set, hl->d_nbr_prefix,
                               n_entries, first, n_tiles);
        }
        HCH_LAUNCH_CHECK("neighbour_kernel");
        for (int l = l0; l < l1; ++l) {            // keep the tap-major copies in step
            hch_status st = transpose_neighbours(hl->lv[l], s);
            if (st != HCH_OK) return st;
        }
        // pattern order of the levels' voxels (stable counting sort by pattern key), then the tap
        // masks of its 64-row tiles
        const int64_t cnt = (int64_t)hl->sort_off[l1] - hl->sort_off[l0];
        if (cnt > 0) {
            {
                hch::LaunchTimer lt(HCH_KERNEL_ID("pattern_scan_kernel"), s, 8.0 * 64.0 * (double)(last - first), 0.0);
                HCH_LAUNCH(hch::pattern_scan_kernel, dim3(hch::PATTERN_BINS, (unsigned)(l1 - l0)), dim3(256), 0, s, hl->set,
                           hl->d_key_total, l0);
            }
            HCH_LAUNCH_CHECK("pattern_scan_kernel");
            {
                hch::LaunchTimer lt(HCH_KERNEL_ID("pattern_scatter_kernel"), s, 5.0 * (double)cnt, 0.0);
                HCH_LAUNCH(hch::pattern_scatter_kernel, dim3((unsigned)(last - first)), dim3(256), 0, s, hl->set,
                           hl->d_nbr_prefix, n_entries, first, (unsigned)(last - first), hl->d_key_total, hl->d_order);
            }
            HCH_LAUNCH_CHECK("pattern_scatter_kernel");
            hch::TileMaskArgs A{};
            A.n_levels = l1 - l0;
            A.tile_prefix[0] = 0;
            for (int l = l0; l < l1; ++l) {
                const Level &L = hl->lv[l];
                A.mask27[l - l0] = L.dmask27; A.tile_mask[l - l0] = L.dtilemask; A.order[l - l0] = L.dorder;
                A.n[l - l0] = (int32_t)L.n_total;
                A.tile_prefix[l - l0 + 1] = A.tile_prefix[l - l0] + (int32_t)((L.n_total + hch::PATTERN_TILE - 1) / hch::PATTERN_TILE);
            }
            const int tiles = A.tile_prefix[A.n_levels];
            hch::LaunchTimer lt(HCH_KERNEL_ID("tile_mask_kernel"), s, 8.0 * (double)cnt, 0.0);
            HCH_LAUNCH(hch::tile_mask_kernel, dim3((unsigned)((tiles + 3) / 4)), dim3(256), 0, s, A);
            HCH_LAUNCH_CHECK("tile_mask_kernel");
        }
    }
    {
        const int first = hl->child_prefix[(size_t)l0 * b], last = hl->child_prefix[(size_t)l1 * b];
        if (last > first) {
            double bytes = 0.0;   // per coarse voxel: position in, 8 indices out; the finer tables once
            for (int l = std::max(l0, 1); l < l1; ++l)
                if (hl->lv[l].ratio == 2) bytes += (double)hl->lv[l].n_total * 44.0 + (double)hl->lv[l - 1].m_total * 10.0 + (double)hl->lv[l - 1].r_total * 3.0;
            const unsigned n_tiles = (unsigned)(last - first);
            const unsigned grid = (n_tiles + hch::NUM_XCD - 1) / hch::NUM_XCD * hch::NUM_XCD;
            hch::LaunchTimer lt(HCH_KERNEL_ID("child_kernel"), s, bytes, 0.0);
            HCH_LAUNCH(hch::child_kernel, dim3(grid), dim3(256), 0, s, hl->set, hl->d_child_prefix,
                               n_entries, first, n_tiles);
        }
        HCH_LAUNCH_CHECK("child_kernel");
    }
    return HCH_OK;
}

extern "C" hch_status hch_build_neighbours(hch_levels *levels, int32_t level, void *stream)
{
    if (!levels || level < -1 || level >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_build_neighbours: bad level");
    if (!levels->d_nbr_prefix) return fail(HCH_EINVAL, "hch_build_neighbours: levels were built without device tables");
    if (level < 0) return launch_index_lists(levels, 0, (int)levels->lv.size(), (hipStream_t)stream);
    return launch_index_lists(levels, level, level + 1, (hipStream_t)stream);
}

extern "C" hch_status hch_build_tap_major(hch_levels *levels, int32_t level, void *stream)
{
    if (!levels || level < -1 || level >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_build_tap_major: bad level");
    if (!levels->d_nbr_prefix) return fail(HCH_EINVAL, "hch_build_tap_major: levels were built without device tables");
    const int l0 = level < 0 ? 0 : level, l1 = level < 0 ? (int)levels->lv.size() : level + 1;
    for (int l = l0; l < l1; ++l) {
        Level &L = levels->lv[l];
        if (!L.dnbr_t && L.n_total > 0 && hipMalloc((void **)&L.dnbr_t, (size_t)L.n_total * 27 * 4) != hipSuccess) {
            L.dnbr_t = nullptr;
            return fail(HCH_ENOMEM, "hch_build_tap_major: hipMalloc failed");
        }
        hch_status st = transpose_neighbours(L, (hipStream_t)stream);
        if (st != HCH_OK) return st;
    }
    return HCH_OK;
}

extern "C" hch_status hch_build_neighbours_range(hch_levels *levels, int32_t first, int32_t count, void *stream)
{
    if (!levels || first < 0 || count < 0 || (int64_t)first + count > (int64_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_build_neighbours_range: bad level range");
    if (!levels->d_nbr_prefix) return fail(HCH_EINVAL, "hch_build_neighbours_range: levels were built without device tables");
    if (count == 0) return HCH_OK;
    return launch_index_lists(levels, first, first + count, (hipStream_t)stream);
}

// ---- PSH construction on the device (psh_device.hip.hpp) ----

namespace {
struct DeviceBlocks {            // device allocations that live until the end of the build call
    std::vector<void *> ptrs;
    ~DeviceBlocks() { for (void *p : ptrs) if (p) (void)hipFree(p); }
    hch_status get(void **out, size_t bytes, int fill, hipStream_t s)
    {
        *out = nullptr;
        hipError_t e = hipMalloc(out, bytes ? bytes : 16);
        if (e != hipSuccess) { *out = nullptr; return fail(HCH_ENOMEM, std::string("hipMalloc: ") + hipGetErrorString(e)); }
        ptrs.push_back(*out);
        if (fill >= 0 && bytes) HCH_HIP(hipMemsetAsync(*out, fill, bytes, s));
        return HCH_OK;
    }
};
struct PairWork {
    int l, v;
    int32_t n, m, r, attempts;
    const uint32_t *phi;         // offset words of the successful attempt (device)
    bool done;
};
}  // namespace

// Fills, for every level: mbar, rbar, attempts, M, R, m_total, r_total, the device tables dH, dT,
// dV, dPhi, dslot3, dphi4, dcoords, dmeta and the host copies H, T, Phi, V.  Levels must have
// ubar, b, coords, N, n_total.
static hch_status device_construct(hch_levels *hl, hipStream_t s)
{
    const int n_levels = (int)hl->lv.size();
    const int batch = hl->lv[0].b;
    DeviceBlocks tmp;
    std::vector<PairWork> work;
    hch_status st;
    for (int l = 0; l < n_levels; ++l) {
        Level &L = hl->lv[l];
        L.mbar.assign((size_t)batch, 0); L.rbar.assign((size_t)batch, 0); L.attempts.assign((size_t)batch, 0);
        L.M.assign((size_t)batch + 1, 0); L.R.assign((size_t)batch + 1, 0);
        for (int v = 0; v < batch; ++v) {
            const int64_t n = L.N[v + 1] - L.N[v];
            const int m = hch::hash_side(n);
            if (m > 256) return fail(HCH_EUNSUPPORTED, "hch_build_levels_device: a model needs a hash table side above 256");
            L.mbar[v] = m;
            L.M[v + 1] = L.M[v] + (int64_t)m * m * m;
            work.push_back(PairWork{l, v, (int32_t)n, m, hch::offset_side_first(n, m), 0, nullptr, false});
        }
        L.m_total = L.M[batch];
        if (L.m_total >= ((int64_t)1 << 31)) return fail(HCH_EUNSUPPORTED, "hch_build_levels_device: super table exceeds 32-bit indexing");
        HCH_HIP(hipMalloc((void **)&L.dH, (size_t)L.m_total * 4));
        HCH_HIP(hipMalloc((void **)&L.dT, (size_t)L.m_total * 6));
        HCH_HIP(hipMalloc((void **)&L.dV, (size_t)L.m_total * 4));
        HCH_HIP(hipMemsetAsync(L.dH, 0xFF, (size_t)L.m_total * 4, s));     // -1 = free slot
        HCH_HIP(hipMemsetAsync(L.dT, 0xFF, (size_t)L.m_total * 6, s));     // 0xFFFF = no position
        if ((st = upload((void **)&L.dcoords, L.coords.data(), L.coords.size() * 4, s)) != HCH_OK) return st;
    }
    const int n_pairs = (int)work.size();
    int32_t *d_fail = nullptr;
    if ((st = tmp.get((void **)&d_fail, (size_t)n_pairs * 4, -1, s)) != HCH_OK) return st;
    std::vector<int32_t> h_fail((size_t)n_pairs);

    std::vector<int> active((size_t)n_pairs);
    for (int i = 0; i < n_pairs; ++i) active[i] = i;
    for (int round = 0; !active.empty(); ++round) {
        if (round >= 24) return fail(HCH_EBUILD, "hch_build_levels_device: perfect hash construction failed");
        const int na = (int)active.size();
        std::vector<hch::PairDesc> desc((size_t)na);
        int64_t cells = 0, vox = 0, slots = 0;
        int32_t max_n = 0, max_r3 = 0, max_m3 = 0;
        for (int a = 0; a < na; ++a) {
            PairWork &w = work[active[a]];
            Level &L = hl->lv[w.l];
            if (w.r > 1024 || w.r > 2 * L.ubar + 1)   // beyond one cell per grid position nothing can improve
                return fail(HCH_EBUILD, "hch_build_levels_device: perfect hash construction failed");
            const int32_t r3 = w.r * w.r * w.r, m3 = w.m * w.m * w.m;
            desc[a] = hch::PairDesc{L.dcoords + 3 * L.N[w.v], L.dH + L.M[w.v], L.dT + 3 * L.M[w.v], w.n, w.m, w.r,
                                    (int32_t)cells, (int32_t)vox, (int32_t)slots, active[a]};
            cells += r3; vox += w.n; slots += m3;
            max_n = std::max(max_n, w.n); max_r3 = std::max(max_r3, r3); max_m3 = std::max(max_m3, m3);
            ++w.attempts;
        }
        if (cells >= ((int64_t)1 << 31) / hch::PSH_CLASSES || vox >= ((int64_t)1 << 31) || slots >= ((int64_t)1 << 31))
            return fail(HCH_EUNSUPPORTED, "hch_build_levels_device: offset tables exceed 32-bit indexing");
        hch::PairDesc *d_desc = nullptr;
        int32_t *d_cnt = nullptr, *d_first = nullptr, *d_fill = nullptr, *d_bucket = nullptr, *d_members = nullptr;
        int32_t *d_counters = nullptr, *d_free = nullptr;
        uint32_t *d_phi = nullptr, *d_res = nullptr;
        int2 *d_cells = nullptr;
        if ((st = tmp.get((void **)&d_desc, desc.size() * sizeof(hch::PairDesc), -1, s)) != HCH_OK) return st;
        HCH_HIP(hipMemcpyAsync(d_desc, desc.data(), desc.size() * sizeof(hch::PairDesc), hipMemcpyHostToDevice, s));
        if ((st = tmp.get((void **)&d_cnt, (size_t)cells * 4, 0, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_first, (size_t)cells * 4, -1, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_fill, (size_t)cells * 4, 0, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_phi, (size_t)cells * 4, 0, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_bucket, (size_t)vox * 4, -1, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_members, (size_t)vox * 4, -1, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_res, (size_t)vox * 4, -1, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_free, (size_t)slots * 4, -1, s)) != HCH_OK) return st;
        if ((st = tmp.get((void **)&d_cells, (size_t)cells * hch::PSH_CLASSES * sizeof(int2), -1, s)) != HCH_OK) return st;
        // counters: [0, CLASSES) buckets per class, then per active pair: free slots, singles placed
        const size_t n_counters = (size_t)hch::PSH_CLASSES + 2 * (size_t)na;
        if ((st = tmp.get((void **)&d_counters, n_counters * 4, 0, s)) != HCH_OK) return st;
        int32_t *d_class_count = d_counters, *d_nfree = d_counters + hch::PSH_CLASSES, *d_rank = d_nfree + na;
        HCH_HIP(hipMemsetAsync(d_fail, 0, (size_t)n_pairs * 4, s));

        const dim3 gv((unsigned)((max_n + 255) / 256), (unsigned)na), gc((unsigned)((max_r3 + 255) / 256), (unsigned)na);
        const dim3 gs((unsigned)((max_m3 + 255) / 256), (unsigned)na);
        HCH_LAUNCH(hch::psh_count_kernel, gv, dim3(256), 0, s, d_desc, d_cnt, d_bucket);
        HCH_LAUNCH(hch::psh_scan_kernel, dim3(1), dim3(1024), 0, s, d_cnt, d_first, (int)cells);
        HCH_LAUNCH(hch::psh_fill_kernel, gv, dim3(256), 0, s, d_desc, d_bucket, d_first, d_fill, d_members, d_res);
        HCH_LAUNCH(hch::psh_classify_kernel, gc, dim3(256), 0, s, d_desc, d_cnt, d_class_count, d_cells, cells);
        HCH_LAUNCH_CHECK("psh construction");
        int32_t class_count[hch::PSH_CLASSES];
        HCH_HIP(hipMemcpyAsync(class_count, d_class_count, sizeof class_count, hipMemcpyDeviceToHost, s));
        HCH_HIP(hipStreamSynchronize(s));
        // largest buckets first: all of 9 voxels and more in one launch, then one size per launch
        for (int k = hch::PSH_CLASSES - 1; k >= 2; --k) {
            if (class_count[k] <= 0) continue;
            HCH_HIP(hipMemsetAsync(d_nfree, 0, (size_t)na * 4, s));
            HCH_LAUNCH(hch::psh_free_list_kernel, gs, dim3(256), 0, s, d_desc, d_nfree, d_free);
            HCH_LAUNCH(hch::psh_place_kernel, dim3((unsigned)((class_count[k] + 3) / 4)), dim3(256), 0, s, d_desc,
                               d_cells + (size_t)k * cells, class_count[k], d_cnt, d_first, d_members, d_res, d_nfree,
                               d_free, d_phi, d_fail);
        }
        HCH_HIP(hipMemsetAsync(d_nfree, 0, (size_t)na * 4, s));
        HCH_LAUNCH(hch::psh_free_list_kernel, gs, dim3(256), 0, s, d_desc, d_nfree, d_free);
        HCH_LAUNCH(hch::psh_place_single_kernel, gc, dim3(256), 0, s, d_desc, d_cnt, d_first, d_members, d_res,
                           d_nfree, d_free, d_rank, d_phi, d_fail);
        HCH_LAUNCH_CHECK("psh construction");
        HCH_HIP(hipMemcpyAsync(h_fail.data(), d_fail, (size_t)n_pairs * 4, hipMemcpyDeviceToHost, s));
        HCH_HIP(hipStreamSynchronize(s));

        std::vector<int> again;
        for (int a = 0; a < na; ++a) {
            PairWork &w = work[active[a]];
            Level &L = hl->lv[w.l];
            if (!h_fail[active[a]]) {
                w.done = true;
                w.phi = d_phi + desc[a].cell_base;
                continue;
            }
            const size_t m3 = (size_t)w.m * w.m * w.m;
            HCH_HIP(hipMemsetAsync(L.dH + L.M[w.v], 0xFF, m3 * 4, s));
            HCH_HIP(hipMemsetAsync(L.dT + 3 * L.M[w.v], 0xFF, m3 * 6, s));
            w.r = hch::offset_side_next(w.r, w.m);
            again.push_back(active[a]);
        }
        active.swap(again);
    }

    // super tables of every level from the pairs' results
    for (int l = 0; l < n_levels; ++l) {
        Level &L = hl->lv[l];
        std::vector<hch::PackDesc> pd((size_t)batch);
        int32_t widest = 0;
        for (int v = 0; v < batch; ++v) {
            const PairWork &w = work[(size_t)l * batch + v];
            L.rbar[v] = w.r; L.attempts[v] = w.attempts;
            L.R[v + 1] = L.R[v] + (int64_t)w.r * w.r * w.r;
        }
        L.r_total = L.R[batch];
        if (L.r_total >= ((int64_t)1 << 31) / 3) return fail(HCH_EUNSUPPORTED, "hch_build_levels_device: super table exceeds 32-bit indexing");
        for (int v = 0; v < batch; ++v) {
            const PairWork &w = work[(size_t)l * batch + v];
            pd[v] = hch::PackDesc{w.phi, w.m * w.m * w.m, w.r * w.r * w.r, (int32_t)L.M[v], (int32_t)L.R[v]};
            widest = std::max(widest, std::max(pd[v].m3, pd[v].r3));
        }
        hch::PackDesc *d_pd = nullptr;
        if ((st = tmp.get((void **)&d_pd, pd.size() * sizeof(hch::PackDesc), -1, s)) != HCH_OK) return st;
        HCH_HIP(hipMemcpyAsync(d_pd, pd.data(), pd.size() * sizeof(hch::PackDesc), hipMemcpyHostToDevice, s));
        HCH_HIP(hipMalloc((void **)&L.dPhi, std::max<size_t>(16, (size_t)L.r_total * 3)));
        HCH_HIP(hipMalloc((void **)&L.dphi4, std::max<size_t>(16, (size_t)L.r_total * 4)));
        HCH_HIP(hipMalloc((void **)&L.dslot3, (size_t)L.m_total * 4 * hch::SLOT_WORDS));
        HCH_LAUNCH(hch::psh_pack_kernel, dim3((unsigned)((widest + 255) / 256), (unsigned)batch), dim3(256), 0, s,
                           d_pd, L.dH, L.dT, L.dslot3, L.dV, L.dphi4, L.dPhi);
        HCH_LAUNCH_CHECK("psh_pack_kernel");
        std::vector<int32_t> meta;
        meta.insert(meta.end(), L.mbar.begin(), L.mbar.end());
        meta.insert(meta.end(), L.rbar.begin(), L.rbar.end());
        for (int64_t x : L.M) meta.push_back((int32_t)x);
        for (int64_t x : L.R) meta.push_back((int32_t)x);
        for (int64_t x : L.N) meta.push_back((int32_t)x);
        if ((st = upload((void **)&L.dmeta, meta.data(), meta.size() * 4, s)) != HCH_OK) return st;
        // host copies for hch_level_info
        L.H.resize((size_t)L.m_total); L.V.resize((size_t)L.m_total);
        L.T.resize((size_t)L.m_total * 3); L.Phi.resize((size_t)L.r_total * 3);
        HCH_HIP(hipMemcpyAsync(L.H.data(), L.dH, L.H.size() * 4, hipMemcpyDeviceToHost, s));
        HCH_HIP(hipMemcpyAsync(L.V.data(), L.dV, L.V.size() * 4, hipMemcpyDeviceToHost, s));
        HCH_HIP(hipMemcpyAsync(L.T.data(), L.dT, L.T.size() * 2, hipMemcpyDeviceToHost, s));
        if (L.r_total) HCH_HIP(hipMemcpyAsync(L.Phi.data(), L.dPhi, L.Phi.size(), hipMemcpyDeviceToHost, s));
        HCH_HIP(hipStreamSynchronize(s));     // `meta` and `pd` die here
    }
    return HCH_OK;
}

// ratios == nullptr: every level halves the resolution (a power of two); else ratios[l] >= 2 is
// the ratio between level l and level l+1, whose side is ceil(side_l / ratios[l])
// Run `fn` on up to `nthr` host threads (the caller's included) and wait for all of them.  An
// exception inside a worker (std::bad_alloc from its vectors, std::system_error) must not leave
// the thread function: it is caught there and reported as false.  Threads that were started are
// always joined, also when starting a further one fails.
template <typename Fn>
static bool run_on_threads(unsigned nthr, Fn fn)
{
    std::atomic<int> failed(0);
    auto guarded = [&]() {
        try { fn(); } catch (...) { failed = 1; }
    };
    std::vector<std::thread> pool;
    struct Joiner {
        std::vector<std::thread> &p;
        ~Joiner() { for (auto &th : p) if (th.joinable()) th.join(); }
    } joiner{pool};
    try {
        pool.reserve(nthr);
        for (unsigned i = 1; i < nthr; ++i) pool.emplace_back(guarded);
    } catch (...) {
        failed = 1;             // fewer threads than wanted: the work is still done below
    }
    guarded();
    for (auto &th : pool) th.join();
    return failed == 0;
}

static hch_status build_impl(const int32_t *coords_xyz, const int64_t *model_offsets,
                             int32_t batch, int32_t resolution, int32_t n_levels, const int32_t *ratios,
                             void *stream, bool with_device, bool device_tables, hch_levels **out)
{
    if (out) *out = nullptr;
    if (!coords_xyz || !model_offsets || !out) return fail(HCH_EINVAL, "hch_build_levels: null pointer");
    if (batch <= 0 || batch > 65535) return fail(HCH_EINVAL, "hch_build_levels: batch must be 1..65535");
    std::vector<int32_t> side((size_t)std::max(n_levels, 1), resolution), ratio_of((size_t)std::max(n_levels, 1), 1);
    if (!ratios) {
        if (resolution < 2 || resolution > 32768 || (resolution & (resolution - 1)))
            return fail(HCH_EINVAL, "hch_build_levels: resolution must be a power of two in 2..32768");
        if (n_levels < 1 || (resolution >> (n_levels - 1)) < 1)
            return fail(HCH_EINVAL, "hch_build_levels: n_levels out of range for this resolution");
        for (int l = 1; l < n_levels; ++l) { side[l] = resolution >> l; ratio_of[l] = 2; }
    } else {
        if (resolution < 2 || resolution > 32768)
            return fail(HCH_EINVAL, "hch_build_levels_ratios: resolution must be in 2..32768");
        if (n_levels < 1) return fail(HCH_EINVAL, "hch_build_levels_ratios: n_levels must be at least 1");
        for (int l = 1; l < n_levels; ++l) {
            if (ratios[l - 1] < 2 || side[l - 1] < 2)
                return fail(HCH_EINVAL, "hch_build_levels_ratios: every ratio must be >= 2 and every level but the last have side >= 2");
            ratio_of[l] = ratios[l - 1];
            side[l] = (side[l - 1] + ratios[l - 1] - 1) / ratios[l - 1];
        }
    }
    if (model_offsets[0] != 0) return fail(HCH_EINVAL, "hch_build_levels: model_offsets[0] must be 0");
    for (int v = 0; v < batch; ++v)
        if (model_offsets[v + 1] <= model_offsets[v])
            return fail(HCH_EINVAL, "hch_build_levels: empty model or decreasing model_offsets");
    const int64_t n_total = model_offsets[batch];
    if (n_total >= ((int64_t)1 << 31) / 27)
        return fail(HCH_EUNSUPPORTED, "hch_build_levels: more than 2^31/27 voxels in a batch");
    for (int64_t i = 0; i < 3 * n_total; ++i)
        if (coords_xyz[i] < 0 || coords_xyz[i] >= resolution)
            return fail(HCH_EINVAL, "hch_build_levels: coordinate outside [0, resolution)");
    // duplicates inside a model (models in parallel on host threads)
    {
        std::atomic<int> next_model(0), dup(0);
        auto check = [&]() {
            std::vector<int64_t> lin;
            for (;;) {
                const int v = next_model.fetch_add(1);
                if (v >= batch) break;
                const int64_t a = model_offsets[v], n = model_offsets[v + 1] - a;
                lin.resize((size_t)n);
                for (int64_t i = 0; i < n; ++i) {
                    const int32_t *p = coords_xyz + 3 * (a + i);
                    lin[i] = ((int64_t)p[0] * resolution + p[1]) * resolution + p[2];
                }
                std::sort(lin.begin(), lin.end());
                if (std::adjacent_find(lin.begin(), lin.end()) != lin.end()) dup = 1;
            }
        };
        const unsigned nthr = std::max(1u, std::min({std::thread::hardware_concurrency(), 16u, (unsigned)batch}));
        if (!run_on_threads(nthr, check)) return fail(HCH_ENOMEM, "hch_build_levels: out of host memory");
        if (dup) return fail(HCH_EINVAL, "hch_build_levels: duplicate voxel inside a model");
    }

    hch_levels *hl = new (std::nothrow) hch_levels;
    if (!hl) return fail(HCH_ENOMEM, "hch_build_levels: out of host memory");
    hipStream_t s = (hipStream_t)stream;
    hch_status st = HCH_OK;

    try {
        hl->lv.resize((size_t)n_levels);
        // ---- occupancy of every level (host) ----
        for (int l = 0; l < n_levels; ++l) {
            Level &L = hl->lv[l];
            L.ubar = side[l];
            L.ratio = ratio_of[l];
            L.b = batch;
            L.N.assign((size_t)batch + 1, 0);
            if (l == 0) {
                L.coords.assign(coords_xyz, coords_xyz + 3 * n_total);
                for (int v = 0; v <= batch; ++v) L.N[v] = model_offsets[v];
            } else {
                const Level &Lf = hl->lv[l - 1];
                std::vector<std::vector<int32_t>> per_model((size_t)batch);
                std::atomic<int> next_model(0);
                auto coarsen = [&]() {
                    for (;;) {
                        const int v = next_model.fetch_add(1);
                        if (v >= batch) break;
                        hch::coarsen_model(Lf.coords.data() + 3 * Lf.N[v], Lf.N[v + 1] - Lf.N[v], Lf.ubar, L.ratio, per_model[v]);
                    }
                };
                {
                    const unsigned nthr = std::max(1u, std::min({std::thread::hardware_concurrency(), 16u, (unsigned)batch}));
                    if (!run_on_threads(nthr, coarsen)) throw std::bad_alloc();
                }
                for (int v = 0; v < batch; ++v) {
                    L.coords.insert(L.coords.end(), per_model[v].begin(), per_model[v].end());
                    L.N[v + 1] = L.N[v] + (int64_t)per_model[v].size() / 3;
                }
            }
            L.n_total = L.N[batch];
            L.max_n = 0;
            for (int v = 0; v < batch; ++v) L.max_n = std::max<int32_t>(L.max_n, (int32_t)(L.N[v + 1] - L.N[v]));
        }

        if (device_tables) {
            if (n_levels > hch::MAX_LEVELS) st = fail(HCH_EUNSUPPORTED, "hch_build_levels: too many levels");
            if (st == HCH_OK) st = device_construct(hl, s);
        }
        // ---- PSH construction of every (level, model), spread over host threads ----
        std::vector<std::vector<hch::ModelTables>> tabs((size_t)n_levels);
        for (auto &t : tabs) t.resize((size_t)batch);
        const int n_tasks = device_tables ? 0 : n_levels * batch;
        std::vector<int> result((size_t)n_tasks, 0);
        std::atomic<int> next(0);
        auto worker = [&]() {
            for (;;) {
                const int t = next.fetch_add(1);
                if (t >= n_tasks) break;
                const int l = t / batch, v = t % batch;     // finest (largest) levels first
                const Level &L = hl->lv[l];
                result[t] = (int)hch::build_model_tables(L.coords.data() + 3 * L.N[v],
                                                         L.N[v + 1] - L.N[v], L.ubar, tabs[l][v]);
            }
        };
        {
            unsigned nthr = std::thread::hardware_concurrency();
            nthr = std::max(1u, std::min(nthr, 16u));
            nthr = std::min<unsigned>(nthr, (unsigned)std::max(1, n_tasks));
            if (!run_on_threads(nthr, worker)) throw std::bad_alloc();
        }
        for (int t = 0; t < n_tasks && st == HCH_OK; ++t) {
            if (result[t] == hch::BUILD_UNSUPPORTED)
                st = fail(HCH_EUNSUPPORTED, "hch_build_levels: a model needs a hash table side above 256");
            else if (result[t] == hch::BUILD_FAILED)
                st = fail(HCH_EBUILD, "hch_build_levels: perfect hash construction failed");
        }

        // ---- super tables (Section 3.2) and upload ----
        for (int l = 0; l < n_levels && st == HCH_OK; ++l) {
            Level &L = hl->lv[l];
            if (device_tables) {      // tables are already resident; only the index lists are missing
                if (hipMalloc((void **)&L.dnbr, (size_t)L.n_total * 27 * 4) != hipSuccess) {
                    L.dnbr = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(nbr27) failed"); break;
                }
                if (l > 0 && L.ratio == 2 && hipMalloc((void **)&L.dchild, (size_t)L.n_total * 8 * 4) != hipSuccess) {
                    L.dchild = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(child8) failed"); break;
                }
                continue;
            }
            L.mbar.resize((size_t)batch); L.rbar.resize((size_t)batch); L.attempts.resize((size_t)batch);
            L.M.assign((size_t)batch + 1, 0); L.R.assign((size_t)batch + 1, 0);
            for (int v = 0; v < batch; ++v) {
                const hch::ModelTables &t = tabs[l][v];
                L.mbar[v] = t.m; L.rbar[v] = t.r; L.attempts[v] = t.attempts;
                L.M[v + 1] = L.M[v] + (int64_t)t.m * t.m * t.m;
                L.R[v + 1] = L.R[v] + (int64_t)t.r * t.r * t.r;
            }
            L.m_total = L.M[batch]; L.r_total = L.R[batch];
            if (L.m_total >= ((int64_t)1 << 31) || L.r_total >= ((int64_t)1 << 31) / 3) {
                st = fail(HCH_EUNSUPPORTED, "hch_build_levels: super table exceeds 32-bit indexing");
                break;
            }
            L.H.resize((size_t)L.m_total); L.V.resize((size_t)L.m_total);
            L.T.resize((size_t)L.m_total * 3); L.Phi.resize((size_t)L.r_total * 3);
            for (int v = 0; v < batch; ++v) {
                hch::ModelTables &t = tabs[l][v];
                std::copy(t.H.begin(), t.H.end(), L.H.begin() + L.M[v]);
                std::copy(t.T.begin(), t.T.end(), L.T.begin() + 3 * L.M[v]);
                std::copy(t.Phi.begin(), t.Phi.end(), L.Phi.begin() + 3 * L.R[v]);
                std::fill(L.V.begin() + L.M[v], L.V.begin() + L.M[v + 1], v);
                t = hch::ModelTables();
            }
            if (!with_device) continue;
            std::vector<int32_t> meta;
            meta.insert(meta.end(), L.mbar.begin(), L.mbar.end());
            meta.insert(meta.end(), L.rbar.begin(), L.rbar.end());
            for (int64_t x : L.M) meta.push_back((int32_t)x);
            for (int64_t x : L.R) meta.push_back((int32_t)x);
            for (int64_t x : L.N) meta.push_back((int32_t)x);

            if ((st = upload((void **)&L.dH, L.H.data(), L.H.size() * 4, s)) != HCH_OK) break;
            if ((st = upload((void **)&L.dV, L.V.data(), L.V.size() * 4, s)) != HCH_OK) break;
            if ((st = upload((void **)&L.dT, L.T.data(), L.T.size() * 2, s)) != HCH_OK) break;
            if ((st = upload((void **)&L.dPhi, L.Phi.data(), L.Phi.size(), s)) != HCH_OK) break;
            if ((st = upload((void **)&L.dcoords, L.coords.data(), L.coords.size() * 4, s)) != HCH_OK) break;
            if ((st = upload((void **)&L.dmeta, meta.data(), meta.size() * 4, s)) != HCH_OK) break;
            constexpr int SW = hch::SLOT_WORDS;
            std::vector<uint32_t> slot3((size_t)L.m_total * SW, 0u), phi4((size_t)L.r_total);
            for (int64_t q = 0; q < L.m_total; ++q) {
                slot3[SW * q + 0] = (uint32_t)L.H[q];
                slot3[SW * q + 1] = (uint32_t)L.T[3 * q] | ((uint32_t)L.T[3 * q + 1] << 16);
                slot3[SW * q + 2] = (uint32_t)L.T[3 * q + 2];
            }
            for (int64_t q = 0; q < L.r_total; ++q)
                phi4[q] = (uint32_t)L.Phi[3 * q] | ((uint32_t)L.Phi[3 * q + 1] << 8) | ((uint32_t)L.Phi[3 * q + 2] << 16);
            if ((st = upload((void **)&L.dslot3, slot3.data(), slot3.size() * 4, s)) != HCH_OK) break;
            if ((st = upload((void **)&L.dphi4, phi4.data(), phi4.size() * 4, s)) != HCH_OK) break;
            if (hipMalloc((void **)&L.dnbr, (size_t)L.n_total * 27 * 4) != hipSuccess) {
                L.dnbr = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(nbr27) failed"); break;
            }
            if (l > 0 && L.ratio == 2 && hipMalloc((void **)&L.dchild, (size_t)L.n_total * 8 * 4) != hipSuccess) {
                L.dchild = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(child8) failed"); break;
            }
            // the staging vectors die at the end of this iteration: finish the copies first
            hipError_t e = hipStreamSynchronize(s);
            if (e != hipSuccess) { st = fail(HCH_EHIP, std::string("hipStreamSynchronize: ") + hipGetErrorString(e)); break; }
        }
        if (st == HCH_OK && with_device) {
            if (n_levels > hch::MAX_LEVELS) st = fail(HCH_EUNSUPPORTED, "hch_build_levels: too many levels");
        }
        if (st == HCH_OK && with_device) {
            // buffers of the pattern order (see launch_index_lists)
            hl->sort_off.assign((size_t)n_levels + 1, 0);
            for (int l = 0; l < n_levels; ++l) hl->sort_off[l + 1] = hl->sort_off[l] + (int32_t)hl->lv[l].n_total;
            const size_t n_all = (size_t)hl->sort_off[n_levels];
            int64_t nbr_tiles = 0;
            for (int l = 0; l < n_levels; ++l)
                for (int v = 0; v < batch; ++v) nbr_tiles += (hl->lv[l].N[v + 1] - hl->lv[l].N[v] + 255) / 256;
            if (hipMalloc((void **)&hl->d_sort_key, std::max<size_t>(n_all, 64)) != hipSuccess) { hl->d_sort_key = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(pattern keys) failed"); }
            if (st == HCH_OK && hipMalloc((void **)&hl->d_order, std::max<size_t>(n_all, 64) * 4) != hipSuccess) { hl->d_order = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(pattern order) failed"); }
            if (st == HCH_OK && hipMalloc((void **)&hl->d_tile_hist, (size_t)std::max<int64_t>(nbr_tiles, 1) * hch::PATTERN_BINS * 4) != hipSuccess) { hl->d_tile_hist = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(tile histograms) failed"); }
            if (st == HCH_OK && hipMalloc((void **)&hl->d_key_total, (size_t)hch::MAX_LEVELS * hch::PATTERN_BINS * 4) != hipSuccess) { hl->d_key_total = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(key totals) failed"); }
            for (int l = 0; l < n_levels && st == HCH_OK; ++l) {
                Level &L = hl->lv[l];
                const size_t tiles = (size_t)((L.n_total + hch::PATTERN_TILE - 1) / hch::PATTERN_TILE);
                if (hipMalloc((void **)&L.dmask27, std::max<size_t>((size_t)L.n_total, 64) * 4) != hipSuccess) { L.dmask27 = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(mask27) failed"); break; }
                if (hipMalloc((void **)&L.dtilemask, std::max<size_t>(tiles, 64) * 4) != hipSuccess) { L.dtilemask = nullptr; st = fail(HCH_ENOMEM, "hipMalloc(tile masks) failed"); break; }
                L.dorder = hl->d_order + hl->sort_off[l];
            }
        }
        if (st == HCH_OK && with_device) {
            hl->set.batch = batch;
            hl->nbr_prefix.assign((size_t)n_levels * batch + 1, 0);
            hl->child_prefix.assign((size_t)n_levels * batch + 1, 0);
            for (int l = 0; l < n_levels; ++l) {
                Level &L = hl->lv[l];
                hl->set.view[l] = L.view();
                hl->set.coords[l] = L.dcoords;
                hl->set.nbr[l] = L.dnbr;
                hl->set.child[l] = L.dchild;
                hl->set.mask27[l] = L.dmask27;
                hl->set.sort_off[l] = hl->sort_off[l];
                hl->set.level_tile0[l] = hl->nbr_prefix[(size_t)l * batch];
                for (int v = 0; v < batch; ++v) {
                    const int32_t tiles = (int32_t)((L.N[v + 1] - L.N[v] + 255) / 256);
                    const size_t e = (size_t)l * batch + v;
                    hl->nbr_prefix[e + 1] = hl->nbr_prefix[e] + tiles;
                    hl->child_prefix[e + 1] = hl->child_prefix[e] + (l > 0 && L.ratio == 2 ? tiles : 0);
                }
            }
            hl->set.sort_key = hl->d_sort_key;
            hl->set.tile_hist = hl->d_tile_hist;
            for (int l = 0; l < n_levels; ++l) {
                hl->set.level_tile0[l] = hl->nbr_prefix[(size_t)l * batch];
                hl->set.level_tiles[l] = hl->nbr_prefix[(size_t)(l + 1) * batch] - hl->nbr_prefix[(size_t)l * batch];
                hl->set.hist_off[l] = hl->set.level_tile0[l] * hch::PATTERN_BINS;
            }
            if ((st = upload((void **)&hl->d_nbr_prefix, hl->nbr_prefix.data(), hl->nbr_prefix.size() * 4, s)) == HCH_OK)
                st = upload((void **)&hl->d_child_prefix, hl->child_prefix.data(), hl->child_prefix.size() * 4, s);
            if (st == HCH_OK) st = hch_build_neighbours(hl, -1, s);
        }
        if (st == HCH_OK && with_device) {
            hipError_t e = hipStreamSynchronize(s);
            if (e != hipSuccess) st = fail(HCH_EHIP, std::string("hipStreamSynchronize: ") + hipGetErrorString(e));
        }
        // occupied-neighbour count of every level (used only for reporting algorithmic traffic)
        if (st == HCH_OK && with_device) {
            unsigned long long *d_cnt = nullptr;
            std::vector<unsigned long long> h_cnt((size_t)n_levels, 0);
            if (hipMalloc((void **)&d_cnt, (size_t)n_levels * 8) != hipSuccess) st = fail(HCH_ENOMEM, "hipMalloc failed");
            if (st == HCH_OK) {
                hipError_t e = hipMemsetAsync(d_cnt, 0, (size_t)n_levels * 8, s);
                for (int l = 0; l < n_levels && e == hipSuccess; ++l) {
                    const int64_t items = hl->lv[l].n_total * 27;
                    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>(4096, (items + 255) / 256));
                    HCH_LAUNCH(hch::count_valid_kernel, dim3(grid), dim3(256), 0, s, hl->lv[l].dnbr, items, d_cnt + l);
                    e = hipGetLastError();
                }
                if (e == hipSuccess) e = hipMemcpyAsync(h_cnt.data(), d_cnt, (size_t)n_levels * 8, hipMemcpyDeviceToHost, s);
                if (e == hipSuccess) e = hipStreamSynchronize(s);
                if (e != hipSuccess) st = fail(HCH_EHIP, std::string("neighbour count: ") + hipGetErrorString(e));
                for (int l = 0; l < n_levels; ++l) hl->lv[l].nbr_valid = (int64_t)h_cnt[l];
            }
            if (d_cnt) (void)hipFree(d_cnt);
        }
    } catch (const std::bad_alloc &) {
        st = fail(HCH_ENOMEM, "hch_build_levels: out of host memory");
    }

    if (st != HCH_OK) { hch_free_levels(hl); return st; }
    *out = hl;
    return HCH_OK;
}

extern "C" hch_status hch_build_levels(const int32_t *coords_xyz, const int64_t *model_offsets,
                                       int32_t batch, int32_t resolution, int32_t n_levels,
                                       void *stream, hch_levels **out)
{
    return build_impl(coords_xyz, model_offsets, batch, resolution, n_levels, nullptr, stream, true, false, out);
}

extern "C" hch_status hch_build_levels_device(const int32_t *coords_xyz, const int64_t *model_offsets,
                                              int32_t batch, int32_t resolution, int32_t n_levels,
                                              void *stream, hch_levels **out)
{
    return build_impl(coords_xyz, model_offsets, batch, resolution, n_levels, nullptr, stream, true, true, out);
}

extern "C" hch_status hch_build_levels_ratios(const int32_t *coords_xyz, const int64_t *model_offsets,
                                              int32_t batch, int32_t resolution, int32_t n_levels,
                                              const int32_t *ratios, int32_t device_tables,
                                              void *stream, hch_levels **out)
{
    if (n_levels > 1 && !ratios) {
        if (out) *out = nullptr;
        return fail(HCH_EINVAL, "hch_build_levels_ratios: null ratios");
    }
    static const int32_t none[1] = {2};
    return build_impl(coords_xyz, model_offsets, batch, resolution, n_levels, ratios ? ratios : none, stream, true,
                      device_tables != 0, out);
}

extern "C" hch_status hch_build_tables_host(const int32_t *coords_xyz, const int64_t *model_offsets,
                                            int32_t batch, int32_t resolution, int32_t n_levels,
                                            hch_levels **out)
{
    return build_impl(coords_xyz, model_offsets, batch, resolution, n_levels, nullptr, nullptr, false, false, out);
}

extern "C" hch_status hch_level_info(const hch_levels *levels, int32_t level, hch_level_desc *out)
{
    if (!levels || !out || level < 0 || level >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_level_info: bad argument");
    const Level &L = levels->lv[level];
    out->ubar = L.ubar; out->batch = L.b;
    out->n_total = L.n_total; out->m_total = L.m_total; out->r_total = L.r_total;
    out->nbr_valid = L.nbr_valid;
    out->mbar = L.mbar.data(); out->rbar = L.rbar.data(); out->attempts = L.attempts.data();
    out->M = L.M.data(); out->R = L.R.data(); out->N = L.N.data();
    out->coords_host = L.coords.data();
    out->H_host = L.H.data(); out->T_host = L.T.data(); out->Phi_host = L.Phi.data();
    out->V_host = L.V.data();
    out->H = L.dH; out->T = L.dT; out->Phi = L.dPhi; out->V = L.dV; out->coords = L.dcoords;
    out->nbr27 = L.dnbr; out->child8 = L.dchild;
    out->row_order = L.dorder; out->tile_taps = L.dtilemask;
    return HCH_OK;
}

// ---------------------------------------------------------------------------------------
// hash2col / col2hash
// ---------------------------------------------------------------------------------------

static hch_status get_level(const hch_levels *levels, int32_t level, const Level **L, const char *who)
{
    if (!levels || level < 0 || level >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, std::string(who) + ": bad level");
    *L = &levels->lv[level];
    if (!(*L)->dnbr) return fail(HCH_EINVAL, std::string(who) + ": levels were built without device tables");
    return HCH_OK;
}

static inline int elem_size(hch_dtype d) { return d == HCH_BF16 ? 2 : 4; }

// voxels per workgroup for the gather / scatter kernels: large tiles when there are many voxels,
// smaller ones when the level is small so that the chip still gets a few thousand workgroups
static int tile_voxels(int64_t n, int lo, int hi)
{
    int64_t tv = n / 2048;
    tv = std::max<int64_t>(lo, std::min<int64_t>(hi, tv));
    return (int)tv;
}

static hch_status do_hash2col(const Level &L, hch_dtype dtype, const void *X, int c_in,
                              int64_t row_begin, int64_t rows, void *col, hipStream_t s)
{
    if (rows == 0) return HCH_OK;
    const int es = elem_size(dtype);
    const int row_bytes = c_in * es;
    // per voxel: 27 indices and its own feature row in (neighbour re-reads are cache hits),
    // 27 rows out (zeros included: the GEMM operand needs them)
    const double bytes = (double)rows * (108.0 + 28.0 * row_bytes);
    const int tv = tile_voxels(rows, 8, 128);
    const size_t lds = (size_t)tv * 27 * 4;
    const unsigned n_tiles = (unsigned)((rows + tv - 1) / tv);
    const unsigned grid = (n_tiles + hch::NUM_XCD - 1) / hch::NUM_XCD * hch::NUM_XCD;
    if (row_bytes % 16 == 0 && aligned16(X) && aligned16(col)) {
        hch::LaunchTimer lt(HCH_KERNEL_ID("hash2col_kernel<unsigned int __vector(4)>"), s, bytes, 0.0);
        HCH_LAUNCH(hch::hash2col_kernel<hch::u32x4>, dim3(grid), dim3(256), lds, s,
                           (const hch::u32x4 *)X, L.dnbr, (hch::u32x4 *)col, row_begin, rows, row_bytes / 16, tv, n_tiles);
    } else {
        hch::LaunchTimer lt(dtype == HCH_F32 ? HCH_KERNEL_ID("hash2col_kernel<float>") : HCH_KERNEL_ID("hash2col_kernel<unsigned short>"), s, bytes, 0.0);
        if (dtype == HCH_F32)
            HCH_LAUNCH(hch::hash2col_kernel<float>, dim3(grid), dim3(256), lds, s,
                               (const float *)X, L.dnbr, (float *)col, row_begin, rows, c_in, tv, n_tiles);
        else
            HCH_LAUNCH(hch::hash2col_kernel<uint16_t>, dim3(grid), dim3(256), lds, s,
                               (const uint16_t *)X, L.dnbr, (uint16_t *)col, row_begin, rows, c_in, tv, n_tiles);
    }
    HCH_LAUNCH_CHECK("hash2col");
    return HCH_OK;
}

extern "C" hch_status hch_hash2col(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                   const void *X, int32_t c_in, int64_t row_begin,
                                   int64_t row_count, void *col, void *stream)
{
    const Level *L;
    hch_status st = get_level(levels, level, &L, "hch_hash2col");
    if (st != HCH_OK) return st;
    if (!X || !col || c_in <= 0 || (dtype != HCH_F32 && dtype != HCH_BF16))
        return fail(HCH_EINVAL, "hch_hash2col: bad argument");
    if (row_begin < 0 || row_count < 0 || row_begin + row_count > L->n_total)
        return fail(HCH_EINVAL, "hch_hash2col: row range outside the level");
    return do_hash2col(*L, dtype, X, c_in, row_begin, row_count, col, (hipStream_t)stream);
}

// planes: dcol is stored tap-major, [27][n][c_in] (the library's own layout between the data
// gradient product and this gather; needs c_in % 4 == 0), instead of [n][27*c_in]
static hch_status do_col2hash(const Level &L, const float *dcol, int c_in, float *dX, bool planes, hipStream_t s)
{
    if (L.n_total == 0) return HCH_OK;
    // per voxel: 27 indices in, one c_in row per occupied neighbour in, one row out
    const double bytes = (double)L.n_total * (108.0 + 4.0 * c_in) + (double)L.nbr_valid * 4.0 * c_in;
    const bool vec = c_in % 4 == 0 && aligned16(dcol) && aligned16(dX);
    if (planes && !vec) return fail(HCH_EINVAL, "col2hash: tap-major layout needs aligned 4-channel units");
    hch::LaunchTimer lt(planes ? HCH_KERNEL_ID("col2hash_kernel<4, true>")
                               : (vec ? HCH_KERNEL_ID("col2hash_kernel<4, false>") : HCH_KERNEL_ID("col2hash_kernel<1, false>")),
                        s, bytes, (double)L.nbr_valid * c_in);
    const int cu = vec ? c_in / 4 : c_in;
    const int tv = std::max(4, std::min(128, 256 / cu));
    const size_t lds = (size_t)tv * 27 * 4;
    const unsigned n_tiles = (unsigned)((L.n_total + tv - 1) / tv);
    const unsigned grid = (n_tiles + hch::NUM_XCD - 1) / hch::NUM_XCD * hch::NUM_XCD;
    if (planes)
        HCH_LAUNCH((hch::col2hash_kernel<4, true>), dim3(grid), dim3(256), lds, s, dcol, L.dnbr, dX,
                           L.n_total, c_in, tv, n_tiles);
    else if (vec)
        HCH_LAUNCH((hch::col2hash_kernel<4, false>), dim3(grid), dim3(256), lds, s, dcol, L.dnbr, dX,
                           L.n_total, c_in, tv, n_tiles);
    else
        HCH_LAUNCH((hch::col2hash_kernel<1, false>), dim3(grid), dim3(256), lds, s, dcol, L.dnbr, dX,
                           L.n_total, c_in, tv, n_tiles);
    HCH_LAUNCH_CHECK("col2hash");
    return HCH_OK;
}

extern "C" hch_status hch_col2hash(const hch_levels *levels, int32_t level, const float *dcol,
                                   int32_t c_in, float *dX, void *stream)
{
    const Level *L;
    hch_status st = get_level(levels, level, &L, "hch_col2hash");
    if (st != HCH_OK) return st;
    if (!dcol || !dX || c_in <= 0) return fail(HCH_EINVAL, "hch_col2hash: bad argument");
    return do_col2hash(*L, dcol, c_in, dX, false, (hipStream_t)stream);
}

// ---------------------------------------------------------------------------------------
// GEMM launches
// ---------------------------------------------------------------------------------------

// slices of a split reduction are multiples of the reduction length of one tile
static inline int k_gran(hch_dtype dtype) { return dtype == HCH_BF16 ? hch::BF16_BK : hch::GEMM_BK; }

// tile shape and split of one product
// hch_set_lean_loops: 0 = every product takes the pointer-based form of its main loop
static std::atomic<int> g_lean_loops{1};

struct GemmPlan {
    int bm, bn, wm;
    int splits, k_per_split;
};

// fwd-like products (M = voxels): wide tiles when there are many row tiles, 64-row tiles and a
// split of the reduction when the level is too small to fill the chip
static GemmPlan plan_rows(int64_t M, int N, int K, bool allow_split, int gran = hch::GEMM_BK)
{
    GemmPlan p;
    p.bn = N <= 16 ? 16 : (N <= 32 ? 32 : 64);
    p.bm = 128; p.wm = 4;
    const int64_t n_tiles = (N + p.bn - 1) / p.bn;
    int64_t blocks = (M + 127) / 128 * n_tiles;
    if (p.bn == 64 && blocks < 1024) { p.bm = 64; p.wm = 2; blocks = (M + 63) / 64 * n_tiles; }
    p.splits = 1; p.k_per_split = K + hch::GEMM_BK;
    if (allow_split && blocks < 512 && K >= 512) {
        // as many slices as fit the chip in one round of workgroups (4 per CU with the 64-row
        // tile, 3 with the 128-row ones): a second, nearly empty round costs as much as a full one
        const int64_t resident = p.bm == 64 ? 1024 : 768;
        int64_t want = std::min<int64_t>(resident / blocks, K / 256);
        want = std::max<int64_t>(1, want);
        int64_t kps = (K + want - 1) / want;
        kps = (kps + gran - 1) / gran * gran;
        p.k_per_split = (int)kps;
        p.splits = (int)((K + kps - 1) / kps);
    }
    return p;
}

// weight-gradient product (M = 27*c_in, N = c_out, reduction over n voxels split in slices)
static GemmPlan plan_wgrad(int64_t n, int c_in, int c_out, int taps = 27, int gran = hch::GEMM_BK)
{
    GemmPlan p;
    const int Kc = taps * c_in;
    p.bn = c_out <= 16 ? 16 : (c_out <= 32 ? 32 : 64);
    p.bm = 128; p.wm = 4;
    const int64_t tiles = (int64_t)((Kc + 127) / 128) * ((c_out + p.bn - 1) / p.bn);
    int64_t want = std::max<int64_t>(1, 768 / tiles);   // one round of workgroups, 3 per CU
    // bf16 kernel: a multiple of 8 slices, each XCD (32 CUs, 96 workgroups at a time) taking
    // whole slices, if that still fills most of the chip
    if (gran == hch::BF16_BK && tiles <= 96 && (96 / tiles) * tiles >= 64) want = 8 * (96 / tiles);
    want = std::min<int64_t>(want, std::max<int64_t>(1, (n + 255) / 256));
    // fp32 kernel: a multiple of 8 slices as well (each XCD takes whole slices and gathers their
    // voxels once for all its tiles) where that costs at most an eighth of the slices
    if (gran != hch::BF16_BK && want >= 8) want = want / 8 * 8;
    int64_t rows = (n + want - 1) / want;
    rows = std::max<int64_t>(gran, (rows + gran - 1) / gran * gran);
    p.k_per_split = (int)rows;
    p.splits = (int)std::max<int64_t>(1, (n + rows - 1) / rows);
    // keep the count a multiple of 8 (rounding the slice length up may have dropped a few slices;
    // the extra ones are empty and write zeros)
    if (want >= 8 && want % 8 == 0 && p.splits <= want) p.splits = (int)((p.splits + 7) / 8 * 8);
    return p;
}

static inline bool k_split_aligned(const GemmPlan &p) { return p.k_per_split % 4 == 0; }

template <typename TIN, int AMODE, bool B_KC>
static hch_status launch_gemm_t(const GemmPlan &plan, const void *A, const void *B, float *C,
                                const int32_t *nbr, int M, int N, int K, int64_t lda, int64_t ldb,
                                int64_t ldc, int64_t c_split_stride, double alg_bytes, hipStream_t s,
                                int c_planes = 0, int taps = 27, int b_wrap = 0, int64_t b_tap_stride = 0,
                                const int32_t *rowmap = nullptr, const uint32_t *tilemask = nullptr, int64_t a_rows = 0,
                                const uint32_t *rowmask = nullptr, int mask_c = 1)
{
    if (M <= 0 || N <= 0) return HCH_OK;
    GemmPlan p = plan;
    // vector path: every 4-element unit is aligned and wholly inside or outside its matrix
    const uintptr_t amask = sizeof(TIN) * 4 - 1;
    const bool a_fast_ok = (AMODE == hch::A_COLS) ? (M % 4 == 0) : (K % 4 == 0 || AMODE == hch::A_GATHER_T);
    const bool b_fast_ok = B_KC ? (K % 4 == 0) : (N % 4 == 0);
    const bool vec = (lda % 4 == 0) && (ldb % 4 == 0) && a_fast_ok && b_fast_ok &&
                     !(reinterpret_cast<uintptr_t>(A) & amask) && !(reinterpret_cast<uintptr_t>(B) & amask) &&
                     (k_split_aligned(p));
    if (b_wrap && !vec) return fail(HCH_EINVAL, "gemm: in-place weight reading needs aligned operands");
    if (!vec || AMODE != hch::A_GATHER || taps != 27) rowmap = nullptr;     // rows in pattern order and tap skipping:
    if (!rowmap) tilemask = nullptr;                                        // the vector path of the 3x3x3 gather only
    if (!vec && p.bm == 64) { p.bm = 128; p.wm = 4; }   // the generic path has the 128-row tiles only
    const int c_vec_ok = (c_planes > 0 ? c_planes % 4 == 0 : ldc % 4 == 0) && (c_split_stride % 4 == 0) && aligned16(C);
    const unsigned m_tiles = (unsigned)((M + p.bm - 1) / p.bm);
    // XCD-contiguous row tiles only where rows are voxels and there are enough tiles to keep
    // every XCD busy (an exact multiple of 8 cannot be told apart from the plain order, so
    // pad it by 8 as well)
    // (in pattern order neighbouring tiles have the same amount of work: chunks of tiles go to the
    // XCDs in turn, see xcd_chunk_tile, and the grid is a whole number of rounds of chunks)
    const bool remap = (AMODE == hch::A_GATHER || AMODE == hch::A_ROWS) && m_tiles >= 256 && !tilemask;
    const unsigned gx = tilemask ? hch::skip_grid(m_tiles, hch::skip_chunk(m_tiles * (unsigned)(p.bm / 64), (unsigned)(p.bm / 64)))
                                 : (remap ? (m_tiles / hch::NUM_XCD + 1) * hch::NUM_XCD : m_tiles);
    const unsigned n_tiles = (unsigned)((N + p.bn - 1) / p.bn);
    // reductions over the voxels cut into a multiple of 8 slices: one XCD per slice
    const int flat = ((AMODE == hch::A_GATHER_T || AMODE == hch::A_COLS) && p.splits >= 8 && p.splits % (int)hch::NUM_XCD == 0) ? p.splits : 0;
    const dim3 grid = flat ? dim3((unsigned)p.splits * m_tiles * n_tiles) : dim3(gx, n_tiles, (unsigned)p.splits);
    // the kernel's name as a profiler prints it: gemm_f32_kernel<TIN, BM, BN, BK, WM, AMODE, B_KC>
    static int ids[2][3][2][4];                        // [lean][planes / skipping][vector path][tile shape]
    static const bool ids_ready = [] { memset(ids, 0xFF, sizeof ids); return true; }();
    (void)ids_ready;
    const int cfg = p.bm == 64 ? 0 : (p.bn == 16 ? 1 : (p.bn == 32 ? 2 : 3));
    const int v = vec ? 1 : 0, pl = c_planes > 0 ? 1 : (tilemask ? 2 : 0);
    if (pl == 1 && p.bn != 64) return fail(HCH_EINVAL, "gemm: plane-wise output needs the 64-column tile");
    // The lean loop (buffer loads, scalar offsets): float gathers of a 3x3x3 neighbourhood whose
    // operands stay below 2 GiB each, so that 32-bit byte offsets reach everything and a negative
    // offset is out of range; row indices must fit the 24-bit multiply.  Gathering along the
    // reduction axis a tile must lie within one tap (rows of a multiple of 32 channels).
    constexpr bool gather_mode = (AMODE == hch::A_GATHER || AMODE == hch::A_GATHER_T);
    constexpr bool lean_mode = (AMODE == hch::A_GATHER || AMODE == hch::A_ROWS || ((AMODE == hch::A_GATHER_T || AMODE == hch::A_COLS) && !B_KC)) &&
                               sizeof(TIN) == 4;
    bool lean = false;
    // rows of 16 channels (not a multiple of 32): tiles of 16 reduction indices, one tap each
    const bool lean16 = AMODE == hch::A_GATHER && !B_KC && lda % 32 == 16 && p.bm == 128 && p.bn == 32 &&
                        (p.splits == 1 || p.k_per_split % 16 == 0);
    if constexpr (lean_mode) {
        const int64_t lim = (int64_t)1 << 31;
        if constexpr (gather_mode) {
            const int64_t idx_rows = AMODE == hch::A_GATHER ? M : K;
            int64_t b_bytes;
            if (AMODE == hch::A_GATHER_T) b_bytes = (int64_t)K * ldb * 4;
            else if (B_KC) b_bytes = ((int64_t)(taps - 1) * (b_tap_stride < 0 ? -b_tap_stride : b_tap_stride) + (int64_t)N * ldb) * 4;
            else b_bytes = (int64_t)taps * lda * ldb * 4;
            lean = vec && c_planes == 0 && taps == 27 && nbr && a_rows > 0 && a_rows < ((int64_t)1 << 23) && lda * 4 < ((int64_t)1 << 23) &&
                   a_rows * lda * 4 < lim && idx_rows * taps * 4 < lim && b_bytes < lim &&
                   (AMODE == hch::A_GATHER_T || ((lda % 32 == 0 || lean16) && (B_KC ? b_wrap == (int)lda : b_wrap == 0)));
        } else {
            // plain operands (the products of the columns algorithm): row-major A needs whole tiles,
            // K and the slices multiples of 32; k-major A and B may end anywhere (their buffers are
            // described slice by slice)
            const int64_t a_bytes = (int64_t)(AMODE == hch::A_ROWS ? M : K) * lda * 4;
            const int64_t b_bytes = (int64_t)(B_KC ? N : K) * ldb * 4;
            lean = vec && c_planes == 0 && b_wrap == 0 && a_bytes < lim && b_bytes < lim &&
                   (AMODE == hch::A_COLS || (K % 32 == 0 && (p.splits == 1 || p.k_per_split % 32 == 0)));
        }
    }
    if (!g_lean_loops.load(std::memory_order_relaxed)) lean = false;
    const int ln = lean ? 1 : 0;
    if (ids[ln][pl][v][cfg] < 0) {
        char nm[128];
        // all eleven template arguments, as a profiler prints the instantiation
        snprintf(nm, sizeof nm, "gemm_f32_kernel<%s, %d, %d, 32, %d, %d, %s, %s, %s, %s, %s>",
                 sizeof(TIN) == 4 ? "float" : "unsigned short", p.bm, p.bm == 64 ? 64 : p.bn, p.wm,
                 (int)AMODE, B_KC ? "true" : "false", v ? "true" : "false", pl == 1 ? "true" : "false",
                 pl == 2 ? "true" : "false", lean ? "true" : "false");
        ids[ln][pl][v][cfg] = hch::Profiler::get().id_for(nm);
    }
    int kid = ids[ln][pl][v][cfg];
    if (lean && lean16)
        kid = tilemask ? HCH_KERNEL_ID("gemm_f32_kernel<float, 128, 32, 16, 4, 2, false, true, false, true, true>")
                       : HCH_KERNEL_ID("gemm_f32_kernel<float, 128, 32, 16, 4, 2, false, true, false, false, true>");
    const bool short_k = AMODE == hch::A_ROWS && B_KC && pl == 1 && vec && p.bm == 128 && K <= 16 && p.splits == 1;
    if (short_k) kid = HCH_KERNEL_ID("gemm_f32_kernel<float, 128, 64, 16, 4, 0, true, true, true, false, false>");
    hch::LaunchTimer lt(kid, s, alg_bytes, 2.0 * M * (double)N * K);
#define HCH_GEMM_ARGS (const TIN *)A, (const TIN *)B, C, nbr, M, N, K, lda, ldb, ldc, p.k_per_split, c_split_stride, c_vec_ok, \
                      m_tiles, c_planes, taps, b_wrap, b_tap_stride, rowmap, tilemask, flat, rowmask, mask_c
#define HCH_GEMM_CASE(BM_, BN_, BK_, WM_, VEC_, PL_)                                                                \
    HCH_LAUNCH((hch::gemm_f32_kernel<TIN, BM_, BN_, BK_, WM_, AMODE, B_KC, VEC_, PL_>), grid, dim3(256), 0, s, HCH_GEMM_ARGS)
#define HCH_GEMM_SKIP_CASE(BM_, BN_, WM_)                                                                           \
    HCH_LAUNCH((hch::gemm_f32_kernel<TIN, BM_, BN_, 32, WM_, hch::A_GATHER, B_KC, true, false, true>), grid, dim3(256), 0, s, HCH_GEMM_ARGS)
    if constexpr (AMODE == hch::A_ROWS && B_KC) {
        if (pl == 1) {
            if (vec) {
                if (p.bm == 64) HCH_GEMM_CASE(64, 64, 32, 2, true, true);
                else if (short_k) HCH_GEMM_CASE(128, 64, 16, 4, true, true);      // a reduction of at most 16: one half-size tile
                else HCH_GEMM_CASE(128, 64, 32, 4, true, true);
            }
            else HCH_GEMM_CASE(128, 64, 32, 4, false, true);
            HCH_LAUNCH_CHECK("gemm_f32_kernel");
            return HCH_OK;
        }
    }
#define HCH_GEMM_LEAN_CASE(BM_, BN_, WM_, SKIP_)                                                                     \
    HCH_LAUNCH((hch::gemm_f32_kernel<TIN, BM_, BN_, 32, WM_, AMODE, B_KC, true, false, SKIP_, true>), grid, dim3(256), 0, s, HCH_GEMM_ARGS)
    if constexpr (lean_mode) {
        if (lean) {
            if constexpr (AMODE == hch::A_GATHER && !B_KC) {
                if (lean16) {
                    if (tilemask) HCH_LAUNCH((hch::gemm_f32_kernel<TIN, 128, 32, 16, 4, AMODE, B_KC, true, false, true, true>), grid, dim3(256), 0, s, HCH_GEMM_ARGS);
                    else HCH_LAUNCH((hch::gemm_f32_kernel<TIN, 128, 32, 16, 4, AMODE, B_KC, true, false, false, true>), grid, dim3(256), 0, s, HCH_GEMM_ARGS);
                    HCH_LAUNCH_CHECK("gemm_f32_kernel");
                    return HCH_OK;
                }
            }
            if constexpr (AMODE == hch::A_GATHER) {
                if (tilemask) {
                    if (p.bm == 64) HCH_GEMM_LEAN_CASE(64, 64, 2, true);
                    else if (p.bn == 16) HCH_GEMM_LEAN_CASE(128, 16, 4, true);
                    else if (p.bn == 32) HCH_GEMM_LEAN_CASE(128, 32, 4, true);
                    else HCH_GEMM_LEAN_CASE(128, 64, 4, true);
                    HCH_LAUNCH_CHECK("gemm_f32_kernel");
                    return HCH_OK;
                }
            }
            if (p.bm == 64) HCH_GEMM_LEAN_CASE(64, 64, 2, false);
            else if (p.bn == 16) HCH_GEMM_LEAN_CASE(128, 16, 4, false);
            else if (p.bn == 32) HCH_GEMM_LEAN_CASE(128, 32, 4, false);
            else HCH_GEMM_LEAN_CASE(128, 64, 4, false);
            HCH_LAUNCH_CHECK("gemm_f32_kernel");
            return HCH_OK;
        }
    }
#undef HCH_GEMM_LEAN_CASE
    if constexpr (AMODE == hch::A_GATHER) {
        if (vec && tilemask) {      // rows in pattern order, absent taps left out
            if (p.bm == 64) HCH_GEMM_SKIP_CASE(64, 64, 2);
            else if (p.bn == 16) HCH_GEMM_SKIP_CASE(128, 16, 4);
            else if (p.bn == 32) HCH_GEMM_SKIP_CASE(128, 32, 4);
            else HCH_GEMM_SKIP_CASE(128, 64, 4);
            HCH_LAUNCH_CHECK("gemm_f32_kernel");
            return HCH_OK;
        }
    }
    if (vec) {
        if (p.bm == 64) HCH_GEMM_CASE(64, 64, 32, 2, true, false);
        else if (p.bn == 16) HCH_GEMM_CASE(128, 16, 32, 4, true, false);
        else if (p.bn == 32) HCH_GEMM_CASE(128, 32, 32, 4, true, false);
        else HCH_GEMM_CASE(128, 64, 32, 4, true, false);
    } else {
        // odd channel counts / unaligned operands: one generic shape is enough
        if (p.bn == 16) HCH_GEMM_CASE(128, 16, 32, 4, false, false);
        else if (p.bn == 32) HCH_GEMM_CASE(128, 32, 32, 4, false, false);
        else HCH_GEMM_CASE(128, 64, 32, 4, false, false);
    }
#undef HCH_GEMM_CASE
#undef HCH_GEMM_SKIP_CASE
#undef HCH_GEMM_ARGS
    HCH_LAUNCH_CHECK("gemm_f32_kernel");
    return HCH_OK;
}

// bf16 operands on the bf16 matrix instruction (gemm_bf16_kernel): whether the operands meet its
// alignment rules; products that do not go to the kernel that widens to fp32 on load
template <int AMODE, bool B_KC>
static bool bf16_mfma_ok(const GemmPlan &p, const void *A, const void *B, int M, int N, int K, int64_t lda,
                         int64_t ldb, int c_planes, int b_wrap)
{
    constexpr bool a_k_fast = (AMODE == hch::A_ROWS || AMODE == hch::A_GATHER);
    if (c_planes > 0 || lda % 8 != 0 || ldb % 8 != 0 || !aligned16(A) || !aligned16(B)) return false;
    if (p.splits > 1 && p.k_per_split % hch::BF16_BK != 0) return false;
    if (b_wrap % hch::BF16_BK != 0) return false;
    if (a_k_fast ? (K % 8 != 0) : (M % 8 != 0 || p.bm != 128)) return false;
    if (B_KC ? (K % 8 != 0) : (N % 8 != 0)) return false;
    return true;
}

template <int AMODE, bool B_KC>
static hch_status launch_gemm_bf16(const GemmPlan &p, const void *A, const void *B, float *C,
                                   const int32_t *nbr, int M, int N, int K, int64_t lda, int64_t ldb,
                                   int64_t ldc, int64_t c_split_stride, double alg_bytes, hipStream_t s,
                                   int taps, int b_wrap, int64_t b_tap_stride, const int32_t *nbr_t, int64_t a_rows = 0)
{
    if (M <= 0 || N <= 0) return HCH_OK;
    // index rows [voxel][tap], or their tap-major copy [tap][voxel] (voxels = rows of the output
    // when gathering along the reduction axis, the reduction length when gathering along the rows)
    const int64_t idx_row_stride = nbr_t ? 1 : taps;
    const int64_t idx_tap_stride = nbr_t ? (AMODE == hch::A_GATHER_T ? K : M) : 1;
    if (nbr_t) nbr = nbr_t;
    const int c_vec_ok = (ldc % 4 == 0) && (c_split_stride % 4 == 0) && aligned16(C);
    const unsigned m_tiles = (unsigned)((M + p.bm - 1) / p.bm);
    const bool remap = (AMODE == hch::A_GATHER || AMODE == hch::A_ROWS) && m_tiles >= 256;
    const unsigned gx = remap ? (m_tiles / hch::NUM_XCD + 1) * hch::NUM_XCD : m_tiles;
    const unsigned n_tiles = (unsigned)((N + p.bn - 1) / p.bn);
    // reductions over the voxels cut into a multiple of 8 slices: one XCD per slice
    const int flat = ((AMODE == hch::A_GATHER_T || AMODE == hch::A_COLS) && p.splits % (int)hch::NUM_XCD == 0) ? p.splits : 0;
    const dim3 grid = flat ? dim3((unsigned)p.splits * m_tiles * n_tiles) : dim3(gx, n_tiles, (unsigned)p.splits);
    // the lean loop: see launch_gemm_t; rows of a multiple of 64 channels here (one tile, one tap)
    constexpr bool lean_mode = (AMODE == hch::A_GATHER || (AMODE == hch::A_GATHER_T && !B_KC));
    bool lean = false;
    if constexpr (lean_mode) {
        const int64_t lim = (int64_t)1 << 31;
        const int64_t idx_rows = AMODE == hch::A_GATHER ? M : K;
        int64_t b_bytes;
        if (AMODE == hch::A_GATHER_T) b_bytes = (int64_t)K * ldb * 2;
        else if (B_KC) b_bytes = ((int64_t)(taps - 1) * (b_tap_stride < 0 ? -b_tap_stride : b_tap_stride) + (int64_t)N * ldb) * 2;
        else b_bytes = (int64_t)taps * lda * ldb * 2;
        lean = taps == 27 && nbr && a_rows > 0 && a_rows < ((int64_t)1 << 23) && lda * 2 < ((int64_t)1 << 23) &&
               a_rows * lda * 2 < lim && idx_rows * taps * 4 < lim && b_bytes < lim &&
               (AMODE == hch::A_GATHER_T || (lda % hch::BF16_BK == 0 && (B_KC ? b_wrap == (int)lda : b_wrap == 0)));
    }
    if (!g_lean_loops.load(std::memory_order_relaxed)) lean = false;
    const bool big = lean && AMODE == hch::A_GATHER && p.bm == 128 && p.bn == 64 && p.splits == 1 && M >= 256 * 1024;
    static int ids[2][5] = {{-1, -1, -1, -1, -1}, {-1, -1, -1, -1, -1}};
    const int cfg = big ? 4 : (p.bm == 64 ? 0 : (p.bn == 16 ? 1 : (p.bn == 32 ? 2 : 3)));
    const int ln = lean ? 1 : 0;
    if (ids[ln][cfg] < 0) {
        char nm[128];
        snprintf(nm, sizeof nm, "gemm_bf16_kernel<%d, %d, %d, %d, %s, %s>", big ? 256 : p.bm, p.bm == 64 ? 64 : p.bn, p.wm,
                 (int)AMODE, B_KC ? "true" : "false", lean ? "true" : "false");
        ids[ln][cfg] = hch::Profiler::get().id_for(nm);
    }
    hch::LaunchTimer lt(ids[ln][cfg], s, alg_bytes, 2.0 * M * (double)N * K);
#define HCH_BF16_CASE(BM_, BN_, WM_)                                                                                 \
    HCH_LAUNCH((hch::gemm_bf16_kernel<BM_, BN_, WM_, AMODE, B_KC>), grid, dim3(256), 0, s,                  \
                       (const uint16_t *)A, (const uint16_t *)B, C, nbr, M, N, K, lda, ldb, ldc, p.k_per_split,     \
                       c_split_stride, c_vec_ok, m_tiles, idx_row_stride, idx_tap_stride, b_wrap, b_tap_stride, flat)
#define HCH_BF16_LEAN_CASE(BM_, BN_, WM_)                                                                            \
    HCH_LAUNCH((hch::gemm_bf16_kernel<BM_, BN_, WM_, AMODE, B_KC, true>), grid, dim3(256), 0, s,                    \
                       (const uint16_t *)A, (const uint16_t *)B, C, nbr, M, N, K, lda, ldb, ldc, p.k_per_split,     \
                       c_split_stride, c_vec_ok, m_tiles, idx_row_stride, idx_tap_stride, b_wrap, b_tap_stride, flat)
    if constexpr (lean_mode) {
        if (lean) {
            if (p.bm == 64) {
                if constexpr (AMODE == hch::A_GATHER) HCH_BF16_LEAN_CASE(64, 64, 2);
                else return fail(HCH_EINVAL, "gemm_bf16: 64-row tiles with a transposed A");
            }
            else if (p.bn == 16) HCH_BF16_LEAN_CASE(128, 16, 4);
            else if (p.bn == 32) HCH_BF16_LEAN_CASE(128, 32, 4);
            else if (big) {
                // many voxels, 64 output columns: 256-row tiles, a wavefront computes 64 x 64 outputs
                // and reads a third fewer operand bytes from LDS per matrix instruction
                if constexpr (AMODE == hch::A_GATHER) {

                    const unsigned mt = (unsigned)((M + 255) / 256);
                    const dim3 g2((mt / hch::NUM_XCD + 1) * hch::NUM_XCD, n_tiles, 1);
                    HCH_LAUNCH((hch::gemm_bf16_kernel<256, 64, 4, AMODE, B_KC, true>), g2, dim3(256), 0, s,
                       (const uint16_t *)A, (const uint16_t *)B, C, nbr, M, N, K, lda, ldb, ldc, p.k_per_split,
                       c_split_stride, c_vec_ok, mt, idx_row_stride, idx_tap_stride, b_wrap, b_tap_stride, flat);
                }
            }
            else HCH_BF16_LEAN_CASE(128, 64, 4);
            HCH_LAUNCH_CHECK("gemm_bf16_kernel");
            return HCH_OK;
        }
    }
#undef HCH_BF16_LEAN_CASE
    if (p.bm == 64) {
        if constexpr (AMODE == hch::A_ROWS || AMODE == hch::A_GATHER) HCH_BF16_CASE(64, 64, 2);
        else return fail(HCH_EINVAL, "gemm_bf16: 64-row tiles with a transposed A");
    }
    else if (p.bn == 16) HCH_BF16_CASE(128, 16, 4);
    else if (p.bn == 32) HCH_BF16_CASE(128, 32, 4);
    else HCH_BF16_CASE(128, 64, 4);
#undef HCH_BF16_CASE
    HCH_LAUNCH_CHECK("gemm_bf16_kernel");
    return HCH_OK;
}

template <int AMODE, bool B_KC>
static hch_status launch_gemm(hch_dtype dtype, const GemmPlan &p, const void *A, const void *B, float *C,
                              const int32_t *nbr, int M, int N, int K, int64_t lda, int64_t ldb,
                              int64_t ldc, int64_t c_split_stride, double alg_bytes, hipStream_t s,
                              int c_planes = 0, int taps = 27, int b_wrap = 0, int64_t b_tap_stride = 0,
                              const int32_t *nbr_t = nullptr, const int32_t *rowmap = nullptr, const uint32_t *tilemask = nullptr,
                              int64_t a_rows = 0 /* rows of the gathered matrix; 0: not known, no lean loop */,
                              const uint32_t *rowmask = nullptr /* per output row: which groups of mask_c columns to store (fp32 kernel) */,
                              int mask_c = 1)
{
    if (dtype == HCH_BF16 && bf16_mfma_ok<AMODE, B_KC>(p, A, B, M, N, K, lda, ldb, c_planes, b_wrap))
        return launch_gemm_bf16<AMODE, B_KC>(p, A, B, C, nbr, M, N, K, lda, ldb, ldc, c_split_stride, alg_bytes, s, taps, b_wrap, b_tap_stride, nbr_t, a_rows);
    if (dtype == HCH_BF16)
        return launch_gemm_t<uint16_t, AMODE, B_KC>(p, A, B, C, nbr, M, N, K, lda, ldb, ldc, c_split_stride, alg_bytes, s, c_planes, taps, b_wrap, b_tap_stride);
    return launch_gemm_t<float, AMODE, B_KC>(p, A, B, C, nbr, M, N, K, lda, ldb, ldc, c_split_stride, alg_bytes, s, c_planes, taps, b_wrap, b_tap_stride,
                                             rowmap, tilemask, a_rows, rowmask, mask_c);
}

// Register-direct gathered product (conv_direct_kernel): shape-only part of the plan, shared by
// the workspace query and the launch.  Used for products with at most 16 output columns (the
// first forward layer, data gradients into few channels): there a staged tile would be written
// to LDS and read back exactly once, and this kernel measured faster; wider outputs go to the
// LDS-tiled kernel, which measured faster there.
struct DirectPlan {
    bool ok;
    int rt, nt, S;
    bool check;
    int J, upt, step_t, step_q;
    int splits, j_per_split;
    unsigned wave_tiles, n_groups;
};

static DirectPlan plan_direct(int64_t M, int c, int N)
{
    DirectPlan d{};
    d.ok = M > 0 && c % 4 == 0 && N % 4 == 0 && N <= 16 && M * std::max(c, N) < ((int64_t)1 << 31) - 64 * std::max(c, N);
    if (!d.ok) return d;
    d.nt = 1; d.rt = 4; d.S = 4;
    d.check = (c % 16 != 0) || (N % (16 * d.nt) != 0);
    d.upt = c / 4;
    d.J = (27 * d.upt + 3) / 4;
    d.step_t = 4 / d.upt;
    d.step_q = 4 % d.upt;
    d.n_groups = (unsigned)((N + 16 * d.nt - 1) / (16 * d.nt));
    d.wave_tiles = (unsigned)((M + 16 * d.rt - 1) / (16 * d.rt));
    // small levels: slices of the reduction until every SIMD has a few waves
    const int64_t waves = (int64_t)d.wave_tiles * d.n_groups;
    int64_t want = waves >= 1536 ? 1 : std::max<int64_t>(1, std::min<int64_t>((2048 + waves - 1) / waves, d.J / (3 * d.S)));
    int jps = (int)((d.J + want - 1) / want);
    jps = (jps + d.S - 1) / d.S * d.S;
    d.j_per_split = jps;
    d.splits = (d.J + jps - 1) / jps;
    return d;
}

static hch_status launch_direct(const DirectPlan &d, const float *X, const int32_t *nbr, const float *Wm,
                                float *out, int64_t M, int c, int N, double alg_bytes, hipStream_t s, int flipped = 0,
                                const int32_t *rowmap = nullptr, const uint32_t *tilemask = nullptr)
{
    const unsigned blocks = (d.wave_tiles + 3) / 4;
    const bool skip = rowmap && tilemask;        // rows in pattern order, absent taps left out, chunks of tiles per XCD
    const dim3 grid(skip ? hch::skip_grid(blocks, hch::skip_chunk(d.wave_tiles, 4)) : (blocks / hch::NUM_XCD + 1) * hch::NUM_XCD, d.n_groups, (unsigned)d.splits);
    static int ids[2][2] = {{-1, -1}, {-1, -1}};
    const int b = d.check ? 1 : 0, k = skip ? 1 : 0;
    if (ids[k][b] < 0) {
        char nm[96];
        snprintf(nm, sizeof nm, "conv_direct_kernel<%d, %d, %d, %s, %s>", d.rt, d.nt, d.S, d.check ? "true" : "false", skip ? "true" : "false");
        ids[k][b] = hch::Profiler::get().id_for(nm);
    }
    hch::LaunchTimer lt(ids[k][b], s, alg_bytes, 2.0 * M * (double)N * 27.0 * c);
#define HCH_DIRECT_CASE(RT_, NT_, S_, CHECK_, SKIP_)                                                                \
    HCH_LAUNCH((hch::conv_direct_kernel<RT_, NT_, S_, CHECK_, SKIP_>), grid, dim3(256), 0, s, X, nbr, Wm, out,  \
                       (int)M, c, N, d.J, d.j_per_split, d.upt, d.step_t, d.step_q, d.wave_tiles, M * (int64_t)N, flipped, \
                       rowmap, tilemask)
    if (skip) { if (d.check) HCH_DIRECT_CASE(4, 1, 4, true, true); else HCH_DIRECT_CASE(4, 1, 4, false, true); }
    else { if (d.check) HCH_DIRECT_CASE(4, 1, 4, true, false); else HCH_DIRECT_CASE(4, 1, 4, false, false); }
#undef HCH_DIRECT_CASE
    HCH_LAUNCH_CHECK("conv_direct_kernel");
    return HCH_OK;
}

// gathered product into exactly 4 output columns (conv_narrow4_kernel)
static bool narrow4_ok(int64_t M, int c, int N)
{
    return N == 4 && (c == 16 || c == 32 || c == 64) && M > 0 && M * (int64_t)c < ((int64_t)1 << 31) - 64 * c;
}

static hch_status launch_narrow4(const float *X, const int32_t *nbr, const float *Wm, float *out, int64_t M, int c,
                                 double alg_bytes, hipStream_t s, int flipped = 0,
                                 const int32_t *rowmap = nullptr, const uint32_t *tilemask = nullptr)
{
    const unsigned wave_tiles = (unsigned)((M + 63) / 64);
    const unsigned blocks = (wave_tiles + 3) / 4;
    const bool skip = rowmap && tilemask;
    const dim3 grid(skip ? hch::skip_grid(blocks, hch::skip_chunk(wave_tiles, 4)) : (blocks / hch::NUM_XCD + 1) * hch::NUM_XCD);
    const int cc = c / 16;
    int kid;
    if (skip) kid = cc == 1 ? HCH_KERNEL_ID("conv_narrow4_kernel<1, true>") : (cc == 2 ? HCH_KERNEL_ID("conv_narrow4_kernel<2, true>") : HCH_KERNEL_ID("conv_narrow4_kernel<4, true>"));
    else kid = cc == 1 ? HCH_KERNEL_ID("conv_narrow4_kernel<1, false>") : (cc == 2 ? HCH_KERNEL_ID("conv_narrow4_kernel<2, false>") : HCH_KERNEL_ID("conv_narrow4_kernel<4, false>"));
    hch::LaunchTimer lt(kid, s, alg_bytes, 2.0 * M * 4.0 * 27.0 * c);
#define HCH_NARROW_CASE(CC_)                                                                                          \
    do {                                                                                                                \
        if (skip) HCH_LAUNCH((hch::conv_narrow4_kernel<CC_, true>), grid, dim3(256), 0, s, X, nbr, Wm, out, (int)M, wave_tiles, flipped, rowmap, tilemask); \
        else HCH_LAUNCH((hch::conv_narrow4_kernel<CC_, false>), grid, dim3(256), 0, s, X, nbr, Wm, out, (int)M, wave_tiles, flipped, rowmap, tilemask);     \
    } while (0)
    if (cc == 1) HCH_NARROW_CASE(1);
    else if (cc == 2) HCH_NARROW_CASE(2);
    else if (cc == 4) HCH_NARROW_CASE(4);
    else return fail(HCH_EINVAL, "conv_narrow4: channel count");
#undef HCH_NARROW_CASE
    HCH_LAUNCH_CHECK("conv_narrow4_kernel");
    return HCH_OK;
}

static hch_status launch_reduce(const float *part, float *out, int64_t n, int splits, hipStream_t s)
{
    const int kid = splits <= 16 ? HCH_KERNEL_ID("splitk_reduce_kernel<1>")
                    : (n >= 65536 || splits <= 256 ? HCH_KERNEL_ID("splitk_reduce_kernel<16>") : HCH_KERNEL_ID("splitk_reduce_kernel<64>"));
    hch::LaunchTimer lt(kid, s, 4.0 * n * (splits + 1.0), (double)n * splits);
    // few slices: a thread per output; many slices: 16 or 64 lanes per output, so that even a
    // small output (a 27 x 4 x 16 weight gradient) spreads over a few hundred workgroups
    if (splits <= 16)
        HCH_LAUNCH(hch::splitk_reduce_kernel<1>, dim3(blocks_for(n)), dim3(256), 0, s, part, out, n, splits, n);
    else if (n >= 65536 || splits <= 256)
        HCH_LAUNCH(hch::splitk_reduce_kernel<16>, dim3((unsigned)((n + 15) / 16)), dim3(256), 0, s, part, out, n, splits, n);
    else
        HCH_LAUNCH(hch::splitk_reduce_kernel<64>, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, s, part, out, n, splits, n);
    HCH_LAUNCH_CHECK("splitk_reduce_kernel");
    return HCH_OK;
}

// workspace layout, all offsets 256-byte aligned:
//   columns algorithm : [ column matrix | split-K partial sums ]
//   fused algorithm   : [ flipped+transposed weights (bwd_data only) | split-K partial sums ]
struct WsLayout { size_t first_bytes, part_bytes; };

// bf16 forward product: with rows of a multiple of 64 channels the kernel takes the weights from a
// copy transposed per tap, Wt[27][c_out][c_in] at the start of the workspace, in which the
// reduction index is the fast one -- its tiles then go to LDS as they are, instead of being
// transposed in registers on every tile (vector instructions that cost matrix time)
static bool fwd_transposed_weights(hch_dtype dtype, int c_in, int c_out)
{
    return dtype == HCH_BF16 && c_in % hch::BF16_BK == 0 && c_out % 8 == 0;
}

static WsLayout ws_layout(const Level &L, int c_in, int c_out, hch_dtype dtype, hch_ws_kind kind, hch_algo algo)
{
    const size_t Kc = (size_t)27 * c_in, n = (size_t)L.n_total;
    WsLayout w{0, 0};
    if (kind == HCH_WS_FWD) {
        const GemmPlan p = plan_rows(L.n_total, c_out, (int)Kc, true, k_gran(dtype));
        if (algo == HCH_ALGO_COLUMNS) w.first_bytes = round_up(n * Kc * elem_size(dtype), 256);
        int splits = p.splits;
        if (algo == HCH_ALGO_FUSED) { const DirectPlan d = plan_direct(L.n_total, c_in, c_out); if (d.ok) splits = std::max(splits, d.splits); }
        if (algo == HCH_ALGO_FUSED && fwd_transposed_weights(dtype, c_in, c_out)) w.first_bytes = round_up(Kc * c_out * elem_size(dtype), 256);
        if (splits > 1) w.part_bytes = round_up((size_t)splits * n * c_out * 4, 256);
    } else if (kind == HCH_WS_BWD_DATA) {
        if (algo == HCH_ALGO_COLUMNS) w.first_bytes = round_up(n * Kc * 4, 256);
        else {
            const GemmPlan p = plan_rows(L.n_total, c_in, 27 * c_out, true, k_gran(dtype));
            w.first_bytes = round_up(Kc * c_out * elem_size(dtype), 256);
            const DirectPlan d = plan_direct(L.n_total, c_out, c_in);
            const int splits = d.ok ? std::max(p.splits, d.splits) : p.splits;
            if (splits > 1) w.part_bytes = round_up((size_t)splits * n * c_in * 4, 256);
        }
    } else if (kind == HCH_WS_BWD_WEIGHT) {
        const GemmPlan p = plan_wgrad(L.n_total, c_in, c_out, 27, k_gran(dtype));
        if (algo == HCH_ALGO_COLUMNS) w.first_bytes = round_up(n * Kc * elem_size(dtype), 256);
        if (p.splits > 1) w.part_bytes = round_up((size_t)p.splits * Kc * c_out * 4, 256);
    }
    return w;
}

extern "C" size_t hch_conv_workspace_bytes(const hch_levels *levels, int32_t level, int32_t c_in,
                                           int32_t c_out, hch_dtype dtype, hch_ws_kind kind, hch_algo algo)
{
    if (!levels || level < 0 || level >= (int32_t)levels->lv.size() || c_in <= 0 || c_out <= 0) return 0;
    if (algo == HCH_ALGO_COLUMNS_RESIDENT) algo = HCH_ALGO_COLUMNS;
    if (algo == HCH_ALGO_FUSED_DENSE) algo = HCH_ALGO_FUSED;     // same workspace as the fused algorithm
    if (algo != HCH_ALGO_COLUMNS && algo != HCH_ALGO_FUSED) return 0;
    const Level &L = levels->lv[level];
    if (kind == HCH_WS_MIN) {
        // hch_conv_fwd with the columns algorithm: room for 1024 rows of the column matrix
        // next to the split-K area
        const WsLayout w = ws_layout(L, c_in, c_out, dtype, HCH_WS_FWD, algo);
        const size_t rows = std::min<size_t>((size_t)L.n_total, 1024);
        const size_t first = algo == HCH_ALGO_COLUMNS ? round_up(rows * 27 * c_in * elem_size(dtype), 256) : w.first_bytes;
        return std::max<size_t>(256, first + w.part_bytes);
    }
    if (kind != HCH_WS_FWD && kind != HCH_WS_BWD_DATA && kind != HCH_WS_BWD_WEIGHT) return 0;
    const WsLayout w = ws_layout(L, c_in, c_out, dtype, kind, algo);
    return std::max<size_t>(256, w.first_bytes + w.part_bytes);
}

// ---------------------------------------------------------------------------------------
// convolution
// ---------------------------------------------------------------------------------------

static hch_status conv_args(const hch_levels *levels, int32_t level, hch_dtype dtype, const void *a,
                            const void *b, const void *c, int32_t c_in, int32_t c_out,
                            const void *ws, hch_algo algo, const Level **L, const char *who)
{
    hch_status st = get_level(levels, level, L, who);
    if (st != HCH_OK) return st;
    if (!a || !b || !c || !ws || c_in <= 0 || c_out <= 0)
        return fail(HCH_EINVAL, std::string(who) + ": null pointer or non-positive channel count");
    if ((int64_t)27 * c_in * c_out >= ((int64_t)1 << 31))
        return fail(HCH_EINVAL, std::string(who) + ": weight tensor too large");
    if (algo != HCH_ALGO_COLUMNS && algo != HCH_ALGO_FUSED)
        return fail(HCH_EINVAL, std::string(who) + ": unknown algorithm");
    if (dtype != HCH_F32 && dtype != HCH_BF16)
        return fail(HCH_EINVAL, std::string(who) + ": unknown dtype");
    if (reinterpret_cast<uintptr_t>(ws) & 255u)
        return fail(HCH_EINVAL, std::string(who) + ": workspace must be 256-byte aligned");
    if ((*L)->n_total >= ((int64_t)1 << 31) / 64)
        return fail(HCH_EUNSUPPORTED, std::string(who) + ": too many voxels");
    // the kernels index feature rows with 32 bits: voxel * channels + channel
    if ((*L)->n_total * (int64_t)std::max(c_in, c_out) >= ((int64_t)1 << 31))
        return fail(HCH_EUNSUPPORTED, std::string(who) + ": a feature matrix of more than 2^31 elements");
    return HCH_OK;
}

extern "C" hch_status hch_conv_fwd(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                   const void *X, const void *W, float *Y, int32_t c_in,
                                   int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                                   void *stream)
{
    const Level *L;
    const bool skip = algo == HCH_ALGO_FUSED;                    // absent taps may be skipped
    if (algo == HCH_ALGO_FUSED_DENSE) algo = HCH_ALGO_FUSED;
    hch_status st = conv_args(levels, level, dtype, X, W, Y, c_in, c_out, workspace, algo, &L, "hch_conv_fwd");
    if (st != HCH_OK) return st;
    if (ws_bytes < hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, HCH_WS_MIN, algo))
        return fail(HCH_EWORKSPACE, "hch_conv_fwd: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    const int Kc = 27 * c_in;
    const int64_t n = L->n_total;
    const WsLayout w = ws_layout(*L, c_in, c_out, dtype, HCH_WS_FWD, algo);
    const GemmPlan p = plan_rows(n, c_out, Kc, true, k_gran(dtype));
    const double es = elem_size(dtype);               // bytes per input element
    float *part = (float *)((char *)workspace + ((ws_bytes - w.part_bytes) & ~(size_t)255));   // split-K area at the end

    if (algo == HCH_ALGO_FUSED) {
        // Y = gathered columns . W, the column matrix never leaves the chip.  Per voxel: 27
        // indices and its feature row in, one output row out; the weights once.
        if (narrow4_ok(n, c_in, c_out) && dtype == HCH_F32 && aligned16(X) && aligned16(W) && aligned16(Y)) {
            const double bytes = (double)n * (108.0 + 4.0 * c_in + 4.0 * c_out) + 4.0 * Kc * c_out;
            return launch_narrow4((const float *)X, L->dnbr, (const float *)W, Y, n, c_in, bytes, s, 0,
                                  skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr);
        }
        const DirectPlan d = plan_direct(n, c_in, c_out);
        if (d.ok && dtype == HCH_F32 && aligned16(X) && aligned16(W) && aligned16(Y)) {
            const double bytes = (double)n * (108.0 + 4.0 * c_in + 4.0 * c_out * d.splits) + 4.0 * Kc * c_out;
            st = launch_direct(d, (const float *)X, L->dnbr, (const float *)W, d.splits > 1 ? part : Y, n, c_in, c_out, bytes, s, 0,
                               skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr);
            if (st != HCH_OK) return st;
            if (d.splits > 1) st = launch_reduce(part, Y, n * c_out, d.splits, s);
            return st;
        }
        const double bytes = (double)n * (108.0 + es * c_in + 4.0 * c_out * p.splits) + es * Kc * c_out;
        if (fwd_transposed_weights(dtype, c_in, c_out) && aligned16(X) && aligned16(W) && aligned16(workspace)) {
            const int64_t wn = (int64_t)Kc * c_out, per_tap = (int64_t)c_in * c_out;
            {
                hch::LaunchTimer lt(HCH_KERNEL_ID("flip_transpose_weights_kernel<unsigned short>"), s, 4.0 * wn, 0.0);
                HCH_LAUNCH(hch::flip_transpose_weights_kernel<uint16_t>, dim3(blocks_for(wn)), dim3(256), 0, s,
                           (const uint16_t *)W, (uint16_t *)workspace, c_in, c_out, 27, 0);
            }
            HCH_LAUNCH_CHECK("flip_transpose_weights_kernel");
            st = launch_gemm<hch::A_GATHER, true>(dtype, p, X, workspace, p.splits > 1 ? part : Y, L->dnbr, (int)n, c_out, Kc,
                                                  c_in, c_in, c_out, n * c_out, bytes, s, 0, 27, c_in, per_tap, L->dnbr_t,
                                                  nullptr, nullptr, n);
            if (st != HCH_OK) return st;
            if (p.splits > 1) st = launch_reduce(part, Y, n * c_out, p.splits, s);
            return st;
        }
        st = launch_gemm<hch::A_GATHER, false>(dtype, p, X, W,
                                               p.splits > 1 ? part : Y, L->dnbr, (int)n, c_out, Kc, c_in,
                                               c_out, c_out, n * c_out, bytes, s, 0, 27, 0, 0, L->dnbr_t,
                                               skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr, n);
        if (st != HCH_OK) return st;
        if (p.splits > 1) st = launch_reduce(part, Y, n * c_out, p.splits, s);
        return st;
    }

    // as many rows of the column matrix as the workspace holds, in multiples of the GEMM tile
    int64_t chunk = (int64_t)(((ws_bytes - w.part_bytes) & ~(size_t)255) / ((size_t)Kc * elem_size(dtype)));
    if (chunk < n) chunk = std::max<int64_t>(128, chunk / 128 * 128);
    for (int64_t r0 = 0; r0 < n; r0 += chunk) {
        const int64_t rows = std::min<int64_t>(chunk, n - r0);
        st = do_hash2col(*L, dtype, X, c_in, r0, rows, workspace, s);
        if (st != HCH_OK) return st;
        const double bytes = es * ((double)rows * Kc + (double)Kc * c_out) + 4.0 * (double)rows * c_out * p.splits;
        // the split plan was made for all n rows; slices of a chunk land in the same places
        st = launch_gemm<hch::A_ROWS, false>(dtype, p, workspace, W,
                                             p.splits > 1 ? part + r0 * c_out : Y + r0 * c_out, nullptr,
                                             (int)rows, c_out, Kc, Kc, c_out, c_out, n * c_out, bytes, s);
        if (st != HCH_OK) return st;
    }
    if (p.splits > 1) st = launch_reduce(part, Y, n * c_out, p.splits, s);
    return st;
}

extern "C" hch_status hch_conv_bwd_data(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                        const void *dY, const void *W, float *dX, int32_t c_in,
                                        int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                                        void *stream)
{
    const Level *L;
    const bool skip = algo == HCH_ALGO_FUSED;
    if (algo == HCH_ALGO_FUSED_DENSE) algo = HCH_ALGO_FUSED;
    hch_status st = conv_args(levels, level, dtype, dY, W, dX, c_in, c_out, workspace, algo, &L, "hch_conv_bwd_data");
    if (st != HCH_OK) return st;
    if (ws_bytes < hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, HCH_WS_BWD_DATA, algo))
        return fail(HCH_EWORKSPACE, "hch_conv_bwd_data: workspace too small");
    hipStream_t s = (hipStream_t)stream;
    const int Kc = 27 * c_in;
    const int64_t n = L->n_total;
    const double es = elem_size(dtype);

    if (algo == HCH_ALGO_FUSED) {
        // dX[q] = sum_k dY[neighbour 26-k of q] . W[k]^T: a gathered product over the output
        // gradients with the flipped, transposed weights; dcol is never formed.
        const WsLayout w = ws_layout(*L, c_in, c_out, dtype, HCH_WS_BWD_DATA, algo);
        void *Wt = workspace;
        float *part = (float *)((char *)workspace + w.first_bytes);
        const int64_t wn = (int64_t)Kc * c_out;
        const int Kd = 27 * c_out;
        // narrow outputs: kernels that read the weights in place (flipped and transposed on the fly)
        if (narrow4_ok(n, c_out, c_in) && dtype == HCH_F32 && aligned16(dY) && aligned16(dX) && aligned16(W)) {
            const double bytes = (double)n * (108.0 + 4.0 * c_out + 4.0 * c_in) + 4.0 * wn;
            return launch_narrow4((const float *)dY, L->dnbr, (const float *)W, dX, n, c_out, bytes, s, 1,
                                  skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr);
        }
        const DirectPlan d = plan_direct(n, c_out, c_in);
        // (gradients whose rows hold a multiple of 32 channels go to the LDS-tiled kernel's lean loop,
        // which measured faster than this one: 56 against 67 us for 32 -> 16 channels on 176k voxels)
        if (d.ok && c_out % 32 != 0 && dtype == HCH_F32 && aligned16(dY) && aligned16(dX) && aligned16(W)) {
            const double bytes = (double)n * (108.0 + 4.0 * c_out + 4.0 * c_in * d.splits) + 4.0 * wn;
            st = launch_direct(d, (const float *)dY, L->dnbr, (const float *)W, d.splits > 1 ? part : dX, n, c_out, c_in, bytes, s, 1,
                               skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr);
            if (st != HCH_OK) return st;
            if (d.splits > 1) st = launch_reduce(part, dX, n * c_in, d.splits, s);
            return st;
        }
        const GemmPlan p = plan_rows(n, c_in, Kd, true, k_gran(dtype));
        if (c_out % k_gran(dtype) == 0 && c_in % 4 == 0 && aligned16(dY) && aligned16(W)) {
            // the LDS-tiled kernel reads W[27][c_in][c_out] in place as the flipped, transposed
            // matrix: tap 26 - t of the weights for rows t*c_out .. (t+1)*c_out - 1
            const int64_t per_tap = (int64_t)c_in * c_out;
            const char *Wlast = (const char *)W + 26 * per_tap * elem_size(dtype);
            const double bytes = (double)n * (108.0 + es * c_out + 4.0 * c_in * p.splits) + es * wn;
            st = launch_gemm<hch::A_GATHER, true>(dtype, p, dY, Wlast, p.splits > 1 ? part : dX, L->dnbr, (int)n, c_in, Kd,
                                                  c_out, c_out, c_in, n * c_in, bytes, s, 0, 27, c_out, -per_tap, L->dnbr_t,
                                                  skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr, n);
            if (st != HCH_OK) return st;
            if (p.splits > 1) st = launch_reduce(part, dX, n * c_in, p.splits, s);
            return st;
        }
        if (dtype == HCH_F32) {
            hch::LaunchTimer lt(HCH_KERNEL_ID("flip_transpose_weights_kernel<float>"), s, 8.0 * wn, 0.0);
            HCH_LAUNCH(hch::flip_transpose_weights_kernel<float>, dim3(blocks_for(wn)), dim3(256), 0, s,
                               (const float *)W, (float *)Wt, c_in, c_out, 27, 1);
        } else {
            hch::LaunchTimer lt(HCH_KERNEL_ID("flip_transpose_weights_kernel<unsigned short>"), s, 4.0 * wn, 0.0);
            HCH_LAUNCH(hch::flip_transpose_weights_kernel<uint16_t>, dim3(blocks_for(wn)), dim3(256), 0, s,
                               (const uint16_t *)W, (uint16_t *)Wt, c_in, c_out, 27, 1);
        }
        HCH_LAUNCH_CHECK("flip_transpose_weights_kernel");
        const double bytes = (double)n * (108.0 + es * c_out + 4.0 * c_in * p.splits) + es * wn;
        st = launch_gemm<hch::A_GATHER, false>(dtype, p, dY, Wt,
                                               p.splits > 1 ? part : dX, L->dnbr, (int)n, c_in, Kd, c_out,
                                               c_in, c_in, n * c_in, bytes, s, 0, 27, 0, 0, L->dnbr_t,
                                               skip ? L->dorder : nullptr, skip ? L->dtilemask : nullptr, n);
        if (st != HCH_OK) return st;
        if (p.splits > 1) st = launch_reduce(part, dX, n * c_in, p.splits, s);
        return st;
    }

    float *dcol = (float *)workspace;
    // dcol[N x Kc] = dY[N x c_out] . W^T   (W is [Kc x c_out]: its rows are B's columns)
    const GemmPlan p = plan_rows(n, Kc, c_out, false, k_gran(dtype));
    // with few input channels dcol is stored tap-major ([27][n][c_in]) between the two kernels:
    // the gather then reads, tap by tap, 16- or 32-byte pieces of nearly consecutive rows that
    // lie next to each other, instead of one such piece out of every 27*c_in-float row.  (With
    // 16 channels or more a piece fills its own memory sectors and the row-major store of the
    // product is the cheaper one: measured.)
    const bool planes = c_in % 4 == 0 && c_in <= 8 && aligned16(dX);
    // Algorithm 2 adds dcol[i][k] to voxel nbr[i][k] and drops it where there is none: in the
    // tap-major form those pieces (two thirds of dcol at the finest level) are not stored; the
    // per-voxel bit sets of existing neighbours come with the index lists.  (Row-major, with 16 or
    // more channels, leaving pieces out of the rows made the product slower by more than the
    // gather gained: 96 -> 111 us and 45 -> 31 us at level 1, 72 -> 81 and 13 -> 13 at level 2.)
    const bool masked = planes && L->dmask27 != nullptr;
    const uint32_t *rowmask = masked ? L->dmask27 : nullptr;
    // bytes: dY and W in; of dcol the pieces that have a destination, and 4 per row for the bit set (all of dcol without it)
    const double bytes = es * ((double)n * c_out + (double)Kc * c_out) +
                         (masked ? 4.0 * ((double)L->nbr_valid * c_in + (double)n) : 4.0 * (double)n * Kc);
    st = launch_gemm<hch::A_ROWS, true>(dtype, p, dY, W, dcol, nullptr,
                                        (int)n, Kc, c_out, c_out, c_out, Kc, 0, bytes, s, planes ? c_in : 0,
                                        27, 0, 0, nullptr, nullptr, nullptr, 0, rowmask, c_in);
    if (st != HCH_OK) return st;
    return do_col2hash(*L, dcol, c_in, dX, planes, s);
}

static hch_status conv_bwd_weight_impl(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                       const void *X, const void *dY, float *dW, int32_t c_in,
                                       int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                                       void *stream, const char *who)
{
    const Level *L;
    const bool resident = algo == HCH_ALGO_COLUMNS_RESIDENT;     // the column matrix is in the workspace already
    if (resident) algo = HCH_ALGO_COLUMNS;
    if (algo == HCH_ALGO_FUSED_DENSE) algo = HCH_ALGO_FUSED;
    hch_status st = conv_args(levels, level, dtype, X, dY, dW, c_in, c_out, workspace, algo, &L, who);
    if (st != HCH_OK) return st;
    if (ws_bytes < hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, HCH_WS_BWD_WEIGHT, algo))
        return fail(HCH_EWORKSPACE, std::string(who) + ": workspace too small");
    hipStream_t s = (hipStream_t)stream;
    const int Kc = 27 * c_in;
    const int64_t n = L->n_total;
    const double es = elem_size(dtype);
    const WsLayout w = ws_layout(*L, c_in, c_out, dtype, HCH_WS_BWD_WEIGHT, algo);
    const GemmPlan p = plan_wgrad(n, c_in, c_out, 27, k_gran(dtype));
    const int64_t wsize = (int64_t)Kc * c_out;
    float *part = (float *)((char *)workspace + w.first_bytes);
    float *dst = (p.splits == 1) ? dW : part;

    // dW[Kc x c_out] = col^T[Kc x N] . dY[N x c_out], reduction over the voxels split in slices
    if (algo == HCH_ALGO_FUSED) {
        const double bytes = (double)n * (108.0 + es * c_in + es * c_out) + 4.0 * wsize * p.splits;
        st = launch_gemm<hch::A_GATHER_T, false>(dtype, p, X, dY, dst,
                                                 L->dnbr, Kc, c_out, (int)n, c_in, c_out, c_out, wsize, bytes, s, 0, 27, 0, 0, L->dnbr_t,
                                                 nullptr, nullptr, n);
    } else {
        void *col = workspace;
        if (!resident) {
            st = do_hash2col(*L, dtype, X, c_in, 0, n, col, s);
            if (st != HCH_OK) return st;
        }
        const double bytes = es * ((double)n * Kc + (double)n * c_out) + 4.0 * (double)wsize * p.splits;
        st = launch_gemm<hch::A_COLS, false>(dtype, p, col, dY, dst, nullptr,
                                             Kc, c_out, (int)n, Kc, c_out, c_out, wsize, bytes, s);
    }
    if (st != HCH_OK) return st;
    if (p.splits > 1) st = launch_reduce(part, dW, wsize, p.splits, s);
    return st;
}

extern "C" hch_status hch_conv_bwd_weight(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                          const void *X, const void *dY, float *dW, int32_t c_in,
                                          int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                                          void *stream)
{
    return conv_bwd_weight_impl(levels, level, dtype, X, dY, dW, c_in, c_out, workspace, ws_bytes, algo, stream,
                                "hch_conv_bwd_weight");
}

// ---------------------------------------------------------------------------------------
// The weight gradient for callers that cannot allocate and bring no workspace: the partial sums of
// the split reduction live in a fixed array in device memory that every GPU the library runs on
// holds until the process ends.
// ---------------------------------------------------------------------------------------

// The array's name is only a host-side handle of the symbol; the device address is asked for
// once per device (each GPU has its own copy at its own address) and only that pointer is
// handed to kernels.
static __device__ __align__(256) unsigned char scratch[HCH_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];
}

static hch_status scratch_address(void **out)
{
    int dev = -1;
    HCH_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(HCH_EUNSUPPORTED, "hch_conv_bwd_weight_noalloc: device ordinal above 63");
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // two threads may both ask; they get the same answer
        HCH_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u))
            return fail(HCH_EHIP, "hch_conv_bwd_weight_noalloc: no usable address for the scratch array");
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return HCH_OK;
}

extern "C" hch_status hch_conv_bwd_weight_noalloc(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                                  const void *X, const void *dY, float *dW, int32_t c_in,
                                                  int32_t c_out, void *stream)
{
    if (!levels || level < 0 || level >= (int32_t)levels->lv.size() || c_in <= 0 || c_out <= 0)
        return fail(HCH_EINVAL, "hch_conv_bwd_weight_noalloc: bad level or channel count");
    if (dtype != HCH_F32 && dtype != HCH_BF16) return fail(HCH_EINVAL, "hch_conv_bwd_weight_noalloc: unknown dtype");
    if ((int64_t)27 * c_in * c_out >= ((int64_t)1 << 31))
        return fail(HCH_EINVAL, "hch_conv_bwd_weight_noalloc: weight tensor too large");
    const size_t need = hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, HCH_WS_BWD_WEIGHT, HCH_ALGO_FUSED);
    if (need == 0 || need > (size_t)HCH_NOALLOC_SCRATCH_BYTES)
        return fail(HCH_EWORKSPACE, "hch_conv_bwd_weight_noalloc: the partial sums of this product need " +
                                        std::to_string(need) + " bytes, the built-in scratch array holds " +
                                        std::to_string((size_t)HCH_NOALLOC_SCRATCH_BYTES) +
                                        "; use hch_conv_bwd_weight with a workspace");
    void *ptr = nullptr;
    hch_status st = scratch_address(&ptr);
    if (st != HCH_OK) return st;
    // every slice of the split reduction writes all of its 27*c_in*c_out partial sums (zeros where
    // its range of voxels is empty) before the reduction kernel reads them: nothing has to be
    // cleared between calls
    return conv_bwd_weight_impl(levels, level, dtype, X, dY, dW, c_in, c_out, ptr, (size_t)HCH_NOALLOC_SCRATCH_BYTES,
                                HCH_ALGO_FUSED, stream, "hch_conv_bwd_weight_noalloc");
}

// ---------------------------------------------------------------------------------------
// pooling, ReLU
// ---------------------------------------------------------------------------------------

extern "C" hch_status hch_pool_fwd(const hch_levels *levels, int32_t level_in, const float *X,
                                   float *Y, int32_t *argmax, int32_t c, void *stream)
{
    if (!levels || level_in < 0 || level_in + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_pool_fwd: level_in must have a coarser level");
    if (!X || !Y || !argmax || c <= 0) return fail(HCH_EINVAL, "hch_pool_fwd: bad argument");
    const Level &Lc = levels->lv[level_in + 1];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, "hch_pool_fwd: these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, "hch_pool_fwd: levels were built without device tables");
    const bool vec = c % 4 == 0 && aligned16(X) && aligned16(Y) && aligned16(argmax);
    const int64_t items = Lc.n_total * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_pool_fwd: too large");
    {
        // per coarse voxel: 8 child indices, its children's rows in; value and switch rows out
        const Level &Lf = levels->lv[level_in];
        const double bytes = (double)Lc.n_total * (32.0 + 8.0 * c) + (double)Lf.n_total * 4.0 * c;
        hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("pool_fwd_kernel<4>") : HCH_KERNEL_ID("pool_fwd_kernel<1>"), (hipStream_t)stream, bytes, 0.0);
        if (vec)
            HCH_LAUNCH(hch::pool_fwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               X, Lc.dchild, Y, argmax, Lc.n_total, c);
        else
            HCH_LAUNCH(hch::pool_fwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               X, Lc.dchild, Y, argmax, Lc.n_total, c);
    }
    HCH_LAUNCH_CHECK("pool_fwd_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_pool_bwd(const hch_levels *levels, int32_t level_in, const float *dY,
                                   const int32_t *argmax, float *dX, int32_t c, void *stream)
{
    if (!levels || level_in < 0 || level_in + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_pool_bwd: level_in must have a coarser level");
    if (!dY || !argmax || !dX || c <= 0) return fail(HCH_EINVAL, "hch_pool_bwd: bad argument");
    const Level &Lc = levels->lv[level_in + 1];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, "hch_pool_bwd: these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, "hch_pool_bwd: levels were built without device tables");
    const bool vec = c % 4 == 0 && aligned16(dY) && aligned16(dX) && aligned16(argmax);
    const int64_t items = Lc.n_total * 8 * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_pool_bwd: too large");
    {
        const Level &Lf = levels->lv[level_in];
        const double bytes = (double)Lc.n_total * (32.0 + 8.0 * c) + (double)Lf.n_total * 4.0 * c;
        hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("pool_bwd_kernel<4>") : HCH_KERNEL_ID("pool_bwd_kernel<1>"), (hipStream_t)stream, bytes, 0.0);
        if (vec)
            HCH_LAUNCH(hch::pool_bwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               dY, argmax, Lc.dchild, dX, Lc.n_total, c);
        else
            HCH_LAUNCH(hch::pool_bwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               dY, argmax, Lc.dchild, dX, Lc.n_total, c);
    }
    HCH_LAUNCH_CHECK("pool_bwd_kernel");
    return HCH_OK;
}

// ---------------------------------------------------------------------------------------
// transposed convolution and max-unpooling (paper Section 4, last paragraphs): the same
// products with the roles of input and output exchanged
// ---------------------------------------------------------------------------------------

extern "C" hch_status hch_deconv_fwd(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                     const void *X, const void *W, float *Y, int32_t c_in,
                                     int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                                     void *stream)
{
    // Y = col2hash(X . W^T): the data-gradient path of the convolution c_out -> c_in
    return hch_conv_bwd_data(levels, level, dtype, X, W, Y, c_out, c_in, workspace, ws_bytes, algo, stream);
}

extern "C" hch_status hch_deconv_bwd_data(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                          const void *dY, const void *W, float *dX, int32_t c_in,
                                          int32_t c_out, void *workspace, size_t ws_bytes,
                                          hch_algo algo, void *stream)
{
    // the adjoint of the above is the forward convolution c_out -> c_in
    return hch_conv_fwd(levels, level, dtype, dY, W, dX, c_out, c_in, workspace, ws_bytes, algo, stream);
}

extern "C" hch_status hch_deconv_bwd_weight(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                            const void *X, const void *dY, float *dW, int32_t c_in,
                                            int32_t c_out, void *workspace, size_t ws_bytes,
                                            hch_algo algo, void *stream)
{
    // dW[27][c_out][c_in] = hash2col(dY)^T . X: the weight gradient of the convolution c_out -> c_in
    // whose input is dY and whose output gradient is X
    return hch_conv_bwd_weight(levels, level, dtype, dY, X, dW, c_out, c_in, workspace, ws_bytes, algo, stream);
}

extern "C" hch_status hch_unpool_fwd(const hch_levels *levels, int32_t level_out, const float *Xc,
                                     const int32_t *argmax, float *Y, int32_t c, void *stream)
{
    return hch_pool_bwd(levels, level_out, Xc, argmax, Y, c, stream);
}

extern "C" hch_status hch_unpool_bwd(const hch_levels *levels, int32_t level_out, const float *dY,
                                     const int32_t *argmax, float *dXc, int32_t c, void *stream)
{
    if (!levels || level_out < 0 || level_out + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_unpool_bwd: level_out must have a coarser level");
    if (!dY || !argmax || !dXc || c <= 0) return fail(HCH_EINVAL, "hch_unpool_bwd: bad argument");
    const Level &Lc = levels->lv[level_out + 1];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, "hch_unpool_bwd: these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, "hch_unpool_bwd: levels were built without device tables");
    const int64_t items = Lc.n_total * c;
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_unpool_bwd: too large");
    if (items == 0) return HCH_OK;
    {
        hch::LaunchTimer lt(HCH_KERNEL_ID("unpool_bwd_kernel"), (hipStream_t)stream, 12.0 * items, 0.0);
        HCH_LAUNCH(hch::unpool_bwd_kernel, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                           dY, argmax, dXc, Lc.n_total, c);
    }
    HCH_LAUNCH_CHECK("unpool_bwd_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_relu_pool_fwd(const hch_levels *levels, int32_t level_in, const float *Y,
                                        float *A, float *P, int32_t *argmax, int32_t c, void *stream)
{
    if (!levels || level_in < 0 || level_in + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_relu_pool_fwd: level_in must have a coarser level");
    if (!Y || !P || !argmax || c <= 0) return fail(HCH_EINVAL, "hch_relu_pool_fwd: bad argument");
    const Level &Lc = levels->lv[level_in + 1];
    const Level &Lf = levels->lv[level_in];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, "hch_relu_pool_fwd: these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, "hch_relu_pool_fwd: levels were built without device tables");
    const bool vec = c % 4 == 0 && aligned16(Y) && (!A || aligned16(A)) && aligned16(P) && aligned16(argmax);
    const int64_t items = Lc.n_total * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_relu_pool_fwd: too large");
    {
        // per fine voxel: its row in (and its rectified row out when A is given); per coarse
        // voxel: 8 indices in, value and switch rows out
        const double bytes = (double)Lf.n_total * (A ? 8.0 : 4.0) * c + (double)Lc.n_total * (32.0 + 8.0 * c);
        hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("relu_pool_fwd_kernel<4>") : HCH_KERNEL_ID("relu_pool_fwd_kernel<1>"),
                            (hipStream_t)stream, bytes, 0.0);
        if (vec)
            HCH_LAUNCH(hch::relu_pool_fwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               Y, Lc.dchild, A, P, argmax, Lc.n_total, c);
        else
            HCH_LAUNCH(hch::relu_pool_fwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               Y, Lc.dchild, A, P, argmax, Lc.n_total, c);
    }
    HCH_LAUNCH_CHECK("relu_pool_fwd_kernel");
    return HCH_OK;
}

// shared by the two forms of the fused backward step: `sign` holds fine rows (A or Y) or, pooled, the rows P
static hch_status pool_relu_bwd_impl(const hch_levels *levels, int32_t level_in, const float *dP,
                                     const int32_t *argmax, const float *sign, bool pooled, float *dY, int32_t c,
                                     void *stream, const char *who)
{
    if (!levels || level_in < 0 || level_in + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, std::string(who) + ": level_in must have a coarser level");
    if (!dP || !argmax || !sign || !dY || c <= 0) return fail(HCH_EINVAL, std::string(who) + ": bad argument");
    const Level &Lc = levels->lv[level_in + 1];
    const Level &Lf = levels->lv[level_in];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, std::string(who) + ": these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, std::string(who) + ": levels were built without device tables");
    const bool vec = c % 4 == 0 && aligned16(dP) && aligned16(argmax) && aligned16(sign) && aligned16(dY);
    const int64_t items = Lc.n_total * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, std::string(who) + ": too large");
    {
        // per fine voxel: its gradient row out (and its row in, unless the pooled rows stand in);
        // per coarse voxel: 8 indices, gradient and switch rows (and the pooled row) in
        const double bytes = (double)Lf.n_total * (pooled ? 4.0 : 8.0) * c + (double)Lc.n_total * (32.0 + (pooled ? 12.0 : 8.0) * c);
        const int kid = pooled ? (vec ? HCH_KERNEL_ID("pool_relu_bwd_kernel<4, true>") : HCH_KERNEL_ID("pool_relu_bwd_kernel<1, true>"))
                               : (vec ? HCH_KERNEL_ID("pool_relu_bwd_kernel<4, false>") : HCH_KERNEL_ID("pool_relu_bwd_kernel<1, false>"));
        hch::LaunchTimer lt(kid, (hipStream_t)stream, bytes, 0.0);
#define HCH_POOL_RELU_BWD(VEC_, POOLED_)                                                                             \
    HCH_LAUNCH((hch::pool_relu_bwd_kernel<VEC_, POOLED_>), dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream, \
                       dP, argmax, Lc.dchild, sign, dY, Lc.n_total, c)
        if (pooled) { if (vec) HCH_POOL_RELU_BWD(4, true); else HCH_POOL_RELU_BWD(1, true); }
        else { if (vec) HCH_POOL_RELU_BWD(4, false); else HCH_POOL_RELU_BWD(1, false); }
#undef HCH_POOL_RELU_BWD
    }
    HCH_LAUNCH_CHECK("pool_relu_bwd_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_pool_relu_bwd(const hch_levels *levels, int32_t level_in, const float *dP,
                                        const int32_t *argmax, const float *A, float *dY, int32_t c,
                                        void *stream)
{
    return pool_relu_bwd_impl(levels, level_in, dP, argmax, A, false, dY, c, stream, "hch_pool_relu_bwd");
}

extern "C" hch_status hch_pool_relu_bwd_pooled(const hch_levels *levels, int32_t level_in, const float *dP,
                                               const int32_t *argmax, const float *P, float *dY, int32_t c,
                                               void *stream)
{
    return pool_relu_bwd_impl(levels, level_in, dP, argmax, P, true, dY, c, stream, "hch_pool_relu_bwd_pooled");
}

// ---------------------------------------------------------------------------------------
// general kernel side / stride / padding (Algorithm 1 and 2 as stated), average pooling
// ---------------------------------------------------------------------------------------

// level_out for a field of stride S read at level_in, or a failure
static hch_status field_levels(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride, int32_t pad,
                               const Level **Li, const Level **Lo, const char *who)
{
    if (!levels) return fail(HCH_EINVAL, std::string(who) + ": null levels");
    if (F < 1 || F > 7) return fail(HCH_EINVAL, std::string(who) + ": kernel side must be 1..7");
    if (stride < 1) return fail(HCH_EINVAL, std::string(who) + ": stride must be positive");
    if (stride == 1 && (F % 2 == 0 || pad != (F - 1) / 2))
        return fail(HCH_EINVAL, std::string(who) + ": a stride-1 field is centred: odd kernel side, padding (F-1)/2");
    if (pad < 0 || pad >= F) return fail(HCH_EINVAL, std::string(who) + ": padding must be in [0, F)");
    if (level_in < 0 || level_in >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, std::string(who) + ": level out of range");
    // the output level: the one whose side relates to level_in's by exactly `stride`
    int shift = 0;
    int64_t prod = 1;
    while (prod < stride && level_in + shift + 1 < (int32_t)levels->lv.size()) {
        ++shift;
        prod *= levels->lv[level_in + shift].ratio;
    }
    if (prod != stride)
        return fail(HCH_EINVAL, std::string(who) + ": no level of this set is `stride` times coarser than level_in");
    *Li = &levels->lv[level_in];
    *Lo = &levels->lv[level_in + shift];
    if (!(*Li)->dslot3 || !(*Lo)->dslot3) return fail(HCH_EINVAL, std::string(who) + ": levels were built without device tables");
    return HCH_OK;
}

extern "C" hch_status hch_field_build(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                      int32_t pad, int32_t *field, int32_t *field_t, void *stream)
{
    const Level *Li, *Lo;
    hch_status st = field_levels(levels, level_in, F, stride, pad, &Li, &Lo, "hch_field_build");
    if (st != HCH_OK) return st;
    if (!field && !field_t) return fail(HCH_EINVAL, "hch_field_build: nothing to build");
    const int F3 = F * F * F;
    hipStream_t s = (hipStream_t)stream;
    if (field) {
        const int64_t items = (int64_t)Lo->max_n * F3;
        hch::LaunchTimer lt(HCH_KERNEL_ID("field_kernel<false>"), s, (double)Lo->n_total * (12.0 + 4.0 * F3), 0.0);
        HCH_LAUNCH(hch::field_kernel<false>, dim3(blocks_for(items), (unsigned)Lo->b), dim3(256), 0, s,
                           Li->view(), Lo->dcoords, Lo->dN(), field, F, stride, pad);
    }
    if (field_t) {
        const int64_t items = (int64_t)Li->max_n * F3;
        hch::LaunchTimer lt(HCH_KERNEL_ID("field_kernel<true>"), s, (double)Li->n_total * (12.0 + 4.0 * F3), 0.0);
        HCH_LAUNCH(hch::field_kernel<true>, dim3(blocks_for(items), (unsigned)Li->b), dim3(256), 0, s,
                           Lo->view(), Li->dcoords, Li->dN(), field_t, F, stride, pad);
    }
    HCH_LAUNCH_CHECK("field_kernel");
    return HCH_OK;
}

// workspace of the three products of a general convolution: [ transposed weights (bwd_data on one
// level) or the column-matrix gradient (bwd_data between two levels) | split partial sums ]
static WsLayout sconv_layout(const Level &Li, const Level &Lo, int taps, int c_in, int c_out, hch_dtype dtype, hch_ws_kind kind)
{
    WsLayout w{0, 0};
    if (kind == HCH_WS_FWD) {
        const GemmPlan p = plan_rows(Lo.n_total, c_out, taps * c_in, true, k_gran(dtype));
        if (p.splits > 1) w.part_bytes = round_up((size_t)p.splits * Lo.n_total * c_out * 4, 256);
    } else if (kind == HCH_WS_BWD_DATA && &Li != &Lo) {
        // between two levels: the gradient of the column matrix, [N_out][taps*c_in] floats
        w.first_bytes = round_up((size_t)Lo.n_total * taps * c_in * 4, 256);
    } else if (kind == HCH_WS_BWD_DATA) {
        const GemmPlan p = plan_rows(Li.n_total, c_in, taps * c_out, true, k_gran(dtype));
        w.first_bytes = round_up((size_t)taps * c_in * c_out * elem_size(dtype), 256);
        if (p.splits > 1) w.part_bytes = round_up((size_t)p.splits * Li.n_total * c_in * 4, 256);
    } else {
        const GemmPlan p = plan_wgrad(Lo.n_total, c_in, c_out, taps, k_gran(dtype));
        if (p.splits > 1) w.part_bytes = round_up((size_t)p.splits * taps * c_in * c_out * 4, 256);
    }
    return w;
}

extern "C" size_t hch_sconv_workspace_bytes(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                            int32_t c_in, int32_t c_out, hch_dtype dtype, hch_ws_kind kind)
{
    const Level *Li, *Lo;
    if (c_in <= 0 || c_out <= 0 || (kind != HCH_WS_FWD && kind != HCH_WS_BWD_DATA && kind != HCH_WS_BWD_WEIGHT)) return 0;
    if (field_levels(levels, level_in, F, stride, stride == 1 ? (F - 1) / 2 : 0, &Li, &Lo, "hch_sconv_workspace_bytes") != HCH_OK) return 0;
    const WsLayout w = sconv_layout(*Li, *Lo, F * F * F, c_in, c_out, dtype, kind);
    return std::max<size_t>(256, w.first_bytes + w.part_bytes);
}

static hch_status sconv_args(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride, hch_dtype dtype,
                             const void *a, const void *b, const void *c, const void *idx, int32_t c_in, int32_t c_out,
                             const void *ws, size_t ws_bytes, hch_ws_kind kind, const Level **Li, const Level **Lo,
                             const char *who)
{
    hch_status st = field_levels(levels, level_in, F, stride, stride == 1 ? (F - 1) / 2 : 0, Li, Lo, who);
    if (st != HCH_OK) return st;
    if (!a || !b || !c || !idx || !ws || c_in <= 0 || c_out <= 0)
        return fail(HCH_EINVAL, std::string(who) + ": null pointer or non-positive channel count");
    if ((int64_t)F * F * F * c_in * c_out >= ((int64_t)1 << 31)) return fail(HCH_EINVAL, std::string(who) + ": weight tensor too large");
    if (dtype != HCH_F32 && dtype != HCH_BF16) return fail(HCH_EINVAL, std::string(who) + ": unknown dtype");
    if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(HCH_EINVAL, std::string(who) + ": workspace must be 256-byte aligned");
    if (std::max((*Li)->n_total, (*Lo)->n_total) >= ((int64_t)1 << 31) / 512)
        return fail(HCH_EUNSUPPORTED, std::string(who) + ": too many voxels");
    if (std::max((*Li)->n_total, (*Lo)->n_total) * (int64_t)std::max(c_in, c_out) >= ((int64_t)1 << 31))
        return fail(HCH_EUNSUPPORTED, std::string(who) + ": a feature matrix of more than 2^31 elements");
    if (ws_bytes < hch_sconv_workspace_bytes(levels, level_in, F, stride, c_in, c_out, dtype, kind))
        return fail(HCH_EWORKSPACE, std::string(who) + ": workspace too small");
    return HCH_OK;
}

extern "C" hch_status hch_sconv_fwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                    hch_dtype dtype, const void *X, const void *W, float *Y, const int32_t *field,
                                    int32_t c_in, int32_t c_out, void *workspace, size_t ws_bytes, void *stream)
{
    const Level *Li, *Lo;
    hch_status st = sconv_args(levels, level_in, F, stride, dtype, X, W, Y, field, c_in, c_out, workspace, ws_bytes,
                               HCH_WS_FWD, &Li, &Lo, "hch_sconv_fwd");
    if (st != HCH_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int taps = F * F * F, K = taps * c_in;
    const int64_t n = Lo->n_total;
    const double es = elem_size(dtype);
    const GemmPlan p = plan_rows(n, c_out, K, true, k_gran(dtype));
    float *part = (float *)workspace;
    const double bytes = (double)n * (4.0 * taps + 4.0 * c_out * p.splits) + es * (double)Li->n_total * c_in + es * K * c_out;
    st = launch_gemm<hch::A_GATHER, false>(dtype, p, X, W, p.splits > 1 ? part : Y, field, (int)n, c_out, K, c_in,
                                           c_out, c_out, n * c_out, bytes, s, 0, taps);
    if (st != HCH_OK) return st;
    if (p.splits > 1) st = launch_reduce(part, Y, n * c_out, p.splits, s);
    return st;
}

extern "C" hch_status hch_sconv_bwd_weight(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                           hch_dtype dtype, const void *X, const void *dY, float *dW,
                                           const int32_t *field, int32_t c_in, int32_t c_out, void *workspace,
                                           size_t ws_bytes, void *stream)
{
    const Level *Li, *Lo;
    hch_status st = sconv_args(levels, level_in, F, stride, dtype, X, dY, dW, field, c_in, c_out, workspace, ws_bytes,
                               HCH_WS_BWD_WEIGHT, &Li, &Lo, "hch_sconv_bwd_weight");
    if (st != HCH_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int taps = F * F * F, K = taps * c_in;
    const int64_t n = Lo->n_total, wsize = (int64_t)K * c_out;
    const double es = elem_size(dtype);
    const GemmPlan p = plan_wgrad(n, c_in, c_out, taps, k_gran(dtype));
    float *part = (float *)workspace;
    const double bytes = (double)n * (4.0 * taps + es * c_out) + es * (double)Li->n_total * c_in + 4.0 * wsize * p.splits;
    st = launch_gemm<hch::A_GATHER_T, false>(dtype, p, X, dY, p.splits == 1 ? dW : part, field, K, c_out, (int)n, c_in,
                                             c_out, c_out, wsize, bytes, s, 0, taps);
    if (st != HCH_OK) return st;
    if (p.splits > 1) st = launch_reduce(part, dW, wsize, p.splits, s);
    return st;
}

extern "C" hch_status hch_sconv_bwd_data(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                         hch_dtype dtype, const void *dY, const void *W, float *dX,
                                         const int32_t *field_t, int32_t c_in, int32_t c_out, void *workspace,
                                         size_t ws_bytes, void *stream)
{
    const Level *Li, *Lo;
    hch_status st = sconv_args(levels, level_in, F, stride, dtype, dY, W, dX, field_t, c_in, c_out, workspace, ws_bytes,
                               HCH_WS_BWD_DATA, &Li, &Lo, "hch_sconv_bwd_data");
    if (st != HCH_OK) return st;
    hipStream_t s = (hipStream_t)stream;
    const int taps = F * F * F, Kd = taps * c_out;
    const int64_t n = Li->n_total, wn = (int64_t)taps * c_in * c_out;
    const double es = elem_size(dtype);
    const WsLayout w = sconv_layout(*Li, *Lo, taps, c_in, c_out, dtype, HCH_WS_BWD_DATA);
    if (Li != Lo) {
        // Between two levels only about one field row in stride^3 of an input voxel has an owner,
        // so the gathered product below would multiply mostly zeros.  Here the paper's own order
        // is the cheaper one: dcol[N_out][taps*c_in] = dY . W^T (Eq.8), then col2hash (Algorithm
        // 2) as a gather through field_t.
        float *dcol = (float *)workspace;
        const int Kc = taps * c_in;
        const int64_t no = Lo->n_total;
        const GemmPlan pc = plan_rows(no, Kc, c_out, false, k_gran(dtype));
        const double gbytes = es * ((double)no * c_out + (double)wn) + 4.0 * (double)no * Kc;
        st = launch_gemm<hch::A_ROWS, true>(dtype, pc, dY, W, dcol, nullptr, (int)no, Kc, c_out, c_out, c_out, Kc, 0, gbytes, s);
        if (st != HCH_OK) return st;
        const bool vec = c_in % 4 == 0 && aligned16(dX);
        const int64_t items = n * (vec ? c_in / 4 : c_in);
        if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_sconv_bwd_data: too large");
        // per input voxel: its index row, one piece of dcol per owner (about taps / stride^3), its row out
        const double cbytes = (double)n * (4.0 * taps + 4.0 * c_in + 4.0 * c_in * taps / ((double)stride * stride * stride));
        hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("field_col2hash_kernel<4>") : HCH_KERNEL_ID("field_col2hash_kernel<1>"), s, cbytes, 0.0);
        if (vec)
            HCH_LAUNCH(hch::field_col2hash_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, s, dcol, field_t, dX, n, taps, c_in);
        else
            HCH_LAUNCH(hch::field_col2hash_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, s, dcol, field_t, dX, n, taps, c_in);
        HCH_LAUNCH_CHECK("field_col2hash_kernel");
        return HCH_OK;
    }
    void *Wt = workspace;
    float *part = (float *)((char *)workspace + w.first_bytes);
    // dX[i] = sum over rows of dY[field_t[i][row]] . W[row]^T: a gathered product over the output
    // gradients through the transposed index rows, weights transposed per tap (not flipped)
    if (dtype == HCH_F32) {
        hch::LaunchTimer lt(HCH_KERNEL_ID("flip_transpose_weights_kernel<float>"), s, 8.0 * wn, 0.0);
        HCH_LAUNCH(hch::flip_transpose_weights_kernel<float>, dim3(blocks_for(wn)), dim3(256), 0, s,
                           (const float *)W, (float *)Wt, c_in, c_out, taps, 0);
    } else {
        hch::LaunchTimer lt(HCH_KERNEL_ID("flip_transpose_weights_kernel<unsigned short>"), s, 4.0 * wn, 0.0);
        HCH_LAUNCH(hch::flip_transpose_weights_kernel<uint16_t>, dim3(blocks_for(wn)), dim3(256), 0, s,
                           (const uint16_t *)W, (uint16_t *)Wt, c_in, c_out, taps, 0);
    }
    HCH_LAUNCH_CHECK("flip_transpose_weights_kernel");
    const GemmPlan p = plan_rows(n, c_in, Kd, true, k_gran(dtype));
    const double bytes = (double)n * (4.0 * taps + 4.0 * c_in * p.splits) + es * (double)Lo->n_total * c_out + es * wn;
    st = launch_gemm<hch::A_GATHER, false>(dtype, p, dY, Wt, p.splits > 1 ? part : dX, field_t, (int)n, c_in, Kd, c_out,
                                           c_in, c_in, n * c_in, bytes, s, 0, taps);
    if (st != HCH_OK) return st;
    if (p.splits > 1) st = launch_reduce(part, dX, n * c_in, p.splits, s);
    return st;
}

// pooling over general receptive fields between level_in and the level `stride` times coarser
static hch_status spool_args(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride, const void *a,
                             const void *b, const void *idx, int32_t c, const Level **Li, const Level **Lo, const char *who)
{
    hch_status st = field_levels(levels, level_in, F, stride, stride == 1 ? (F - 1) / 2 : 0, Li, Lo, who);
    if (st != HCH_OK) return st;
    if (!a || !b || !idx || c <= 0) return fail(HCH_EINVAL, std::string(who) + ": null pointer or non-positive channel count");
    if (std::max((*Li)->n_total, (*Lo)->n_total) * (int64_t)c > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, std::string(who) + ": too large");
    return HCH_OK;
}

extern "C" hch_status hch_spool_max_fwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                        const float *X, const int32_t *field, float *Y, int32_t *argmax,
                                        int32_t c, void *stream)
{
    const Level *Li, *Lo;
    hch_status st = spool_args(levels, level_in, F, stride, X, Y, field, c, &Li, &Lo, "hch_spool_max_fwd");
    if (st != HCH_OK) return st;
    if (!argmax) return fail(HCH_EINVAL, "hch_spool_max_fwd: null argmax");
    const int taps = F * F * F;
    const bool vec = c % 4 == 0 && aligned16(X) && aligned16(Y) && aligned16(argmax);
    const int64_t items = Lo->n_total * (vec ? c / 4 : c);
    const double bytes = (double)Lo->n_total * (4.0 * taps + 8.0 * c) + (double)Li->n_total * 4.0 * c;
    hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("field_pool_fwd_kernel<4>") : HCH_KERNEL_ID("field_pool_fwd_kernel<1>"),
                        (hipStream_t)stream, bytes, 0.0);
    if (vec)
        HCH_LAUNCH(hch::field_pool_fwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                           X, field, Y, argmax, Lo->n_total, taps, c);
    else
        HCH_LAUNCH(hch::field_pool_fwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                           X, field, Y, argmax, Lo->n_total, taps, c);
    HCH_LAUNCH_CHECK("field_pool_fwd_kernel");
    return HCH_OK;
}

// backward of pooling where the fields partition the input level (F = stride): through the forward rows
template <bool MAXPOOL>
static hch_status launch_field_unpool(const float *dY, const int32_t *argmax, const int32_t *field, float *dX,
                                      int64_t n_out, int64_t n_in, int taps, int c, hipStream_t s)
{
    const bool vec = c % 4 == 0 && aligned16(dY) && aligned16(dX) && (!MAXPOOL || aligned16(argmax));
    const int64_t items = n_out * taps * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "field pooling backward: too large");
    const double bytes = (double)n_out * (4.0 * taps + (MAXPOOL ? 8.0 : 4.0) * c) + (double)n_in * 4.0 * c;
    const int kid = MAXPOOL ? (vec ? HCH_KERNEL_ID("field_unpool_kernel<4, true>") : HCH_KERNEL_ID("field_unpool_kernel<1, true>"))
                            : (vec ? HCH_KERNEL_ID("field_unpool_kernel<4, false>") : HCH_KERNEL_ID("field_unpool_kernel<1, false>"));
    hch::LaunchTimer lt(kid, s, bytes, 0.0);
    if (vec)
        HCH_LAUNCH((hch::field_unpool_kernel<4, MAXPOOL>), dim3(blocks_for(items)), dim3(256), 0, s,
                           dY, argmax, field, dX, n_out, taps, c, 1.0f / taps);
    else
        HCH_LAUNCH((hch::field_unpool_kernel<1, MAXPOOL>), dim3(blocks_for(items)), dim3(256), 0, s,
                           dY, argmax, field, dX, n_out, taps, c, 1.0f / taps);
    HCH_LAUNCH_CHECK("field_unpool_kernel");
    return HCH_OK;
}

// The fields of a pooling with F = stride > 1 and NO padding partition the input level, and every
// input voxel lies in the field of an occupied output voxel (its parent): only then may the
// backward pass write dX through the forward rows.  With padding an input voxel can fall into the
// field of a position that is not occupied on the output level, and no forward row reaches it.
static inline bool fields_partition(int32_t F, int32_t stride, int32_t pad) { return F == stride && stride > 1 && pad == 0; }

extern "C" hch_status hch_spool_max_bwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                        int32_t pad, const float *dY, const int32_t *argmax, const int32_t *field,
                                        const int32_t *field_t, float *dX, int32_t c, void *stream)
{
    const Level *Li, *Lo;
    const bool partition = field && fields_partition(F, stride, pad);
    if (pad < 0 || pad >= F) return fail(HCH_EINVAL, "hch_spool_max_bwd: padding must be in [0, F)");
    if (!partition && !field_t)
        return fail(HCH_EINVAL, "hch_spool_max_bwd: field_t is needed unless F = stride > 1, pad = 0 and field is given");
    hch_status st = spool_args(levels, level_in, F, stride, dY, dX, partition ? field : field_t, c, &Li, &Lo, "hch_spool_max_bwd");
    if (st != HCH_OK) return st;
    if (!argmax) return fail(HCH_EINVAL, "hch_spool_max_bwd: null argmax");
    const int taps = F * F * F;
    if (partition) return launch_field_unpool<true>(dY, argmax, field, dX, Lo->n_total, Li->n_total, taps, c, (hipStream_t)stream);
    const bool vec = c % 4 == 0 && aligned16(dY) && aligned16(dX) && aligned16(argmax);
    const int64_t items = Li->n_total * (vec ? c / 4 : c);
    const double bytes = (double)Li->n_total * (4.0 * taps + 4.0 * c) + (double)Lo->n_total * 8.0 * c;
    hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("field_pool_bwd_kernel<4>") : HCH_KERNEL_ID("field_pool_bwd_kernel<1>"),
                        (hipStream_t)stream, bytes, 0.0);
    if (vec)
        HCH_LAUNCH(hch::field_pool_bwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                           dY, argmax, field_t, dX, Li->n_total, taps, c);
    else
        HCH_LAUNCH(hch::field_pool_bwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                           dY, argmax, field_t, dX, Li->n_total, taps, c);
    HCH_LAUNCH_CHECK("field_pool_bwd_kernel");
    return HCH_OK;
}

static hch_status launch_field_avg(const float *src, const int32_t *idx, float *dst, int64_t n_dst, int64_t n_src,
                                   int taps, int c, hipStream_t s)
{
    const bool vec = c % 4 == 0 && aligned16(src) && aligned16(dst);
    const int64_t items = n_dst * (vec ? c / 4 : c);
    const double bytes = (double)n_dst * (4.0 * taps + 4.0 * c) + (double)n_src * 4.0 * c;
    hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("field_avg_kernel<4>") : HCH_KERNEL_ID("field_avg_kernel<1>"), s, bytes, 0.0);
    if (vec)
        HCH_LAUNCH(hch::field_avg_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, s, src, idx, dst, n_dst, taps, c, 1.0f / taps);
    else
        HCH_LAUNCH(hch::field_avg_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, s, src, idx, dst, n_dst, taps, c, 1.0f / taps);
    HCH_LAUNCH_CHECK("field_avg_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_spool_avg_fwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                        const float *X, const int32_t *field, float *Y, int32_t c, void *stream)
{
    const Level *Li, *Lo;
    hch_status st = spool_args(levels, level_in, F, stride, X, Y, field, c, &Li, &Lo, "hch_spool_avg_fwd");
    if (st != HCH_OK) return st;
    return launch_field_avg(X, field, Y, Lo->n_total, Li->n_total, F * F * F, c, (hipStream_t)stream);
}

extern "C" hch_status hch_spool_avg_bwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                        int32_t pad, const float *dY, const int32_t *field, const int32_t *field_t,
                                        float *dX, int32_t c, void *stream)
{
    const Level *Li, *Lo;
    const bool partition = field && fields_partition(F, stride, pad);
    if (pad < 0 || pad >= F) return fail(HCH_EINVAL, "hch_spool_avg_bwd: padding must be in [0, F)");
    if (!partition && !field_t)
        return fail(HCH_EINVAL, "hch_spool_avg_bwd: field_t is needed unless F = stride > 1, pad = 0 and field is given");
    hch_status st = spool_args(levels, level_in, F, stride, dY, dX, partition ? field : field_t, c, &Li, &Lo, "hch_spool_avg_bwd");
    if (st != HCH_OK) return st;
    if (partition) return launch_field_unpool<false>(dY, nullptr, field, dX, Lo->n_total, Li->n_total, F * F * F, c, (hipStream_t)stream);
    return launch_field_avg(dY, field_t, dX, Li->n_total, Lo->n_total, F * F * F, c, (hipStream_t)stream);
}

extern "C" hch_status hch_avgpool_fwd(const hch_levels *levels, int32_t level_in, const float *X, float *Y,
                                      int32_t c, void *stream)
{
    if (!levels || level_in < 0 || level_in + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_avgpool_fwd: level_in must have a coarser level");
    if (!X || !Y || c <= 0) return fail(HCH_EINVAL, "hch_avgpool_fwd: bad argument");
    const Level &Lc = levels->lv[level_in + 1];
    const Level &Lf = levels->lv[level_in];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, "hch_avgpool_fwd: these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, "hch_avgpool_fwd: levels were built without device tables");
    const bool vec = c % 4 == 0 && aligned16(X) && aligned16(Y);
    const int64_t items = Lc.n_total * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_avgpool_fwd: too large");
    {
        const double bytes = (double)Lf.n_total * 4.0 * c + (double)Lc.n_total * (32.0 + 4.0 * c);
        hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("avgpool_fwd_kernel<4>") : HCH_KERNEL_ID("avgpool_fwd_kernel<1>"),
                            (hipStream_t)stream, bytes, 8.0 * Lc.n_total * c);
        if (vec)
            HCH_LAUNCH(hch::avgpool_fwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               X, Lc.dchild, Y, Lc.n_total, c);
        else
            HCH_LAUNCH(hch::avgpool_fwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               X, Lc.dchild, Y, Lc.n_total, c);
    }
    HCH_LAUNCH_CHECK("avgpool_fwd_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_avgpool_bwd(const hch_levels *levels, int32_t level_in, const float *dY, float *dX,
                                      int32_t c, void *stream)
{
    if (!levels || level_in < 0 || level_in + 1 >= (int32_t)levels->lv.size())
        return fail(HCH_EINVAL, "hch_avgpool_bwd: level_in must have a coarser level");
    if (!dY || !dX || c <= 0) return fail(HCH_EINVAL, "hch_avgpool_bwd: bad argument");
    const Level &Lc = levels->lv[level_in + 1];
    const Level &Lf = levels->lv[level_in];
    if (Lc.ratio != 2) return fail(HCH_EUNSUPPORTED, "hch_avgpool_bwd: these two levels are not in ratio 2; use hch_field_build with hch_spool_* / hch_sconv_*");
    if (!Lc.dchild) return fail(HCH_EINVAL, "hch_avgpool_bwd: levels were built without device tables");
    const bool vec = c % 4 == 0 && aligned16(dY) && aligned16(dX);
    const int64_t items = Lc.n_total * (vec ? c / 4 : c);
    if (items > MAX_GRID_ITEMS) return fail(HCH_EUNSUPPORTED, "hch_avgpool_bwd: too large");
    {
        const double bytes = (double)Lf.n_total * 4.0 * c + (double)Lc.n_total * (32.0 + 4.0 * c);
        hch::LaunchTimer lt(vec ? HCH_KERNEL_ID("avgpool_bwd_kernel<4>") : HCH_KERNEL_ID("avgpool_bwd_kernel<1>"),
                            (hipStream_t)stream, bytes, 0.0);
        if (vec)
            HCH_LAUNCH(hch::avgpool_bwd_kernel<4>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               dY, Lc.dchild, dX, Lc.n_total, c);
        else
            HCH_LAUNCH(hch::avgpool_bwd_kernel<1>, dim3(blocks_for(items)), dim3(256), 0, (hipStream_t)stream,
                               dY, Lc.dchild, dX, Lc.n_total, c);
    }
    HCH_LAUNCH_CHECK("avgpool_bwd_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_relu_fwd(const float *x, float *y, int64_t n, void *stream)
{
    if (!x || !y || n < 0) return fail(HCH_EINVAL, "hch_relu_fwd: bad argument");
    if (n == 0) return HCH_OK;
    {
        hch::LaunchTimer lt(HCH_KERNEL_ID("relu_fwd_kernel"), (hipStream_t)stream, 8.0 * n, 0.0);
        const int64_t n4 = (aligned16(x) && aligned16(y)) ? n / 4 : 0;
        HCH_LAUNCH(hch::relu_fwd_kernel, dim3(blocks_for(std::max(n4, n - 4 * n4))), dim3(256), 0,
                           (hipStream_t)stream, x, y, n, n4);
    }
    HCH_LAUNCH_CHECK("relu_fwd_kernel");
    return HCH_OK;
}

extern "C" hch_status hch_relu_bwd(const float *y, const float *dy, float *dx, int64_t n, void *stream)
{
    if (!y || !dy || !dx || n < 0) return fail(HCH_EINVAL, "hch_relu_bwd: bad argument");
    if (n == 0) return HCH_OK;
    {
        hch::LaunchTimer lt(HCH_KERNEL_ID("relu_bwd_kernel"), (hipStream_t)stream, 12.0 * n, 0.0);
        const int64_t n4 = (aligned16(y) && aligned16(dy) && aligned16(dx)) ? n / 4 : 0;
        HCH_LAUNCH(hch::relu_bwd_kernel, dim3(blocks_for(std::max(n4, n - 4 * n4))), dim3(256), 0,
                           (hipStream_t)stream, y, dy, dx, n, n4);
    }
    HCH_LAUNCH_CHECK("relu_bwd_kernel");
    return HCH_OK;
}

// ---------------------------------------------------------------------------------------
// per-kernel timing
// ---------------------------------------------------------------------------------------

extern "C" int32_t hch_set_lean_loops(int32_t enabled)
{
    return g_lean_loops.exchange(enabled ? 1 : 0);
}

extern "C" hch_status hch_probe_mfma(hch_dtype dtype, int32_t iters, int32_t workgroups, float *sink, void *stream)
{
    if (!sink || iters <= 0 || workgroups <= 0 || (dtype != HCH_F32 && dtype != HCH_BF16))
        return fail(HCH_EINVAL, "hch_probe_mfma: bad argument");
    hipStream_t s = (hipStream_t)stream;
    const double waves = 4.0 * workgroups, per = dtype == HCH_BF16 ? 16384.0 : 2048.0;
    hch::LaunchTimer lt(dtype == HCH_BF16 ? HCH_KERNEL_ID("mfma_probe_kernel<true>") : HCH_KERNEL_ID("mfma_probe_kernel<false>"),
                        s, 0.0, waves * iters * 8.0 * per);
    if (dtype == HCH_BF16) HCH_LAUNCH(hch::mfma_probe_kernel<true>, dim3((unsigned)workgroups), dim3(256), 0, s, sink, iters);
    else HCH_LAUNCH(hch::mfma_probe_kernel<false>, dim3((unsigned)workgroups), dim3(256), 0, s, sink, iters);
    HCH_LAUNCH_CHECK("mfma_probe_kernel");
    return HCH_OK;
}

extern "C" int32_t hch_kernel_count(void) { return hch::Profiler::get().count(); }

extern "C" const char *hch_kernel_name(int32_t id)
{
    thread_local std::string buf;
    buf = hch::Profiler::get().name(id);
    return buf.c_str();
}

extern "C" hch_status hch_profile_enable(int32_t kernel_id, int32_t on)
{
    if (kernel_id >= hch::Profiler::get().count()) return fail(HCH_EINVAL, "hch_profile_enable: unknown kernel id");
    hch::Profiler::get().enable(kernel_id, on != 0);
    return HCH_OK;
}

extern "C" hch_status hch_profile_read(int32_t kernel_id, hch_kernel_stats *out)
{
    if (!out || kernel_id < 0 || kernel_id >= hch::Profiler::get().count())
        return fail(HCH_EINVAL, "hch_profile_read: bad argument");
    hch::Profiler::get().collect();
    const hch::KernelStats st = hch::Profiler::get().read(kernel_id);
    out->launches = st.launches; out->ms = st.ms; out->bytes = st.bytes; out->flops = st.flops;
    return HCH_OK;
}

extern "C" hch_status hch_profile_reset(void)
{
    hch::Profiler::get().collect();
    hch::Profiler::get().reset();
    return HCH_OK;
}
