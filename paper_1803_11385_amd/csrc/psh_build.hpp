// Host-side construction of perfect spatial hash tables (paper Section 3.1, 5.2).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

namespace hch {

// Tables of one model at one level.
struct ModelTables {
    int m = 0;                    // hash table side
    int r = 0;                    // offset table side
    int attempts = 0;             // offset table sizes tried
    std::vector<int32_t> H;       // m^3, data index or -1
    std::vector<uint16_t> T;      // m^3 x 3, position tag, 0xFFFF on empty slots
    std::vector<uint8_t> Phi;     // r^3 x 3
};

enum BuildResult { BUILD_OK = 0, BUILD_UNSUPPORTED = 1, BUILD_FAILED = 2 };

int hash_side(int64_t n);                 // smallest m with m^3 > n
int offset_side_first(int64_t n, int m);  // smallest r with 6 r^3 >= n, then coprime to m
int offset_side_next(int r, int m);       // smallest larger r with >= 2x the cells, coprime to m

// xyz: n x 3 positions in [0, ubar); data index = row number.  Input is assumed validated.
BuildResult build_model_tables(const int32_t *xyz, int64_t n, int ubar, ModelTables &out);

// Parents floor(p / ratio) of a model's voxels on the grid of side ceil(ubar_fine / ratio), unique,
// ordered by linear position.
void coarsen_model(const int32_t *xyz, int64_t n, int ubar_fine, int ratio, std::vector<int32_t> &out_xyz);

}  // namespace hch
