/*
 * hch -- the hot path of H-CNN (spatial-hashing based CNN for 3D shapes) on one
 * AMD MI355X (gfx950): 3x3x3 convolution and 2x2x2 max-pooling over the sparse
 * surface voxels of a mini-batch of shapes held in per-level perfect spatial hash
 * (PSH) tables.
 *
 * C ABI.  Plain pointers and sizes only.  Every function returns an hch_status
 * (0 = HCH_OK); nothing throws, aborts or prints.  hch_last_error() returns a
 * thread-local message for the last non-OK status.
 *
 * Pointer kinds are stated per argument: HOST = ordinary process memory,
 * DEVICE = memory of the current HIP device (e.g. torch tensor storage).
 * `stream` is a hipStream_t passed as void* (NULL = the default stream).  Kernels
 * are enqueued on it and NOT synchronised, except where stated.
 *
 * Data layout (differs from the paper, Section 3.2, which stores a level's data
 * array channel-major c x N): feature / gradient tensors are VOXEL-MAJOR rows,
 *     X[N_l][c]      row i = the c features of the voxel with global data index i,
 * so one neighbour fetch is one contiguous read.  Global data index = N*[v] + the
 * voxel's rank inside model v (Eq.6).  At the finest level the rank is the order of
 * the caller's coordinates; at coarser levels voxels of a model are ordered by their
 * linear position (x*u + y)*u + z.
 * Weights are W[27][c_in][c_out], tap k = (dx+1)*9 + (dy+1)*3 + (dz+1) for the
 * neighbour offset (dx,dy,dz) in {-1,0,1}^3  (the paper's W is c_out x (c_in*27)
 * with column i_c*27 + k: the same numbers transposed).
 * The column matrix of hash2col (Algorithm 1) is col[N_l][27*c_in], element
 * (i, k*c_in + c) = X[neighbour k of voxel i][c], or 0 where that neighbour is
 * empty or outside the grid.
 */
#ifndef HCH_H
#define HCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HCH_OK = 0,
    HCH_EINVAL = 1,        /* null pointer, bad size, coordinates out of range / duplicated ... */
    HCH_ENOMEM = 2,        /* host or device allocation failed                                   */
    HCH_EBUILD = 3,        /* PSH construction did not succeed even with singleton buckets       */
    HCH_EHIP = 4,          /* a HIP runtime call failed (message has the HIP error string)       */
    HCH_EUNSUPPORTED = 5,  /* a model needs a hash table side above 256 (8-bit offsets), ...     */
    HCH_EWORKSPACE = 6     /* workspace smaller than hch_conv_workspace_bytes(..., HCH_WS_MIN)   */
} hch_status;

typedef enum {
    HCH_F32 = 0,           /* X, W, dY are float; all arithmetic in fp32                          */
    HCH_BF16 = 1           /* X, W, dY are bfloat16 bit patterns (uint16); products accumulate in
                              fp32; outputs Y, dX, dW are float                                   */
} hch_dtype;

typedef struct hch_levels hch_levels;   /* opaque; owned by the library */

/* Read-only view of one level of the mini-batch "super-PSH" (Section 3.2).  All
 * pointers are owned by the hch_levels object and stay valid until hch_free_levels. */
typedef struct {
    int32_t ubar;            /* grid resolution of this level                                   */
    int32_t batch;           /* b                                                               */
    int64_t n_total;         /* N*[b]: occupied voxels of the whole batch                       */
    int64_t m_total;         /* M*[b]: hash slots of the whole batch                            */
    int64_t r_total;         /* R*[b]: offset-table cells of the whole batch                    */
    int64_t nbr_valid;       /* occupied entries of nbr27 (centre included); 0 for host-only    */
    /* HOST arrays */
    const int32_t *mbar;     /* [b]   hash table side per model (Section 5.2: m^3 > n)          */
    const int32_t *rbar;     /* [b]   offset table side per model                               */
    const int32_t *attempts; /* [b]   number of offset-table sizes tried during construction    */
    const int64_t *M;        /* [b+1] exclusive prefix of m^3, leading 0                        */
    const int64_t *R;        /* [b+1] exclusive prefix of r^3                                   */
    const int64_t *N;        /* [b+1] exclusive prefix of n                                     */
    const int32_t *coords_host; /* [n_total][3] voxel positions in data order                   */
    const int32_t *H_host;   /* host copies of the four super tables below, same shapes         */
    const uint16_t *T_host;
    const uint8_t *Phi_host;
    const int32_t *V_host;
    /* DEVICE arrays */
    const int32_t *H;        /* [m_total]     H*: local data index of the slot, -1 = redundant  */
    const uint16_t *T;       /* [m_total][3]  T*: position tag, 0xFFFF x3 on redundant slots    */
    const uint8_t *Phi;      /* [r_total][3]  Phi*: per-axis offsets, each < m                  */
    const int32_t *V;        /* [m_total]     V*: model index of the slot (0-based)             */
    const int32_t *coords;   /* [n_total][3]  voxel positions in data order                     */
    const int32_t *nbr27;    /* [n_total][27] global data index of neighbour k, or -1           */
    const int32_t *child8;   /* [n_total][8]  global data index AT THE NEXT FINER LEVEL of child
                                k = dx*4 + dy*2 + dz at 2p + (dx,dy,dz), or -1; NULL at level 0  */
    const int32_t *row_order;/* [n_total]     the level's data indices in "pattern order": sorted
                                (stably) by a 6-bit key, one bit per pair of opposite edge-adjacent
                                neighbours (taps k and 26-k, k = 1, 3, .., 11; first pair = most
                                significant bit): set if either exists.  Consecutive entries have
                                similar sets of neighbours.  NULL for host-only level sets        */
    const uint32_t *tile_taps;/* [ceil(n_total/64)] bit k of entry b: some voxel among
                                row_order[64b .. 64b+63] has neighbour k.  The fused products
                                work on such tiles and leave out the taps a tile lacks            */
} hch_level_desc;

const char *hch_last_error(void);

/*
 * Build the multi-level PSH of a mini-batch (Section 3.1, 3.2, 5.2).
 *
 *   coords_xyz     HOST  [n_total][3] int32, finest level, 0 <= x,y,z < resolution; the
 *                        voxels of model v are rows model_offsets[v] .. model_offsets[v+1]-1;
 *                        no duplicates inside a model
 *   model_offsets  HOST  [batch+1] int64, model_offsets[0] = 0, strictly increasing
 *   resolution     grid side of the finest level: a power of two, 2 .. 32768 (positions are
 *                  tagged with 16 bits per axis and 0xFFFF marks an empty slot)
 *   n_levels       number of levels, >= 1; level l has side resolution >> l (must stay >= 1);
 *                  a coarse voxel is occupied iff one of its 8 children is (Section 5.1)
 *
 * Per model and level: hash table side m = smallest with m^3 > n; offset table side r starts
 * at the smallest with 6 r^3 >= n and, whenever construction fails, grows to the smallest
 * side with at least double the cells (Section 5.2); both are kept coprime.  The tables are
 * concatenated into the super tables with prefix arrays M*, R*, N* and the model index V*.
 * Construction runs on the host; the tables are then uploaded and the per-voxel neighbour and
 * child index lists are produced on the device by PSH lookups (hch_build_neighbours).
 * BLOCKS until everything is resident.  *out is owned by the library; release it with
 * hch_free_levels.  Errors: HCH_EINVAL (arguments, range, duplicates, empty model),
 * HCH_EUNSUPPORTED (m > 256), HCH_EBUILD, HCH_ENOMEM, HCH_EHIP; *out is NULL on error.
 */
hch_status hch_build_levels(const int32_t *coords_xyz, const int64_t *model_offsets,
                            int32_t batch, int32_t resolution, int32_t n_levels,
                            void *stream, hch_levels **out);

/*
 * The same object with the tables CONSTRUCTED ON THE DEVICE (Section 5.2 and the conclusion name
 * GPU construction as future work).  Host work: argument checks and the occupancy of the coarser
 * levels; then one set of launches builds every (level, model) pair: buckets of positions sharing
 * p mod r are placed largest first, all buckets of one size in parallel, each claiming its slots
 * with compare-and-swap and backing off to the next candidate offset on a conflict; pairs that
 * fail are repeated with the next offset-table side.  Sizes (m, first r, growth of r), table
 * formats and everything computed through the tables (neighbour and child lists, every
 * convolution and pooling result) are the same as with hch_build_levels; the tables themselves
 * are valid but differ from the host-built ones and from run to run (which of two racing buckets
 * gets a slot depends on timing), and `attempts` / r may differ.  Same arguments, ownership and
 * errors as hch_build_levels; BLOCKS.
 */
hch_status hch_build_levels_device(const int32_t *coords_xyz, const int64_t *model_offsets,
                                   int32_t batch, int32_t resolution, int32_t n_levels,
                                   void *stream, hch_levels **out);

/*
 * Level sets whose resolutions are in ratios other than 2 (Section 4: unlike an octree, a PSH can
 * be generated on a grid of arbitrary resolution, which is what allows any stride):
 *   resolution  grid side of the finest level, any integer 2 .. 32768
 *   ratios      HOST [n_levels - 1], ratios[l] >= 2: level l+1 has side ceil(side_l / ratios[l]) and
 *               holds the voxels floor(p / ratios[l]) of level l's voxels p (occupied iff one of the
 *               ratios[l]^3 positions below it is), ordered by linear position per model
 *   device_tables  0: tables constructed on the host as in hch_build_levels; else on the device
 * Everything else as hch_build_levels.  child8 exists only between levels in ratio 2, and only
 * there hch_pool_*, hch_relu_pool_*, hch_avgpool_*, hch_unpool_* apply (HCH_EUNSUPPORTED
 * elsewhere); between any two levels use hch_field_build with hch_sconv_* and hch_spool_*.
 */
hch_status hch_build_levels_ratios(const int32_t *coords_xyz, const int64_t *model_offsets,
                                   int32_t batch, int32_t resolution, int32_t n_levels,
                                   const int32_t *ratios, int32_t device_tables,
                                   void *stream, hch_levels **out);

/*
 * The host half of hch_build_levels only: occupancy of every level, PSH construction and the
 * super tables, kept in host memory.  Touches no GPU.  The object serves hch_level_info (all
 * DEVICE pointers are NULL) and hch_free_levels; every other call rejects it with HCH_EINVAL.
 */
hch_status hch_build_tables_host(const int32_t *coords_xyz, const int64_t *model_offsets,
                                 int32_t batch, int32_t resolution, int32_t n_levels,
                                 hch_levels **out);

void hch_free_levels(hch_levels *levels);

int32_t hch_num_levels(const hch_levels *levels);

/* Fill *out with the view of `level` (0 = finest).  HCH_EINVAL if out of range. */
hch_status hch_level_info(const hch_levels *levels, int32_t level, hch_level_desc *out);

/*
 * (Re)compute on the device, by hash lookups through the level's PSH (Eq.1, Eq.4-6 and the
 * tag test of Section 3.1), the "pre-stored neighbour information" of Section 5.3:
 * nbr27 of `level`, and child8 of `level` (looked up in level-1's tables) when level > 0.
 * This is the index side of the traversal of Algorithm 1, done once per level and batch
 * instead of once per channel.  level = -1 does every level (two launches in all).
 * Asynchronous on `stream`.
 */
hch_status hch_build_neighbours(hch_levels *levels, int32_t level, void *stream);

/* The same for levels first .. first+count-1 (two launches for the whole range), so that a
 * caller can build the finest level on one stream and the coarser ones beside it on another. */
hch_status hch_build_neighbours_range(hch_levels *levels, int32_t first, int32_t count, void *stream);

/*
 * Optional tap-major copy of nbr27, [27][N_l] instead of [N_l][27], of `level` (-1: every level).
 * The products with bf16 inputs are bound by the number of cache accesses of their gathers, and
 * the 27 indices of a voxel one tap at a time cost one access per voxel; from the copy the
 * indices that a tile of voxels needs for a tap are consecutive.  The first call on a level
 * allocates N_l * 108 bytes (owned by `levels`); the copy is refreshed by this call and by every
 * later hch_build_neighbours* on that level, and used by hch_conv_* (bf16) when present.
 * Results do not depend on it.  Asynchronous on `stream` apart from the allocation.
 */
hch_status hch_build_tap_major(hch_levels *levels, int32_t level, void *stream);

/*
 * hash2col (Algorithm 1), rows [row_begin, row_begin + row_count) of the column matrix:
 *   X    DEVICE [N_l][c_in]              (float or bf16 per dtype)
 *   col  DEVICE [row_count][27*c_in]     same element type as X; written completely
 *                                        (zeros for empty neighbours)
 */
hch_status hch_hash2col(const hch_levels *levels, int32_t level, hch_dtype dtype,
                        const void *X, int32_t c_in, int64_t row_begin, int64_t row_count,
                        void *col, void *stream);

/*
 * col2hash (Algorithm 2): dX[j][:] = sum over (i,k) with neighbour k of voxel i equal to j of
 * dcol[i][k*c_in + :].  dcol DEVICE [N_l][27*c_in] float; dX DEVICE [N_l][c_in] float,
 * overwritten (no need to zero it).  The sum is taken per destination row in fixed tap
 * order, so results are bit-reproducible run to run.
 */
hch_status hch_col2hash(const hch_levels *levels, int32_t level, const float *dcol,
                        int32_t c_in, float *dX, void *stream);

/* How a convolution call computes its products.  Both give the same results up to the order
 * of fp32 additions.
 *   HCH_ALGO_COLUMNS  the paper's three steps: hash2col writes the column matrix to the
 *                     workspace, a dense GEMM consumes it, col2hash folds gradients back.
 *   HCH_ALGO_FUSED    the same products with the column matrix gathered through the index rows
 *                     straight into the GEMM's operand tile, so it never goes to memory.
 *   HCH_ALGO_COLUMNS_RESIDENT  hch_conv_bwd_weight only: as HCH_ALGO_COLUMNS, but the workspace
 *                     still holds the column matrix of X that hch_conv_fwd(HCH_ALGO_COLUMNS) left
 *                     at its start (same level, c_in, dtype and X; a workspace of at least the
 *                     HCH_WS_FWD size, so that the forward pass ran in one piece, and not used by
 *                     another call since), so hash2col is not run again.  The caller vouches for
 *                     the contents; sizes as for HCH_ALGO_COLUMNS.
 *   HCH_ALGO_FUSED_DENSE  HCH_ALGO_FUSED without its tap compaction: where the fused algorithm
 *                     would compact, tap by tap, the voxels whose neighbour exists and multiply
 *                     only those rows, this one multiplies whole rows of the column matrix, zeros
 *                     included (what the paper's dense GEMM does).  For measurement.  */
typedef enum { HCH_ALGO_COLUMNS = 0, HCH_ALGO_FUSED = 1, HCH_ALGO_COLUMNS_RESIDENT = 2, HCH_ALGO_FUSED_DENSE = 3 } hch_algo;

typedef enum {
    HCH_WS_FWD = 0,         /* hch_conv_fwd: everything in one pass                            */
    HCH_WS_BWD_DATA = 1,    /* hch_conv_bwd_data: required size                                */
    HCH_WS_BWD_WEIGHT = 2,  /* hch_conv_bwd_weight: required size                              */
    HCH_WS_MIN = 3          /* smallest workspace hch_conv_fwd accepts                         */
} hch_ws_kind;

/* Bytes of DEVICE workspace for a 3x3x3 stride-1 convolution on `level` (at least 256).
 * Returns 0 on bad arguments.  With HCH_ALGO_COLUMNS the workspace holds the column matrix
 * (N_l x 27*c_in elements) and, for small levels, partial sums of a split reduction;
 * hch_conv_fwd accepts any size >= the HCH_WS_MIN value and walks the voxels in chunks when
 * given less than HCH_WS_FWD; the two backward calls need their full size.  With
 * HCH_ALGO_FUSED only the partial sums and one rearranged copy of the weights live there
 * (bwd_data: flipped and transposed; fwd with bf16 inputs and c_in a multiple of 64:
 * transposed per tap). */
size_t hch_conv_workspace_bytes(const hch_levels *levels, int32_t level, int32_t c_in,
                                int32_t c_out, hch_dtype dtype, hch_ws_kind kind, hch_algo algo);

/*
 * Convolution forward (Eq.2 = Eq.3):  Y = hash2col(X) . W
 *   X  DEVICE [N_l][c_in], W DEVICE [27][c_in][c_out]  (dtype);  Y DEVICE [N_l][c_out] float,
 *   overwritten.  workspace DEVICE, ws_bytes as above, 256-byte aligned.  No bias.
 * Errors of the three convolution calls: HCH_EINVAL (null pointer, channel count <= 0, level,
 * dtype or algorithm unknown, workspace misaligned, 27*c_in*c_out >= 2^31), HCH_EWORKSPACE
 * (ws_bytes below the required size), HCH_EUNSUPPORTED (N_l >= 2^31/64, or a feature matrix of
 * 2^31 elements or more, N_l * max(c_in, c_out): rows are indexed with 32 bits), HCH_EHIP (a
 * launch failed).  Nothing is written on error.
 */
hch_status hch_conv_fwd(const hch_levels *levels, int32_t level, hch_dtype dtype,
                        const void *X, const void *W, float *Y, int32_t c_in, int32_t c_out,
                        void *workspace, size_t ws_bytes, hch_algo algo, void *stream);

/*
 * Back-propagation to the input (Eq.8 followed by col2hash, Algorithm 2):
 *   dcol = dY . W^T ;  dX = col2hash(dcol)
 *   dY DEVICE [N_l][c_out], W DEVICE [27][c_in][c_out] (dtype); dX DEVICE [N_l][c_in] float,
 *   overwritten.
 */
hch_status hch_conv_bwd_data(const hch_levels *levels, int32_t level, hch_dtype dtype,
                             const void *dY, const void *W, float *dX, int32_t c_in,
                             int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                             void *stream);

/*
 * Weight gradient (Eq.7):  dW = hash2col(X)^T . dY
 *   X DEVICE [N_l][c_in], dY DEVICE [N_l][c_out] (dtype); dW DEVICE [27][c_in][c_out] float,
 *   overwritten.  Partial sums over blocks of voxels are combined in a fixed order
 *   (bit-reproducible).
 */
hch_status hch_conv_bwd_weight(const hch_levels *levels, int32_t level, hch_dtype dtype,
                               const void *X, const void *dY, float *dW, int32_t c_in,
                               int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                               void *stream);

/*
 * hch_conv_bwd_weight with HCH_ALGO_FUSED for callers that can neither allocate device memory nor
 * hand over a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The call itself allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine): the partial sums of its split reduction go to an array of HCH_NOALLOC_SCRATCH_BYTES
 * bytes that is part of the library's device image, so every GPU the library runs on holds that
 * much memory until the process ends.  Same arguments (minus workspace and algorithm), same
 * kernels, same bits in dW as hch_conv_bwd_weight(..., HCH_ALGO_FUSED).
 * Errors: as hch_conv_bwd_weight, and HCH_EWORKSPACE when the product's partial sums,
 * hch_conv_workspace_bytes(levels, level, c_in, c_out, dtype, HCH_WS_BWD_WEIGHT, HCH_ALGO_FUSED),
 * exceed HCH_NOALLOC_SCRATCH_BYTES (nothing is launched then; the library's split planning fills
 * one round of workgroups, which keeps those sums below 24 MiB for every level and channel count,
 * so this only guards against a change of that planning).
 * All calls on one GPU share the one array: calls that may overlap on a GPU (different streams,
 * different host threads) race on it and must be serialised by the caller; calls on the same
 * stream are ordered.  The array keeps the last call's partial sums; every call overwrites all the
 * entries it later reads, so nothing needs clearing in between.
 */
#define HCH_NOALLOC_SCRATCH_BYTES (32u << 20)
hch_status hch_conv_bwd_weight_noalloc(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                       const void *X, const void *dY, float *dW, int32_t c_in,
                                       int32_t c_out, void *stream);

/*
 * 2x2x2 stride-2 max-pooling from level_in (fine) to level_in + 1 (coarse) (Section 4,
 * pooling): per coarse voxel and channel the maximum over the OCCUPIED children, and the
 * switch = global data index (at level_in) of the child holding it; the first child in
 * k order wins ties, a NaN never replaces an earlier value.
 *   X DEVICE [N_fine][c] float; Y DEVICE [N_coarse][c] float; argmax DEVICE [N_coarse][c] int32.
 */
hch_status hch_pool_fwd(const hch_levels *levels, int32_t level_in, const float *X, float *Y,
                        int32_t *argmax, int32_t c, void *stream);

/*
 * Max-pool backward (= max-unpooling, Section 4): dX[argmax[o][ch]][ch] = dY[o][ch], every
 * other element of dX is 0.  dX DEVICE [N_fine][c] float is overwritten completely.
 * argmax must hold, per coarse voxel, indices of its own children (what hch_pool_fwd wrote).
 */
hch_status hch_pool_bwd(const hch_levels *levels, int32_t level_in, const float *dY,
                        const int32_t *argmax, float *dX, int32_t c, void *stream);

/*
 * Transposed convolution (Section 4: "flips the input and output of the forward convolution
 * using a transposed kernel", i.e. Eq.8 followed by col2hash) and its two gradients.
 *   W DEVICE [27][c_out][c_in] are the weights of the FORWARD convolution c_out -> c_in that is
 *   being transposed;  X DEVICE [N_l][c_in];  Y DEVICE [N_l][c_out] float, overwritten.
 *   hch_deconv_fwd        Y  = col2hash(X . W^T)
 *   hch_deconv_bwd_data   dX = hash2col(dY) . W               (dX [N_l][c_in])
 *   hch_deconv_bwd_weight dW = hash2col(dY)^T . X             (dW [27][c_out][c_in])
 * Workspace: hch_conv_workspace_bytes with the channel counts exchanged (c_out, c_in) and the
 * kinds HCH_WS_BWD_DATA, HCH_WS_FWD, HCH_WS_BWD_WEIGHT respectively.
 */
hch_status hch_deconv_fwd(const hch_levels *levels, int32_t level, hch_dtype dtype, const void *X,
                          const void *W, float *Y, int32_t c_in, int32_t c_out, void *workspace,
                          size_t ws_bytes, hch_algo algo, void *stream);
hch_status hch_deconv_bwd_data(const hch_levels *levels, int32_t level, hch_dtype dtype,
                               const void *dY, const void *W, float *dX, int32_t c_in, int32_t c_out,
                               void *workspace, size_t ws_bytes, hch_algo algo, void *stream);
hch_status hch_deconv_bwd_weight(const hch_levels *levels, int32_t level, hch_dtype dtype,
                                 const void *X, const void *dY, float *dW, int32_t c_in,
                                 int32_t c_out, void *workspace, size_t ws_bytes, hch_algo algo,
                                 void *stream);

/*
 * Max-unpooling from level_out + 1 (coarse) to level_out (fine) (Section 4): the receptive field
 * of every coarse voxel is zero except at its recorded switch, which receives the coarse value.
 *   Xc DEVICE [N_coarse][c];  argmax as written by hch_pool_fwd;  Y DEVICE [N_fine][c], overwritten.
 * Backward: dXc[o][ch] = dY[argmax[o][ch]][ch].
 */
hch_status hch_unpool_fwd(const hch_levels *levels, int32_t level_out, const float *Xc,
                          const int32_t *argmax, float *Y, int32_t c, void *stream);
hch_status hch_unpool_bwd(const hch_levels *levels, int32_t level_out, const float *dY,
                          const int32_t *argmax, float *dXc, int32_t c, void *stream);

/*
 * Convolutions with a general kernel side F, stride and padding (Algorithm 1 and 2 as the paper
 * states them, Section 4: receptive field [p*S - P, p*S - P + F - 1]^3 on the input level for
 * output voxel p; [p - (F-1)/2, p + (F-1)/2]^3 when S = 1), and 2x2x2 average pooling (Section 4:
 * a convolution whose weights all equal 1/F^3).  Stride S reads level_in and writes the level
 * of the same hch_levels object whose grid is S times coarser: level_in + log2(S) when the levels
 * halve the resolution (hch_build_levels), or wherever the ratios given to
 * hch_build_levels_ratios multiply up to S; HCH_EINVAL if there is no such level.  F = 1..7;
 * S = 1 needs odd F and P = (F-1)/2.
 *
 * hch_field_build fills the index rows of the traversal by hash lookups (the general form of
 * the "pre-stored neighbour information"); both are caller-owned DEVICE buffers, either may be
 * NULL:
 *   field    [N_out][F^3]  input data index at row (fx*F + fy)*F + fz of output voxel o's field,
 *                          or -1 (empty, or outside the grid)
 *   field_t  [N_in][F^3]   data index of the output voxel whose field holds input voxel i at that
 *                          row, or -1: Algorithm 2's scatter turned into a gather
 * The products take them as arguments (W is [F^3][c_in][c_out], row as above):
 *   hch_sconv_fwd         Y[N_out][c_out]  = gathered columns . W                (Eq.3)
 *   hch_sconv_bwd_weight  dW               = gathered columns^T . dY             (Eq.7)
 *   hch_sconv_bwd_data    dX[N_in][c_in]   = sum_rows dY[field_t[i][row]] . W[row]^T   (Eq.8 + Alg.2)
 * X / dX live on level_in, Y / dY on the output level; dtype, outputs (fp32, overwritten),
 * workspace rules (256-byte aligned, at least hch_sconv_workspace_bytes) and errors as for
 * hch_conv_*.  With F = 3, S = 1, P = 1 `field` equals nbr27 and the results equal hch_conv_*'s.
 */
hch_status hch_field_build(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                           int32_t pad, int32_t *field, int32_t *field_t, void *stream);
size_t hch_sconv_workspace_bytes(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                 int32_t c_in, int32_t c_out, hch_dtype dtype, hch_ws_kind kind);
hch_status hch_sconv_fwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                         hch_dtype dtype, const void *X, const void *W, float *Y, const int32_t *field,
                         int32_t c_in, int32_t c_out, void *workspace, size_t ws_bytes, void *stream);
hch_status hch_sconv_bwd_weight(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                                hch_dtype dtype, const void *X, const void *dY, float *dW,
                                const int32_t *field, int32_t c_in, int32_t c_out, void *workspace,
                                size_t ws_bytes, void *stream);
hch_status hch_sconv_bwd_data(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                              hch_dtype dtype, const void *dY, const void *W, float *dX,
                              const int32_t *field_t, int32_t c_in, int32_t c_out, void *workspace,
                              size_t ws_bytes, void *stream);

/*
 * Pooling over general receptive fields (Section 4: pooling is a convolution-like traversal with
 * stride S > 1, and "any stride sizes" are possible because a PSH can be built on a grid of any
 * resolution), between level_in and the level S times coarser, through the index rows of
 * hch_field_build(levels, level_in, F, S, pad, field, field_t):
 *   hch_spool_max_fwd  Y[o][ch] = maximum of X over the occupied entries of field[o][:], argmax the
 *                      entry's data index; rules as for hch_pool_fwd (first maximum in row order,
 *                      NaN never replaces, empty field: 0 and -1)
 *   hch_spool_max_bwd  dX[q][ch] = sum of dY[o][ch] over the outputs o = field_t[q][:] whose switch
 *                      for ch is q (at most one when fields do not overlap, F <= S); dX is
 *                      written completely
 *   hch_spool_avg_fwd  Y[o] = (sum of the occupied entries' rows) / F^3     (weights 1/F^3)
 *   hch_spool_avg_bwd  dX[q] = (sum of dY[o] over o = field_t[q][:]) / F^3
 * The two backward calls take `pad` (the padding the index rows were built with) and both `field`
 * and `field_t`, either of which may be NULL: when F = S > 1 and pad = 0 the fields partition the
 * input level and every input voxel lies in the field of an occupied output voxel, so, given
 * `field`, each output voxel writes the rows of its own field (faster than the gather through
 * `field_t`, same result); in every other case `field_t` is needed (HCH_EINVAL without it) and
 * `field` is ignored: with padding an input voxel can fall into the field of an unoccupied
 * position, which no forward row reaches.
 * X, dX DEVICE [N_in][c] float;  Y, dY DEVICE [N_out][c] float;  argmax DEVICE [N_out][c] int32.
 * With F = 2, S = 2, pad = 0 on levels in ratio 2 the results equal hch_pool_* / hch_avgpool_*.
 */
hch_status hch_spool_max_fwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                             const float *X, const int32_t *field, float *Y, int32_t *argmax,
                             int32_t c, void *stream);
hch_status hch_spool_max_bwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                             int32_t pad, const float *dY, const int32_t *argmax, const int32_t *field,
                             const int32_t *field_t, float *dX, int32_t c, void *stream);
hch_status hch_spool_avg_fwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                             const float *X, const int32_t *field, float *Y, int32_t c, void *stream);
hch_status hch_spool_avg_bwd(const hch_levels *levels, int32_t level_in, int32_t F, int32_t stride,
                             int32_t pad, const float *dY, const int32_t *field, const int32_t *field_t,
                             float *dX, int32_t c, void *stream);

/*
 * 2x2x2 average pooling from level_in to level_in + 1 and its adjoint (the average-unpooling of
 * Section 4).  Y[o] = (sum over the occupied children of o of X[child]) / 8: an empty child
 * counts as zero, as in a convolution with weights 1/8.  Backward: every occupied child of o
 * receives dY[o] / 8; dX is written completely.
 *   X, dX DEVICE [N_fine][c];  Y, dY DEVICE [N_coarse][c]
 */
hch_status hch_avgpool_fwd(const hch_levels *levels, int32_t level_in, const float *X, float *Y,
                           int32_t c, void *stream);
hch_status hch_avgpool_bwd(const hch_levels *levels, int32_t level_in, const float *dY, float *dX,
                           int32_t c, void *stream);

/*
 * The two steps that sit between a convolution and the next level in the paper's networks
 * (Section 5.1: Convolution -> ReLU -> Pooling), fused into one pass each; results are
 * identical to calling the separate functions.
 *   hch_relu_pool_fwd:  A = max(Y, 0) (DEVICE [N_fine][c], written completely), then
 *                       P, argmax = hch_pool_fwd(A).  A may be NULL: the rectified rows are
 *                       then not stored (a training step needs only their sign, which Y has).
 *   hch_pool_relu_bwd:  dY = hch_relu_bwd(A, hch_pool_bwd(dP, argmax)), written completely.
 *                       Only the sign of A is read, so Y may be passed in its place.
 *   hch_pool_relu_bwd_pooled:  the same result from the pooled rows P (DEVICE [N_coarse][c]) that
 *                       hch_relu_pool_fwd wrote with this argmax: the child a switch names
 *                       carries the maximum, so A[argmax[o][ch]][ch] = P[o][ch] and P's sign
 *                       decides.  Neither A nor Y is read: a training step need not keep them.
 */
hch_status hch_relu_pool_fwd(const hch_levels *levels, int32_t level_in, const float *Y, float *A,
                             float *P, int32_t *argmax, int32_t c, void *stream);
hch_status hch_pool_relu_bwd(const hch_levels *levels, int32_t level_in, const float *dP,
                             const int32_t *argmax, const float *A, float *dY, int32_t c,
                             void *stream);
hch_status hch_pool_relu_bwd_pooled(const hch_levels *levels, int32_t level_in, const float *dP,
                                    const int32_t *argmax, const float *P, float *dY, int32_t c,
                                    void *stream);

/* Element-wise ReLU over a compact data array of n floats (Section 4, "other CNN
 * operations"): y = max(x, 0);  backward dx = (y > 0) ? dy : 0.  In-place use is allowed. */
hch_status hch_relu_fwd(const float *x, float *y, int64_t n, void *stream);
hch_status hch_relu_bwd(const float *y, const float *dy, float *dx, int64_t n, void *stream);

/*
 * Measurement aid: a kernel that does nothing but matrix instructions, so that a benchmark can
 * state the rate the chip's matrix pipes actually reach next to the rates of the products above.
 * `workgroups` workgroups of 4 wavefronts each run `iters` iterations of 8 independent
 * instructions (HCH_F32: v_mfma_f32_16x16x4_f32, 2048 flops each; HCH_BF16:
 * v_mfma_f32_16x16x32_bf16, 16384 flops each), i.e. workgroups * 4 * iters * 8 instructions.
 *   sink  DEVICE [workgroups * 256] float, overwritten.  Asynchronous on `stream`.
 */
hch_status hch_probe_mfma(hch_dtype dtype, int32_t iters, int32_t workgroups, float *sink, void *stream);

/*
 * Measurement and test aid: the products of a convolution have two forms of their main loop,
 * one that addresses memory with guarded 64-bit pointers and works for every shape, and a lean
 * one (loads through buffer descriptors, scalar offsets) that the library takes when the
 * operands allow it.  Both multiply the same tiles in the same order, so their results agree bit
 * for bit; `enabled` = 0 makes every later call take the first form, 1 (the default) restores the
 * choice.  Process-wide, not synchronised with calls running on other threads.  Returns the
 * previous setting.
 */
int32_t hch_set_lean_loops(int32_t enabled);

/*
 * Optional per-kernel timing, for benchmarks.  A kernel gets an id in [0, hch_kernel_count())
 * the first time it is launched; hch_kernel_name gives the name of its __global__ function,
 * template arguments included, as a profiler prints it (the pointer is valid until the next
 * call on the same thread).  hch_profile_enable(id, on): launches of that kernel are bracketed
 * by two HIP events on their stream while on != 0; id = -1 switches every kernel, also ones
 * that have not run yet.  Off by default.  hch_profile_read blocks until the bracketed launches
 * so far have finished and returns, for one kernel, the number of timed launches, the sum of
 * their durations, and the sums of their ALGORITHMIC bytes and flops (every operand moved
 * once, as counted from the launch's shapes; not a hardware counter).  hch_profile_reset clears
 * the sums.
 */
typedef struct {
    int64_t launches;
    double ms;
    double bytes;
    double flops;
} hch_kernel_stats;

int32_t hch_kernel_count(void);
const char *hch_kernel_name(int32_t kernel_id);
hch_status hch_profile_enable(int32_t kernel_id, int32_t on);
hch_status hch_profile_read(int32_t kernel_id, hch_kernel_stats *out);
hch_status hch_profile_reset(void);

#ifdef __cplusplus
}
#endif
#endif /* HCH_H */
