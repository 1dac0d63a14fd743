/*
 * CPU oracle for the H-CNN hot path -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow, double-precision restatement of what the paper's method
 * computes: perfect-spatial-hash construction and lookup (Section 3.1, Eq.1,
 * Section 5.2), the mini-batch "super" tables and their prefix arrays
 * (Section 3.2), the hash2col / col2hash traversals (Algorithms 1 and 2, Eq.4-6),
 * convolution as a matrix product and its two gradients (Eq.2, 3, 7, 8) and
 * max-pooling with switches (Section 4, pooling / unpooling paragraphs).
 *
 * It keeps the paper's own layouts and notation:
 *   - the data array D* of a level is a row-major  c x N  matrix (channel-major,
 *     one column per occupied voxel);
 *   - the column matrix D~ is  (c * F^3) x N_o , row index  i_c * F^3 + row ;
 *   - W is  c_out x (c_in * F^3) ;
 *   - the traversals iterate over (channel, output HASH SLOT) exactly as the
 *     algorithms do, reading the voxel position back from the position tag.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the GPU path.
 *
 * Readings of points the paper leaves open (each is a convention that the GPU
 * library restates independently):
 *   - Eq.1 is read per axis as (h0(p) + Phi[h1(p)]) mod m, the form the worked
 *     2-D example of Section 3.1 evaluates;
 *   - d-dimensional tables are flattened with z fastest: lin_k(x,y,z)=(x*k+y)*k+z;
 *   - the row stride of D~ per channel is F^3 (the algorithms print F);
 *   - a receptive field is walked x-slowest / z-fastest ("spatial arrangement");
 *   - positions outside [0,u)^3 are empty and are never hashed;
 *   - model indices are 0-based: M*[v], R*[v], N*[v] are model v's bases;
 *   - empty hash slots carry H=-1, T=(0xFFFF,0xFFFF,0xFFFF); unused offset
 *     cells are (0,0,0); V* is filled for every slot of a model;
 *   - max-pooling takes the maximum over OCCUPIED children only, the first
 *     child in walk order wins ties (a later child replaces only if strictly
 *     greater), and the switch is the global data index at the fine level.
 *
 * PSH construction (Section 5.2 defers the details to the original PSH paper,
 * which is not available): parity unpinned by the paper beyond the size rules
 * and validity; the deterministic procedure below is this build's own.
 *   m = min{k : k^3 > n};  r = min{k : 6 k^3 >= n}, raised until gcd(r,m)=1;
 *   buckets g = lin_r(p mod r), processed by (count descending, g ascending),
 *   voxels inside a bucket in data order; for a bucket whose first voxel is q0,
 *   candidate t = 0,1,.. places q0 at slot unlin_m((s0 + t) mod m^3) with
 *   s0 = ((g * 2654435761) mod 2^32) mod m^3, i.e. offset = slot - h0(q0) mod m;
 *   the first candidate that sends every voxel of the bucket to a free slot is
 *   taken; if none exists the attempt fails and r grows to
 *   min{k > r : k^3 >= 2 r^3} (again raised to be coprime with m).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#define ORC_OK 0
#define ORC_EINVAL 1
#define ORC_ECAP 2      /* offset table capacity handed in is too small */
#define ORC_EBUILD 3
#define ORC_EUNSUPPORTED 5

/* ------------------------------------------------------------------------- */
/* Section 5.2: table sizes                                                  */
/* ------------------------------------------------------------------------- */

/* smallest m with m^3 > n  (strict: at least one redundant slot, as in the
 * 3x3 table that holds the 8 pixels of the worked example) */
int orc_mbar(int64_t n)
{
    int64_t m = 1;
    while (m * m * m <= n) m++;
    return (int)m;
}

static int gcd_int(int a, int b)
{
    while (b) { int t = a % b; a = b; b = t; }
    return a;
}

/* smallest r with r^3 >= sigma*n, sigma = 1/(2d) = 1/6, then made coprime to m */
int orc_rbar0(int64_t n, int mbar)
{
    int64_t r = 1;
    while (6 * r * r * r < n) r++;
    while (gcd_int((int)r, mbar) != 1) r++;
    return (int)r;
}

/* "increase r by cube-root of 2": smallest larger r whose capacity is doubled */
int orc_rbar_next(int rbar, int mbar)
{
    int64_t r0 = rbar, r = rbar + 1;
    while (r * r * r < 2 * r0 * r0 * r0) r++;
    while (gcd_int((int)r, mbar) != 1) r++;
    return (int)r;
}

/* ------------------------------------------------------------------------- */
/* Section 3.1 / 5.2: construction of one model's PSH                         */
/* ------------------------------------------------------------------------- */

typedef struct { int64_t g; int64_t count; } bucket_key;

static int cmp_bucket(const void *a, const void *b)
{
    const bucket_key *x = (const bucket_key *)a, *y = (const bucket_key *)b;
    if (x->count != y->count) return x->count > y->count ? -1 : 1;
    if (x->g != y->g) return x->g < y->g ? -1 : 1;
    return 0;
}

/* One attempt with a fixed r.  Returns 1 on success, 0 on failure. */
static int psh_attempt(const int32_t *p, int64_t n, int m, int r,
                       int32_t *H, uint16_t *T, uint8_t *Phi)
{
    int64_t m3 = (int64_t)m * m * m, r3 = (int64_t)r * r * r;
    int64_t i, j;
    int ok = 1;

    for (i = 0; i < m3; i++) { H[i] = -1; T[3*i] = T[3*i+1] = T[3*i+2] = 0xFFFF; }
    memset(Phi, 0, (size_t)(3 * r3));

    /* bucket membership: counting sort of the data indices by bucket, which
     * keeps data order inside a bucket */
    int64_t *count = (int64_t *)calloc((size_t)r3 + 1, sizeof(int64_t));
    int64_t *start = (int64_t *)calloc((size_t)r3 + 1, sizeof(int64_t));
    int64_t *member = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    int64_t *gof = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    for (i = 0; i < n; i++) {
        int64_t g = (((int64_t)(p[3*i] % r)) * r + p[3*i+1] % r) * r + p[3*i+2] % r;
        gof[i] = g;
        count[g]++;
    }
    for (i = 0; i < r3; i++) start[i+1] = start[i] + count[i];
    {
        int64_t *fill = (int64_t *)calloc((size_t)r3 + 1, sizeof(int64_t));
        for (i = 0; i < n; i++) { int64_t g = gof[i]; member[start[g] + fill[g]++] = i; }
        free(fill);
    }

    int64_t nb = 0;
    for (i = 0; i < r3; i++) if (count[i] > 0) nb++;
    bucket_key *order = (bucket_key *)malloc((size_t)(nb > 0 ? nb : 1) * sizeof(bucket_key));
    nb = 0;
    for (i = 0; i < r3; i++) if (count[i] > 0) { order[nb].g = i; order[nb].count = count[i]; nb++; }
    qsort(order, (size_t)nb, sizeof(bucket_key), cmp_bucket);

    int64_t *slot_of = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));

    for (j = 0; j < nb && ok; j++) {
        int64_t g = order[j].g, cnt = order[j].count;
        const int64_t *mem = member + start[g];
        const int32_t *q0 = p + 3 * mem[0];
        int a0 = q0[0] % m, a1 = q0[1] % m, a2 = q0[2] % m;
        int64_t s0 = (int64_t)(((uint64_t)g * 2654435761ULL) & 0xFFFFFFFFULL) % m3;
        int found = 0;
        int64_t t;
        for (t = 0; t < m3 && !found; t++) {
            int64_t e = (s0 + t) % m3;
            int sx = (int)(e / ((int64_t)m * m)), sy = (int)((e / m) % m), sz = (int)(e % m);
            int ox = (sx - a0 + m) % m, oy = (sy - a1 + m) % m, oz = (sz - a2 + m) % m;
            int64_t k, placed = 0;
            int good = 1;
            for (k = 0; k < cnt; k++) {
                const int32_t *q = p + 3 * mem[k];
                int64_t s = (((int64_t)((q[0] % m + ox) % m)) * m + (q[1] % m + oy) % m) * m
                            + (q[2] % m + oz) % m;
                if (H[s] != -1) { good = 0; break; }
                H[s] = (int32_t)mem[k];          /* provisional: also exposes */
                slot_of[k] = s;                  /* clashes inside the bucket */
                placed++;
            }
            if (!good) {
                for (k = 0; k < placed; k++) H[slot_of[k]] = -1;
                continue;
            }
            found = 1;
            Phi[3*g] = (uint8_t)ox; Phi[3*g+1] = (uint8_t)oy; Phi[3*g+2] = (uint8_t)oz;
            for (k = 0; k < cnt; k++) {
                const int32_t *q = p + 3 * mem[k];
                int64_t s = slot_of[k];
                T[3*s] = (uint16_t)q[0]; T[3*s+1] = (uint16_t)q[1]; T[3*s+2] = (uint16_t)q[2];
            }
        }
        if (!found) ok = 0;
    }

    free(slot_of); free(order); free(gof); free(member); free(start); free(count);
    return ok;
}

/*
 * Build the PSH of one model.  coords: [n][3] with 0 <= x,y,z < ubar, no
 * duplicates; data index of a voxel = its position in coords.
 * H [m^3], T [m^3][3] must be sized from orc_mbar(n); Phi has room for phi_cap
 * cells (3 bytes each).  On ORC_OK *rbar_out holds the offset-table side and
 * *attempts_out the number of r values tried.  ORC_ECAP: grow Phi and call again.
 */
int orc_psh_build(const int32_t *coords, int64_t n, int ubar,
                  int32_t *H, uint16_t *T, uint8_t *Phi, int64_t phi_cap,
                  int *rbar_out, int *attempts_out)
{
    int64_t i;
    if (n <= 0 || ubar <= 0 || ubar > 32768) return ORC_EINVAL;
    if (n >= ((int64_t)1 << 31)) return ORC_EINVAL;
    for (i = 0; i < 3 * n; i++) if (coords[i] < 0 || coords[i] >= ubar) return ORC_EINVAL;
    int m = orc_mbar(n);
    if (m > 256) return ORC_EUNSUPPORTED;      /* an 8-bit offset must reach every slot */
    int r = orc_rbar0(n, m);
    int attempts = 0;
    for (;;) {
        if ((int64_t)r * r * r > phi_cap) { *rbar_out = r; return ORC_ECAP; }
        attempts++;
        if (psh_attempt(coords, n, m, r, H, T, Phi)) break;
        if (r >= ubar) return ORC_EBUILD;       /* singleton buckets cannot fail */
        r = orc_rbar_next(r, m);
    }
    *rbar_out = r;
    if (attempts_out) *attempts_out = attempts;
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Section 3.2: one level of the mini-batch super-PSH                          */
/* ------------------------------------------------------------------------- */

typedef struct {
    int32_t b;            /* models in the batch                              */
    int32_t ubar;         /* grid resolution of this level                    */
    const int32_t *mbar;  /* [b]   hash-table side per model                  */
    const int32_t *rbar;  /* [b]   offset-table side per model                */
    const int64_t *M;     /* [b+1] exclusive prefix of m^3  (M*[0] = 0)       */
    const int64_t *R;     /* [b+1] exclusive prefix of r^3                    */
    const int64_t *N;     /* [b+1] exclusive prefix of n                      */
    const int32_t *H;     /* [M[b]]     H*: local data index or -1            */
    const uint16_t *T;    /* [M[b]][3]  T*: position tag                      */
    const uint8_t *Phi;   /* [R[b]][3]  Phi*: offsets                         */
    const int32_t *V;     /* [M[b]]     V*: model index of the slot           */
} orc_level;

/* prefix arrays M*, R*, N* (leading 0, b+1 entries) and V* */
void orc_super_prefix(int32_t b, const int32_t *mbar, const int32_t *rbar, const int64_t *n,
                      int64_t *M, int64_t *R, int64_t *N)
{
    int32_t i;
    M[0] = R[0] = N[0] = 0;
    for (i = 0; i < b; i++) {
        M[i+1] = M[i] + (int64_t)mbar[i] * mbar[i] * mbar[i];
        R[i+1] = R[i] + (int64_t)rbar[i] * rbar[i] * rbar[i];
        N[i+1] = N[i] + n[i];
    }
}

void orc_fill_V(int32_t b, const int64_t *M, int32_t *V)
{
    int32_t v; int64_t s;
    for (v = 0; v < b; v++) for (s = M[v]; s < M[v+1]; s++) V[s] = v;
}

/* Eq.1 with Eq.4 and Eq.5: super hash index of position p in model v.
 * Caller guarantees 0 <= p < ubar on every axis. */
static int64_t super_hash_index(const orc_level *L, int v, int x, int y, int z)
{
    int m = L->mbar[v], r = L->rbar[v];
    int64_t iphi = L->R[v] + (((int64_t)(x % r)) * r + y % r) * r + z % r;   /* Eq.4 */
    int hx = (x % m + L->Phi[3*iphi]) % m;                                  /* Eq.1 */
    int hy = (y % m + L->Phi[3*iphi+1]) % m;
    int hz = (z % m + L->Phi[3*iphi+2]) % m;
    return L->M[v] + (((int64_t)hx) * m + hy) * m + hz;                     /* Eq.5 */
}

/* Full query protocol of Section 3.1 on the super tables: global data index
 * (Eq.6) of voxel p of model v, or -1 when p is off the model or off the grid. */
int64_t orc_lookup(const orc_level *L, int v, int x, int y, int z)
{
    if (x < 0 || y < 0 || z < 0 || x >= L->ubar || y >= L->ubar || z >= L->ubar) return -1;
    int64_t iH = super_hash_index(L, v, x, y, z);
    if (L->H[iH] == -1) return -1;
    if (L->T[3*iH] != x || L->T[3*iH+1] != y || L->T[3*iH+2] != z) return -1;
    return L->N[v] + L->H[iH];                                              /* Eq.6 */
}

/* raw slot (for the worked-example pin): the super hash index itself */
int64_t orc_hash_slot(const orc_level *L, int v, int x, int y, int z)
{
    return super_hash_index(L, v, x, y, z);
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1 / 2 traversal                                                  */
/* ------------------------------------------------------------------------- */

/* lower corner of the receptive field of output voxel p (one axis) */
static int field_lo(int p, int F, int Ss, int Sp)
{
    if (Ss == 1) return p - (F - 1) / 2;
    return p * Ss - Sp;
}

/*
 * hash2col (Algorithm 1).  Din: c x N_i (row-major), out Dt: (c*F^3) x N_o.
 * Li / Lo are the input / output levels (the same level when Ss == 1).
 * Every entry of Dt that belongs to an occupied output voxel is written
 * (value or 0); there are no other columns.
 */
void orc_hash2col(const orc_level *Li, const orc_level *Lo, int c, const double *Din,
                  int F, int Ss, int Sp, double *Dt)
{
    int64_t Mo = Lo->M[Lo->b], Ni = Li->N[Li->b], No = Lo->N[Lo->b];
    int F3 = F * F * F;
    int64_t ithrd;
    #pragma omp parallel for schedule(static)
    for (ithrd = 0; ithrd < (int64_t)c * Mo; ithrd++) {
        int ic = (int)(ithrd / Mo);
        int64_t iHo = ithrd - (int64_t)ic * Mo;
        if (Lo->H[iHo] == -1) continue;
        int v = Lo->V[iHo];
        int64_t col = Lo->N[v] + Lo->H[iHo];
        int px = Lo->T[3*iHo], py = Lo->T[3*iHo+1], pz = Lo->T[3*iHo+2];
        int lx = field_lo(px, F, Ss, Sp), ly = field_lo(py, F, Ss, Sp), lz = field_lo(pz, F, Ss, Sp);
        int row = 0, fx, fy, fz;
        for (fx = 0; fx < F; fx++) for (fy = 0; fy < F; fy++) for (fz = 0; fz < F; fz++) {
            int64_t iD = orc_lookup(Li, v, lx + fx, ly + fy, lz + fz);
            double val = 0.0;
            if (iD >= 0) val = Din[(int64_t)ic * Ni + iD];
            Dt[((int64_t)ic * F3 + row) * No + col] = val;
            row++;
        }
    }
}

/*
 * col2hash (Algorithm 2).  dDt: (c*F^3) x N_o, out dDin: c x N_i, zeroed first.
 * Channels are independent; within a channel the sum runs in slot order.
 */
void orc_col2hash(const orc_level *Li, const orc_level *Lo, int c, const double *dDt,
                  int F, int Ss, int Sp, double *dDin)
{
    int64_t Mo = Lo->M[Lo->b], Ni = Li->N[Li->b], No = Lo->N[Lo->b];
    int F3 = F * F * F;
    int ic;
    memset(dDin, 0, (size_t)c * (size_t)Ni * sizeof(double));
    #pragma omp parallel for schedule(static)
    for (ic = 0; ic < c; ic++) {
        int64_t iHo;
        for (iHo = 0; iHo < Mo; iHo++) {
            if (Lo->H[iHo] == -1) continue;
            int v = Lo->V[iHo];
            int64_t col = Lo->N[v] + Lo->H[iHo];
            int px = Lo->T[3*iHo], py = Lo->T[3*iHo+1], pz = Lo->T[3*iHo+2];
            int lx = field_lo(px, F, Ss, Sp), ly = field_lo(py, F, Ss, Sp), lz = field_lo(pz, F, Ss, Sp);
            int row = 0, fx, fy, fz;
            for (fx = 0; fx < F; fx++) for (fy = 0; fy < F; fy++) for (fz = 0; fz < F; fz++) {
                int64_t iD = orc_lookup(Li, v, lx + fx, ly + fy, lz + fz);
                if (iD >= 0)
                    dDin[(int64_t)ic * Ni + iD] += dDt[((int64_t)ic * F3 + row) * No + col];
                row++;
            }
        }
    }
}

/*
 * The traversal's index side alone ("pre-stored neighbour information",
 * Section 5.3): for each occupied output voxel (column col) and field position
 * row, the global input data index or -1.  out: N_o x F^3 (int32).
 */
void orc_field_indices(const orc_level *Li, const orc_level *Lo, int F, int Ss, int Sp,
                       int32_t *out)
{
    int64_t Mo = Lo->M[Lo->b];
    int F3 = F * F * F;
    int64_t iHo;
    #pragma omp parallel for schedule(static)
    for (iHo = 0; iHo < Mo; iHo++) {
        if (Lo->H[iHo] == -1) continue;
        int v = Lo->V[iHo];
        int64_t col = Lo->N[v] + Lo->H[iHo];
        int px = Lo->T[3*iHo], py = Lo->T[3*iHo+1], pz = Lo->T[3*iHo+2];
        int lx = field_lo(px, F, Ss, Sp), ly = field_lo(py, F, Ss, Sp), lz = field_lo(pz, F, Ss, Sp);
        int row = 0, fx, fy, fz;
        for (fx = 0; fx < F; fx++) for (fy = 0; fy < F; fy++) for (fz = 0; fz < F; fz++) {
            out[col * F3 + row] = (int32_t)orc_lookup(Li, v, lx + fx, ly + fy, lz + fz);
            row++;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* plain matrix product, row-major, double:  C[m x n] = op(A) * op(B)         */
/*   ta == 0: A is m x k;  ta != 0: A is stored k x m and used transposed     */
/*   tb == 0: B is k x n;  tb != 0: B is stored n x k and used transposed     */
/* ------------------------------------------------------------------------- */
void orc_matmul(const double *A, const double *B, double *C,
                int64_t m, int64_t k, int64_t n, int ta, int tb)
{
    int64_t i;
    #pragma omp parallel for schedule(static)
    for (i = 0; i < m; i++) {
        int64_t j, l;
        double *Ci = C + i * n;
        for (j = 0; j < n; j++) Ci[j] = 0.0;
        if (!tb) {
            for (l = 0; l < k; l++) {
                double a = ta ? A[l * m + i] : A[i * k + l];
                const double *Bl = B + l * n;
                for (j = 0; j < n; j++) Ci[j] += a * Bl[j];
            }
        } else {
            for (j = 0; j < n; j++) {
                const double *Bj = B + j * k;
                double s = 0.0;
                for (l = 0; l < k; l++) s += (ta ? A[l * m + i] : A[i * k + l]) * Bj[l];
                Ci[j] = s;
            }
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Convolution and its gradients (Eq.3, Eq.7, Eq.8); 3x3x3 stride 1 is F=3,   */
/* Ss=1; the general F / stride form is kept because the algorithms state it. */
/* Dt / dDt are scratch of (c_in*F^3) x N_o doubles supplied by the caller.   */
/* ------------------------------------------------------------------------- */

/* D_o = W * D~_i          W: c_out x (c_in F^3),  D_o: c_out x N_o */
void orc_conv_fwd(const orc_level *Li, const orc_level *Lo, int c_in, int c_out,
                  const double *Din, const double *W, int F, int Ss, int Sp,
                  double *Dt, double *Dout)
{
    int64_t No = Lo->N[Lo->b];
    orc_hash2col(Li, Lo, c_in, Din, F, Ss, Sp, Dt);
    orc_matmul(W, Dt, Dout, c_out, (int64_t)c_in * F * F * F, No, 0, 0);
}

/* dW = dD_o * D~_i^T      dW: c_out x (c_in F^3) */
void orc_conv_bwd_weight(const orc_level *Li, const orc_level *Lo, int c_in, int c_out,
                         const double *Din, const double *dDout, int F, int Ss, int Sp,
                         double *Dt, double *dW)
{
    int64_t No = Lo->N[Lo->b];
    orc_hash2col(Li, Lo, c_in, Din, F, Ss, Sp, Dt);
    orc_matmul(dDout, Dt, dW, c_out, No, (int64_t)c_in * F * F * F, 0, 1);
}

/* dD~_i = W^T * dD_o ,  then col2hash      dDin: c_in x N_i */
void orc_conv_bwd_data(const orc_level *Li, const orc_level *Lo, int c_in, int c_out,
                       const double *dDout, const double *W, int F, int Ss, int Sp,
                       double *dDt, double *dDin)
{
    int64_t No = Lo->N[Lo->b];
    orc_matmul(W, dDout, dDt, (int64_t)c_in * F * F * F, c_out, No, 1, 0);
    orc_col2hash(Li, Lo, c_in, dDt, F, Ss, Sp, dDin);
}

/* ------------------------------------------------------------------------- */
/* Eq.2 evaluated directly at chosen voxels (no column matrix): used to check  */
/* sampled outputs at sizes where D~ would not fit.  3x3x3, stride 1.          */
/* ------------------------------------------------------------------------- */

/* Y[s][o] for the voxels whose global data indices are idx[0..ns);
 * coords: N x 3 positions of the level's data rows, model: their model index. */
void orc_conv_fwd_at(const orc_level *L, int c_in, int c_out, const double *Din,
                     const double *W, const int32_t *coords, const int32_t *model,
                     const int64_t *idx, int64_t ns, double *out)
{
    int64_t N = L->N[L->b], s;
    #pragma omp parallel for schedule(dynamic, 16)
    for (s = 0; s < ns; s++) {
        int64_t i = idx[s];
        int v = model[i], k = 0, dx, dy, dz, o, ci;
        for (o = 0; o < c_out; o++) out[s * c_out + o] = 0.0;
        for (dx = -1; dx <= 1; dx++) for (dy = -1; dy <= 1; dy++) for (dz = -1; dz <= 1; dz++, k++) {
            int64_t j = orc_lookup(L, v, coords[3*i] + dx, coords[3*i+1] + dy, coords[3*i+2] + dz);
            if (j < 0) continue;
            for (o = 0; o < c_out; o++) {
                double acc = 0.0;
                for (ci = 0; ci < c_in; ci++)
                    acc += W[(int64_t)o * c_in * 27 + ci * 27 + k] * Din[(int64_t)ci * N + j];
                out[s * c_out + o] += acc;
            }
        }
    }
}

/* dX[s][ci] = sum_k sum_o W[o, ci*27+k] * dY[o, q - delta_k]  at voxels idx[] */
void orc_conv_bwd_data_at(const orc_level *L, int c_in, int c_out, const double *dDout,
                          const double *W, const int32_t *coords, const int32_t *model,
                          const int64_t *idx, int64_t ns, double *out)
{
    int64_t N = L->N[L->b], s;
    #pragma omp parallel for schedule(dynamic, 16)
    for (s = 0; s < ns; s++) {
        int64_t i = idx[s];
        int v = model[i], k = 0, dx, dy, dz, o, ci;
        for (ci = 0; ci < c_in; ci++) out[s * c_in + ci] = 0.0;
        for (dx = -1; dx <= 1; dx++) for (dy = -1; dy <= 1; dy++) for (dz = -1; dz <= 1; dz++, k++) {
            /* output voxel p whose k-th field position is q:  p = q - delta_k */
            int64_t j = orc_lookup(L, v, coords[3*i] - dx, coords[3*i+1] - dy, coords[3*i+2] - dz);
            if (j < 0) continue;
            for (ci = 0; ci < c_in; ci++) {
                double acc = 0.0;
                for (o = 0; o < c_out; o++)
                    acc += W[(int64_t)o * c_in * 27 + ci * 27 + k] * dDout[(int64_t)o * N + j];
                out[s * c_in + ci] += acc;
            }
        }
    }
}

/* dW[o, ci*27+k] = sum_p dY[o,p] * X[ci, p + delta_k]  for chosen (o, ci, k) triples */
void orc_conv_bwd_weight_at(const orc_level *L, int c_in, int c_out, const double *Din,
                            const double *dDout, const int32_t *coords, const int32_t *model,
                            const int32_t *triples, int64_t nt, double *out)
{
    int64_t N = L->N[L->b], t;
    (void)c_in; (void)c_out;
    #pragma omp parallel for schedule(dynamic, 1)
    for (t = 0; t < nt; t++) {
        int o = triples[3*t], ci = triples[3*t+1], k = triples[3*t+2];
        int dx = k / 9 - 1, dy = (k / 3) % 3 - 1, dz = k % 3 - 1;
        double acc = 0.0;
        int64_t i;
        for (i = 0; i < N; i++) {
            int64_t j = orc_lookup(L, model[i], coords[3*i] + dx, coords[3*i+1] + dy, coords[3*i+2] + dz);
            if (j >= 0) acc += dDout[(int64_t)o * N + i] * Din[(int64_t)ci * N + j];
        }
        out[t] = acc;
    }
}

/* ------------------------------------------------------------------------- */
/* Max-pooling with switches, and its backward (= max-unpooling)               */
/* ------------------------------------------------------------------------- */

/*
 * Pooling as the strided traversal of Algorithm 1 (stride Ss, field F, pad Sp):
 * Li is the fine level, Lo the coarse one.  Dout: c x N_o, sw: c x N_o (int32,
 * global fine data index of the maximum).  Every occupied coarse voxel is
 * assumed to have at least one occupied fine voxel in its field (true for the
 * hierarchy: a coarse voxel exists iff one of its children does); if not, the
 * output is 0 and the switch -1.
 */
void orc_pool_max_fwd(const orc_level *Li, const orc_level *Lo, int c, const double *Din,
                      int F, int Ss, int Sp, double *Dout, int32_t *sw)
{
    int64_t Mo = Lo->M[Lo->b], Ni = Li->N[Li->b], No = Lo->N[Lo->b];
    int64_t ithrd;
    #pragma omp parallel for schedule(static)
    for (ithrd = 0; ithrd < (int64_t)c * Mo; ithrd++) {
        int ic = (int)(ithrd / Mo);
        int64_t iHo = ithrd - (int64_t)ic * Mo;
        if (Lo->H[iHo] == -1) continue;
        int v = Lo->V[iHo];
        int64_t col = Lo->N[v] + Lo->H[iHo];
        int px = Lo->T[3*iHo], py = Lo->T[3*iHo+1], pz = Lo->T[3*iHo+2];
        int lx = field_lo(px, F, Ss, Sp), ly = field_lo(py, F, Ss, Sp), lz = field_lo(pz, F, Ss, Sp);
        int fx, fy, fz;
        double best = 0.0;
        int64_t arg = -1;
        for (fx = 0; fx < F; fx++) for (fy = 0; fy < F; fy++) for (fz = 0; fz < F; fz++) {
            int64_t iD = orc_lookup(Li, v, lx + fx, ly + fy, lz + fz);
            if (iD < 0) continue;
            double val = Din[(int64_t)ic * Ni + iD];
            if (arg < 0 || val > best) { best = val; arg = iD; }
        }
        Dout[(int64_t)ic * No + col] = best;
        sw[(int64_t)ic * No + col] = (int32_t)arg;
    }
}

/* dDin (c x N_i) = 0 everywhere except at the switches, which receive dDout */
void orc_pool_max_bwd(int c, int64_t Ni, int64_t No, const double *dDout, const int32_t *sw,
                      double *dDin)
{
    int ic; int64_t j;
    memset(dDin, 0, (size_t)c * (size_t)Ni * sizeof(double));
    for (ic = 0; ic < c; ic++)
        for (j = 0; j < No; j++) {
            int32_t a = sw[(int64_t)ic * No + j];
            if (a >= 0) dDin[(int64_t)ic * Ni + a] = dDout[(int64_t)ic * No + j];
        }
}

/* ------------------------------------------------------------------------- */
/* Transposed convolution and max-unpooling (Section 4, last paragraphs)       */
/* ------------------------------------------------------------------------- */

/*
 * Transposed convolution: D~_o = W^T * D_i, then col2hash -- "exactly how the error
 * back-propagation is handled".  W: c_i x (c_o * F^3) is the weight matrix of the forward
 * convolution c_o -> c_i that is being transposed; Din: c_i x N; Dout: c_o x N.
 * Dt is scratch of (c_o*F^3) x N doubles.
 */
void orc_deconv_fwd(const orc_level *L, int c_i, int c_o, const double *Din, const double *W,
                    int F, double *Dt, double *Dout)
{
    int64_t N = L->N[L->b];
    orc_matmul(W, Din, Dt, (int64_t)c_o * F * F * F, c_i, N, 1, 0);
    orc_col2hash(L, L, c_o, Dt, F, 1, 0, Dout);
}

/* Max-unpooling: the receptive field of every coarse voxel is zero except at the recorded
 * switch, which receives the coarse value.  (Same routing as orc_pool_max_bwd.)
 * Its backward reads the fine gradient back at the switches. */
void orc_unpool_max_bwd(int c, int64_t Nf, int64_t Nc, const double *dDfine, const int32_t *sw,
                        double *dDcoarse)
{
    int ic; int64_t j;
    for (ic = 0; ic < c; ic++)
        for (j = 0; j < Nc; j++) {
            int32_t a = sw[(int64_t)ic * Nc + j];
            dDcoarse[(int64_t)ic * Nc + j] = a >= 0 ? dDfine[(int64_t)ic * Nf + a] : 0.0;
        }
}

/* number of OpenMP threads the parallel loops above will use */
#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
/* number of threads the loops above use from now on (for timing the oracle at 1 thread) */
void orc_set_threads(int n) { if (n >= 1) omp_set_num_threads(n); }
#else
int orc_threads(void) { return 1; }
void orc_set_threads(int n) { (void)n; }
#endif
