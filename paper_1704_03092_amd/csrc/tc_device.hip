// Device side of libstrassen_tc (gfx950 / CDNA4 only).
//
//  planner kernels   scatter vectors and block scatter vectors of the matrix view (Sec. 2.3)
//  fused kernel      the general primitive of Sec. 3, eq. (straprim1), generalised to <= 4 signed blocks per
//                    operand and <= 4 signed destinations: gather blocks of A and B through the scatter
//                    vectors, add them in registers, stage the sums in LDS (Sec. 4.1 "packing"), multiply
//                    tiles on the FP64 matrix cores, add the tile to every destination block of C from
//                    registers (Sec. 4.2).  Level 0 is the same kernel with one term and one destination.
//  lincomb kernel    element-wise  dst_d = g_d * (sum_t c_t src_t) + f_d * dst_d  on matrix views; used for
//                    the dense operand sums of the Naive variant and to accumulate a dense product M into the
//                    blocks of C (AB and Naive variants), Sec. 4.1.
//
// Matrix-core instruction: v_mfma_f64_4x4x4_4b_f64.  One instruction multiplies four independent 4x4x4
// blocks; measured on MI355X it sustains twice the rate of v_mfma_f64_16x16x4_f64.  Register layout (lane l):
//   A operand: block (l/4)%4, row l%4, k = l/16        B operand: block (l/4)%4, column l%4, k = l/16
//   D result : block (l/4)%4, column l%4, row l/16
// A 16x16 output patch is covered by 4 instructions whose B operand has its four column blocks rotated by
// s = 0..3 positions: block slot b of instruction s multiplies row block b by column block (b + s) % 4.
#include <hip/hip_runtime.h>

#include "tc_internal.h"

namespace tc {

namespace {

constexpr int TM = 128;      // tile rows (free bundle I)
constexpr int TN = 128;      // tile columns (free bundle J)
constexpr int NTHREADS = 512;  // 8 waves: 2 along the rows x 4 along the columns, each owning 64 x 32 outputs
constexpr int GROUP_M = 8;   // tile rows per rasterisation group

// Contracted entries per pipeline step.  A gathered element needs more than 16 entries' worth of matrix-core
// work to arrive, so the step is made as deep as the registers allow: 32 for one or two terms per operand.
template <int NT>
struct Cfg {
    static constexpr int KT = (NT <= 2) ? 32 : 16;
    static constexpr int NE = TM * KT / NTHREADS;  // elements of each operand tile a thread gathers per k-step
    static constexpr int NQ = KT / 4;              // matrix-core instruction groups ("quarters") per k-step
};

// LDS tile layout: element (k, x) of a KT x 128 tile lives at k * PITCH + x.  Instruction group q of a k-step
// takes k = 16 * (q / 4) + 4 * (lane / 16) + q % 4, so one fragment load touches rows k and k + 4 in each half-wave;
// with PITCH = 132 those rows start 16 bank-pairs apart and the load is conflict-free, every fragment address is one
// per-lane base plus a compile-time offset, and the transposing store (lanes with consecutive k) sees 2-way
// conflicts at worst.
constexpr int PITCH = 132;

__device__ __forceinline__ const double* pick_src(int space, const double* user, const double* W, int64_t off) {
    return (space == 0 ? user : W) + off;
}

// Scatter vectors are reached through pointers stored in the product descriptors; telling the compiler that they
// point to global memory keeps their loads off the flat path (a pending flat load forces a full wait before the
// next LDS access).
typedef const __attribute__((address_space(1))) int64_t* gvec_t;
__device__ __forceinline__ gvec_t as_global(const int64_t* p) { return (gvec_t)p; }
typedef const __attribute__((address_space(1))) double* gdbl_t;

// Non-matrix VALU instructions do not overlap with v_mfma_f64_4x4x4 on this chip (measured: every integer or
// fp64 VALU instruction adds its full issue time), so the main loop is written to need as few of them as possible:
// the gather tables hold ready-made byte addresses (one 64-bit add per loaded element), the k-step loop is
// unrolled over the two LDS buffers so that every LDS address is a per-lane base plus a constant, and an
// operand with a single +1 term is stored as loaded.
template <int NT>
struct FusedSmem {
    static constexpr int KT = Cfg<NT>::KT;
    static constexpr int TILE = KT * PITCH;
    double a[2][TILE];
    double b[2][TILE];
    int64_t a_fix[NT][TM];      // per term: address of row x of the A blocks (base + 8 * rscat), kSentinel where padded
    int64_t b_fix[NT][TN];      // per term: address of column x of the B blocks (base + 8 * cscat)
    int64_t a_step[2][NT][KT];  // per term: 8 * cscat_A of the contracted entries of a k-step (two steps in flight)
    int64_t b_step[2][NT][KT];  // per term: 8 * rscat_B
    int64_t dump[2][NT][KT];    // where threads that own no table entry store theirs (keeps that store branch-free)
};

// Each thread gathers NE elements of the A tile and NE of the B tile per k-step, for every term.
//   MODE 0: lanes run along the 128 free entries (x); element e of a thread is (x = tid % 128, k = tid / 128 + 4e)
//   MODE 1: lanes run along the contracted entries (k); element e is (k = tid % KT, x = tid / KT + (512 / KT) e)
// The loads of a k-step are issued during the matrix-core work on the previous one and, after it, summed with
// their signs (the operand sum of Sec. 4.1) and stored into the other LDS buffer.
// CHECKED: entries of the zero padding (negative table sum) read the operand's element 0 and count as zero.
template <int MODE, int NT, bool CHECKED>
__device__ __forceinline__ void issue_loads(double (&ld)[NT][Cfg<NT>::NE], unsigned& padmask, const double* __restrict__ safe,
                                            const int64_t* __restrict__ fixed_tab /* [NT][128] */,
                                            const int64_t* __restrict__ step_tab /* [NT][KT] */, int nterms, int tid) {
    constexpr int KT = Cfg<NT>::KT, NE = Cfg<NT>::NE;
    padmask = 0;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (t > 0 && t >= nterms) {  // absent term: contributes zeros (its coefficient is zero as well)
#pragma unroll
            for (int e = 0; e < NE; ++e) ld[t][e] = 0.0;
        } else {
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                int64_t addr;
                if (MODE == 0)
                    addr = fixed_tab[t * 128 + (tid & 127)] + step_tab[t * KT + (tid >> 7) + 4 * e];
                else
                    addr = step_tab[t * KT + (tid % KT)] + fixed_tab[t * 128 + (tid / KT) + (NTHREADS / KT) * e];
                if (CHECKED) {
                    padmask |= (addr < 0 ? 1u : 0u) << (t * NE + e);
                    ld[t][e] = *(gdbl_t)(addr < 0 ? (int64_t)safe : addr);
                } else {
                    ld[t][e] = *(gdbl_t)addr;
                }
            }
        }
    }
}

template <int MODE, int NT, bool CHECKED>
__device__ __forceinline__ void stage_sums(double* __restrict__ dst, const double (&ld)[NT][Cfg<NT>::NE], unsigned padmask,
                                           const double* __restrict__ coef, bool plain) {
    constexpr int KT = Cfg<NT>::KT, NE = Cfg<NT>::NE;
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        double v;
        if (NT == 1 && !CHECKED) {
            v = plain ? ld[0][e] : coef[0] * ld[0][e];
        } else {
            v = 0.0;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const double x = (CHECKED && ((padmask >> (t * NE + e)) & 1u)) ? 0.0 : ld[t][e];
                v = (t == 0) ? coef[0] * x : __builtin_fma(coef[t], x, v);
            }
        }
        dst[(MODE == 0) ? 4 * e * PITCH : (NTHREADS / KT) * e] = v;
    }
}

__device__ __forceinline__ int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }

template <int AMODE, int BMODE, int NT>
struct FusedState {
    static constexpr int KT = Cfg<NT>::KT, NE = Cfg<NT>::NE, NQ = Cfg<NT>::NQ, TILE = KT * PITCH;
    FusedSmem<NT>* S;
    const Product* P;
    int tid, nA, nB, nk, kfull;
    bool plainA, plainB;       // single term with coefficient +1: staged as loaded
    bool early;                // this wave issues its gather before the matrix-core work of a k-step, its partner on
                               // the same SIMD a quarter of the way in: one of the two always has MFMAs to issue
    const double *safeA, *safeB;
    // scatter entries of later k-steps
    gvec_t ent_ptr;
    int ent_limit;             // k entries that exist for this thread's term, counted from its own k
    int64_t* ent_dst;
    // per-lane LDS bases
    const double* fa;
    const double* fb[4];
    double* sa;                // where this thread stages its A elements (buffer 0)
    double* sb;
    double acc[4][2][4];
    double la[NT][NE], lb[NT][NE];
    unsigned pa, pb;
    bool issued_fast;          // the loads in flight were issued without padding checks

    // gather of k-step `target` (table slot SLOT = target % 2)
    template <int SLOT>
    __device__ __forceinline__ void issue(int target) {
        if (target < nk) {
            issued_fast = target < kfull;  // no padding anywhere in that k-step
            if (issued_fast) {
                issue_loads<AMODE, NT, false>(la, pa, safeA, &S->a_fix[0][0], &S->a_step[SLOT][0][0], nA, tid);
                issue_loads<BMODE, NT, false>(lb, pb, safeB, &S->b_fix[0][0], &S->b_step[SLOT][0][0], nB, tid);
            } else {
                issue_loads<AMODE, NT, true>(la, pa, safeA, &S->a_fix[0][0], &S->a_step[SLOT][0][0], nA, tid);
                issue_loads<BMODE, NT, true>(lb, pb, safeB, &S->b_fix[0][0], &S->b_step[SLOT][0][0], nB, tid);
            }
        }
    }

    // operand sums of the loads in flight into LDS buffer BUF
    template <int BUF>
    __device__ __forceinline__ void stage() {
        if (issued_fast) {
            stage_sums<AMODE, NT, false>(sa + BUF * TILE, la, 0, P->A.coef, plainA);
            stage_sums<BMODE, NT, false>(sb + BUF * TILE, lb, 0, P->B.coef, plainB);
        } else {
            stage_sums<AMODE, NT, true>(sa + BUF * TILE, la, pa, P->A.coef, false);
            stage_sums<BMODE, NT, true>(sb + BUF * TILE, lb, pb, P->B.coef, false);
        }
    }

    template <int CUR, int Q>
    __device__ __forceinline__ void read_frags(double (&af)[4], double (&bf)[8]) {
        constexpr int ROW = 16 * (Q / 4) + (Q % 4);
#pragma unroll
        for (int x = 0; x < 4; ++x) af[x] = fa[CUR * TILE + ROW * PITCH + x * 16];
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int s = 0; s < 4; ++s) bf[y * 4 + s] = fb[s][CUR * TILE + ROW * PITCH + y * 16];
    }

    __device__ __forceinline__ void multiply(const double (&af)[4], const double (&bf)[8]) {
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    acc[x][y][s] = __builtin_amdgcn_mfma_f64_4x4x4f64(af[x], bf[y * 4 + s], acc[x][y][s], 0, 0, 0);
    }

    // instruction groups Q .. NQ-1 of the k-step in LDS buffer CUR; the fragments of group Q are in af/bf[Q % 2] and
    // those of group Q + 1 are read while group Q multiplies
    template <int CUR, int Q, int SLOT>
    __device__ __forceinline__ void groups(double (&af)[2][4], double (&bf)[2][8], int step) {
        if constexpr (Q < NQ) {
            if constexpr (Q + 1 < NQ) read_frags<CUR, Q + 1>(af[(Q + 1) & 1], bf[(Q + 1) & 1]);
            multiply(af[Q & 1], bf[Q & 1]);
            if constexpr (Q + 1 == NQ / 4) {
                if (!early) issue<SLOT>(step + 1);
            }
            groups<CUR, Q + 1, SLOT>(af, bf, step);
        }
    }

    // One k-step: gather k-step step + 1, multiply the tiles of this step (LDS buffer CUR), stage k-step step + 1.
    template <int CUR>
    __device__ __forceinline__ void step_body(int step) {
        constexpr int NXT = CUR ^ 1;
        if (early) issue<NXT>(step + 1);
        // table entry of k-step step + 2; unconditional load: ent_ptr always points at readable memory
        const int kn = (step + 2) * KT;
        const bool have = kn < ent_limit;
        const int64_t raw_entry = ent_ptr[have ? kn : 0];

        double af[2][4], bf[2][8];
        read_frags<CUR, 0>(af[0], bf[0]);
        groups<CUR, 0, NXT>(af, bf, step);

        if (step + 1 < nk) stage<NXT>();
        ent_dst[CUR * NT * KT] = have ? raw_entry * 8 : kSentinel;  // every thread stores: no branch around the wait
        __syncthreads();
    }
};

template <int AMODE, int BMODE, int NT>
__global__ __launch_bounds__(NTHREADS, 2) void fused_kernel(const Product* __restrict__ prods, int first, int tiles_m, int tiles_n,
                                                            const double* __restrict__ Au, const double* __restrict__ Bu,
                                                            double* __restrict__ Cu, double* __restrict__ W, double alpha, double beta) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    FusedSmem<NT>& S = *reinterpret_cast<FusedSmem<NT>*>(smem_raw);
    const int tid = threadIdx.x;
    typedef FusedState<AMODE, BMODE, NT> State;
    constexpr int KT = State::KT;

    // ---- which tile: spread consecutive logical ids over one XCD (block b runs on XCD b % 8), then walk
    //      GROUP_M tile rows at a time so that co-resident workgroups share A and B panels in that XCD's L2 ----
    const int total = gridDim.x, bid = blockIdx.x;
    const int q8 = total >> 3, r8 = total & 7, xcd = bid & 7;
    const int lid = xcd * q8 + (xcd < r8 ? xcd : r8) + (bid >> 3);
    const int per_prod = tiles_m * tiles_n;
    const int pidx = lid / per_prod;
    int rem = lid - pidx * per_prod;
    const int gsz = GROUP_M * tiles_n;
    const int grp = rem / gsz;
    const int gm0 = grp * GROUP_M;
    const int gh = (tiles_m - gm0) < GROUP_M ? (tiles_m - gm0) : GROUP_M;
    rem -= grp * gsz;
    const int tm = gm0 + rem % gh, tn = rem / gh;
    const Product& P = prods[first + pidx];
    const int64_t i0 = (int64_t)tm * TM, j0 = (int64_t)tn * TN;
    const int nA = P.A.nterms, nB = P.B.nterms;

    State st;
    st.S = &S;
    st.P = &P;
    st.tid = tid;
    st.nA = nA;
    st.nB = nB;
    st.nk = (int)((P.kb + KT - 1) / KT);
    st.plainA = nA == 1 && P.A.coef[0] == 1.0;
    st.plainB = nB == 1 && P.B.coef[0] == 1.0;
    const double* Abase = pick_src(P.A.space, Au, W, P.A.base_off);
    const double* Bbase = pick_src(P.B.space, Bu, W, P.B.base_off);
    st.safeA = Abase;
    st.safeB = Bbase;
    st.pa = st.pb = 0;
    st.issued_fast = false;

    // ---- tile-fixed gather tables; how much of the tile and of the k range is free of zero padding ----
    int64_t klimit = P.kb;       // k entries that are real in every term of both operands
    bool tile_full = true;       // every row and column of the tile is real in every term
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (t < nA) {
            klimit = min64(klimit, P.A.cs_len - P.A.coff[t]);
            tile_full = tile_full && (i0 + TM <= min64(P.mb, P.A.rs_len - P.A.roff[t]));
        }
        if (t < nB) {
            klimit = min64(klimit, P.B.rs_len - P.B.roff[t]);
            tile_full = tile_full && (j0 + TN <= min64(P.nb, P.B.cs_len - P.B.coff[t]));
        }
    }
    st.kfull = tile_full ? (int)(klimit / KT) : 0;  // k-steps [0, kfull) need no checks
    for (int e = tid; e < NT * TM; e += NTHREADS) {
        const int t = e / TM, x = e % TM;
        const int64_t gi = i0 + x;
        int64_t val = kSentinel;
        if (t < nA && gi < P.mb && P.A.roff[t] + gi < P.A.rs_len) val = (int64_t)Abase + 8 * as_global(P.A.rs)[P.A.roff[t] + gi];
        S.a_fix[t][x] = val;
        const int64_t gj = j0 + x;
        val = kSentinel;
        if (t < nB && gj < P.nb && P.B.coff[t] + gj < P.B.cs_len) val = (int64_t)Bbase + 8 * as_global(P.B.cs)[P.B.coff[t] + gj];
        S.b_fix[t][x] = val;
    }
    // Threads 0..KT*NT-1 fetch the column scatter entries of A for a k-step (one per term and k), threads
    // 256..256+KT*NT-1 the row scatter entries of B, two k-steps ahead of the tile that uses them.
    st.ent_ptr = as_global(reinterpret_cast<const int64_t*>(&P));  // dummy target for threads without an entry
    st.ent_limit = 0;
    st.ent_dst = &S.dump[0][0][0];
    {
        const bool isB = tid >= 256;
        const int q = tid & 255, t = q / KT, kl = q % KT;
        if (t < NT) {
            const Operand& op = isB ? P.B : P.A;
            st.ent_dst = isB ? &S.b_step[0][t][kl] : &S.a_step[0][t][kl];
            if (t < op.nterms) {
                const int64_t off0 = isB ? op.roff[t] : op.coff[t];
                st.ent_ptr = as_global(isB ? op.rs : op.cs) + off0 + kl;
                st.ent_limit = (int)(min64(P.kb, (isB ? op.rs_len : op.cs_len) - off0) - kl);
            }
        }
    }
    st.ent_dst[0] = (0 < st.ent_limit) ? 8 * st.ent_ptr[0] : kSentinel;
    st.ent_dst[NT * KT] = (KT < st.ent_limit) ? 8 * st.ent_ptr[KT] : kSentinel;
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int l16 = lane & 15, lk = lane >> 4;
    st.early = wm == 0;
    // per-lane bases; everything else in an LDS address is a compile-time offset
    st.fa = &S.a[0][0] + 4 * lk * PITCH + wm * 64 + l16;
#pragma unroll
    for (int s = 0; s < 4; ++s) st.fb[s] = &S.b[0][0] + 4 * lk * PITCH + wn * 32 + ((l16 + 4 * s) & 15);
    st.sa = &S.a[0][0] + ((AMODE == 0) ? (tid >> 7) * PITCH + (tid & 127) : (tid % KT) * PITCH + (tid / KT));
    st.sb = &S.b[0][0] + ((BMODE == 0) ? (tid >> 7) * PITCH + (tid & 127) : (tid % KT) * PITCH + (tid / KT));

    // ---- prologue: k-step 0 into LDS buffer 0 ----
    st.template issue<0>(0);
    st.template stage<0>();
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int s = 0; s < 4; ++s) st.acc[x][y][s] = 0.0;
    __syncthreads();

    for (int step = 0; step < st.nk; step += 2) {
        st.template step_body<0>(step);
        if (step + 1 < st.nk) st.template step_body<1>(step + 1);
    }

    // ---- epilogue: add alpha * tile to every destination block of C (Sec. 4.2) ----
    // the operand tiles are dead: reuse their LDS for the destinations' scatter tables
    int64_t(*c_rs)[TM] = reinterpret_cast<int64_t(*)[TM]>(&S.a[0][0]);
    int64_t(*c_cs)[TN] = reinterpret_cast<int64_t(*)[TN]>(&S.b[0][0]);
    const int nC = P.C.nterms;
    for (int e = tid; e < NT * TM; e += NTHREADS) {
        const int d = e / TM, x = e % TM;
        const int64_t gi = i0 + x, gj = j0 + x;
        int64_t val = kSentinel;
        if (d < nC && gi < P.mb && P.C.roff[d] + gi < P.C.rs_len) val = as_global(P.C.rs)[P.C.roff[d] + gi];
        c_rs[d][x] = val;
        val = kSentinel;
        if (d < nC && gj < P.nb && P.C.coff[d] + gj < P.C.cs_len) val = as_global(P.C.cs)[P.C.coff[d] + gj];
        c_cs[d][x] = val;
    }
    __syncthreads();
    double* Cbase = (P.C.space == 0 ? Cu : W) + P.C.base_off;
    const int dj = lane & 3, dblk = (lane >> 2) & 3, di = lane >> 4;
#pragma unroll
    for (int d = 0; d < NT; ++d) {
        if (d >= nC) break;
        const double g = P.C.coef[d];
        const double f = P.overwrite ? 0.0 : (((P.first_mask >> d) & 1u) ? beta : 1.0);
        int64_t rsv[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) rsv[x] = c_rs[d][wm * 64 + x * 16 + dblk * 4 + di];
#pragma unroll
        for (int y = 0; y < 2; ++y) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int64_t csv = c_cs[d][wn * 32 + y * 16 + ((dblk + s) & 3) * 4 + dj];
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int64_t off = rsv[x] + csv;
                    if (off >= 0) {
                        const double v = g * (alpha * st.acc[x][y][s]);
                        Cbase[off] = (f == 0.0) ? v : __builtin_fma(f, Cbase[off], v);
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// element-wise linear combination on matrix views
// ---------------------------------------------------------------------------------------------------------
template <bool ROWS_FAST>
__global__ __launch_bounds__(256) void lincomb_kernel(const Product* __restrict__ prods, int index, const double* __restrict__ srcU,
                                                      double* __restrict__ Cu, double* __restrict__ W, double beta, int slow_per_block) {
    const Product& P = prods[index];
    // a block covers 256 entries of the fast direction and slow_per_block of the slow one
    const int64_t fast = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t slow0 = (int64_t)blockIdx.y * slow_per_block;
    const int64_t nfast = ROWS_FAST ? P.mb : P.nb, nslow = ROWS_FAST ? P.nb : P.mb;
    if (fast >= nfast) return;
    const double* src = (P.A.space == 0 ? srcU : W) + P.A.base_off;
    double* dst = (P.C.space == 0 ? Cu : W) + P.C.base_off;
    const int nS = P.A.nterms, nD = P.C.nterms;
    int64_t sfix[kMaxTerms], dfix[kMaxTerms];
#pragma unroll
    for (int t = 0; t < kMaxTerms; ++t) {
        sfix[t] = dfix[t] = kSentinel;
        if (t < nS) {
            const int64_t g = (ROWS_FAST ? P.A.roff[t] : P.A.coff[t]) + fast;
            const int64_t len = ROWS_FAST ? P.A.rs_len : P.A.cs_len;
            if (g < len) sfix[t] = (ROWS_FAST ? P.A.rs : P.A.cs)[g];
        }
        if (t < nD) {
            const int64_t g = (ROWS_FAST ? P.C.roff[t] : P.C.coff[t]) + fast;
            const int64_t len = ROWS_FAST ? P.C.rs_len : P.C.cs_len;
            if (g < len) dfix[t] = (ROWS_FAST ? P.C.rs : P.C.cs)[g];
        }
    }
    for (int e = 0; e < slow_per_block; ++e) {
        const int64_t sl = slow0 + e;
        if (sl >= nslow) break;
        double v = 0.0;
#pragma unroll
        for (int t = 0; t < kMaxTerms; ++t) {
            if (t >= nS) break;
            const int64_t g = (ROWS_FAST ? P.A.coff[t] : P.A.roff[t]) + sl;
            const int64_t len = ROWS_FAST ? P.A.cs_len : P.A.rs_len;
            if (g < len && sfix[t] >= 0) v = __builtin_fma(P.A.coef[t], src[sfix[t] + (ROWS_FAST ? P.A.cs : P.A.rs)[g]], v);
        }
#pragma unroll
        for (int d = 0; d < kMaxTerms; ++d) {
            if (d >= nD) break;
            const int64_t g = (ROWS_FAST ? P.C.coff[d] : P.C.roff[d]) + sl;
            const int64_t len = ROWS_FAST ? P.C.cs_len : P.C.rs_len;
            if (g < len && dfix[d] >= 0) {
                const int64_t off = dfix[d] + (ROWS_FAST ? P.C.cs : P.C.rs)[g];
                const double f = P.overwrite ? 0.0 : (((P.first_mask >> d) & 1u) ? beta : 1.0);
                const double gv = P.C.coef[d] * v;
                dst[off] = (f == 0.0) ? gv : __builtin_fma(f, dst[off], gv);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// planner kernels (Sec. 2.3, "Block Scatter Matrix View")
// ---------------------------------------------------------------------------------------------------------
// scat[i] = sum_d i_d * stride_d   where   i = sum_d i_d * prod_{l<d} len_l   (first index of the bundle fastest)
__global__ __launch_bounds__(256) void scatter_kernel(const BundleDesc* __restrict__ descs, int64_t* __restrict__ store) {
    const BundleDesc& b = descs[blockIdx.y];
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < b.total; i += (int64_t)gridDim.x * blockDim.x) {
        int64_t rest = i, loc = 0;
        for (int d = 0; d < b.ndim; ++d) {
            const int64_t len = b.len[d];
            const int64_t digit = rest % len;
            rest /= len;
            loc += digit * b.stride[d];
        }
        store[b.out_off + i] = loc;
    }
}

// bs[q] = common difference of the entries of block q, 0 if they are not equally spaced; a block holding a
// single entry is recorded as regular with stride 1.
__global__ __launch_bounds__(256) void block_scatter_kernel(const BundleDesc* __restrict__ descs, int bs_block, int64_t* __restrict__ store) {
    const BundleDesc& b = descs[blockIdx.y];
    const int64_t nblk = (b.total + bs_block - 1) / bs_block;
    for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nblk; q += (int64_t)gridDim.x * blockDim.x) {
        const int64_t lo = q * bs_block;
        const int64_t hi = (lo + bs_block < b.total) ? lo + bs_block : b.total;
        const int64_t* v = store + b.out_off;
        int64_t s = (hi - lo >= 2) ? v[lo + 1] - v[lo] : 1;
        for (int64_t e = lo + 1; e < hi; ++e)
            if (v[e] - v[e - 1] != s) s = 0;
        store[b.bs_off + q] = s;
    }
}

template <int AMODE, int BMODE, int NT>
int launch_fused_t(const Product* prods, int first, int count, int tiles_m, int tiles_n, const double* A, const double* B, double* C,
                   double* W, double alpha, double beta, hipStream_t stream) {
    static bool configured = false;
    const size_t smem = sizeof(FusedSmem<NT>);
    static_assert(sizeof(FusedSmem<NT>) <= 160 * 1024, "LDS budget of one CU");
    auto kern = fused_kernel<AMODE, BMODE, NT>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return (int)e;
        configured = true;
    }
    const int64_t blocks = (int64_t)count * tiles_m * tiles_n;
    if (blocks <= 0 || blocks > 0x7fffffff) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), smem, stream, prods, first, tiles_m, tiles_n, A, B, C, W, alpha, beta);
    return (int)hipGetLastError();
}

template <int NT>
int launch_fused_modes(const FusedConfig& cfg, const Product* prods, int first, int count, int tiles_m, int tiles_n, const double* A,
                       const double* B, double* C, double* W, double alpha, double beta, hipStream_t stream) {
    switch (cfg.a_mode * 2 + cfg.b_mode) {
        case 0: return launch_fused_t<0, 0, NT>(prods, first, count, tiles_m, tiles_n, A, B, C, W, alpha, beta, stream);
        case 1: return launch_fused_t<0, 1, NT>(prods, first, count, tiles_m, tiles_n, A, B, C, W, alpha, beta, stream);
        case 2: return launch_fused_t<1, 0, NT>(prods, first, count, tiles_m, tiles_n, A, B, C, W, alpha, beta, stream);
        default: return launch_fused_t<1, 1, NT>(prods, first, count, tiles_m, tiles_n, A, B, C, W, alpha, beta, stream);
    }
}

}  // namespace

int dev_malloc(void** p, size_t bytes) { return (int)hipMalloc(p, bytes); }
int dev_free(void* p) { return (int)hipFree(p); }
int dev_upload(void* dst, const void* src, size_t bytes, void* stream) {
    // the source is pageable host memory owned by the plan: the copy is complete when this returns
    (void)stream;
    return (int)hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice);
}
int dev_download(void* dst, const void* src, size_t bytes) { return (int)hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost); }
int dev_stream_sync(void* stream) { return (int)hipStreamSynchronize((hipStream_t)stream); }

int launch_planner(const BundleDesc* descs_dev, int nvec, int64_t max_total, int bs_block, int64_t* store_dev, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    int64_t bx = (max_total + 255) / 256;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(scatter_kernel, dim3((unsigned)bx, (unsigned)nvec), dim3(256), 0, st, descs_dev, store_dev);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
    int64_t nblk = (max_total + bs_block - 1) / bs_block;
    bx = (nblk + 255) / 256;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(block_scatter_kernel, dim3((unsigned)bx, (unsigned)nvec), dim3(256), 0, st, descs_dev, bs_block, store_dev);
    return (int)hipGetLastError();
}

int launch_fused(const FusedConfig& cfg, const Product* prods_dev, int first, int count, int64_t mb, int64_t nb, const double* A,
                 const double* B, double* C, double* W, double alpha, double beta, void* stream) {
    const int64_t tiles_m = (mb + TM - 1) / TM, tiles_n = (nb + TN - 1) / TN;
    if (tiles_m <= 0 || tiles_n <= 0 || tiles_m > (1 << 20) || tiles_n > (1 << 20)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    switch (cfg.max_terms) {
        case 1: return launch_fused_modes<1>(cfg, prods_dev, first, count, (int)tiles_m, (int)tiles_n, A, B, C, W, alpha, beta, st);
        case 2: return launch_fused_modes<2>(cfg, prods_dev, first, count, (int)tiles_m, (int)tiles_n, A, B, C, W, alpha, beta, st);
        case 4: return launch_fused_modes<4>(cfg, prods_dev, first, count, (int)tiles_m, (int)tiles_n, A, B, C, W, alpha, beta, st);
        default: return (int)hipErrorInvalidValue;
    }
}

int launch_lincomb(const Product* prods_dev, int index, int64_t mb, int64_t nb, int lanes_along_rows, const double* A, const double* B,
                   double* C, double* W, int src_role, double beta, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const double* src = src_role == 0 ? A : B;
    const int64_t nfast = lanes_along_rows ? mb : nb, nslow = lanes_along_rows ? nb : mb;
    if (nfast <= 0 || nslow <= 0) return 0;
    int64_t per = 16;
    while ((nslow + per - 1) / per > 65535) per *= 2;
    const int64_t gx = (nfast + 255) / 256, gy = (nslow + per - 1) / per;
    if (gx > 0x7fffffff || per > (1 << 30)) return (int)hipErrorInvalidValue;
    if (lanes_along_rows)
        hipLaunchKernelGGL(lincomb_kernel<true>, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, st, prods_dev, index, src, C, W, beta, (int)per);
    else
        hipLaunchKernelGGL(lincomb_kernel<false>, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, st, prods_dev, index, src, C, W, beta, (int)per);
    return (int)hipGetLastError();
}

}  // namespace tc
