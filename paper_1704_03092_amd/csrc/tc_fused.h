// The fused kernel of libstrassen_tc (gfx950 / CDNA4 only): the general primitive of Sec. 3, eq. (straprim1),
// generalised to <= 4 signed blocks per operand and <= 4 signed destinations.  It gathers blocks of A and B through
// the scatter vectors, adds them in registers, stages the sums in LDS (Sec. 4.1 "packing"), multiplies tiles on the
// FP64 matrix cores and adds the tile to every destination block of C from registers (Sec. 4.2).  Level 0 is the same
// kernel with one term and one destination.
//
// Matrix-core instruction: v_mfma_f64_4x4x4_4b_f64.  One instruction multiplies four independent 4x4x4 blocks;
// measured on MI355X it sustains twice the rate of v_mfma_f64_16x16x4_f64.  Register layout (lane l):
//   A operand: block (l/4)%4, row l%4, k = l/16        B operand: block (l/4)%4, column l%4, k = l/16
//   D result : block (l/4)%4, column l%4, row l/16
// A 16x16 output patch is covered by 4 instructions whose B operand has its four column blocks rotated by
// s = 0..3 positions: block slot b of instruction s multiplies row block b by column block (b + s) % 4.
//
// Other VALU instructions do not overlap with these MFMAs on this chip (measured: every integer or fp64 VALU
// instruction adds its full issue time), so the main loop is written to need as few of them as possible: the
// gather tables hold ready-made byte addresses (one 64-bit add per load), the k-step loop is unrolled over the two
// LDS buffers so that every LDS address is a per-lane base plus a constant, and an operand with a single +1 term is
// stored as loaded.  A wave-wide global load costs the CU's address pipeline the same whatever its width, so
// operands whose consecutive entries are contiguous and 16-byte aligned are gathered two elements per load.
#pragma once
#include <hip/hip_runtime.h>

#include "tc_internal.h"

namespace tc {
namespace fused {

constexpr int TM = 128;        // tile rows (free bundle I)
constexpr int TN = 128;        // tile columns (free bundle J)
constexpr int NTHREADS = 512;  // 8 waves: 2 along the rows x 4 along the columns, each owning 64 x 32 outputs
constexpr int GROUP_M = 8;     // tile rows per rasterisation group

// Contracted entries per pipeline step.  A gathered element needs more than 16 entries' worth of matrix-core
// work to arrive, so the step is made as deep as the registers allow: 32 for one or two terms per operand.
template <int NT>
struct Cfg {
    static constexpr int KT = (NT <= 2) ? 32 : 16;
    static constexpr int NE = TM * KT / NTHREADS;  // elements of each operand tile a thread gathers per k-step
    static constexpr int NQ = KT / 4;              // matrix-core instruction groups per k-step
    // The second wave of a SIMD issues its gather after this many groups, when its partner's burst of loads has
    // drained from the CU's address pipeline (a burst lasts longer the more terms there are); measured optimum.
    static constexpr int LATE = (NT == 1) ? 3 : (NT == 2) ? 4 : 3;
};

// LDS tile layout: element (k, x) of a KT x 128 tile lives at k * PITCH + x.  Instruction group q of a k-step
// takes k = 16 * (q / 4) + 4 * (lane / 16) + q % 4, so one fragment load touches rows k and k + 4 in each half-wave;
// with PITCH = 132 those rows start 16 bank-pairs apart and the load is conflict-free, and every fragment address
// is one per-lane base plus a compile-time offset.
constexpr int PITCH = 132;
constexpr int OPITCH = 130;  // row pitch of the output tile staged in LDS by the epilogue

// Scatter vectors are reached through pointers stored in the product descriptors; telling the compiler that they
// point to global memory keeps their loads off the flat path (a pending flat load forces a full wait before the
// next LDS access).
typedef const __attribute__((address_space(1))) int64_t* gvec_t;
__device__ __forceinline__ gvec_t as_global(const int64_t* p) { return (gvec_t)p; }
typedef const __attribute__((address_space(1))) double* gdbl_t;
typedef double double2_t __attribute__((ext_vector_type(2)));
typedef const __attribute__((address_space(1))) double2_t* gdbl2_t;

template <int NT>
struct Smem {
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

// Which elements of a KT x 128 operand tile a thread gathers in a k-step.
//   MODE 0: lanes run along the 128 free entries x (the operand is contiguous along its free bundle)
//   MODE 1: lanes run along the contracted entries k (contiguous along the contracted bundle); a wave covers 16 k
//           (one 128-byte line) times 4 x, which also makes the transposing LDS store hit every bank pair twice
//   VEC   : an element pair per load: (x, x+1) in mode 0, (k, k+1) in mode 1
// Load e of a thread is element (K0 + CK * e, X0 + CX * e).
template <int MODE, int NT, bool VEC>
struct Map {
    static constexpr int KT = Cfg<NT>::KT;
    static constexpr int KB = KT / 16;
    static constexpr int N = VEC ? Cfg<NT>::NE / 2 : Cfg<NT>::NE;  // loads per thread, term and k-step
    static constexpr int CK = (MODE == 0) ? (VEC ? 8 : 4) : 0;
    static constexpr int CX = (MODE == 1) ? (VEC ? 64 / KB : 32 / KB) : 0;
    __device__ static __forceinline__ int k0(int tid) {
        const int lane = tid & 63, w = tid >> 6;
        if (MODE == 0) return VEC ? (tid >> 6) : (tid >> 7);
        return VEC ? 2 * ((lane & 7) + 8 * (w % KB)) : (lane & 15) + 16 * (w % KB);
    }
    __device__ static __forceinline__ int x0(int tid) {
        const int lane = tid & 63, w = tid >> 6;
        if (MODE == 0) return VEC ? 2 * (tid & 63) : (tid & 127);
        return VEC ? (lane >> 3) + 8 * (w / KB) : (lane >> 4) + 4 * (w / KB);
    }
};

// Per-thread LDS addresses of one operand for the unchecked gather: table entries and staging position.
struct Bases {
    const int64_t* fix;   // &fix_tab[0][x0]
    const int64_t* step;  // &step_tab[slot 0][0][k0]
    double* stage;        // &tile[buffer 0][k0 * PITCH + x0]
};

// Issue the loads of one k-step for every term; absent terms (index >= nterms) contribute zeros.
template <int MODE, int NT, bool VEC>
__device__ __forceinline__ void issue_fast(double (&ld)[NT][Cfg<NT>::NE], const Bases& b, int slot_off, int nterms) {
    typedef Map<MODE, NT, VEC> M;
    constexpr int KT = Cfg<NT>::KT;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (t > 0 && t >= nterms) {
#pragma unroll
            for (int e = 0; e < Cfg<NT>::NE; ++e) ld[t][e] = 0.0;
        } else {
#pragma unroll
            for (int e = 0; e < M::N; ++e) {
                const int64_t addr = b.fix[t * 128 + M::CX * e] + b.step[slot_off + t * KT + M::CK * e];
                if (VEC) {
                    const double2_t v = *(gdbl2_t)addr;
                    ld[t][2 * e] = v.x;
                    ld[t][2 * e + 1] = v.y;
                } else {
                    ld[t][e] = *(gdbl_t)addr;
                }
            }
        }
    }
}

// Signed sum of the terms (the operand sum of Sec. 4.1) into the LDS tile.
template <int MODE, int NT, bool VEC>
__device__ __forceinline__ void stage_fast(const double (&ld)[NT][Cfg<NT>::NE], double* __restrict__ dst, const double* __restrict__ coef,
                                           bool plain) {
    typedef Map<MODE, NT, VEC> M;
#pragma unroll
    for (int e = 0; e < M::N; ++e) {
        double v[2];
#pragma unroll
        for (int h = 0; h < (VEC ? 2 : 1); ++h) {
            const int i = VEC ? 2 * e + h : e;
            if (NT == 1) {
                v[h] = plain ? ld[0][i] : coef[0] * ld[0][i];
            } else {
                v[h] = coef[0] * ld[0][i];
#pragma unroll
                for (int t = 1; t < NT; ++t) v[h] = __builtin_fma(coef[t], ld[t][i], v[h]);
            }
        }
        double* p = dst + M::CK * e * PITCH + M::CX * e;
        if (!VEC) {
            p[0] = v[0];
        } else if (MODE == 0) {
            double2_t vv = {v[0], v[1]};
            *reinterpret_cast<double2_t*>(p) = vv;
        } else {
            p[0] = v[0];
            p[PITCH] = v[1];
        }
    }
}

// Gather with padding checks (tiles or k-steps that touch the zero padding of a Strassen block or the ragged edge):
// entries of the padding (negative table sum) read the operand's element 0 and count as zero.  Scalar mapping.
template <int MODE, int NT>
__device__ __forceinline__ void issue_checked(double (&ld)[NT][Cfg<NT>::NE], unsigned& padmask, const double* __restrict__ safe,
                                              const int64_t* __restrict__ fixed_tab, const int64_t* __restrict__ step_tab, int nterms, int tid) {
    typedef Map<MODE, NT, false> M;
    constexpr int KT = Cfg<NT>::KT, NE = Cfg<NT>::NE;
    const int k0 = M::k0(tid), x0 = M::x0(tid);
    padmask = 0;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (t > 0 && t >= nterms) {
                ld[t][e] = 0.0;
            } else {
                const int64_t addr = fixed_tab[t * 128 + x0 + M::CX * e] + step_tab[t * KT + k0 + M::CK * e];
                padmask |= (addr < 0 ? 1u : 0u) << (t * NE + e);
                ld[t][e] = *(gdbl_t)(addr < 0 ? (int64_t)safe : addr);
            }
        }
    }
}

template <int MODE, int NT>
__device__ __forceinline__ void stage_checked(const double (&ld)[NT][Cfg<NT>::NE], unsigned padmask, double* __restrict__ tile,
                                              const double* __restrict__ coef, int tid) {
    typedef Map<MODE, NT, false> M;
    constexpr int NE = Cfg<NT>::NE;
    double* dst = tile + M::k0(tid) * PITCH + M::x0(tid);
#pragma unroll
    for (int e = 0; e < NE; ++e) {
        double v = 0.0;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const double x = ((padmask >> (t * NE + e)) & 1u) ? 0.0 : ld[t][e];
            v = (t == 0) ? coef[0] * x : __builtin_fma(coef[t], x, v);
        }
        dst[M::CK * e * PITCH + M::CX * e] = v;
    }
}

__device__ __forceinline__ int64_t min64(int64_t a, int64_t b) { return a < b ? a : b; }

template <int AMODE, int BMODE, int NT, bool VA, bool VB>
struct State {
    static constexpr int KT = Cfg<NT>::KT, NE = Cfg<NT>::NE, NQ = Cfg<NT>::NQ, TILE = KT * PITCH;
    Smem<NT>* S;
    const Product* P;
    int tid, nA, nB, nk, kfull;
    bool plainA, plainB;       // single term with coefficient +1: staged as loaded
    bool early;                // this wave issues its gather before the matrix-core work of a k-step, its partner on
                               // the same SIMD after Cfg::LATE groups: one of the two always has MFMAs to issue
    const double *safeA, *safeB;
    // scatter entries of later k-steps
    gvec_t ent_ptr;
    int ent_limit;             // k entries that exist for this thread's term, counted from its own k
    int64_t* ent_dst;
    Bases ba, bb;
    // per-lane fragment bases
    const double* fa;
    const double* fb[4];
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
                issue_fast<AMODE, NT, VA>(la, ba, SLOT * NT * KT, nA);
                issue_fast<BMODE, NT, VB>(lb, bb, SLOT * NT * KT, nB);
            } else {
                issue_checked<AMODE, NT>(la, pa, safeA, &S->a_fix[0][0], &S->a_step[SLOT][0][0], nA, tid);
                issue_checked<BMODE, NT>(lb, pb, safeB, &S->b_fix[0][0], &S->b_step[SLOT][0][0], nB, tid);
            }
        }
    }

    // operand sums of the loads in flight into LDS buffer BUF
    template <int BUF>
    __device__ __forceinline__ void stage() {
        if (issued_fast) {
            stage_fast<AMODE, NT, VA>(la, ba.stage + BUF * TILE, P->A.coef, plainA);
            stage_fast<BMODE, NT, VB>(lb, bb.stage + BUF * TILE, P->B.coef, plainB);
        } else {
            stage_checked<AMODE, NT>(la, pa, &S->a[BUF][0], P->A.coef, tid);
            stage_checked<BMODE, NT>(lb, pb, &S->b[BUF][0], P->B.coef, tid);
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
            if constexpr (Q + 1 == Cfg<NT>::LATE) {
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

template <int AMODE, int BMODE, int NT, bool VA, bool VB>
__global__ __launch_bounds__(NTHREADS, 2) void fused_kernel(const Product* __restrict__ prods, int first, int tiles_m, int tiles_n,
                                                            const double* __restrict__ Au, const double* __restrict__ Bu,
                                                            double* __restrict__ Cu, double* __restrict__ W, double alpha, double beta, int c_mode) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Smem<NT>& S = *reinterpret_cast<Smem<NT>*>(smem_raw);
    const int tid = threadIdx.x;
    typedef State<AMODE, BMODE, NT, VA, VB> St;
    constexpr int KT = St::KT;

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

    St st;
    st.S = &S;
    st.P = &P;
    st.tid = tid;
    st.nA = nA;
    st.nB = nB;
    st.nk = (int)((P.kb + KT - 1) / KT);
    st.plainA = nA == 1 && P.A.coef[0] == 1.0;
    st.plainB = nB == 1 && P.B.coef[0] == 1.0;
    const double* Abase = (P.A.space == 0 ? Au : W) + P.A.base_off;
    const double* Bbase = (P.B.space == 0 ? Bu : W) + P.B.base_off;
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
    {
        typedef Map<AMODE, NT, VA> MA;
        typedef Map<BMODE, NT, VB> MB;
        st.ba.fix = &S.a_fix[0][0] + MA::x0(tid);
        st.ba.step = &S.a_step[0][0][0] + MA::k0(tid);
        st.ba.stage = &S.a[0][0] + MA::k0(tid) * PITCH + MA::x0(tid);
        st.bb.fix = &S.b_fix[0][0] + MB::x0(tid);
        st.bb.step = &S.b_step[0][0][0] + MB::k0(tid);
        st.bb.stage = &S.b[0][0] + MB::k0(tid) * PITCH + MB::x0(tid);
    }

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
    // The accumulators hold 4x4 blocks scattered over the tile; they are transposed through LDS (the operand buffers
    // are dead) so that each wave-wide access to C covers 64 consecutive entries of C's contiguous direction.
    // The gather tables' LDS is reused for the destinations' scatter tables.
    constexpr int NPASS = (sizeof(S.a) + sizeof(S.b) >= (size_t)TN * OPITCH * sizeof(double)) ? 1 : 2;
    constexpr int CP = TN / NPASS;  // tile columns staged per pass
    static_assert(sizeof(S.a) + sizeof(S.b) >= (size_t)CP * OPITCH * sizeof(double), "output staging does not fit");
    int64_t(*c_rs)[TM] = reinterpret_cast<int64_t(*)[TM]>(&S.a_fix[0][0]);
    int64_t(*c_cs)[TN] = reinterpret_cast<int64_t(*)[TN]>(&S.b_fix[0][0]);
    double* otile = &S.a[0][0];  // [CP columns][OPITCH], rows fastest
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
    double* Cbase = (P.C.space == 0 ? Cu : W) + P.C.base_off;
    const int dj = lane & 3, dblk = (lane >> 2) & 3, di = lane >> 4;
#pragma unroll 1
    for (int pass = 0; pass < NPASS; ++pass) {
        if (pass > 0) __syncthreads();  // the previous pass has been read out
        if (wn / (4 / NPASS) == pass) {
            const int cw = (wn % (4 / NPASS)) * 32;
#pragma unroll
            for (int y = 0; y < 2; ++y)
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int x = 0; x < 4; ++x)
                        otile[(cw + y * 16 + ((dblk + s) & 3) * 4 + dj) * OPITCH + wm * 64 + x * 16 + dblk * 4 + di] = alpha * st.acc[x][y][s];
        }
        __syncthreads();
        for (int d = 0; d < nC; ++d) {
            const double g = P.C.coef[d];
            const double f = P.overwrite ? 0.0 : (((P.first_mask >> d) & 1u) ? beta : 1.0);
            constexpr int BATCH = CP / 4;  // elements per thread, destination and pass: all their loads are issued together
            static_assert(BATCH == TM / (NTHREADS / CP), "both thread mappings cover the pass");
            if (c_mode == 0) {
                // lanes along the rows: thread = (row r, column group cg), columns cg + 4 j
                const int r = tid & 127, cg = tid >> 7;
                const int64_t rsd = c_rs[d][r];
                for (int j0b = 0; j0b < CP / 4; j0b += BATCH) {
                    int64_t off[BATCH];
                    double cur[BATCH];
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) {
                        off[b] = rsd + c_cs[d][pass * CP + cg + 4 * (j0b + b)];
                        cur[b] = (f != 0.0 && off[b] >= 0) ? Cbase[off[b]] : 0.0;
                    }
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) {
                        const double v = g * otile[(cg + 4 * (j0b + b)) * OPITCH + r];
                        if (off[b] >= 0) Cbase[off[b]] = (f == 0.0) ? v : __builtin_fma(f, cur[b], v);
                    }
                }
            } else {
                // lanes along the columns: thread = (column c, row group rg), rows rg + RS j
                constexpr int RS = NTHREADS / CP;
                const int c = tid % CP, rg = tid / CP;
                const int64_t csd = c_cs[d][pass * CP + c];
                for (int j0b = 0; j0b < TM / RS; j0b += BATCH) {
                    int64_t off[BATCH];
                    double cur[BATCH];
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) {
                        off[b] = c_rs[d][rg + RS * (j0b + b)] + csd;
                        cur[b] = (f != 0.0 && off[b] >= 0) ? Cbase[off[b]] : 0.0;
                    }
#pragma unroll
                    for (int b = 0; b < BATCH; ++b) {
                        const double v = g * otile[c * OPITCH + rg + RS * (j0b + b)];
                        if (off[b] >= 0) Cbase[off[b]] = (f == 0.0) ? v : __builtin_fma(f, cur[b], v);
                    }
                }
            }
        }
    }
}

template <int AMODE, int BMODE, int NT, bool VA, bool VB>
int launch_one(const Product* prods, int first, int count, int tiles_m, int tiles_n, const double* A, const double* B, double* C,
               double* W, double alpha, double beta, int c_mode, hipStream_t stream) {
    static bool configured = false;
    static_assert(sizeof(Smem<NT>) <= 160 * 1024, "LDS budget of one CU");
    const size_t smem = sizeof(Smem<NT>);
    auto kern = fused_kernel<AMODE, BMODE, NT, VA, VB>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return (int)e;
        configured = true;
    }
    const int64_t blocks = (int64_t)count * tiles_m * tiles_n;
    if (blocks <= 0 || blocks > 0x7fffffff) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), smem, stream, prods, first, tiles_m, tiles_n, A, B, C, W, alpha, beta, c_mode);
    return (int)hipGetLastError();
}

// vec: bit 0 = pair-wise gather of A, bit 1 = of B
template <int NT>
int launch_nt(int a_mode, int b_mode, int vec, int c_mode, const Product* prods, int first, int count, int tiles_m, int tiles_n, const double* A,
              const double* B, double* C, double* W, double alpha, double beta, hipStream_t stream);

#define TC_FUSED_CASE(AM, BM, VA, VB) \
    case ((AM) * 8 + (BM) * 4 + (VA) * 2 + (VB)): \
        return launch_one<AM, BM, NT, (VA) != 0, (VB) != 0>(prods, first, count, tiles_m, tiles_n, A, B, C, W, alpha, beta, c_mode, stream);

#define TC_FUSED_DEFINE_LAUNCH(NTV)                                                                                                  \
    template <>                                                                                                                      \
    int launch_nt<NTV>(int a_mode, int b_mode, int vec, int c_mode, const Product* prods, int first, int count, int tiles_m, int tiles_n,        \
                       const double* A, const double* B, double* C, double* W, double alpha, double beta, hipStream_t stream) {      \
        constexpr int NT = NTV;                                                                                                      \
        switch (a_mode * 8 + b_mode * 4 + (vec & 1) * 2 + ((vec >> 1) & 1)) {                                                        \
            TC_FUSED_CASE(0, 0, 0, 0) TC_FUSED_CASE(0, 0, 0, 1) TC_FUSED_CASE(0, 0, 1, 0) TC_FUSED_CASE(0, 0, 1, 1)                  \
            TC_FUSED_CASE(0, 1, 0, 0) TC_FUSED_CASE(0, 1, 0, 1) TC_FUSED_CASE(0, 1, 1, 0) TC_FUSED_CASE(0, 1, 1, 1)                  \
            TC_FUSED_CASE(1, 0, 0, 0) TC_FUSED_CASE(1, 0, 0, 1) TC_FUSED_CASE(1, 0, 1, 0) TC_FUSED_CASE(1, 0, 1, 1)                  \
            TC_FUSED_CASE(1, 1, 0, 0) TC_FUSED_CASE(1, 1, 0, 1) TC_FUSED_CASE(1, 1, 1, 0) TC_FUSED_CASE(1, 1, 1, 1)                  \
        }                                                                                                                            \
        return (int)hipErrorInvalidValue;                                                                                            \
    }

}  // namespace fused
}  // namespace tc
