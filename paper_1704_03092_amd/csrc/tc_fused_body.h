// The fused kernel of libstrassen_tc (gfx950 / CDNA4 only): the general primitive displayed at the start of Sec. 3,
// generalised to <= 4 signed blocks per operand and <= 4 signed destinations.  It gathers blocks of A and B through
// the scatter vectors, adds them in registers, stages the sums in LDS (Sec. 4.1 "packing"), multiplies tiles on the
// FP64 matrix cores and adds the tile to every destination block of C from registers (Sec. 4.2).  Level 0 is the same
// kernel with one term and one destination.
//
// Matrix-core instruction: v_mfma_f64_16x16x4_f64, one per 16 x 16 output patch and four contracted entries.
// Register layout (lane l; probed on the device for the result):
//   A operand: row l % 16, k = l / 16        B operand: column l % 16, k = l / 16
//   D result v (0..3): row 4 v + l / 16, column l % 16
// Lane l % 16 stands for tile rows (columns) 2 (l % 16) + {0, 1} of a 32-wide strip, so that one 16-byte LDS read
// delivers the fragments of two patches without any shuffling.  (TC_MFMA16 = 0 builds the kernel on
// v_mfma_f64_4x4x4_4b_f64 instead, which it was written for: the same operand layout read as four independent 4 x 4
// blocks, a patch covered by four instructions whose B operand has its column blocks rotated by s = 0..3.  Measured
// with nothing else in the loop the two sustain 77.7 and 76.7 TFLOP/s: tc_bench_mfma_peak.)
//
// Other VALU instructions delay these MFMAs on this chip (measured: integer or fp64 VALU work added to an MFMA loop
// adds its issue time), so the main loop needs few of them: the gather tables hold ready-made byte addresses (one
// 64-bit add per load), the k-step loop is unrolled over the two LDS buffers so that every LDS address is a
// per-lane base plus a constant, and an operand whose leading coefficient is +1 starts its sum from the gathered
// element itself.  A wave-wide global load costs the CU's address pipeline the same whatever its width, so
// operands whose consecutive entry pairs are contiguous are gathered two elements per load.
//
// This file is compiled for two workgroup geometries (TC_GEO_SMALL, set by the including header):
//   tc::fused        128 x 128 tiles, 512 threads (8 waves, 2 x 4), one workgroup per compute unit: all kernel families
//   tc::fused_small  128 x 64 tiles, 256 threads (4 waves, 2 x 2), two workgroups per compute unit: single-term products
//                    only.  Less arithmetic per gathered element (1.5 x the operand reads), but one workgroup's
//                    set-up, first gathers and destination update overlap the other's matrix-core work, and twice
//                    as many tiles are in flight.  Measured: ahead of the large shape for tiles gathered by stride
//                    at every size (25 % for a handful of tiles, 8 % at k = 256, 1 % at 16384^3), 3 - 4 % behind
//                    for tiles gathered through the tables.  Its vector instructions outside the matrix-core loop
//                    are costly (each waits for a matrix-core instruction of the other workgroup to end), which is
//                    why set-up and epilogue keep workgroup-wide quantities on the scalar unit.
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "tc_internal.h"

namespace tc {
#if TC_GEO_SMALL
namespace fused_small {
constexpr bool SMALL = true;
constexpr int TN = 64;         // tile columns (free bundle J)
constexpr int NTHREADS = 256;  // 4 waves: 2 along the rows x 2 along the columns, each owning 64 x 32 outputs
constexpr int WGS_PER_CU = 2;
#else
namespace fused {
constexpr bool SMALL = false;
constexpr int TN = 128;        // tile columns (free bundle J)
constexpr int NTHREADS = 512;  // 8 waves: 2 along the rows x 4 along the columns, each owning 64 x 32 outputs
constexpr int WGS_PER_CU = 1;
#endif
constexpr int TM = 128;        // tile rows (free bundle I)
constexpr int NW = NTHREADS / 64;  // waves
constexpr int WN = TN / 32;        // waves along the columns
constexpr int GROUP_M = 8;     // tile rows per rasterisation group
constexpr int MAXC = 4;        // destinations of a product

// LDS tile layout: element (k, x) of a KT x 128 tile lives at k * PITCH + x.  Instruction group q of a k-step
// takes k = 16 * (q / 4) + krow(lane / 16) + q % 4 with krow = 0, 8, 4, 12, so every fragment address is one
// per-lane base plus a compile-time offset; PITCH = 132 keeps both the fragment reads and the transposing stores
// of the staging step (nearly) free of bank conflicts.
constexpr int PITCH = 132;
constexpr int OPITCH = 130;  // row pitch of the output tile staged in LDS by the epilogue

// One kernel family per (NTA, NTB) = terms of the operand sums of A and B.
//   EXACT : every product of the launch has exactly NTA and NTB terms; the term loops are compile-time.
//   !EXACT: up to NTA / NTB terms, counted at run time (a four-term sum that lost a block to the zero padding).
// The k-step is 32 deep, 16 deep for the (4,4) family, the run-time-counted one and the small geometry (registers, LDS).
// How far ahead the gathers run and how they are turned over is described at Cfg::D / Cfg::ROLL.
// Build-time switches of the schedule (measurement aids; the defaults are the measured optima).
#ifndef TC_ROLL
#define TC_ROLL 1      // 1: the families with exact term counts gather in a rolling fashion (see Cfg::ROLL); 0: one burst per k-step
#endif
#ifndef TC_MFMA16
#define TC_MFMA16 1    // 1: v_mfma_f64_16x16x4_f64 (one instruction per 16 x 16 output patch and four contracted entries);
                       // 0: v_mfma_f64_4x4x4_4b_f64 (four, with rotated B fragments)
#endif
#ifndef TC_PIN8
#define TC_PIN8 1      // KT = 32: keep the compiler from moving the parts of a rolling gather across instruction groups
#endif
#ifndef TC_PIN4
#define TC_PIN4 1      // KT = 16: likewise
#endif

template <int NTA_, int NTB_, bool EXACT_>
struct Cfg {
    static constexpr int NTA = NTA_, NTB = NTB_;
    static constexpr bool EXACT = EXACT_;
#ifndef TC_KT32_SUM
#define TC_KT32_SUM 6  // 32-deep k-steps for families with at most this many terms in both sums together (all but (4,4):
                       // measured +2 % on the four-term families, two-level ABC 75.4 -> 77.0 TFLOP/s at 16384^3)
#endif
    static constexpr int KT = (!SMALL && EXACT && NTA + NTB <= TC_KT32_SUM) ? 32 : 16;  // (small geometry: LDS for two workgroups)
    static constexpr bool SINGLE = EXACT && NTA == 1 && NTB == 1;
    // D = how many k-steps ahead of the multiplying step a gather is issued; SETS = register sets for gathers in
    // flight.  ROLL (every family with exact term counts): D = 2 with ONE set that is turned over piecewise.  The tile of
    // the next k-step is cut into NQ parts (the first half of the groups takes A's, the second half B's); next to
    // instruction group g a wave waits for part g of the loads it issued one k-step earlier, adds the terms, stores
    // the sums to the other LDS buffer and at once re-issues that part's loads for the k-step after the next.
    // Every load has exactly one k-step to arrive, the waits are for the oldest loads in flight only, and loads and
    // LDS stores are spread evenly over the step.  (Issuing a whole k-step of a multi-term tile in one burst, 16 to
    // 32 loads per wave, fills the address queue of the CU: the profiler counts cycles with that queue full for the
    // multi-term families.)  Without ROLL (the run-time-counted family; build-time alternatives): multi-term sums
    // D = 1, issue at the start (first wave of a SIMD) or in the middle (second wave) of a step, store after its last
    // group; single-term operands D = 2 with two sets (issued during step s, stored to LDS during step s + 1), which
    // was the fastest single-term schedule with the 4x4x4 instruction (TC_ROLL_SINGLE = 0).
#ifndef TC_C_POLICY
#define TC_C_POLICY 2  // cache policy of the destination accesses by stride: 2 = non-temporal (every element of C is read and written once per launch)
#endif
#ifndef TC_ROLL_SINGLE
#define TC_ROLL_SINGLE 1  // the single-term family in 128 x 128 tiles rolls too (8192^3 classical 69.7 -> 72.2 TFLOP/s)
#endif
    static constexpr bool ROLL = TC_ROLL && EXACT && (!SINGLE || SMALL || TC_ROLL_SINGLE);
    static constexpr int D = (SINGLE || ROLL) ? 2 : 1;
    static constexpr int SETS = (SINGLE && !ROLL) ? 2 : 1;
    // The table-free loop fetches no scatter entries (they are fetched where it hands over to the table loop).  Not
    // in the four-term family with its 16-deep k-steps, which measured 2 % slower without the fetch in its loop; in
    // the 128 x 64 geometry every vector instruction saved counts (it waits for the partner workgroup's matrix cores).
    static constexpr bool NOENT_AFF = KT == 32 || SMALL;
    static constexpr int NEA = TM * KT / NTHREADS;  // elements of the A tile (per term) a thread gathers per k-step
    static constexpr int NEB = TN * KT / NTHREADS;  // of the B tile
    static constexpr int NQ = KT / 4;              // matrix-core instruction groups per k-step
    static constexpr int TILE = KT * PITCH;
    // Schedule inside a k-step without ROLL, in instruction groups completed (measured optima).  The two waves of a
    // SIMD do their loads and LDS stores at different times so that one of them always has MFMAs to issue: the
    // first wave issues its gather before group 0, its partner after ISSUE_LATE groups, when the first burst of
    // loads has drained from the CU's address pipeline.  With two sets the second wave stores right before it
    // issues and the first wave three quarters into the step; with D = 1 both store after the last group.
    static constexpr int ISSUE_LATE = (SETS == 2) ? 5 : (NQ == 8 ? 4 : 3);
    static constexpr int STAGE_EARLY = (SETS == 2) ? 6 : NQ;
    static constexpr int STAGE_LATE = (SETS == 2) ? 4 : NQ;
    // Measured: every rolling family is fastest when each part stays next to its instruction group (8192^3, two-term
    // families 65.3 -> 68 TFLOP/s executed; the four-term families lose 10 - 20 % without).
    static constexpr bool PIN = SETS == 1 && (D == 1 || (NQ == 8 ? TC_PIN8 : TC_PIN4));
    static_assert(SETS == 1 || NQ == 8, "the two-set schedule is written for 8 groups");
    static_assert(NEA % (NQ / 2) == 0 && (NEA / (NQ / 2)) % 2 == 0 && NEB % (NQ / 2) == 0 && (NEB / (NQ / 2)) % 2 == 0,
                  "a part of a rolling gather holds whole element pairs");
};

// Scatter vectors are reached through pointers stored in the product descriptors; telling the compiler that they
// point to global memory keeps their loads off the flat path (a pending flat load forces a full wait before the
// next LDS access).
typedef const __attribute__((address_space(1))) int64_t* gvec_t;
__device__ __forceinline__ gvec_t as_global(const int64_t* p) { return (gvec_t)p; }
typedef const __attribute__((address_space(1))) double* gdbl_t;
typedef double double2_t __attribute__((ext_vector_type(2)));
typedef double double4_t __attribute__((ext_vector_type(4)));
typedef double2_t double2_u __attribute__((aligned(8)));  // an element pair in global memory: 8-byte aligned only
typedef const __attribute__((address_space(1))) double2_u* gdbl2_t;

template <class CF>
struct Smem {
    static constexpr int KT = CF::KT, NTA = CF::NTA, NTB = CF::NTB;
    double a[2][CF::TILE];
    double b[2][CF::TILE];
    int64_t a_fix[NTA][TM];      // per term: address of row x of the A blocks (base + 8 * rscat), kSentinel where padded
    int64_t b_fix[NTB][TN];      // per term: address of column x of the B blocks (base + 8 * cscat)
    int64_t a_step[2][NTA][KT];  // per term: 8 * cscat_A of the contracted entries of a k-step (two table slots)
    int64_t b_step[2][NTB][KT];  // per term: 8 * rscat_B
    int64_t dump[2][64];         // where threads that own no table entry store theirs (keeps that store branch-free)
    int64_t c_rs[MAXC][TM];      // epilogue: row and column scatter entries of every destination
    int64_t c_cs[MAXC][TN];
};

// Which elements of a KT x TX operand tile a thread gathers in a k-step (TX = TM for A, TN for B).
//   MODE 0: lanes run along the free entries x (the operand is contiguous along its free bundle): LX lanes per
//           contracted entry, the workgroup's threads cover RK contracted entries per load
//   MODE 1: lanes run along the contracted entries k (contiguous along the contracted bundle); a wave covers 16 k
//           (one 128-byte line) times 4 x (8 x with pairs).  With pairs, each half-wave takes half a line (4 pairs)
//           of 8 columns, so that its 32 transposing LDS stores fall into 32 different bank pairs
//   VEC   : an element pair per load: (x, x+1) in mode 0, (k, k+1) in mode 1
// Load e of a thread is element (K0 + CK * e, X0 + CX * e).
template <int MODE, int KT, bool VEC, int TX>
struct Map {
    static constexpr int NE = TX * KT / NTHREADS;
    static constexpr int KB = KT / 16;
    static constexpr int N = VEC ? NE / 2 : NE;  // loads per thread, term and k-step
    static constexpr int LX = VEC ? TX / 2 : TX, RK = NTHREADS / LX;
    static constexpr int CK = (MODE == 0) ? RK : 0;
    static constexpr int CX = (MODE == 1) ? (VEC ? 8 : 4) * NW / KB : 0;
    static_assert(MODE != 0 || (KT % RK == 0 && N * RK == KT), "mode 0 covers the k-step");
    static_assert(MODE != 1 || (TX % CX == 0 && N * CX == TX), "mode 1 covers the tile's free entries");
    __device__ static __forceinline__ int k0(int tid) {
        const int lane = tid & 63, w = tid >> 6;
        if (MODE == 0) return tid / LX;
        return VEC ? 2 * ((lane & 3) + 4 * (lane >> 5) + 8 * (w % KB)) : (lane & 15) + 16 * (w % KB);
    }
    __device__ static __forceinline__ int x0(int tid) {
        const int lane = tid & 63, w = tid >> 6;
        if (MODE == 0) return (VEC ? 2 : 1) * (tid % LX);
        return VEC ? ((lane >> 2) & 7) + 8 * (w / KB) : (lane >> 4) + 4 * (w / KB);
    }
};

// Per-thread LDS addresses of one operand for the unchecked gather: table entries and staging position.
struct Bases {
    const int64_t* fix;   // &fix_tab[0][x0]
    const int64_t* step;  // &step_tab[slot 0][0][k0]
    double* stage;        // &tile[buffer 0][k0 * PITCH + x0]
    int64_t fixv[4];      // lanes along the free entries: every load of a thread has the same x, its table entries live here
};

// Issue the loads of one k-step for every term; absent terms (index >= nterms) contribute zeros.
template <int MODE, int NT, int KT, bool VEC, bool EXACT, int TX>
__device__ __forceinline__ void issue_fast(double (&ld)[NT][TX * KT / NTHREADS], const Bases& b, int slot_off, int nterms) {
    typedef Map<MODE, KT, VEC, TX> M;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        if (!EXACT && t > 0 && t >= nterms) {
#pragma unroll
            for (int e = 0; e < M::NE; ++e) ld[t][e] = 0.0;
        } else {
#pragma unroll
            for (int e = 0; e < M::N; ++e) {
                const int64_t addr = (M::CX == 0 ? b.fixv[t] : b.fix[t * TX + M::CX * e]) + b.step[slot_off + t * KT + M::CK * e];
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

// Gather without tables, for operands whose row and column scatter vectors are both runs of a constant stride
// (plain matrices, the dense temporaries; what the block scatter vectors of Sec. 2.3 call regular): the address of
// load e of term t is a wave-uniform base (scalar registers, scalar arithmetic) plus one per-lane 32-bit offset
// that never changes.  No LDS reads and no vector ALU work per load.  Pairs only (VEC mapping).
template <int NT>
struct Affine {
    uint32_t voff;    // per lane: byte offset of its element pair inside the wave's patch
    int64_t u0[NT];   // per term: byte address of the wave's patch for load 0 of k-step 0
    int64_t dE, dS;   // bytes from one load to the next, from one k-step to the next
    int last;         // last k-step that exists: gathers issued ahead of the end read that one again
};

// BUF: the loads are buffer loads, whose descriptor base (scalar registers), scalar offset and per-lane offset are
// added by the address unit, where a global load needs a 64-bit vector add per load.  Measured at 16384^3: the
// two-term families gain 1 % from buffer loads; the (1,1) family with two k-steps in flight loses 2 % (its issue
// points were tuned with the adds between the loads) and the four-term families lose 6 % (four descriptors per
// operand spill scalar registers), so those keep global loads.  (Global loads in their scalar-base form, which
// also needs no vector add, measured 2 % slower for the (1,1) family as well: back-to-back loads without the adds
// between them delay the matrix-core instructions of the partner wave more.)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

template <int MODE, int NT, int KT, bool BUF, int TX>
__device__ __forceinline__ void issue_affine(double (&ld)[NT][TX * KT / NTHREADS], const Affine<NT>& a, int target) {
    typedef Map<MODE, KT, true, TX> M;
    typedef const __attribute__((address_space(1))) char* gbyte_t;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int64_t ub = a.u0[t] + (int64_t)(target < a.last ? target : a.last) * a.dS;
        if constexpr (BUF) {
            // raw buffer over the address space from ub on: no stride, no range limit that matters
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)ub, 0, -1, 0x00020000);
#pragma unroll
            for (int e = 0; e < M::N; ++e) {
                const double2_t v =
                    __builtin_bit_cast(double2_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)a.voff, (int)(e * a.dE), 0));
                ld[t][2 * e] = v.x;
                ld[t][2 * e + 1] = v.y;
            }
        } else {
#pragma unroll
            for (int e = 0; e < M::N; ++e) {
                const double2_t v = *(gdbl2_t)((gbyte_t)(ub + e * a.dE) + a.voff);
                ld[t][2 * e] = v.x;
                ld[t][2 * e + 1] = v.y;
            }
        }
    }
}

// A wave-uniform value, marked as such for the compiler (it then lives in scalar registers and everything derived
// from it is scalar arithmetic; without the mark a value that crosses a branch can end up in a vector register, and
// a buffer load whose scalar operand sits there is turned into a loop over the lanes).
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const int lo = __builtin_amdgcn_readfirstlane((int)(uint32_t)(uint64_t)v);
    const int hi = __builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// Per-operand set-up of the table-free gather.  sx / sk: element strides along the free / the contracted bundle;
// fx: element offset of the tile's first free entry in each term (its scatter entry); offk: first contracted entry of
// each term.
template <int MODE, int NT, int KT, int TX>
__device__ __forceinline__ void setup_affine(Affine<NT>& a, const double* base, int64_t sx, int64_t sk, const int64_t (&fx)[NT], const int64_t* offk,
                                             int tid, int last) {
    typedef Map<MODE, KT, true, TX> M;
    // the wave's patch starts at the element of its lane 0; every other lane is a fixed distance from it
    const int t0 = tid & ~63;
    const int wk = __builtin_amdgcn_readfirstlane(M::k0(t0)), wx = __builtin_amdgcn_readfirstlane(M::x0(t0));
    a.voff = (uint32_t)(8 * ((M::k0(tid) - wk) * sk + (M::x0(tid) - wx) * sx));
    a.dE = uniform64(MODE == 0 ? 8 * M::CK * sk : 8 * M::CX * sx);
    a.dS = uniform64(8 * KT * sk);
    a.last = __builtin_amdgcn_readfirstlane(last);
#pragma unroll
    for (int t = 0; t < NT; ++t) a.u0[t] = uniform64((int64_t)base + 8 * (fx[t] + wx * sx + (offk[t] + wk) * sk));
}

// The packing rule of Sec. 4.1 applied to a tile: its TX free entries [off[t] + tile0, + TX) of every term are
// regular iff every block scatter entry involved is non-zero (the entries are then equal) and consecutive blocks join
// up with the same stride; only then may the tile be gathered by stride.  bs: block scatter vector for blocks of 16
// entries (block offsets and tile origins are multiples of 16).  Lane l of the wave looks at block l % 8 of term l / 8.
// Returns the common stride and each term's first scatter entry; every wave of the workgroup computes the same answer.
template <int NT, int TX>
__device__ __forceinline__ bool tile_regular(gvec_t scat, gvec_t bs, const int64_t* off, int64_t tile0, int lane, int64_t& stride,
                                             int64_t (&first)[NT]) {
    static_assert(NT * 8 <= 64, "one lane per block and term");
    const int t = (lane >> 3) < NT && (lane & 7) < TX / 16 ? (lane >> 3) : NT, j = lane & 7;  // (a 64-wide tile has four blocks)
    int64_t v = 0, f = 0;
    bool ok = true;
    if (t < NT) {
        const int64_t f0 = off[t] + tile0 + 16 * j;
        v = bs[f0 >> 4];
        f = scat[f0];
        ok = v > 0 && (j == 0 || f - scat[f0 - 1] == v);
    }
    const int64_t s0 = uniform64(v);  // lane 0: block 0 of term 0
    ok = ok && (t >= NT || v == s0);
    if (!__all(ok ? 1 : 0)) return false;
    stride = s0;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
        const int lo = __builtin_amdgcn_readlane((int)(uint32_t)(uint64_t)f, 8 * u);
        const int hi = __builtin_amdgcn_readlane((int)(uint32_t)((uint64_t)f >> 32), 8 * u);
        first[u] = (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
    }
    return true;
}

// Signed sum of the terms (the operand sum of Sec. 4.1) into the LDS tile.
template <int MODE, int NT, int KT, bool VEC, bool UNIT, int TX>
__device__ __forceinline__ void stage_fast(const double (&ld)[NT][TX * KT / NTHREADS], double* __restrict__ dst, const double* __restrict__ coef) {
    typedef Map<MODE, KT, VEC, TX> M;
#pragma unroll
    for (int e = 0; e < M::N; ++e) {
        double v[2];
#pragma unroll
        for (int h = 0; h < (VEC ? 2 : 1); ++h) {
            const int i = VEC ? 2 * e + h : e;
            if (NT == 1) {
                v[h] = UNIT ? ld[0][i] : coef[0] * ld[0][i];
            } else {
                v[h] = UNIT ? ld[0][i] : coef[0] * ld[0][i];
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
template <int MODE, int NT, int KT, int TX>
__device__ __forceinline__ void issue_checked(double (&ld)[NT][TX * KT / NTHREADS], unsigned& padmask, const double* __restrict__ safe,
                                              const int64_t* __restrict__ fixed_tab, const int64_t* __restrict__ step_tab, int nterms, int tid) {
    typedef Map<MODE, KT, false, TX> M;
    constexpr int NE = M::NE;
    const int k0 = M::k0(tid), x0 = M::x0(tid);
    padmask = 0;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int e = 0; e < NE; ++e) {
            if (t > 0 && t >= nterms) {
                ld[t][e] = 0.0;
            } else {
                const int64_t addr = fixed_tab[t * TX + x0 + M::CX * e] + step_tab[t * KT + k0 + M::CK * e];
                padmask |= (addr < 0 ? 1u : 0u) << (t * NE + e);
                ld[t][e] = *(gdbl_t)(addr < 0 ? (int64_t)safe : addr);
            }
        }
    }
}

template <int MODE, int NT, int KT, int TX>
__device__ __forceinline__ void stage_checked(const double (&ld)[NT][TX * KT / NTHREADS], unsigned padmask, double* __restrict__ tile,
                                              const double* __restrict__ coef, int tid) {
    typedef Map<MODE, KT, false, TX> M;
    constexpr int NE = M::NE;
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

// ---- the same four steps for a part of a tile: loads [E0, E1) of every term (rolling gather, Cfg::ROLL) ----
template <int MODE, int NT, int KT, bool VEC, int TX, int E0, int E1>
__device__ __forceinline__ void issue_fast_part(double (&ld)[NT][TX * KT / NTHREADS], const Bases& b, int slot_off) {
    typedef Map<MODE, KT, VEC, TX> M;
#pragma unroll
    for (int e = E0; e < E1; ++e) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int64_t addr = (M::CX == 0 ? b.fixv[t] : b.fix[t * TX + M::CX * e]) + b.step[slot_off + t * KT + M::CK * e];
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

template <int MODE, int NT, int KT, bool BUF, int TX, int E0, int E1>
__device__ __forceinline__ void issue_affine_part(double (&ld)[NT][TX * KT / NTHREADS], const Affine<NT>& a, int target) {
    typedef const __attribute__((address_space(1))) char* gbyte_t;
    // Without buffer descriptors: the per-lane offset is re-read through an empty asm statement so that its widening
    // to 64 bits stays next to the loads, which then take the scalar base + 32-bit lane offset form (no vector add).
    uint32_t vo = a.voff;
    if constexpr (!BUF) asm volatile("" : "+v"(vo));
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int64_t ub = a.u0[t] + (int64_t)(target < a.last ? target : a.last) * a.dS;
        if constexpr (BUF) {
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)ub, 0, -1, 0x00020000);
#pragma unroll
            for (int e = E0; e < E1; ++e) {
                const double2_t v =
                    __builtin_bit_cast(double2_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)a.voff, (int)(e * a.dE), 0));
                ld[t][2 * e] = v.x;
                ld[t][2 * e + 1] = v.y;
            }
        } else {
#pragma unroll
            for (int e = E0; e < E1; ++e) {
                const double2_t v = *(gdbl2_t)((gbyte_t)(ub + e * a.dE) + vo);
                ld[t][2 * e] = v.x;
                ld[t][2 * e + 1] = v.y;
            }
        }
    }
}

template <int MODE, int NT, int KT, bool VEC, bool UNIT, int TX, int E0, int E1>
__device__ __forceinline__ void stage_fast_part(const double (&ld)[NT][TX * KT / NTHREADS], double* __restrict__ dst, const double* __restrict__ coef) {
    typedef Map<MODE, KT, VEC, TX> M;
#pragma unroll
    for (int e = E0; e < E1; ++e) {
        double v[2];
#pragma unroll
        for (int h = 0; h < (VEC ? 2 : 1); ++h) {
            const int i = VEC ? 2 * e + h : e;
            v[h] = UNIT ? ld[0][i] : coef[0] * ld[0][i];
#pragma unroll
            for (int t = 1; t < NT; ++t) v[h] = __builtin_fma(coef[t], ld[t][i], v[h]);
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

template <int MODE, int NT, int KT, int TX, int E0, int E1>
__device__ __forceinline__ void issue_checked_part(double (&ld)[NT][TX * KT / NTHREADS], unsigned& padmask, const double* __restrict__ safe,
                                                   const int64_t* __restrict__ fixed_tab, const int64_t* __restrict__ step_tab, int tid) {
    typedef Map<MODE, KT, false, TX> M;
    constexpr int NE = M::NE;
    const int k0 = M::k0(tid), x0 = M::x0(tid);
#pragma unroll
    for (int e = E0; e < E1; ++e) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int64_t addr = fixed_tab[t * TX + x0 + M::CX * e] + step_tab[t * KT + k0 + M::CK * e];
            const unsigned bit = 1u << (t * NE + e);
            padmask = addr < 0 ? (padmask | bit) : (padmask & ~bit);
            ld[t][e] = *(gdbl_t)(addr < 0 ? (int64_t)safe : addr);
        }
    }
}

template <int MODE, int NT, int KT, int TX, int E0, int E1>
__device__ __forceinline__ void stage_checked_part(const double (&ld)[NT][TX * KT / NTHREADS], unsigned padmask, double* __restrict__ tile,
                                                   const double* __restrict__ coef, int tid) {
    typedef Map<MODE, KT, false, TX> M;
    constexpr int NE = M::NE;
    double* dst = tile + M::k0(tid) * PITCH + M::x0(tid);
#pragma unroll
    for (int e = E0; e < E1; ++e) {
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

template <int AMODE, int BMODE, class CF, bool VA, bool VB>
struct State {
    static constexpr int KT = CF::KT, NEA = CF::NEA, NEB = CF::NEB, NQ = CF::NQ, TILE = CF::TILE, D = CF::D, SETS = CF::SETS, NTA = CF::NTA,
                         NTB = CF::NTB;
    static_assert(NTA * NEA <= 32 && NTB * NEB <= 32, "padding masks are 32 bits");
    Smem<CF>* S;
    const Product* P;
    int tid, nA, nB, nk, kfull;
    bool unitA, unitB;         // the first coefficient is +1
    bool early;                // first of the two waves of its SIMD
    bool all_fast;             // no k-step needs checks: gathers issued ahead of the end re-read entries that exist
    double coefA[NTA], coefB[NTB];
    const double *safeA, *safeB;
    // scatter entries of later k-steps
    gvec_t ent_ptr;
    int ent_limit;             // k entries that exist for this thread's term, counted from its own k
    int64_t* ent_dst;
    int ent_stride;            // distance between the two table slots at ent_dst
    Bases ba, bb;
    // per-lane fragment bases
    const double* fa;
    static constexpr int NS = TC_MFMA16 ? 1 : 4;  // B fragments per 16 x 16 output patch (rotations of the four column blocks)
    const double* fb[NS];
#if TC_MFMA16
    double4_t acc[4][2];
#else
    double acc[4][2][4];
#endif
    double la[SETS][NTA][NEA], lb[SETS][NTB][NEB];  // register sets of the gathers in flight
    unsigned pa[SETS], pb[SETS];
    bool issued_fast[SETS];    // the loads of a set were issued without padding checks
    Affine<NTA> afa;           // table-free gather (valid when the product qualifies)
    Affine<NTB> afb;

    // gather of k-step `target` into register set SET, with the table slot SLOT (= target % 2).
    // FAST: the caller knows that the k-step has no padding (target < kfull); otherwise that is decided here.
    template <int SET, int SLOT, bool FAST, bool AFF = false>
    __device__ __forceinline__ void issue(int target) {
        if constexpr (FAST && AFF) {
            constexpr bool BUF = SETS == 1 && NTA <= 2 && NTB <= 2;  // (four descriptors per operand would spill scalar registers)
            issue_affine<AMODE, NTA, KT, BUF, TM>(la[SET], afa, target);
            issue_affine<BMODE, NTB, KT, BUF, TN>(lb[SET], afb, target);
            return;
        }
        if (!FAST) issued_fast[SET] = target < kfull;
        if (FAST || issued_fast[SET]) {
            issue_fast<AMODE, NTA, KT, VA, CF::EXACT, TM>(la[SET], ba, SLOT * NTA * KT, nA);
            issue_fast<BMODE, NTB, KT, VB, CF::EXACT, TN>(lb[SET], bb, SLOT * NTB * KT, nB);
        } else {
            issue_checked<AMODE, NTA, KT, TM>(la[SET], pa[SET], safeA, &S->a_fix[0][0], &S->a_step[SLOT][0][0], nA, tid);
            issue_checked<BMODE, NTB, KT, TN>(lb[SET], pb[SET], safeB, &S->b_fix[0][0], &S->b_step[SLOT][0][0], nB, tid);
        }
    }

    // operand sums of register set SET into LDS buffer BUF
    // UNIT: the first coefficient of both operand sums is +1 (a single term is then stored as loaded)
    template <int SET, int BUF, bool FAST, bool UNIT>
    __device__ __forceinline__ void stage() {
        if (FAST || issued_fast[SET]) {
            stage_fast<AMODE, NTA, KT, VA, UNIT, TM>(la[SET], ba.stage + BUF * TILE, coefA);
            stage_fast<BMODE, NTB, KT, VB, UNIT, TN>(lb[SET], bb.stage + BUF * TILE, coefB);
        } else {
            stage_checked<AMODE, NTA, KT, TM>(la[SET], pa[SET], &S->a[BUF][0], coefA, tid);
            stage_checked<BMODE, NTB, KT, TN>(lb[SET], pb[SET], &S->b[BUF][0], coefB, tid);
        }
    }

    // Rolling gather: part G of a k-step's tile.  Parts 0 .. NQ/2 - 1 belong to A, the others to B; part g of an
    // operand is registers [g * PER, (g + 1) * PER) of every term, whatever mapping loaded them.  Whether a k-step was
    // (and is) gathered without padding checks follows from its number alone.
    // roll_stage: part G of k-step `target` (in flight in the set) goes to LDS buffer BUF.
    template <int BUF, int G, bool FAST, bool UNIT>
    __device__ __forceinline__ void roll_stage(int target) {
        constexpr int H = NQ / 2;
        constexpr bool IS_A = G < H;
        constexpr int g = IS_A ? G : G - H, PER = (IS_A ? NEA : NEB) / H;
        constexpr int S0 = g * PER, S1 = (g + 1) * PER;  // as scalar loads
        const bool fast = FAST || target < kfull;
        if constexpr (IS_A) {
            constexpr int E0 = VA ? S0 / 2 : S0, E1 = VA ? S1 / 2 : S1;
            if (fast)
                stage_fast_part<AMODE, NTA, KT, VA, UNIT, TM, E0, E1>(la[0], ba.stage + BUF * TILE, coefA);
            else
                stage_checked_part<AMODE, NTA, KT, TM, S0, S1>(la[0], pa[0], &S->a[BUF][0], coefA, tid);
        } else {
            constexpr int E0 = VB ? S0 / 2 : S0, E1 = VB ? S1 / 2 : S1;
            if (fast)
                stage_fast_part<BMODE, NTB, KT, VB, UNIT, TN, E0, E1>(lb[0], bb.stage + BUF * TILE, coefB);
            else
                stage_checked_part<BMODE, NTB, KT, TN, S0, S1>(lb[0], pb[0], &S->b[BUF][0], coefB, tid);
        }
    }
    // roll_issue: the loads of part G of k-step `target`, with table slot SLOT (= target % 2)
    template <int SLOT, int G, bool FAST, bool AFF>
    __device__ __forceinline__ void roll_issue(int target) {
        constexpr int H = NQ / 2;
        constexpr bool IS_A = G < H;
        constexpr int g = IS_A ? G : G - H, PER = (IS_A ? NEA : NEB) / H;
        constexpr int S0 = g * PER, S1 = (g + 1) * PER;
        constexpr bool BUF = NTA <= 2 && NTB <= 2;  // (four descriptors per operand would spill scalar registers)
        const bool fast = FAST || target < kfull;
        if constexpr (IS_A) {
            constexpr int E0 = VA ? S0 / 2 : S0, E1 = VA ? S1 / 2 : S1;
            if constexpr (FAST && AFF) {
                issue_affine_part<AMODE, NTA, KT, BUF, TM, S0 / 2, S1 / 2>(la[0], afa, target);
            } else {
                if (fast)
                    issue_fast_part<AMODE, NTA, KT, VA, TM, E0, E1>(la[0], ba, SLOT * NTA * KT);
                else
                    issue_checked_part<AMODE, NTA, KT, TM, S0, S1>(la[0], pa[0], safeA, &S->a_fix[0][0], &S->a_step[SLOT][0][0], tid);
            }
        } else {
            constexpr int E0 = VB ? S0 / 2 : S0, E1 = VB ? S1 / 2 : S1;
            if constexpr (FAST && AFF) {
                issue_affine_part<BMODE, NTB, KT, BUF, TN, S0 / 2, S1 / 2>(lb[0], afb, target);
            } else {
                if (fast)
                    issue_fast_part<BMODE, NTB, KT, VB, TN, E0, E1>(lb[0], bb, SLOT * NTB * KT);
                else
                    issue_checked_part<BMODE, NTB, KT, TN, S0, S1>(lb[0], pb[0], safeB, &S->b_fix[0][0], &S->b_step[SLOT][0][0], tid);
            }
        }
    }
    // Every part of k-step `target`, in the order in which the loop turns the parts over (the hardware returns loads
    // in issue order and the waits count loads, so the loop's first trip must find them in that order).
    template <int SLOT, bool FAST, bool AFF, int G = 0>
    __device__ __forceinline__ void roll_issue_all(int target) {
        if constexpr (G < NQ) {
            roll_issue<SLOT, G, FAST, AFF>(target);
            roll_issue_all<SLOT, FAST, AFF, G + 1>(target);
        }
    }

    template <int CUR, int Q>
    __device__ __forceinline__ void read_frags(double (&af)[4], double (&bf)[2 * NS]) {
        constexpr int ROW = 16 * (Q / 4) + (Q % 4);
#pragma unroll
        for (int xp = 0; xp < 2; ++xp) {
            const double2_t v = *reinterpret_cast<const double2_t*>(fa + CUR * TILE + ROW * PITCH + xp * 32);
            af[2 * xp] = v.x;
            af[2 * xp + 1] = v.y;
        }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const double2_t v = *reinterpret_cast<const double2_t*>(fb[s] + CUR * TILE + ROW * PITCH);
            bf[s] = v.x;
            bf[NS + s] = v.y;
        }
    }

    __device__ __forceinline__ void multiply(const double (&af)[4], const double (&bf)[2 * NS]) {
#if TC_MFMA16
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int x = 0; x < 4; ++x) acc[x][y] = __builtin_amdgcn_mfma_f64_16x16x4f64(af[x], bf[y], acc[x][y], 0, 0, 0);
#else
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                    acc[x][y][s] = __builtin_amdgcn_mfma_f64_4x4x4f64(af[x], bf[y * 4 + s], acc[x][y][s], 0, 0, 0);
#endif
    }

    // With one register set the compiler must not move the waits for gathered data up into the MFMA groups;
    // with two sets the data has long arrived and free scheduling measured faster.
    __device__ static __forceinline__ void pin() {
        if constexpr (CF::PIN) __builtin_amdgcn_sched_barrier(0);
    }

    // What a wave does besides MFMAs once DONE instruction groups of k-step `step` (LDS buffer CUR) are complete.
    // D = 2, two sets: the loads of step + 2 go to register set CUR (its previous contents, k-step `step`, were
    //        stored one step ago), and set CUR ^ 1 (k-step step + 1, issued one step ago) is stored to LDS buffer CUR ^ 1.
    // ROLL (D = 2, one set): part G of the set (k-step step + 1, issued one step ago) is stored to LDS buffer CUR ^ 1
    //        and that part's loads of step + 2 are issued into the same registers right away.
    // D = 1: the loads of step + 1 are issued and, after the last group, stored.
    // ROLE: 0 = first wave of the SIMD, 1 = second, 2 = decided at run time (member `early`).
    template <int CUR, int DONE, int ROLE, bool FAST, bool UNIT, bool AFF>
    __device__ __forceinline__ void between_groups(int step) {
        constexpr int NXT = CUR ^ 1;
        if constexpr (CF::ROLL) {
            constexpr int G = DONE - 1;  // part g is turned over after instruction group g
            if constexpr (G >= 0 && G < NQ) {
                pin();
                roll_stage<NXT, G, FAST, UNIT>(step + 1);
                roll_issue<CUR, G, FAST, AFF>(step + 2);
                pin();
            }
        } else {
            constexpr int ISET = (D == 2) ? CUR : 0, SSET = (D == 2) ? NXT : 0, ISLOT = (D == 2) ? CUR : NXT;
            if constexpr (ROLE != 1 && DONE == CF::STAGE_EARLY) {
                pin();
                if (ROLE == 0 || early) stage<SSET, NXT, FAST, UNIT>();
                pin();
            }
            if constexpr (ROLE != 0 && DONE == CF::STAGE_LATE) {
                pin();
                if (ROLE == 1 || !early) stage<SSET, NXT, FAST, UNIT>();
                pin();
            }
            if constexpr (ROLE != 1 && DONE == 0) {
                pin();
                if (ROLE == 0 || early) issue<ISET, ISLOT, FAST, AFF>(step + D);
                pin();
            }
            if constexpr (ROLE != 0 && DONE == CF::ISSUE_LATE) {
                pin();
                if (ROLE == 1 || !early) issue<ISET, ISLOT, FAST, AFF>(step + D);
                pin();
            }
        }
    }

    // instruction groups Q .. NQ-1 of the k-step in LDS buffer CUR; the fragments of group Q are in af/bf[Q % 2] and
    // those of group Q + 1 are read while group Q multiplies
    template <int CUR, int Q, int ROLE, bool FAST, bool UNIT, bool AFF>
    __device__ __forceinline__ void groups(double (&af)[2][4], double (&bf)[2][2 * NS], int step) {
        if constexpr (Q < NQ) {
            if constexpr (Q + 1 < NQ) read_frags<CUR, Q + 1>(af[(Q + 1) & 1], bf[(Q + 1) & 1]);
            // D = 2: a wave in the first half of its k-step outranks its SIMD partner in the second half, which
            // keeps the two from drifting far apart (measured +1.5 %; with D = 1 it costs 2 %)
            if constexpr (SETS == 2 && (Q * 2) % NQ == 0) __builtin_amdgcn_s_setprio(1 - (Q * 2) / NQ);
            multiply(af[Q & 1], bf[Q & 1]);
            between_groups<CUR, Q + 1, ROLE, FAST, UNIT, AFF>(step);
            groups<CUR, Q + 1, ROLE, FAST, UNIT, AFF>(af, bf, step);
        }
    }

    // One k-step.  The scatter entries of k-step step + D + 1 are fetched first (so that waiting for them at the end
    // of the step does not wait for the gather issued after them) and stored to the free table slot at the end.
    template <int CUR, int ROLE, bool FAST, bool UNIT, bool AFF>
    __device__ __forceinline__ void step_body(int step) {
        constexpr int ESLOT = (D == 2) ? (CUR ^ 1) : CUR;
        const int kn = (step + D + 1) * KT;
        const bool have = kn < ent_limit;
        int64_t raw_entry = 0;
        constexpr bool NOENT = AFF && CF::NOENT_AFF;
        if constexpr (!NOENT) raw_entry = ent_ptr[have ? kn : 0];  // unconditional load: ent_ptr always points at readable memory

        between_groups<CUR, 0, ROLE, FAST, UNIT, AFF>(step);
        double af[2][4], bf[2][2 * NS];
        read_frags<CUR, 0>(af[0], bf[0]);
        groups<CUR, 0, ROLE, FAST, UNIT, AFF>(af, bf, step);

        // every thread stores: no branch around the wait.  (Past the end raw_entry is the thread's first entry.)
        // The table-free loop runs to the tile's last k-step and needs no entries at all.
        if constexpr (!NOENT) ent_dst[ESLOT ? ent_stride : 0] = (have || all_fast) ? raw_entry * 8 : kSentinel;
        __syncthreads();
    }

    // k-steps [0, end) (end even) of a tile whose gathers up to k-step end + D - 1 need no padding checks.  The
    // wave's role is a compile-time property of this loop and there is no control flow inside it, so the compiler's
    // wait counts for the loads in flight are exact.
    template <int ROLE, bool UNIT, bool AFF>
    __device__ __forceinline__ void run_fast(int end) {
        // A rolling gather enters its loop with k-step 1 in flight, issued here, straight ahead of the loop and in
        // the loop's own order, so that the loop's load counts are exact from its first trip on.
        if constexpr (CF::ROLL) {
            roll_issue_all<1, true, AFF>(1);
            if constexpr (!(AFF && CF::NOENT_AFF)) __syncthreads();  // table slot 1 has been read by every thread (step 0 refills it)
        }
        for (int step = 0; step < end; step += 2) {
            step_body<0, ROLE, true, UNIT, AFF>(step);
            step_body<1, ROLE, true, UNIT, AFF>(step + 1);
        }
    }
    template <int ROLE, bool UNIT>
    __device__ __forceinline__ void run_fast(int end, bool affine) {
        if constexpr (VA && VB) {
            if (affine) {
                run_fast<ROLE, UNIT, true>(end);
                return;
            }
        }
        run_fast<ROLE, UNIT, false>(end);
    }

    // k-steps [begin, nk) (both even): padding decided per k-step
    __device__ __forceinline__ void run_checked(int begin) {
        if constexpr (CF::ROLL) {
            if (begin == 0) {
                roll_issue_all<1, false, false>(1);
                __syncthreads();  // table slot 1 has been read by every thread (step 0 refills it)
            }
        }
        for (int step = begin; step < nk; step += 2) {
            step_body<0, 2, false, false, false>(step);
            step_body<1, 2, false, false, false>(step + 1);
        }
    }
};

// Which tile a logical workgroup id stands for: product pidx of the launch, tile row tm, tile column tn.  Ids walk
// GROUP_M tile rows at a time, so that workgroups resident together share A and B panels in their XCD's L2.
struct TileId {
    int pidx, tm, tn;
};
__device__ __forceinline__ TileId tile_of(int lid, int tiles_m, int tiles_n) {
    const int per_prod = tiles_m * tiles_n;
    TileId t;
    t.pidx = lid / per_prod;
    int rem = lid - t.pidx * per_prod;
    const int gsz = GROUP_M * tiles_n;
    const int grp = rem / gsz;
    const int gm0 = grp * GROUP_M;
    const int gh = (tiles_m - gm0) < GROUP_M ? (tiles_m - gm0) : GROUP_M;
    rem -= grp * gsz;
    t.tm = gm0 + rem % gh;
    t.tn = rem / gh;
    return t;
}

// The same with the divisions done by multiplication, so that they stay on the scalar unit (an integer division by
// a run-time value compiles to vector floating-point code, and vector instructions of a workgroup that is setting
// up its tile wait for the matrix-core instructions of the workgroup it shares the compute unit with).
// TileDiv holds floor(2^32 / d) for the three divisors (2^32 - 1 for d = 1), computed by the host.
struct TileDiv {
    unsigned per_prod, gsz, gh_last, tail_tiles;
};
__host__ inline unsigned tile_div_rcp(int64_t d) { return d <= 1 ? 0xffffffffu : (unsigned)(((uint64_t)1 << 32) / (uint64_t)d); }
// x / d and the remainder for x < 2^32, d >= 1: the estimate from rcp is at most one too small
__device__ __forceinline__ unsigned div_by(unsigned x, unsigned d, unsigned rcp, unsigned& rem) {
    unsigned q = __umulhi(x, rcp);
    unsigned r = x - q * d;
    if (r >= d) ++q, r -= d;
    if (r >= d) ++q, r -= d;
    rem = r;
    return q;
}
__device__ __forceinline__ TileId tile_of(int lid, int tiles_m, int tiles_n, const TileDiv& dv) {
    TileId t;
    unsigned rem, in_group, rest;
    t.pidx = (int)div_by((unsigned)lid, (unsigned)(tiles_m * tiles_n), dv.per_prod, rem);
    const int grp = (int)div_by(rem, (unsigned)(GROUP_M * tiles_n), dv.gsz, in_group);
    const int gm0 = grp * GROUP_M;
    if (tiles_m - gm0 >= GROUP_M) {
        t.tm = gm0 + (int)(in_group % GROUP_M);
        t.tn = (int)(in_group / GROUP_M);
    } else {  // the last, shorter group of tile rows
        t.tn = (int)div_by(in_group, (unsigned)(tiles_m - gm0), dv.gh_last, rest);
        t.tm = gm0 + (int)rest;
    }
    return t;
}

// Workgroups [0, main_count) compute one whole tile each.  The tiles left over after the last full round of the
// machine (tail_tiles of them, logical ids main_count ...) are cut along the contracted bundle into chunks of tail_kc
// entries, one workgroup per (tile, chunk): workgroup main_count + c * tail_tiles + t stores the raw accumulators of
// chunk c of tail tile t as a dense TM x TN tile at partial + TM * TN * (c * tail_tiles + t); tail_fixup_kernel adds
// the chunks in a fixed order and updates the destinations.
template <int AMODE, int BMODE, class CF, bool VA, bool VB>
__global__ __launch_bounds__(NTHREADS, 2) void fused_kernel(const Product* __restrict__ prods, int first, int tiles_m, int tiles_n,
                                                            const double* __restrict__ Au, const double* __restrict__ Bu,
                                                            double* __restrict__ Cu, double* __restrict__ W, double alpha, double beta, int c_mode,
                                                            int main_count, int tail_tiles, int tail_kc, double* __restrict__ partial,
                                                            TileDiv tdiv) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    Smem<CF>& S = *reinterpret_cast<Smem<CF>*>(smem_raw);
    const int tid = threadIdx.x;
    typedef State<AMODE, BMODE, CF, VA, VB> St;
    constexpr int KT = CF::KT, NTA = CF::NTA, NTB = CF::NTB, D = CF::D, SETS = CF::SETS;

    // ---- which tile ----
    const int bid = blockIdx.x;
    const bool part = bid >= main_count;  // a chunk of a tail tile
    int lid;
    int64_t kbeg = 0;
    if (!part) {
        // Block b runs on XCD b % 8.  Each round of the device (one or two blocks per compute unit) hands every XCD a run of consecutive logical ids (tiles that
        // share panels of A and B in that XCD's L2), so the tiles of the ragged last rows, which run the slower
        // checked loops, are spread over all XCDs; ids are walked from the last to the first, so that those tiles
        // are not the ones everything else waits for at the end.
        constexpr int ROUND = 256 * WGS_PER_CU, PX = ROUND / 8;  // workgroups per round of the device, per XCD
        const int whole_rounds = main_count / ROUND * ROUND;
        int v = bid;
        if (bid < whole_rounds) {
            const int q = bid >> 3;
            v = ((q / PX) * 8 + (bid & 7)) * PX + (q % PX);
        }
        lid = main_count - 1 - v;
    } else {
        unsigned t;
        const unsigned chunk = div_by((unsigned)(bid - main_count), (unsigned)tail_tiles, tdiv.tail_tiles, t);
        lid = main_count + (int)t;
        kbeg = (int64_t)chunk * tail_kc;
    }
    const TileId tile = tile_of(lid, tiles_m, tiles_n, tdiv);
    const Product& P = prods[first + tile.pidx];
    const int64_t i0 = (int64_t)tile.tm * TM, j0 = (int64_t)tile.tn * TN;
    const int nA = CF::EXACT ? NTA : P.A.nterms, nB = CF::EXACT ? NTB : P.B.nterms;
    const int64_t kb = part ? min64(P.kb - kbeg, (int64_t)tail_kc) : P.kb;  // contracted entries of this workgroup
    // a chunk sees the contracted bundle from entry kbeg on: shifted vectors, shortened lengths
    const int64_t* const acs = P.A.cs + kbeg;
    const int64_t* const brs = P.B.rs + kbeg;
    const int64_t acs_len = P.A.cs_len - kbeg, brs_len = P.B.rs_len - kbeg;

    St st;
    st.S = &S;
    st.P = &P;
    st.tid = tid;
    st.nA = nA;
    st.nB = nB;
    st.nk = (int)((kb + KT - 1) / KT);
    st.nk += st.nk & 1;  // the k loop runs two steps per trip; a k-step past the end gathers only zero padding
    st.unitA = P.A.coef[0] == 1.0;
    st.unitB = P.B.coef[0] == 1.0;
#pragma unroll
    for (int t = 0; t < NTA; ++t) st.coefA[t] = P.A.coef[t];
#pragma unroll
    for (int t = 0; t < NTB; ++t) st.coefB[t] = P.B.coef[t];
    const double* Abase = (P.A.space == 0 ? Au : W) + P.A.base_off;
    const double* Bbase = (P.B.space == 0 ? Bu : W) + P.B.base_off;
    st.safeA = Abase;
    st.safeB = Bbase;
#pragma unroll
    for (int d = 0; d < SETS; ++d) {
        st.pa[d] = st.pb[d] = 0;
        st.issued_fast[d] = false;
    }

    // ---- tile-fixed gather tables; how much of the tile and of the k range is free of zero padding ----
    // A tile at the ragged edge still runs the unchecked loops if every row (column) that some destination keeps is
    // real in every term of A (B): the other rows are then gathered from the tile's first row instead (any readable
    // address will do, the epilogue drops them).  With pair-wise gathers along the rows a term's last odd row counts
    // as missing, since its pair would reach past the block.
    // (Row and column counts fit 32 bits: a launch has at most 2^20 tiles per direction.  In 32 bits these
    // workgroup-wide quantities are computed by the scalar unit; 64-bit comparisons would run on the vector unit.)
    int64_t klimit = kb;         // k entries that are real in every term of both operands
    int minA = TM, minB = TN;    // rows / columns of the tile that are real (and pair-complete) in every term
    int maxCr = 0, maxCc = 0;    // rows / columns that some destination keeps
    bool wholeC = true;          // every destination keeps the whole tile
    int effA[NTA], effB[NTB];
    const int i0s = tile.tm * TM, j0s = tile.tn * TN, mb32 = (int)P.mb, nb32 = (int)P.nb;
    auto clip = [](int v, int hi) { return v < 0 ? 0 : (v > hi ? hi : v); };
    auto least = [](int a, int b) { return a < b ? a : b; };
#pragma unroll
    for (int t = 0; t < NTA; ++t) {
        effA[t] = 0;
        if (t < nA) {
            klimit = min64(klimit, acs_len - P.A.coff[t]);
            effA[t] = clip(least(mb32, (int)P.A.rs_len - (int)P.A.roff[t]) - i0s, TM);
            if (AMODE == 0 && VA) effA[t] &= ~1;
            minA = effA[t] < minA ? effA[t] : minA;
        }
    }
#pragma unroll
    for (int t = 0; t < NTB; ++t) {
        effB[t] = 0;
        if (t < nB) {
            klimit = min64(klimit, brs_len - P.B.roff[t]);
            effB[t] = clip(least(nb32, (int)P.B.cs_len - (int)P.B.coff[t]) - j0s, TN);
            if (BMODE == 0 && VB) effB[t] &= ~1;
            minB = effB[t] < minB ? effB[t] : minB;
        }
    }
    for (int d = 0; d < P.C.nterms; ++d) {
        const int r = clip(least(mb32, (int)P.C.rs_len - (int)P.C.roff[d]) - i0s, TM);
        const int c = clip(least(nb32, (int)P.C.cs_len - (int)P.C.coff[d]) - j0s, TN);
        maxCr = r > maxCr ? r : maxCr;
        maxCc = c > maxCc ? c : maxCc;
        wholeC = wholeC && r == TM && c == TN;
    }
    // Destinations whose rows and columns are each one run of a constant stride, all of the tile inside them: the
    // epilogue computes their addresses (a scalar base per wave and element, a fixed offset per lane) and no scatter
    // entries are fetched for them.
    // (A chunk of a tail tile goes to its dense slot of the partial buffer: the same case.)
    const bool c_affine = part || (wholeC && P.C.rs_stride >= 0 && P.C.cs_stride >= 0 && P.C.rs_stride < ((int64_t)1 << 20) &&
                                   P.C.cs_stride < ((int64_t)1 << 20));
    const bool whole = minA == TM && minB == TN;  // nothing missing at all
    const bool rows_ok = minA == TM || (minA >= 1 && minA >= maxCr), cols_ok = minB == TN || (minB >= 1 && minB >= maxCc);
    const bool tile_full = rows_ok && cols_ok;
    st.kfull = tile_full ? (int)(klimit / KT) : 0;  // k-steps [0, kfull) need no checks
    // No padding anywhere in the tile: the unchecked loop runs to the end.  The gathers it issues for the D k-steps
    // past the end are never used; their table entries (and computed addresses) repeat ones that exist.
    st.all_fast = CF::EXACT && st.kfull == st.nk;
    // Table-free gather (the stride path of Sec. 4.1) for a tile whose operands are regular: along the contracted
    // bundle the whole scatter vector must be one run of a constant stride (known from the plan); along the free
    // bundle either the same holds, or the block scatter vectors say that this tile's 128 rows (columns) are regular
    // in every term.  Gathered pair-wise only.
    constexpr int64_t kStrideLimit = (int64_t)1 << 20;  // keeps the per-lane and per-load byte offsets within 31 bits
    bool affine = false;
    if constexpr (VA && VB && CF::EXACT) {
        // (computed addresses of missing rows would leave the operand.)  A tile whose last k-steps are padded takes
        // the table-free loop for the k-steps before them, if there are any, and the tables for the rest.
        if (whole && (st.all_fast || st.kfull - D >= 2) && P.A.cs_stride >= 0 && P.B.rs_stride >= 0 && P.A.cs_stride < kStrideLimit && P.B.rs_stride < kStrideLimit) {
            int64_t sxA = P.A.rs_stride, sxB = P.B.cs_stride;
            int64_t fA[NTA], fB[NTB];
            bool ok = true;
            if (sxA >= 0) {
#pragma unroll
                for (int t = 0; t < NTA; ++t) fA[t] = (P.A.roff[t] + i0) * sxA;
            } else {
                ok = P.A.rbs != nullptr && tile_regular<NTA, TM>(as_global(P.A.rs), as_global(P.A.rbs), P.A.roff, i0, tid & 63, sxA, fA);
            }
            if (ok) {
                if (sxB >= 0) {
#pragma unroll
                    for (int t = 0; t < NTB; ++t) fB[t] = (P.B.coff[t] + j0) * sxB;
                } else {
                    ok = P.B.cbs != nullptr && tile_regular<NTB, TN>(as_global(P.B.cs), as_global(P.B.cbs), P.B.coff, j0, tid & 63, sxB, fB);
                }
            }
            affine = ok && sxA < kStrideLimit && sxB < kStrideLimit;
            if (affine) {
                // A: free bundle = rows, contracted = columns; B: free bundle = columns, contracted = rows
                setup_affine<AMODE, NTA, KT, TM>(st.afa, Abase + kbeg * P.A.cs_stride, sxA, P.A.cs_stride, fA, P.A.coff, tid, st.nk - 1);
                setup_affine<BMODE, NTB, KT, TN>(st.afb, Bbase + kbeg * P.B.rs_stride, sxB, P.B.rs_stride, fB, P.B.roff, tid, st.nk - 1);
            }
        }
    }
    // Such a tile needs no table for its gathers: its first k-steps (one per register set) are issued here, before
    // the tables are fetched, so that the two latencies overlap.
    if constexpr (VA && VB && CF::EXACT) {
        if (affine) {
            st.template issue<0, 0, true, true>(0);
            if constexpr (SETS == 2) st.template issue<1, 1, true, true>(1);
#pragma unroll
            for (int d = 0; d < SETS; ++d) st.issued_fast[d] = true;
        }
    }
    // A tile that is gathered by stride from its first k-step to its last reads none of the gather tables: they are
    // not filled.  (Set-up work is not free even where its latency is hidden: with two workgroups per compute unit
    // every vector instruction of the one setting up waits for a matrix-core instruction of the other to end.)
    const bool lean = affine && st.all_fast;
    for (int e = tid; e < (lean ? 0 : NTA * TM); e += NTHREADS) {
        const int t = e / TM, x = e % TM;
        int64_t val = kSentinel;
        int eff = 0;
#pragma unroll
        for (int u = 0; u < NTA; ++u) eff = (t == u) ? effA[u] : eff;
        if (t < nA) {
            if (tile_full && x >= eff)
                val = (int64_t)Abase + 8 * as_global(P.A.rs)[P.A.roff[t] + i0];
            else if (i0s + x < mb32 && (int)P.A.roff[t] + i0s + x < (int)P.A.rs_len)
                val = (int64_t)Abase + 8 * as_global(P.A.rs)[P.A.roff[t] + i0 + x];
        }
        S.a_fix[t][x] = val;
    }
    for (int e = tid; e < (lean ? 0 : NTB * TN); e += NTHREADS) {
        const int t = e / TN, x = e % TN;
        int64_t val = kSentinel;
        int eff = 0;
#pragma unroll
        for (int u = 0; u < NTB; ++u) eff = (t == u) ? effB[u] : eff;
        if (t < nB) {
            if (tile_full && x >= eff)
                val = (int64_t)Bbase + 8 * as_global(P.B.cs)[P.B.coff[t] + j0];
            else if (j0s + x < nb32 && (int)P.B.coff[t] + j0s + x < (int)P.B.cs_len)
                val = (int64_t)Bbase + 8 * as_global(P.B.cs)[P.B.coff[t] + j0 + x];
        }
        S.b_fix[t][x] = val;
    }
    // Scatter entries of the destinations (used by the epilogue; fetched here so that their latency is hidden).
    int64_t(*c_rs)[TM] = S.c_rs;
    int64_t(*c_cs)[TN] = S.c_cs;
    // A chunk of a tail tile has one destination: its dense slot of the partial buffer, contiguous along the
    // direction c_mode makes the lanes run, written as is (no alpha, no previous contents).
    const int nC = part ? 1 : P.C.nterms;
    for (int e = tid; e < (c_affine ? 0 : nC * TM); e += NTHREADS) {  // (the entries of destinations that do not exist are never read)
        const int d = e / TM, x = e % TM;
        const int gi = i0s + x, gj = j0s + x;
        int64_t val = kSentinel;
        if (part) {
            if (d == 0) val = c_mode == 0 ? x : TN * x;
        } else if (d < nC && gi < mb32 && (int)P.C.roff[d] + gi < (int)P.C.rs_len) {
            val = as_global(P.C.rs)[P.C.roff[d] + gi];
        }
        c_rs[d][x] = val;
        val = kSentinel;
        if (part) {
            if (d == 0) val = c_mode == 0 ? TM * x : x;
        } else if (d < nC && gj < nb32 && (int)P.C.coff[d] + gj < (int)P.C.cs_len) {
            val = as_global(P.C.cs)[P.C.coff[d] + gj];
        }
        if (x < TN) c_cs[d][x] = val;
    }
    // Threads 0..KT*NTA-1 fetch the column scatter entries of A for a k-step (one per term and k), the second half
    // of the workgroup (from thread NTHREADS / 2 on) the row scatter entries of B, D + 1 k-steps ahead of the tile that uses them.
    static_assert(KT * NTA <= NTHREADS / 2 && KT * NTB <= NTHREADS / 2, "one owner thread per table entry");
    st.ent_ptr = as_global(reinterpret_cast<const int64_t*>(&P));  // dummy target for threads without an entry
    st.ent_limit = 0;
    st.ent_dst = &S.dump[0][0];
    st.ent_stride = 64;
    if (!lean) {
        const bool isB = tid >= NTHREADS / 2;
        const int q = tid % (NTHREADS / 2), t = q / KT, kl = q % KT;
        if (t < (isB ? NTB : NTA)) {
            const Operand& op = isB ? P.B : P.A;
            st.ent_dst = isB ? &S.b_step[0][t][kl] : &S.a_step[0][t][kl];
            st.ent_stride = (isB ? NTB : NTA) * KT;
            if (t < (isB ? nB : nA)) {
                const int64_t off0 = isB ? op.roff[t] : op.coff[t];
                const int64_t avail = min64(kb, (isB ? brs_len : acs_len) - off0) - kl;
                if (avail > 0) {  // otherwise the thread keeps the dummy target and stores sentinels
                    st.ent_ptr = as_global(isB ? brs : acs) + off0 + kl;
                    st.ent_limit = (int)avail;
                }
            }
        }
    }
    st.ent_dst[0] = (0 < st.ent_limit) ? 8 * st.ent_ptr[0] : kSentinel;
    st.ent_dst[st.ent_stride] = (KT < st.ent_limit) ? 8 * st.ent_ptr[KT] : kSentinel;
    __syncthreads();

    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l16 = lane & 15, lk = lane >> 4;
    // per-lane bases; everything else in an LDS address is a compile-time offset
    // Fragment x of a lane is tile row 32 * (x / 2) + 2 * l16 + x % 2 of the wave's 64 rows, fragment (y, s) column
    // 2 * ((l16 + 4 s) % 16) + y of its 32 columns: two fragments per 16-byte LDS read, conflict-free, and every
    // read address is a per-lane base plus a constant that fits the instruction's offset field.
    // Lane group lk = lane / 16 takes the contracted entries krow + q (+ 16 per further four groups).  Measured: a
    // 16-byte LDS read is conflict-free only if lanes l and l + 16 of each half-wave are a multiple of 256 bytes
    // apart, i.e. 8 tile rows with PITCH = 132; the two half-waves may differ.
    const int krow = 8 * (lk & 1) + 4 * (lk >> 1);
    st.fa = &S.a[0][0] + krow * PITCH + wm * 64 + 2 * l16;
#pragma unroll
    for (int s = 0; s < St::NS; ++s) st.fb[s] = &S.b[0][0] + krow * PITCH + wn * 32 + 2 * ((l16 + 4 * s) & 15);
    {
        typedef Map<AMODE, KT, VA, TM> MA;
        typedef Map<BMODE, KT, VB, TN> MB;
        st.ba.fix = &S.a_fix[0][0] + MA::x0(tid);
        st.ba.step = &S.a_step[0][0][0] + MA::k0(tid);
        st.ba.stage = &S.a[0][0] + MA::k0(tid) * PITCH + MA::x0(tid);
        st.bb.fix = &S.b_fix[0][0] + MB::x0(tid);
        st.bb.step = &S.b_step[0][0][0] + MB::k0(tid);
        st.bb.stage = &S.b[0][0] + MB::k0(tid) * PITCH + MB::x0(tid);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            st.ba.fixv[t] = (MA::CX == 0 && t < NTA) ? st.ba.fix[t * TM] : 0;
            st.bb.fixv[t] = (MB::CX == 0 && t < NTB) ? st.bb.fix[t * TN] : 0;
        }
    }

    // ---- prologue: k-step 0 into LDS buffer 0; with D = 2 also the gather of k-step 1 (into the second register
    //      set; a rolling gather issues it ahead of its loop) and the scatter entries of k-step 2 ----
    if (!affine) st.template issue<0, 0, false>(0);
    if constexpr (D == 2 && SETS == 2) {
        if (!affine) st.template issue<1, 1, false>(1);
        __syncthreads();  // table slot 0 has been read by every thread
        st.ent_dst[0] = (2 * KT < st.ent_limit || st.all_fast) ? 8 * st.ent_ptr[2 * KT < st.ent_limit ? 2 * KT : 0] : kSentinel;
    }
    st.template stage<0, 0, false, false>();
    if constexpr (CF::ROLL) {  // (k-step 1 is issued where the loops begin)
        __syncthreads();  // table slot 0 has been read by every thread
        st.ent_dst[0] = (2 * KT < st.ent_limit || st.all_fast) ? 8 * st.ent_ptr[2 * KT < st.ent_limit ? 2 * KT : 0] : kSentinel;
    }
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 2; ++y)
#pragma unroll
            for (int s = 0; s < 4; ++s) st.acc[x][y][s] = 0.0;  // (the four results of a lane: rotations s, or rows 4 s + lane / 16)
    __syncthreads();

    // k-steps whose gathers need no padding checks run in a loop specialised for the wave's role on its SIMD
    // (wm = 0: first, wm = 1: second); the remaining ones (ragged edge, zero padding, the last D steps) decide per step.
    st.early = wm == 0;
    // (sums whose terms are counted at run time only occur for blocks a few tiles wide: they take the general loop)
    int nfast = CF::EXACT ? st.kfull - D : 0;
    nfast = nfast < 2 ? 0 : (nfast & ~1);
    if (st.all_fast) nfast = st.nk;
    if (nfast > 0) {
        const bool role0 = CF::ROLL || __builtin_amdgcn_readfirstlane(wm) == 0;  // (a rolling gather is the same for both waves of a SIMD)
        if (CF::EXACT && st.unitA && st.unitB) {  // a loop of its own: no multiply (or no arithmetic at all) per element
            if (role0)
                st.template run_fast<0, CF::EXACT>(nfast, affine);
            else
                st.template run_fast<1, CF::EXACT>(nfast, affine);
        } else {
            if (role0)
                st.template run_fast<0, false>(nfast, affine);
            else
                st.template run_fast<1, false>(nfast, affine);
        }
        if constexpr (D == 2) st.issued_fast[SETS - 1] = true;  // the gather of k-step nfast + 1 is in flight (issued unchecked)
        if constexpr (VA && VB && CF::EXACT && CF::NOENT_AFF) {
            // the table-free loop of these families fetches no scatter entries: those of the first k-step that the
            // loop below gathers (nfast + 2; the gather of nfast + 1 is in flight) are fetched here
            if (affine && !st.all_fast) {
                const int kn = (nfast + 2) * KT;
                st.ent_dst[0] = kn < st.ent_limit ? 8 * st.ent_ptr[kn] : kSentinel;
                __syncthreads();
            }
        }
    }
    st.run_checked(nfast);

    // ---- epilogue: add alpha * tile to every destination block of C (Sec. 4.2) ----
    // The accumulators hold 4x4 blocks scattered over the tile; they are transposed through LDS (the operand buffers
    // are dead) so that each wave-wide access to C covers 64 consecutive entries of C's contiguous direction.
    constexpr int NPASS = (sizeof(S.a) + sizeof(S.b) >= (size_t)TN * OPITCH * sizeof(double)) ? 1 : 2;
    constexpr int CP = TN / NPASS;  // tile columns staged per pass
    static_assert(sizeof(S.a) + sizeof(S.b) >= (size_t)CP * OPITCH * sizeof(double), "output staging does not fit");
    double* otile = &S.a[0][0];  // [CP columns][OPITCH], rows fastest
    double* Cbase = part ? partial + (int64_t)(bid - main_count) * (TM * TN) : (P.C.space == 0 ? Cu : W) + P.C.base_off;
    if (part) alpha = 1.0;
    const int dj = lane & 3, dblk = (lane >> 2) & 3, di = lane >> 4;
    constexpr int CG = NTHREADS / TM;  // column groups of the row-wise mapping
    constexpr int BATCH = CP / CG;     // elements per thread, destination and pass: all their loads are issued together
    constexpr int RS = NTHREADS / CP;
    static_assert(BATCH == TM / RS, "both thread mappings cover the pass");
    // c_mode 0, lanes along the rows: thread = (row r, column group cg), columns cg + CG b.
    // c_mode 1, lanes along the columns: thread = (column c, row group rg), rows rg + RS b.
    // Either way element b of a thread has one fixed and one stepping scatter entry, and sits at a fixed step in the
    // staged tile.
    const int e_r = tid % TM, e_cg = tid / TM, e_c = tid % CP, e_rg = tid / CP;
    const int s_first = c_mode == 0 ? e_cg * OPITCH + e_r : e_c * OPITCH + e_rg, s_step = c_mode == 0 ? CG * OPITCH : RS;
    const int o_step = c_mode == 0 ? CG : RS;
    auto factor = [&](int d) -> double { return (part || P.overwrite) ? 0.0 : (((P.first_mask >> d) & 1u) ? beta : 1.0); };
    auto staged = [&](int b) -> double { return otile[s_first + s_step * b]; };
    // One destination's share of a pass.  The thread's offsets are read first; where none of a wave's is a sentinel (every
    // tile but those on a ragged edge) the wave takes a path without per-element conditions, on which the loads of C,
    // the reads of the staged tile and the stores are each issued as one batch.  (With a condition around every element
    // the compiler orders the work element by element, and every element then waits for its own LDS read.)
    // (The tile is staged as accumulated; alpha joins the destination's sign: +-alpha * x rounds like +-(alpha * x).)
    auto apply = [&](int d, int pass) {
        const double g = part ? 1.0 : P.C.coef[d] * alpha, f = factor(d);
        const int64_t o_fixed = c_mode == 0 ? c_rs[d][e_r] : c_cs[d][pass * CP + e_c];
        const int64_t* o_var = c_mode == 0 ? &c_cs[d][pass * CP + e_cg] : &c_rs[d][e_rg];
        int64_t off[BATCH];
        bool edge = false;
#pragma unroll
        for (int b = 0; b < BATCH; ++b) off[b] = o_fixed + o_var[o_step * b], edge |= off[b] < 0;
        if (!__builtin_amdgcn_ballot_w64(edge)) {
            double cur[BATCH];
            if (f != 0.0) {
#pragma unroll
                for (int b = 0; b < BATCH; ++b) cur[b] = Cbase[off[b]];
#pragma unroll
                for (int b = 0; b < BATCH; ++b) cur[b] = __builtin_fma(f, cur[b], g * staged(b));
            } else {
#pragma unroll
                for (int b = 0; b < BATCH; ++b) cur[b] = g * staged(b);
            }
#pragma unroll
            for (int b = 0; b < BATCH; ++b) Cbase[off[b]] = cur[b];
        } else {
            double cur[BATCH];
#pragma unroll
            for (int b = 0; b < BATCH; ++b) cur[b] = (f != 0.0 && off[b] >= 0) ? Cbase[off[b]] : 0.0;
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const double v = g * staged(b);
                if (off[b] >= 0) Cbase[off[b]] = (f == 0.0) ? v : __builtin_fma(f, cur[b], v);
            }
        }
    };
    // The same for destinations addressed by stride (c_affine): element b of a thread is at a base that is the same
    // for the whole wave (kept in scalar registers, stepped by scalar additions) plus the lane's fixed offset, so the
    // vector unit only combines: the loads and stores are buffer instructions (scalar descriptor at the base of the
    // wave's first element, the step to element b as scalar offset, the lane's offset as vector offset).
    // (The lane direction is a compile-time parameter here, so that the staged tile is read at constant offsets.)
    auto apply_affine = [&](auto lane_dir, int d, int pass) {
        constexpr int c_mode = decltype(lane_dir)::value;
        auto staged = [&](int b) -> double {
            return c_mode == 0 ? otile[e_cg * OPITCH + e_r + CG * OPITCH * b] : otile[e_c * OPITCH + e_rg + RS * b];
        };
        const double g = part ? 1.0 : P.C.coef[d] * alpha, f = factor(d);
        const int wave_first = __builtin_amdgcn_readfirstlane(tid & ~63);  // the wave's first thread
        // (a chunk's slot is a dense TM x TN tile, contiguous along the direction the lanes run)
        const int64_t rsS = part ? (c_mode == 0 ? 1 : TN) : P.C.rs_stride, csS = part ? (c_mode == 0 ? TM : 1) : P.C.cs_stride;
        // lanes along the rows: row e_r, columns pass * CP + e_cg + CG * b; along the columns: column pass * CP + e_c, rows e_rg + RS * b
        const int64_t row0 = (part ? 0 : P.C.roff[d] + i0) + (c_mode == 0 ? 0 : wave_first / CP);
        const int64_t col0 = (part ? 0 : P.C.coff[d] + j0) + pass * CP + (c_mode == 0 ? wave_first / TM : 0);
        // (strides below 2^20: the lane's offset is below 2^30 bytes, the last element's step below 2^31)
        typedef unsigned int word2_t __attribute__((ext_vector_type(2)));
        const int64_t ub = uniform64(reinterpret_cast<int64_t>(Cbase + (row0 * rsS + col0 * csS)));
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)ub, 0, -1, 0x00020000);
        const int step = 8 * (c_mode == 0 ? CG * (int)csS : RS * (int)rsS);
        const int lane_off = 8 * (c_mode == 0 ? e_r * (int)rsS : e_c * (int)csS);
        double cur[BATCH];
        if (f != 0.0) {
#pragma unroll
            for (int b = 0; b < BATCH; ++b) cur[b] = __builtin_bit_cast(double, __builtin_amdgcn_raw_buffer_load_b64(rsrc, lane_off, b * step, TC_C_POLICY));
            if (f == 1.0 && g == 1.0) {  // one instruction per element instead of two, with the same result
#pragma unroll
                for (int b = 0; b < BATCH; ++b) cur[b] += staged(b);
            } else {
#pragma unroll
                for (int b = 0; b < BATCH; ++b) cur[b] = __builtin_fma(f, cur[b], g * staged(b));
            }
        } else {
#pragma unroll
            for (int b = 0; b < BATCH; ++b) cur[b] = g * staged(b);
        }
#pragma unroll
        for (int b = 0; b < BATCH; ++b) __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(word2_t, cur[b]), rsrc, lane_off, b * step, TC_C_POLICY);
    };
#pragma unroll 1
    for (int pass = 0; pass < NPASS; ++pass) {
        if (pass > 0) __syncthreads();  // the previous pass has been read out
        if (wn / (WN / NPASS) == pass) {
            const int cw = (wn % (WN / NPASS)) * 32;
#pragma unroll
            for (int y = 0; y < 2; ++y)
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
#if TC_MFMA16
                        // result s of the lane: row 4 s + lane / 16 of A's 16 lanes, column lane % 16 of B's
                        otile[(cw + 2 * (lane & 15) + y) * OPITCH + wm * 64 + 32 * (x >> 1) + 2 * (4 * s + di) + (x & 1)] = st.acc[x][y][s];
#else
                        otile[(cw + 2 * (((dblk + s) & 3) * 4 + dj) + y) * OPITCH + wm * 64 + 32 * (x >> 1) + 2 * (dblk * 4 + di) + (x & 1)] =
                            st.acc[x][y][s];
#endif
                    }
        }
        __syncthreads();
#pragma unroll
        for (int d = 0; d < MAXC; ++d) {
            if (d < nC) {
                if (!c_affine)
                    apply(d, pass);
                else if (c_mode == 0)
                    apply_affine(std::integral_constant<int, 0>{}, d, pass);
                else
                    apply_affine(std::integral_constant<int, 1>{}, d, pass);
            }
        }
    }
}

// Tail of a launch cut into chunks (see fused_kernel): tiles = tail tiles, chunks per tile, kc = entries per chunk
// (a multiple of 64), partial = room for tiles * chunks dense TM x TN tiles.  tiles = 0: every tile is computed whole.
struct TailSplit {
    int tiles, chunks, kc;
    double* partial;
};

template <int AMODE, int BMODE, class CF, bool VA, bool VB>
int launch_one(const Product* prods, int first, int count, int tiles_m, int tiles_n, const double* A, const double* B, double* C,
               double* W, double alpha, double beta, int c_mode, const TailSplit& tail, hipStream_t stream) {
    static_assert(sizeof(Smem<CF>) * WGS_PER_CU <= 160 * 1024, "LDS budget of one CU");
    const size_t smem = sizeof(Smem<CF>);
    auto kern = fused_kernel<AMODE, BMODE, CF, VA, VB>;
    // The kernel's dynamic LDS size must be raised once per device and instantiation; callers may launch from several
    // host threads and on several devices, so the record of what has been done is an atomic bit per device.
    static std::atomic<uint64_t> configured{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    const uint64_t bit = (dev >= 0 && dev < 64) ? (uint64_t)1 << dev : 0;
    if (!bit || !(configured.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return (int)e;
        configured.fetch_or(bit, std::memory_order_release);
    }
    const int64_t total = (int64_t)count * tiles_m * tiles_n;
    if (total <= 0 || tail.tiles < 0 || tail.tiles > total) return (int)hipErrorInvalidValue;
    if (tail.tiles > 0 && (tail.chunks < 2 || tail.kc < 64 || tail.kc % 64 != 0 || !tail.partial)) return (int)hipErrorInvalidValue;
    const int64_t main_count = total - tail.tiles;
    const int64_t blocks = main_count + (int64_t)tail.tiles * tail.chunks;
    if (blocks > 0x7fffffff) return (int)hipErrorInvalidValue;
    const TileDiv tdiv{tile_div_rcp((int64_t)tiles_m * tiles_n), tile_div_rcp((int64_t)GROUP_M * tiles_n), tile_div_rcp(tiles_m % GROUP_M),
                       tile_div_rcp(tail.tiles)};
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(NTHREADS), smem, stream, prods, first, tiles_m, tiles_n, A, B, C, W, alpha, beta, c_mode,
                       (int)main_count, tail.tiles, tail.kc, tail.partial, tdiv);
    return (int)hipGetLastError();
}

// One launcher per kernel family, each defined in a translation unit of its own.  vec: bit 0 = pair-wise gather of A,
// bit 1 = of B.
template <int NTA, int NTB, bool EXACT>
int launch_family(int a_mode, int b_mode, int vec, int c_mode, const Product* prods, int first, int count, int tiles_m, int tiles_n,
                  const double* A, const double* B, double* C, double* W, double alpha, double beta, const TailSplit& tail, hipStream_t stream);

#define TC_FUSED_CASE(AM, BM, VA, VB) \
    case ((AM) * 8 + (BM) * 4 + (VA) * 2 + (VB)): \
        return launch_one<AM, BM, CF, (VA) != 0, (VB) != 0>(prods, first, count, tiles_m, tiles_n, A, B, C, W, alpha, beta, c_mode, tail, stream);

#define TC_FUSED_DEFINE_LAUNCH(NTAV, NTBV, EXACTV)                                                                                   \
    template <>                                                                                                                      \
    int launch_family<NTAV, NTBV, EXACTV>(int a_mode, int b_mode, int vec, int c_mode, const Product* prods, int first, int count,   \
                                          int tiles_m, int tiles_n, const double* A, const double* B, double* C, double* W,          \
                                          double alpha, double beta, const TailSplit& tail, hipStream_t stream) {                    \
        typedef Cfg<NTAV, NTBV, EXACTV> CF;                                                                                          \
        switch (a_mode * 8 + b_mode * 4 + (vec & 1) * 2 + ((vec >> 1) & 1)) {                                                        \
            TC_FUSED_CASE(0, 0, 0, 0) TC_FUSED_CASE(0, 0, 0, 1) TC_FUSED_CASE(0, 0, 1, 0) TC_FUSED_CASE(0, 0, 1, 1)                  \
            TC_FUSED_CASE(0, 1, 0, 0) TC_FUSED_CASE(0, 1, 0, 1) TC_FUSED_CASE(0, 1, 1, 0) TC_FUSED_CASE(0, 1, 1, 1)                  \
            TC_FUSED_CASE(1, 0, 0, 0) TC_FUSED_CASE(1, 0, 0, 1) TC_FUSED_CASE(1, 0, 1, 0) TC_FUSED_CASE(1, 0, 1, 1)                  \
            TC_FUSED_CASE(1, 1, 0, 0) TC_FUSED_CASE(1, 1, 0, 1) TC_FUSED_CASE(1, 1, 1, 0) TC_FUSED_CASE(1, 1, 1, 1)                  \
        }                                                                                                                            \
        return (int)hipErrorInvalidValue;                                                                                            \
    }

// Sum of the chunks of every tail tile, in chunk order, added to the destinations exactly as the fused kernel's
// epilogue does for a whole tile (Sec. 4.2).  Grid: (tail tile, slice of FixGeo::FIX_SLOW entries of the slow direction); a
// thread owns FIX_PER elements and issues the loads of all their chunks together before it adds them (one workgroup
// per tile with one element at a time took 0.25 ms for 16 tiles of 16 chunks).  LANES_ROWS: lanes run along the
// tile's rows (the partial tiles were written with c_mode 0, rows contiguous); otherwise along its columns.
constexpr int FIX_PER = 2;         // elements per thread
constexpr int FIX_MAXCHUNKS = 16;  // chunks whose loads are in flight together
// Along the lanes' direction a tile has FE entries (its rows, or its columns), along the other SE; a workgroup covers
// all FE of them times FIX_SLOW of the others.
template <bool LANES_ROWS>
struct FixGeo {
    static constexpr int FE = LANES_ROWS ? TM : TN, SE = LANES_ROWS ? TN : TM;
    static constexpr int GROUPS = NTHREADS / FE;        // thread groups along the slow direction
    static constexpr int FIX_SLOW = FIX_PER * GROUPS;   // slow entries per workgroup
    static constexpr int SLICES = SE / FIX_SLOW;        // workgroups per tail tile
};

template <bool LANES_ROWS>
__global__ __launch_bounds__(NTHREADS) void tail_fixup_kernel(const Product* __restrict__ prods, int first, int tiles_m, int tiles_n,
                                                              int main_count, int tail_tiles, int chunks, const double* __restrict__ partial,
                                                              double* __restrict__ Cu, double* __restrict__ W, double alpha, double beta) {
    typedef FixGeo<LANES_ROWS> FG;
    const int t = blockIdx.x, tid = threadIdx.x;
    const TileId tile = tile_of(main_count + t, tiles_m, tiles_n);
    const Product& P = prods[first + tile.pidx];
    const int64_t i0 = (int64_t)tile.tm * TM, j0 = (int64_t)tile.tn * TN;
    double* Cbase = (P.C.space == 0 ? Cu : W) + P.C.base_off;
    const int nC = P.C.nterms;
    const int fast = tid % FG::FE, sg = tid / FG::FE;  // position along the lanes' direction; the other: slice + sg + GROUPS j
    const int64_t gfast = (LANES_ROWS ? i0 : j0) + fast;
    const int64_t lim_fast = LANES_ROWS ? P.mb : P.nb, lim_slow = LANES_ROWS ? P.nb : P.mb;
    int64_t fix[MAXC];
#pragma unroll
    for (int d = 0; d < MAXC; ++d) {
        fix[d] = kSentinel;
        if (d < nC && gfast < lim_fast) {
            const int64_t g = (LANES_ROWS ? P.C.roff[d] : P.C.coff[d]) + gfast;
            if (g < (LANES_ROWS ? P.C.rs_len : P.C.cs_len)) fix[d] = as_global(LANES_ROWS ? P.C.rs : P.C.cs)[g];
        }
    }
    const int64_t stride_c = (int64_t)tail_tiles * (TM * TN);  // from one chunk of a tile to the next
    double v[FIX_PER];
    int slow[FIX_PER];
#pragma unroll
    for (int j = 0; j < FIX_PER; ++j) {
        slow[j] = blockIdx.y * FG::FIX_SLOW + sg + FG::GROUPS * j;
        v[j] = 0.0;
    }
    for (int c0 = 0; c0 < chunks; c0 += FIX_MAXCHUNKS) {
        double x[FIX_PER][FIX_MAXCHUNKS];
#pragma unroll
        for (int j = 0; j < FIX_PER; ++j) {
            const double* src = partial + (int64_t)t * (TM * TN) + slow[j] * FG::FE + fast + c0 * stride_c;
#pragma unroll
            for (int c = 0; c < FIX_MAXCHUNKS; ++c) x[j][c] = (c0 + c < chunks) ? src[c * stride_c] : 0.0;
        }
#pragma unroll
        for (int j = 0; j < FIX_PER; ++j)
#pragma unroll
            for (int c = 0; c < FIX_MAXCHUNKS; ++c)
                if (c0 + c < chunks) v[j] = (c0 + c == 0) ? x[j][c] : v[j] + x[j][c];  // chunk order, whatever the batch size
    }
#pragma unroll
    for (int j = 0; j < FIX_PER; ++j) {
        const int64_t gslow = (LANES_ROWS ? j0 : i0) + slow[j];
        if (gslow >= lim_slow) continue;
        const double av = alpha * v[j];
        for (int d = 0; d < nC; ++d) {
            const int64_t g = (LANES_ROWS ? P.C.coff[d] : P.C.roff[d]) + gslow;
            if (fix[d] < 0 || g >= (LANES_ROWS ? P.C.cs_len : P.C.rs_len)) continue;
            const int64_t off = fix[d] + as_global(LANES_ROWS ? P.C.cs : P.C.rs)[g];
            const double f = P.overwrite ? 0.0 : (((P.first_mask >> d) & 1u) ? beta : 1.0);
            const double gv = P.C.coef[d] * av;
            Cbase[off] = (f == 0.0) ? gv : __builtin_fma(f, Cbase[off], gv);
        }
    }
}

// Launch of the kernel above for the tail tiles of one fused launch.
inline int launch_tail_fixup(bool lanes_rows, const Product* prods, int first, int tiles_m, int tiles_n, int main_count, int tail_tiles, int chunks,
                             const double* partial, double* C, double* W, double alpha, double beta, hipStream_t st) {
    if (lanes_rows)
        hipLaunchKernelGGL(tail_fixup_kernel<true>, dim3((unsigned)tail_tiles, FixGeo<true>::SLICES), dim3(NTHREADS), 0, st, prods, first, tiles_m,
                           tiles_n, main_count, tail_tiles, chunks, partial, C, W, alpha, beta);
    else
        hipLaunchKernelGGL(tail_fixup_kernel<false>, dim3((unsigned)tail_tiles, FixGeo<false>::SLICES), dim3(NTHREADS), 0, st, prods, first, tiles_m,
                           tiles_n, main_count, tail_tiles, chunks, partial, C, W, alpha, beta);
    return (int)hipGetLastError();
}

}  // namespace fused / fused_small
}  // namespace tc
