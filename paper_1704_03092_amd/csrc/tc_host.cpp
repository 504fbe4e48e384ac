// Host side of libstrassen_tc: argument validation, bundle classification and ordering, Strassen schedule,
// launch program, and the C ABI declared in include/strassen_tc.h.  All arithmetic on tensor data happens in
// tc_device.hip; this file only decides what to launch.
#include "strassen_tc.h"
#include "tc_internal.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <string>
#include <vector>

namespace {

using tc::BundleDesc;
using tc::Operand;
using tc::Product;

// The seven products of one-level Strassen (Sec. 2.2, the display of M_0..M_6); quadrants numbered X0 X1 / X2 X3.
// Row r:  M_r = (sum_q kU[r][q] A_q) (sum_q kV[r][q] B_q);   C_q += kW[r][q] M_r.
const int kU[7][4] = {{1, 0, 0, 1}, {0, 0, 1, 1}, {1, 0, 0, 0}, {0, 0, 0, 1}, {1, 1, 0, 0}, {-1, 0, 1, 0}, {0, 1, 0, -1}};
const int kV[7][4] = {{1, 0, 0, 1}, {1, 0, 0, 0}, {0, 1, 0, -1}, {-1, 0, 1, 0}, {0, 0, 0, 1}, {1, 1, 0, 0}, {0, 0, 1, 1}};
const int kW[7][4] = {{1, 0, 0, 1}, {0, 0, 1, -1}, {0, 1, 0, 1}, {1, 0, 1, 0}, {-1, 1, 0, 0}, {0, 0, 0, 1}, {1, 0, 0, 0}};

struct Dim {
    char label;
    int64_t len;
    int64_t sA, sB, sC;  // stride in each tensor that carries the label (0 where absent)
};

enum StepKind { STEP_FUSED = 0, STEP_LINCOMB = 1 };

struct Step {
    StepKind kind;
    int first, count;     // device products [first, first + count)
    tc::FusedConfig cfg;  // STEP_FUSED
    int64_t rows, cols;   // extents
    int lanes_along_rows; // STEP_LINCOMB
    int src_role;         // STEP_LINCOMB: which caller tensor a space-0 source refers to (0 = A, 1 = B)
    // STEP_FUSED: the last tail_tiles tiles are cut into tail_chunks chunks of tail_kc contracted entries (0: none)
    int tail_tiles = 0, tail_chunks = 0;
    int64_t tail_kc = 0;
    double free_frac = 0.0;  // STEP_FUSED: share of the tiles gathered by stride (what the model prices; tails not looked at)
};

// vector ids inside the plan's store
enum { V_RSA = 0, V_CSA, V_RSB, V_CSB, V_RSC, V_CSC, V_RSM, V_CSM, V_RSTA, V_CSTA, V_RSTB, V_CSTB, V_COUNT };

int64_t round_up(int64_t x, int64_t q) { return (x + q - 1) / q * q; }

static_assert(TC_STATIC_WORKSPACE_BYTES == tc::kStaticWorkspaceBytes, "the public limit is the size of the device array");

}  // namespace

struct tc_plan {
    int64_t m = 1, n = 1, k = 1;
    int level_requested = 0, level = 0, variant = TC_VARIANT_ABC, bs_block = 16;
    bool host_only = false;
    int a_mode = 0, b_mode = 0, c_mode = 0;
    int a_vec = 0, b_vec = 0;
    int64_t mb = 0, nb = 0, kb = 0;
    std::vector<Dim> I, J, P;
    std::vector<tc_product_t> sched;  // block-level view of the products, for inspection
    std::vector<Product> prods;       // device descriptors (host copy)
    std::vector<Step> steps;
    int n_launches = 0;
    size_t workspace_bytes = 0;
    int64_t wsM = 0, wsTA = 0, wsTB = 0;  // offsets (elements) of the temporaries inside the workspace
    int64_t wsPart = 0;                   // offset of the chunks of split tail tiles
    int64_t m_peel = 0, n_peel = 0;       // rows / columns left to classical edge products (dynamic peeling)
    // device
    std::vector<BundleDesc> bundles;      // V_COUNT entries (temporaries may be unused: total = 0)
    int64_t store_entries = 0;
    int64_t* store_dev = nullptr;         // scatter vectors followed by block scatter vectors
    BundleDesc* bundles_dev = nullptr;
    Product* prods_dev = nullptr;
};

namespace {

int check_desc(const tc_tensor_desc_t* T) {
    if (!T) return TC_ERR_NULL;
    if (T->ndim < 0 || T->ndim > TC_MAX_NDIM) return TC_ERR_NDIM;
    if (T->ndim > 0 && (!T->len || !T->stride || !T->idx)) return TC_ERR_NULL;
    for (int d = 0; d < T->ndim; ++d) {
        if (T->len[d] < 0) return TC_ERR_LENGTH;
        if (T->stride[d] < 0) return TC_ERR_STRIDE;
        if (T->len[d] > 1 && T->stride[d] == 0) return TC_ERR_STRIDE;
        for (int e = 0; e < d; ++e)
            if (T->idx[e] == T->idx[d]) return TC_ERR_LABEL;
    }
    return TC_OK;
}

int find(const tc_tensor_desc_t* T, char c) {
    for (int d = 0; d < T->ndim; ++d)
        if (T->idx[d] == c) return d;
    return -1;
}

// Are the elements of T pairwise distinct (no two multi-indices share a location)?  First a sufficient condition
// that costs nothing: sorted by stride, every dimension steps over the whole extent of the ones before it (all
// layouts that nest, with or without padding).  Layouts that interleave dimensions can still be free of overlap
// (lengths (2, 3) with strides (3, 2): locations 0, 3, 2, 5, 4, 7); those are decided exactly by listing and sorting
// the locations, for tensors of up to kExactDistinctLimit elements.  Larger interleaved layouts are refused.
constexpr int64_t kExactDistinctLimit = (int64_t)1 << 22;

bool distinct_elements(const tc_tensor_desc_t* T) {
    std::vector<std::pair<int64_t, int64_t>> d;  // (stride, len)
    for (int i = 0; i < T->ndim; ++i)
        if (T->len[i] > 1) d.push_back({T->stride[i], T->len[i]});
    std::sort(d.begin(), d.end());
    int64_t extent = 1;  // 1 + largest offset so far
    bool nested = true;
    for (auto& p : d) {
        if (p.first < extent) nested = false;
        extent += (p.second - 1) * p.first;
    }
    if (nested) return true;
    int64_t total = 1;
    for (auto& p : d) {
        if (total > kExactDistinctLimit / p.second) return false;
        total *= p.second;
    }
    std::vector<int64_t> loc(1, 0);
    loc.reserve((size_t)total);
    for (auto& p : d) {
        const size_t have = loc.size();
        for (int64_t i = 1; i < p.second; ++i)
            for (size_t e = 0; e < have; ++e) loc.push_back(loc[e] + i * p.first);
    }
    std::sort(loc.begin(), loc.end());
    return std::adjacent_find(loc.begin(), loc.end()) == loc.end();
}

int64_t min_stride(const std::vector<Dim>& bundle, int which) {
    int64_t best = INT64_MAX;
    for (const Dim& d : bundle) {
        if (d.len <= 1) continue;
        int64_t s = which == 0 ? d.sA : which == 1 ? d.sB : d.sC;
        best = std::min(best, s);
    }
    return best;
}

// Pairs (2q, 2q+1) of consecutive entries of `lane` (the bundle the gather lanes run along) are contiguous in
// memory iff the bundle's fastest dimension has stride 1 and no pair straddles its end: its length is even, or it
// is the bundle's only dimension (the odd last entry then sits in a ragged tile, which is gathered entry by entry).
// Pairs are only 8-byte aligned in general; the kernel's 16-byte loads do not need more.
bool pairs_contiguous(const std::vector<Dim>& lane, int which) {
    auto stride = [which](const Dim& d) { return which == 0 ? d.sA : which == 1 ? d.sB : d.sC; };
    int nontrivial = 0;
    for (const Dim& d : lane) nontrivial += d.len > 1;
    for (const Dim& d : lane) {
        if (d.len <= 1) continue;
        return stride(d) == 1 && (d.len % 2 == 0 || nontrivial == 1);
    }
    return false;  // the bundle has a single entry: nothing to pair
}

BundleDesc make_bundle(const std::vector<Dim>& bundle, int which);

// How many 128-byte lines the first 256 entries of a bundle's scatter vector touch in tensor `which`, over the 16
// lines that 256 consecutive elements would: 1 for a contiguous run, 16 if every entry sits in a line of its own.
// (A gather along such a bundle fetches that multiple of the operand's bytes, and the lines are seldom still cached
// when their other entries come up.)
double line_amplification(const std::vector<Dim>& bundle, int which) {
    const BundleDesc b = make_bundle(bundle, which);
    const int64_t window = std::min<int64_t>(b.total, 256);
    if (window < 32) return 1.0;
    std::vector<int64_t> lines;
    int64_t idx[TC_MAX_NDIM] = {0};
    int64_t off = 0;
    for (int64_t e = 0; e < window; ++e) {
        lines.push_back(off >> 4);  // (arithmetic shift: negative strides fall into lines too)
        for (int d = 0; d < b.ndim; ++d) {
            off += b.stride[d];
            if (++idx[d] < b.len[d]) break;
            off -= b.stride[d] * b.len[d];
            idx[d] = 0;
        }
    }
    std::sort(lines.begin(), lines.end());
    const int64_t distinct = std::unique(lines.begin(), lines.end()) - lines.begin();
    return (double)distinct / (double)((window + 15) / 16);
}

void order_bundle(std::vector<Dim>& bundle, int which) {
    std::stable_sort(bundle.begin(), bundle.end(), [which](const Dim& x, const Dim& y) {
        int64_t sx = which == 0 ? x.sA : which == 1 ? x.sB : x.sC;
        int64_t sy = which == 0 ? y.sA : which == 1 ? y.sB : y.sC;
        // dimensions of length 1 carry no information; keep them last
        bool tx = x.len <= 1, ty = y.len <= 1;
        if (tx != ty) return ty;
        return sx < sy;
    });
}

BundleDesc make_bundle(const std::vector<Dim>& bundle, int which) {
    BundleDesc b;
    std::memset(&b, 0, sizeof b);
    b.ndim = (int)bundle.size();
    b.total = 1;
    for (int d = 0; d < b.ndim; ++d) {
        b.len[d] = bundle[d].len;
        b.stride[d] = which == 0 ? bundle[d].sA : which == 1 ? bundle[d].sB : bundle[d].sC;
        b.total *= bundle[d].len;
    }
    return b;
}

BundleDesc make_dense(int64_t len, int64_t stride) {
    BundleDesc b;
    std::memset(&b, 0, sizeof b);
    b.ndim = 1;
    b.len[0] = len;
    b.stride[0] = stride;
    b.total = len;
    return b;
}

// Stride s with scat[i] == i * s for every entry of the bundle's scatter vector (its dimensions, fastest first, merge
// into one run: each stride is the previous stride times the previous length), or -1.
int64_t affine_stride(const BundleDesc& b) {
    int64_t stride = -1, next = 0;
    for (int d = 0; d < b.ndim; ++d) {
        if (b.len[d] <= 1) continue;
        if (stride < 0)
            stride = b.stride[d];
        else if (b.stride[d] != next)
            return -1;
        next = b.stride[d] * b.len[d];
    }
    return stride < 0 ? 0 : stride;
}

void block_tables(int level, std::vector<std::vector<int>>& U, std::vector<std::vector<int>>& V, std::vector<std::vector<int>>& W) {
    // L-level coefficients as the Kronecker product of the one-level triples, on the 2^L x 2^L block grid.
    int g = 1 << level, R = 1;
    for (int l = 0; l < level; ++l) R *= 7;
    U.assign(R, std::vector<int>(g * g, 0));
    V = U;
    W = U;
    for (int r = 0; r < R; ++r) {
        int Q = 1;
        for (int l = 0; l < level; ++l) Q *= 4;
        for (int q = 0; q < Q; ++q) {
            int cu = 1, cv = 1, cw = 1, br = 0, bc = 0, rr = r, qq = q;
            // digit l of r (product at recursion depth) pairs with digit l of q (quadrant at that depth); least
            // significant digit = innermost level
            int rd[4], qd[4];
            for (int l = 0; l < level; ++l) {
                rd[l] = rr % 7;
                rr /= 7;
                qd[l] = qq % 4;
                qq /= 4;
            }
            for (int l = level - 1; l >= 0; --l) {  // outermost first
                cu *= kU[rd[l]][qd[l]];
                cv *= kV[rd[l]][qd[l]];
                cw *= kW[rd[l]][qd[l]];
                br = 2 * br + (qd[l] >> 1);
                bc = 2 * bc + (qd[l] & 1);
            }
            U[r][br * g + bc] = cu;
            V[r][br * g + bc] = cv;
            W[r][br * g + bc] = cw;
        }
    }
}

void set_operand(Operand& op, const int64_t* rs, const int64_t* cs, int64_t rs_len, int64_t cs_len, int space, int64_t base_off) {
    std::memset(&op, 0, sizeof op);
    op.rs = rs;
    op.cs = cs;
    op.rs_len = rs_len;
    op.cs_len = cs_len;
    op.space = space;
    op.base_off = base_off;
    op.rs_stride = op.cs_stride = -1;
}

void add_term(Operand& op, int64_t roff, int64_t coff, double coef) {
    op.roff[op.nterms] = roff;
    op.coff[op.nterms] = coff;
    op.coef[op.nterms] = coef;
    ++op.nterms;
}

// Put a term with coefficient +1 first (every Strassen operand sum has one): the kernel then starts the sum from
// the gathered element itself instead of a product.
void lead_with_plus(Operand& op) {
    for (int t = 0; t < op.nterms; ++t)
        if (op.coef[t] == 1.0) {
            std::swap(op.roff[0], op.roff[t]);
            std::swap(op.coff[0], op.coff[t]);
            std::swap(op.coef[0], op.coef[t]);
            return;
        }
}

// Kernel family of a product: sums of one, two or four terms on both sides have kernels specialised for exactly
// those counts (key 8 * n_a + n_b); a three-term sum (a four-term sum that lost a block to the zero padding) runs
// in the family that counts terms at run time (key 0).
int terms_class(int n_a, int n_b) { return (n_a != 3 && n_b != 3) ? 8 * n_a + n_b : 0; }

extern const tc_model_params_t kDefaultModel;
void choose_tiles(const tc_plan_t* p, Step& s, const tc_model_params_t& mp, int tile_mode, int tail_mode, int64_t* chunk_elems);
int64_t count_table_free(const tc_plan_t* p, const Step& s);

int build_plan(tc_plan_t* p, const tc_tensor_desc_t* A, const tc_tensor_desc_t* B, const tc_tensor_desc_t* C, int level, int variant,
               const tc_options_t* opts, void* stream) {
    int rc;
    if ((rc = check_desc(A)) || (rc = check_desc(B)) || (rc = check_desc(C))) return rc;
    if (level < 0 || level > 2) return TC_ERR_LEVEL;
    if (variant < TC_VARIANT_NAIVE || variant > TC_VARIANT_HYBRID) return TC_ERR_VARIANT;
    p->bs_block = 16;
    bool no_merge = false, no_peel = false, no_repack = false;
    int tail_mode = 0;  // 0: the model decides, -1: never, 2..16: that many chunks wherever a launch has a tail
    int tile_mode = 0;  // 0: the model decides, 64 / 128: tile columns of the single-term launches
    int split = 1;
    if (opts) {
        if (opts->tail_split < -1 || opts->tail_split == 1 || opts->tail_split > 16) return TC_ERR_STATE;
        tail_mode = opts->tail_split;
        if (opts->tile_n != 0 && opts->tile_n != 64 && opts->tile_n != 128) return TC_ERR_STATE;
        tile_mode = opts->tile_n;
        if (opts->bs_block < 0 || opts->bs_block > (1 << 20)) return TC_ERR_STATE;
        if (opts->bs_block > 0) p->bs_block = opts->bs_block;
        p->host_only = opts->host_only != 0;
        no_merge = opts->no_merge != 0;
        no_peel = opts->no_peel != 0;
        no_repack = opts->no_repack != 0;
        if (opts->split_k > 4 || opts->split_k < -1) return TC_ERR_STATE;
        split = std::max(opts->split_k, 1);  // -1 has been resolved by the caller (tc_plan_ex)
    }
    // ---- bundles (Sec. 2.3): every label in exactly two tensors ----
    const tc_tensor_desc_t* T[3] = {A, B, C};
    for (int t = 0; t < 3; ++t) {
        for (int d = 0; d < T[t]->ndim; ++d) {
            char c = T[t]->idx[d];
            int ia = find(A, c), ib = find(B, c), ic = find(C, c);
            if ((ia >= 0) + (ib >= 0) + (ic >= 0) != 2) return TC_ERR_LABEL;
            int64_t len = T[t]->len[d];
            if ((ia >= 0 && A->len[ia] != len) || (ib >= 0 && B->len[ib] != len) || (ic >= 0 && C->len[ic] != len)) return TC_ERR_LENGTH;
        }
    }
    if (!distinct_elements(C)) return TC_ERR_STRIDE;
    for (int d = 0; d < A->ndim; ++d) {
        char c = A->idx[d];
        int ib = find(B, c), ic = find(C, c);
        Dim dim{c, A->len[d], A->stride[d], ib >= 0 ? B->stride[ib] : 0, ic >= 0 ? C->stride[ic] : 0};
        (ic >= 0 ? p->I : p->P).push_back(dim);
    }
    for (int d = 0; d < B->ndim; ++d) {
        char c = B->idx[d];
        int ic = find(C, c);
        if (ic >= 0) p->J.push_back(Dim{c, B->len[d], 0, B->stride[d], C->stride[ic]});
    }
    p->m = p->n = p->k = 1;
    for (auto& d : p->I) p->m *= d.len;
    for (auto& d : p->J) p->n *= d.len;
    for (auto& d : p->P) p->k *= d.len;

    // ---- which way does each operand run contiguously, and the order inside each bundle ----
    // The order inside a bundle is free as long as both tensors sharing it use the same one (Sec. 2.3); it is
    // chosen so that the operand whose smallest stride lies in that bundle is read along it.
    p->a_mode = min_stride(p->P, 0) < min_stride(p->I, 0) ? 1 : 0;
    p->b_mode = min_stride(p->P, 1) < min_stride(p->J, 1) ? 1 : 0;
    p->c_mode = min_stride(p->J, 2) < min_stride(p->I, 2) ? 1 : 0;  // 1: C runs contiguously along its columns
    order_bundle(p->I, p->a_mode == 0 ? 0 : 2);
    order_bundle(p->J, p->b_mode == 0 ? 1 : 2);
    order_bundle(p->P, p->a_mode == 1 ? 0 : (p->b_mode == 1 ? 1 : 0));

    p->a_vec = pairs_contiguous(p->a_mode == 0 ? p->I : p->P, 0);
    p->b_vec = pairs_contiguous(p->b_mode == 0 ? p->J : p->P, 1);

    // ---- Strassen partition of the matrix view (Sec. 3) ----
    p->level_requested = level;
    p->variant = variant;
    while (level > 0 && std::min(p->m, std::min(p->n, p->k)) < (1 << level)) --level;
    p->level = level;
    if (variant == TC_VARIANT_HYBRID && level < 1) variant = TC_VARIANT_ABC;  // nothing to store without a Strassen level
    const int g = 1 << level;
    // Block extents: the matrix view is cut at multiples of the extent; the last block of each direction may be
    // short (or empty) and is completed with zeros (Sec. 3, last paragraph: zero padding of the whole bundle).
    // Extents are even (pair-wise gathers never straddle a block).  Where an operand reads the bundle through its
    // block scatter vector (the bundle is no single constant-stride run in that operand) they are multiples of the
    // 16 entries of a block, so that blocks of the vector do not straddle Strassen blocks.  Small units keep the
    // blocks of a direction equally long wherever the length allows: operand sums whose blocks end at different rows
    // need the padding-checked loop in the tiles where they differ.
    auto unit = [](const std::vector<Dim>& bundle, std::initializer_list<int> readers) {
        for (int which : readers)
            if (affine_stride(make_bundle(bundle, which)) < 0) return 16;
        return 2;
    };
    auto extent = [g](int64_t len, int q) { return g == 1 ? len : round_up((len + g - 1) / g, q); };
    // Dynamic peeling of the row and column bundles (Sec. 3, last paragraph): the Strassen products cover the largest
    // leading part that is a whole number of equal blocks, classical edge products (appended after the schedule) the
    // rest.  While the Strassen schedule is generated, m and n stand for that leading part.
    const int64_t m_full = p->m, n_full = p->n;
    // (Only the schedules that sum blocks inside the multiplying kernel gain: single-block products have no blocks of
    // different length to reconcile, the edge products would only add to them.)
    const bool sums_in_kernel = variant == TC_VARIANT_ABC || variant == TC_VARIANT_AB;
    if (level > 0 && !no_peel) {
        // Long bundles are cut at a whole number of 128-wide tiles per block if that leaves at most a tenth to the edge
        // product: the Strassen products then have no ragged tiles at all (every tile of theirs can be gathered by
        // stride), and the fringe is done once, by the single-term kernel, instead of once per block.  Otherwise at
        // a whole number of block units, which at least makes the blocks equally long.
        auto leading = [g, sums_in_kernel](int64_t len, int q) {
            const int64_t tiles = (int64_t)g * 128, coarse = len / tiles * tiles;
            if (coarse == len) return len;
            if (coarse * 10 >= len * 9) return coarse;
            const int64_t cut = (int64_t)g * q, fine = len / cut * cut;
            return sums_in_kernel && fine != len && fine >= tiles ? fine : len;
        };
        p->m = leading(m_full, unit(p->I, {0}));
        p->n = leading(n_full, unit(p->J, {1}));
    }
    p->m_peel = m_full - p->m, p->n_peel = n_full - p->n;
    p->mb = extent(p->m, unit(p->I, {0}));
    p->nb = extent(p->n, unit(p->J, {1}));
    p->kb = extent(p->k, unit(p->P, {0, 1}));

    // ---- vectors in the device store ----
    p->bundles.resize(V_COUNT);
    p->bundles[V_RSA] = make_bundle(p->I, 0);
    p->bundles[V_CSA] = make_bundle(p->P, 0);
    p->bundles[V_RSB] = make_bundle(p->P, 1);
    p->bundles[V_CSB] = make_bundle(p->J, 1);
    p->bundles[V_RSC] = make_bundle(p->I, 2);
    p->bundles[V_CSC] = make_bundle(p->J, 2);
    const bool empty = p->m == 0 || p->n == 0;
    // split_k (level 0): chunks of the contracted bundle, each at least 64 entries and a multiple of 16 long
    int64_t kc = p->k;
    if (level > 0 || empty) split = 1;
    while (split > 1 && round_up((p->k + split - 1) / split, 16) < 64) --split;
    if (split > 1) {
        kc = round_up((p->k + split - 1) / split, 16);
        split = (int)((p->k + kc - 1) / kc);
    }
    const bool use_S = split > 1;
    const bool use_H = !empty && p->k > 0 && variant == TC_VARIANT_HYBRID;  // first-level operand sums: one first-level block
    const int64_t hsub = level == 2 ? 2 : 1;  // second-level blocks per first-level block and direction
    const bool use_M = !empty && p->k > 0 && level > 0 && (variant == TC_VARIANT_AB || variant == TC_VARIANT_NAIVE);
    const bool use_T = use_M && variant == TC_VARIANT_NAIVE;
    p->bundles[V_RSM] = make_dense(use_M || use_S ? p->mb : 0, 1);
    p->bundles[V_CSM] = make_dense(use_M ? p->nb : use_S ? split * p->nb : 0, p->mb);  // the chunks' temporaries side by side
    const int64_t tm = use_H ? hsub * p->mb : p->mb, tn = use_H ? hsub * p->nb : p->nb, tk = use_H ? hsub * p->kb : p->kb;  // temporaries' extents
    // Repacking (the explicit packing of Sec. 4.1, done once per contraction instead of once per tile): an operand
    // that can only be gathered element by element, and whose consecutive entries along the gather direction lie in
    // different memory lines, is first copied into a dense temporary by one element-wise pass; the products then
    // read the temporary by stride.  (Such an operand arises when both A and B have their unit-stride index in the
    // contracted bundle: the bundle's order can follow only one of them.)  Worth it if the tiles re-read the
    // operand at least four times.  The stored-sum schedules have temporaries of their own and do not repack.
    const bool can_repack = !no_repack && !empty && p->k > 0 && !use_S && !use_H && !use_T;
    const bool repack_a = can_repack && !p->a_vec && n_full >= 4 * 128 && line_amplification(p->a_mode == 0 ? p->I : p->P, 0) >= 8.0;
    const bool repack_b = can_repack && !p->b_vec && m_full >= 4 * 128 && line_amplification(p->b_mode == 0 ? p->J : p->P, 1) >= 8.0;
    const bool own_T = use_T || use_H;
    p->bundles[V_RSTA] = make_dense(own_T ? tm : repack_a ? m_full : 0, 1);
    p->bundles[V_CSTA] = make_dense(own_T ? tk : repack_a ? p->k : 0, own_T ? tm : m_full);
    p->bundles[V_RSTB] = make_dense(own_T ? tk : repack_b ? p->k : 0, 1);
    p->bundles[V_CSTB] = make_dense(own_T ? tn : repack_b ? n_full : 0, own_T ? tk : p->k);
    int64_t off = 0;
    for (auto& b : p->bundles) {
        b.out_off = off;
        off += b.total;
    }
    for (auto& b : p->bundles) {
        b.bs_off = off;
        off += (b.total + p->bs_block - 1) / p->bs_block;
    }
    p->store_entries = off;
    if (use_S) {
        p->wsM = 0;
        p->workspace_bytes = (size_t)(split * p->mb * p->nb) * sizeof(double);
    }
    if (use_H) {
        p->wsTA = 0;
        p->wsTB = tm * tk;
        p->workspace_bytes = (size_t)(tm * tk + tk * tn) * sizeof(double);
    }
    if (use_M) {
        int64_t w = 0;
        p->wsM = w;
        w += p->mb * p->nb;
        if (use_T) {
            p->wsTA = w;
            w += p->mb * p->kb;
            p->wsTB = w;
            w += p->kb * p->nb;
        }
        p->workspace_bytes = (size_t)w * sizeof(double);
    }
    if (repack_a || repack_b) {
        int64_t w = (int64_t)(p->workspace_bytes / sizeof(double));
        if (repack_a) p->wsTA = w, w += m_full * p->k;
        if (repack_b) p->wsTB = w, w += p->k * n_full;
        p->workspace_bytes = (size_t)w * sizeof(double);
    }
    // where the products read A and B, and how
    const int a_mode = repack_a ? 0 : p->a_mode, b_mode = repack_b ? 1 : p->b_mode;  // the temporaries: A rows, B columns contiguous
    const int a_vec = repack_a ? 1 : p->a_vec, b_vec = repack_b ? 1 : p->b_vec;

    if (!p->host_only) {
        // look up this GPU's static workspace now, so that tc_contract_static finds the address ready
        void* static_ws = nullptr;
        if (tc::dev_static_workspace(&static_ws)) return TC_ERR_HIP;
        if (tc::dev_malloc((void**)&p->store_dev, sizeof(int64_t) * (size_t)std::max<int64_t>(p->store_entries, 1))) return TC_ERR_HIP;
        if (tc::dev_malloc((void**)&p->bundles_dev, sizeof(BundleDesc) * V_COUNT)) return TC_ERR_HIP;
        if (tc::dev_upload(p->bundles_dev, p->bundles.data(), sizeof(BundleDesc) * V_COUNT, stream)) return TC_ERR_HIP;
        int64_t max_total = 0;
        for (auto& b : p->bundles) max_total = std::max(max_total, b.total);
        if (max_total > 0 && tc::launch_planner(p->bundles_dev, V_COUNT, max_total, p->bs_block, p->store_dev, stream)) return TC_ERR_HIP;
    }
    auto vec = [p](int id) -> const int64_t* { return p->store_dev ? p->store_dev + p->bundles[id].out_off : nullptr; };
    auto setop = [&](Operand& op, int rs_id, int cs_id, int64_t rs_len, int64_t cs_len, int space, int64_t base_off) {
        set_operand(op, vec(rs_id), vec(cs_id), rs_len, cs_len, space, base_off);
        op.rs_id = rs_id;
        op.cs_id = cs_id;
        op.rs_stride = affine_stride(p->bundles[rs_id]);
        op.cs_stride = affine_stride(p->bundles[cs_id]);
        // the kernel reads the block scatter vectors (blocks of 16 entries) to find tiles whose rows / columns are regular
        const bool use_bs = p->store_dev && p->bs_block == 16;
        op.rbs = use_bs ? p->store_dev + p->bundles[rs_id].bs_off : nullptr;
        op.cbs = use_bs ? p->store_dev + p->bundles[cs_id].bs_off : nullptr;
    };

    auto set_a = [&](Operand& op, int64_t rows) {
        if (repack_a)
            setop(op, V_RSTA, V_CSTA, rows, p->k, 1, p->wsTA);
        else
            setop(op, V_RSA, V_CSA, rows, p->k, 0, 0);
    };
    auto set_b = [&](Operand& op, int64_t cols) {
        if (repack_b)
            setop(op, V_RSTB, V_CSTB, p->k, cols, 1, p->wsTB);
        else
            setop(op, V_RSB, V_CSB, p->k, cols, 0, 0);
    };

    struct Pending {
        Product pr;
        tc_product_t view;
    };
    std::vector<char> touched(g * g, 0);  // blocks of C written so far: the first product to write one applies beta
    // Turn a list of products into launches (and, for AB / Naive, their temporaries and element-wise passes).
    auto emit = [&](std::vector<Pending>& list, const tc::FusedConfig& user_cfg_base, bool fusedC_) {
        // Products whose destination sets are disjoint may share one launch (ABC); otherwise one launch each.
        std::vector<int> phase(list.size(), 0);
        int nphase = 0;
        const bool merge = fusedC_ && !no_merge;
        {
            std::vector<std::vector<char>> used;  // per phase: blocks written, and operand class
            std::vector<int> pclass;
            for (size_t e = 0; e < list.size(); ++e) {
                const tc_product_t& v = list[e].view;
                int cls = terms_class(list[e].pr.A.nterms, list[e].pr.B.nterms);
                int chosen = -1;
                if (merge) {
                    for (int ph = 0; ph < nphase && chosen < 0; ++ph) {
                        bool ok = pclass[ph] == cls;
                        for (int d = 0; d < v.n_c && ok; ++d) ok = !used[ph][v.c_row[d] * g + v.c_col[d]];
                        if (ok) chosen = ph;
                    }
                }
                if (chosen < 0) {
                    chosen = nphase++;
                    used.push_back(std::vector<char>(g * g, 0));
                    pclass.push_back(cls);
                }
                for (int d = 0; d < v.n_c; ++d) used[chosen][v.c_row[d] * g + v.c_col[d]] = 1;
                phase[e] = chosen;
            }
        }
        // emit in phase order; the first product (in that order) to write a block of C applies beta to it
        const bool fusedC = fusedC_;
        for (int ph = 0; ph < nphase; ++ph) {
            int first_dev = (int)p->prods.size(), count = 0, cls = 0;
            for (size_t e = 0; e < list.size(); ++e) {
                if (phase[e] != ph) continue;
                Pending& q = list[e];
                uint32_t first_mask = 0;
                for (int d = 0; d < q.view.n_c; ++d) {
                    char& t = touched[q.view.c_row[d] * g + q.view.c_col[d]];
                    if (!t) first_mask |= 1u << d, q.view.c_first[d] = 1;
                    t = 1;
                }
                q.view.launch = (int)p->steps.size();
                cls = terms_class(q.pr.A.nterms, q.pr.B.nterms);  // merged launches hold one class
                if (fusedC) {
                    q.pr.first_mask = first_mask;
                    p->prods.push_back(q.pr);
                    ++count;
                } else {
                    // temporaries: dense, column-major, one block extent each
                    Product acc;  // M -> destinations of C
                    std::memset(&acc, 0, sizeof acc);
                    setop(acc.A, V_RSM, V_CSM, p->mb, p->nb, 1, p->wsM);
                    add_term(acc.A, 0, 0, 1.0);
                    acc.C = q.pr.C;
                    acc.mb = p->mb;
                    acc.nb = p->nb;
                    acc.first_mask = first_mask;
                    Product mul = q.pr;  // (sum A)(sum B) -> M
                    setop(mul.C, V_RSM, V_CSM, p->mb, p->nb, 1, p->wsM);
                    add_term(mul.C, 0, 0, 1.0);
                    mul.first_mask = 1;
                    mul.overwrite = 1;
                    tc::FusedConfig cfg = user_cfg_base;
                    cfg.c_mode = 0;  // M is dense with contiguous rows
                    if (variant == TC_VARIANT_NAIVE) {
                        Product sa, sb;  // operand sums -> TA, TB
                        std::memset(&sa, 0, sizeof sa);
                        std::memset(&sb, 0, sizeof sb);
                        sa.A = q.pr.A;
                        setop(sa.C, V_RSTA, V_CSTA, p->mb, p->kb, 1, p->wsTA);
                        add_term(sa.C, 0, 0, 1.0);
                        sa.mb = p->mb, sa.nb = p->kb, sa.first_mask = 1, sa.overwrite = 1;
                        sb.A = q.pr.B;
                        setop(sb.C, V_RSTB, V_CSTB, p->kb, p->nb, 1, p->wsTB);
                        add_term(sb.C, 0, 0, 1.0);
                        sb.mb = p->kb, sb.nb = p->nb, sb.first_mask = 1, sb.overwrite = 1;
                        int i0 = (int)p->prods.size();
                        p->prods.push_back(sa);
                        p->prods.push_back(sb);
                        p->steps.push_back(Step{STEP_LINCOMB, i0, 1, {}, p->mb, p->kb, p->a_mode == 0 ? 1 : 0, 0});
                        p->steps.push_back(Step{STEP_LINCOMB, i0 + 1, 1, {}, p->kb, p->nb, p->b_mode == 1 ? 1 : 0, 1});
                        setop(mul.A, V_RSTA, V_CSTA, p->mb, p->kb, 1, p->wsTA);
                        add_term(mul.A, 0, 0, 1.0);
                        setop(mul.B, V_RSTB, V_CSTB, p->kb, p->nb, 1, p->wsTB);
                        add_term(mul.B, 0, 0, 1.0);
                        cfg = tc::FusedConfig{0, 1, 1, 1, 1, 1, 1, 1, 0, 128};  // dense temporaries: block extents are multiples of 16
                    } else {
                        cfg.nta = terms_class(q.pr.A.nterms, q.pr.B.nterms) / 8;
                        cfg.ntb = terms_class(q.pr.A.nterms, q.pr.B.nterms) % 8;
                    }
                    int i1 = (int)p->prods.size();
                    p->prods.push_back(mul);
                    p->prods.push_back(acc);
                    q.view.launch = (int)p->steps.size();
                    p->steps.push_back(Step{STEP_FUSED, i1, 1, cfg, p->mb, p->nb, 0, 0});
                    p->steps.push_back(Step{STEP_LINCOMB, i1 + 1, 1, {}, p->mb, p->nb, p->c_mode == 0 ? 1 : 0, 0});
                }
                p->sched.push_back(q.view);
            }
            if (fusedC && count > 0) {
                tc::FusedConfig cfg = user_cfg_base;
                cfg.nta = cls / 8;
                cfg.ntb = cls % 8;
                p->steps.push_back(Step{STEP_FUSED, first_dev, count, cfg, p->mb, p->nb, 0, 0});
            }
        }
        };

    // ---- schedule ----
    if (empty) return TC_OK;  // nothing to do at run time
    if (p->k == 0) {
        // C := beta * C : one element-wise pass with no source term
        Product pr;
        std::memset(&pr, 0, sizeof pr);
        set_operand(pr.A, nullptr, nullptr, 0, 0, 0, 0);
        set_operand(pr.B, nullptr, nullptr, 0, 0, 0, 0);
        setop(pr.C, V_RSC, V_CSC, p->m, p->n, 0, 0);
        add_term(pr.C, 0, 0, 1.0);
        pr.mb = p->m;
        pr.nb = p->n;
        pr.first_mask = 1;
        p->prods.push_back(pr);
        p->steps.push_back(Step{STEP_LINCOMB, 0, 1, {}, p->m, p->n, p->c_mode == 0 ? 1 : 0, 0});
    } else if (use_S) {
        // chunk s: A[:, s kc : (s+1) kc) * B[s kc : (s+1) kc), :] -> temporary s (one launch for all chunks), then
        // C := beta C + alpha-scaled sum of the temporaries (one element-wise pass)
        const int first = (int)p->prods.size();
        for (int s = 0; s < split; ++s) {
            Product mul;
            std::memset(&mul, 0, sizeof mul);
            setop(mul.A, V_RSA, V_CSA, p->m, p->k, 0, 0);
            add_term(mul.A, 0, s * kc, 1.0);
            setop(mul.B, V_RSB, V_CSB, p->k, p->n, 0, 0);
            add_term(mul.B, s * kc, 0, 1.0);
            setop(mul.C, V_RSM, V_CSM, p->mb, split * p->nb, 1, p->wsM);
            add_term(mul.C, 0, s * p->nb, 1.0);
            mul.mb = p->mb, mul.nb = p->nb, mul.kb = kc;
            mul.first_mask = 1, mul.overwrite = 1;
            p->prods.push_back(mul);
            tc_product_t view;
            std::memset(&view, 0, sizeof view);
            view.n_a = view.n_b = view.n_c = 1;
            view.a_sign[0] = view.b_sign[0] = view.c_sign[0] = 1;
            view.c_first[0] = s == 0;
            view.launch = 0;
            p->sched.push_back(view);
        }
        tc::FusedConfig cfg{p->a_mode, p->b_mode, 1, 1, p->a_vec, p->b_vec, 0, 0, 0, 128};  // temporaries: contiguous rows
        p->steps.push_back(Step{STEP_FUSED, first, split, cfg, p->mb, p->nb, 0, 0});
        Product acc;
        std::memset(&acc, 0, sizeof acc);
        setop(acc.A, V_RSM, V_CSM, p->mb, split * p->nb, 1, p->wsM);
        for (int s = 0; s < split; ++s) add_term(acc.A, 0, s * p->nb, 1.0);
        setop(acc.C, V_RSC, V_CSC, p->m, p->n, 0, 0);
        add_term(acc.C, 0, 0, 1.0);
        acc.mb = p->mb, acc.nb = p->nb;
        acc.first_mask = 1;
        p->prods.push_back(acc);
        p->steps.push_back(Step{STEP_LINCOMB, first + split, 1, {}, p->mb, p->nb, p->c_mode == 0 ? 1 : 0, 0});
    } else if (use_H) {
        // The first level stored, the rest fused.  For each first-level product r: operand sums of two first-level
        // blocks go to the dense temporaries TA, TB (a single +1 block is used in place).  One level: TA * TB is
        // one product added to the first-level destinations of r.  Two levels: the seven second-level products of
        // TA * TB are scheduled like one-level ABC, each adding to the second-level blocks of every first-level
        // destination of r (up to 2 x 2 blocks of the 4 x 4 grid of C).
        std::vector<std::vector<int>> U1, V1, W1, U2, V2, W2;
        block_tables(1, U1, V1, W1);
        block_tables(level - 1, U2, V2, W2);
        const int h = (int)hsub, R2 = (int)U2.size();
        const int64_t MB = hsub * p->mb, NB = hsub * p->nb, KB = hsub * p->kb;
        struct Blk {
            int r, c, sign;
        };
        for (int r = 0; r < 7; ++r) {
            std::vector<Blk> oa, ob, oc;
            for (int i = 0; i < 2; ++i)
                for (int j = 0; j < 2; ++j) {
                    if (U1[r][i * 2 + j] && i * MB < p->m && j * KB < p->k) oa.push_back({i, j, U1[r][i * 2 + j]});
                    if (V1[r][i * 2 + j] && i * KB < p->k && j * NB < p->n) ob.push_back({i, j, V1[r][i * 2 + j]});
                    if (W1[r][i * 2 + j] && i * MB < p->m && j * NB < p->n) oc.push_back({i, j, W1[r][i * 2 + j]});
                }
            if (oa.empty() || ob.empty() || oc.empty()) continue;
            // where the second level reads its operands: (vectors, lengths, space, offset of the first-level block, real extents)
            struct Src {
                int rs, cs;  // vector ids
                int64_t rs_len, cs_len, r0, c0, rows, cols;
                int space;
                int64_t base;
                bool direct;
            };
            auto real = [](int64_t total, int64_t start, int64_t ext) { return std::min(ext, total - start); };
            Src sa, sb;
            sa.direct = oa.size() == 1 && oa[0].sign == 1;
            sb.direct = ob.size() == 1 && ob[0].sign == 1;
            if (sa.direct) {
                sa = Src{V_RSA, V_CSA, p->m, p->k, oa[0].r * MB, oa[0].c * KB, real(p->m, oa[0].r * MB, MB), real(p->k, oa[0].c * KB, KB), 0, 0, true};
            } else {
                Product sum;
                std::memset(&sum, 0, sizeof sum);
                setop(sum.A, V_RSA, V_CSA, p->m, p->k, 0, 0);
                int64_t rows = 0, cols = 0;
                for (const Blk& b : oa) {
                    add_term(sum.A, b.r * MB, b.c * KB, b.sign);
                    rows = std::max(rows, real(p->m, b.r * MB, MB));
                    cols = std::max(cols, real(p->k, b.c * KB, KB));
                }
                setop(sum.C, V_RSTA, V_CSTA, MB, KB, 1, p->wsTA);
                add_term(sum.C, 0, 0, 1.0);
                sum.mb = MB, sum.nb = KB, sum.first_mask = 1, sum.overwrite = 1;
                p->steps.push_back(Step{STEP_LINCOMB, (int)p->prods.size(), 1, {}, MB, KB, p->a_mode == 0 ? 1 : 0, 0});
                p->prods.push_back(sum);
                sa = Src{V_RSTA, V_CSTA, MB, KB, 0, 0, rows, cols, 1, p->wsTA, false};
            }
            if (sb.direct) {
                sb = Src{V_RSB, V_CSB, p->k, p->n, ob[0].r * KB, ob[0].c * NB, real(p->k, ob[0].r * KB, KB), real(p->n, ob[0].c * NB, NB), 0, 0, true};
            } else {
                Product sum;
                std::memset(&sum, 0, sizeof sum);
                setop(sum.A, V_RSB, V_CSB, p->k, p->n, 0, 0);
                int64_t rows = 0, cols = 0;
                for (const Blk& b : ob) {
                    add_term(sum.A, b.r * KB, b.c * NB, b.sign);
                    rows = std::max(rows, real(p->k, b.r * KB, KB));
                    cols = std::max(cols, real(p->n, b.c * NB, NB));
                }
                setop(sum.C, V_RSTB, V_CSTB, KB, NB, 1, p->wsTB);
                add_term(sum.C, 0, 0, 1.0);
                sum.mb = KB, sum.nb = NB, sum.first_mask = 1, sum.overwrite = 1;
                p->steps.push_back(Step{STEP_LINCOMB, (int)p->prods.size(), 1, {}, KB, NB, p->b_mode == 1 ? 1 : 0, 1});
                p->prods.push_back(sum);
                sb = Src{V_RSTB, V_CSTB, KB, NB, 0, 0, rows, cols, 1, p->wsTB, false};
            }
            std::vector<Pending> list;
            for (int q = 0; q < R2; ++q) {
                Pending e;
                std::memset(&e.pr, 0, sizeof e.pr);
                std::memset(&e.view, 0, sizeof e.view);
                setop(e.pr.A, sa.rs, sa.cs, sa.rs_len, sa.cs_len, sa.space, sa.base);
                setop(e.pr.B, sb.rs, sb.cs, sb.rs_len, sb.cs_len, sb.space, sb.base);
                setop(e.pr.C, V_RSC, V_CSC, p->m, p->n, 0, 0);
                e.pr.mb = p->mb, e.pr.nb = p->nb, e.pr.kb = p->kb;
                for (int i = 0; i < h; ++i)
                    for (int j = 0; j < h; ++j) {
                        if (U2[q][i * h + j] && i * p->mb < sa.rows && j * p->kb < sa.cols) {
                            add_term(e.pr.A, sa.r0 + i * p->mb, sa.c0 + j * p->kb, U2[q][i * h + j]);
                            for (const Blk& b : oa)  // what the product means on the 4 x 4 grid
                                if (e.view.n_a < 4) {
                                    const int t = e.view.n_a++;
                                    e.view.a_row[t] = h * b.r + i, e.view.a_col[t] = h * b.c + j, e.view.a_sign[t] = b.sign * U2[q][i * h + j];
                                }
                        }
                        if (V2[q][i * h + j] && i * p->kb < sb.rows && j * p->nb < sb.cols) {
                            add_term(e.pr.B, sb.r0 + i * p->kb, sb.c0 + j * p->nb, V2[q][i * h + j]);
                            for (const Blk& b : ob)
                                if (e.view.n_b < 4) {
                                    const int t = e.view.n_b++;
                                    e.view.b_row[t] = h * b.r + i, e.view.b_col[t] = h * b.c + j, e.view.b_sign[t] = b.sign * V2[q][i * h + j];
                                }
                        }
                        if (W2[q][i * h + j])
                            for (const Blk& b : oc) {
                                const int bi = h * b.r + i, bj = h * b.c + j;
                                if (bi * p->mb < p->m && bj * p->nb < p->n) {
                                    add_term(e.pr.C, bi * p->mb, bj * p->nb, b.sign * W2[q][i * h + j]);
                                    const int t = e.view.n_c++;
                                    e.view.c_row[t] = bi, e.view.c_col[t] = bj, e.view.c_sign[t] = b.sign * W2[q][i * h + j];
                                }
                            }
                    }
                lead_with_plus(e.pr.A);
                lead_with_plus(e.pr.B);
                if (e.pr.A.nterms == 0 || e.pr.B.nterms == 0 || e.pr.C.nterms == 0) continue;
                list.push_back(e);
            }
            tc::FusedConfig cfg{sa.direct ? p->a_mode : 0, sb.direct ? p->b_mode : 1, 1, 1, sa.direct ? p->a_vec : 1, sb.direct ? p->b_vec : 1,
                                sa.space, sb.space, p->c_mode, 128};
            emit(list, cfg, true);
        }
    } else {
        for (int which = 0; which < 2; ++which) {
            if (!(which == 0 ? repack_a : repack_b)) continue;
            Product cp;
            std::memset(&cp, 0, sizeof cp);
            const int64_t rows = which == 0 ? m_full : p->k, cols = which == 0 ? p->k : n_full;
            setop(cp.A, which == 0 ? V_RSA : V_RSB, which == 0 ? V_CSA : V_CSB, rows, cols, 0, 0);
            add_term(cp.A, 0, 0, 1.0);
            setop(cp.C, which == 0 ? V_RSTA : V_RSTB, which == 0 ? V_CSTA : V_CSTB, rows, cols, 1, which == 0 ? p->wsTA : p->wsTB);
            add_term(cp.C, 0, 0, 1.0);
            cp.mb = rows, cp.nb = cols, cp.first_mask = 1, cp.overwrite = 1;
            p->steps.push_back(Step{STEP_LINCOMB, (int)p->prods.size(), 1, {}, rows, cols, (which == 0 ? p->a_mode == 0 : p->b_mode == 1) ? 1 : 0, which});
            p->prods.push_back(cp);
        }
        std::vector<std::vector<int>> U, V, W;
        block_tables(level, U, V, W);
        const int R = (int)U.size();
        std::vector<Pending> list;
        for (int r = 0; r < R; ++r) {
            Pending e;
            std::memset(&e.pr, 0, sizeof e.pr);
            std::memset(&e.view, 0, sizeof e.view);
            set_a(e.pr.A, p->m);
            set_b(e.pr.B, p->n);
            setop(e.pr.C, V_RSC, V_CSC, p->m, p->n, 0, 0);
            e.pr.mb = p->mb;
            e.pr.nb = p->nb;
            e.pr.kb = p->kb;
            for (int bi = 0; bi < g; ++bi)
                for (int bk = 0; bk < g; ++bk)
                    if (U[r][bi * g + bk] && bi * p->mb < p->m && bk * p->kb < p->k) {
                        add_term(e.pr.A, bi * p->mb, bk * p->kb, U[r][bi * g + bk]);
                        e.view.a_row[e.view.n_a] = bi, e.view.a_col[e.view.n_a] = bk, e.view.a_sign[e.view.n_a] = U[r][bi * g + bk], ++e.view.n_a;
                    }
            for (int bk = 0; bk < g; ++bk)
                for (int bj = 0; bj < g; ++bj)
                    if (V[r][bk * g + bj] && bk * p->kb < p->k && bj * p->nb < p->n) {
                        add_term(e.pr.B, bk * p->kb, bj * p->nb, V[r][bk * g + bj]);
                        e.view.b_row[e.view.n_b] = bk, e.view.b_col[e.view.n_b] = bj, e.view.b_sign[e.view.n_b] = V[r][bk * g + bj], ++e.view.n_b;
                    }
            for (int bi = 0; bi < g; ++bi)
                for (int bj = 0; bj < g; ++bj)
                    if (W[r][bi * g + bj] && bi * p->mb < p->m && bj * p->nb < p->n) {
                        add_term(e.pr.C, bi * p->mb, bj * p->nb, W[r][bi * g + bj]);
                        e.view.c_row[e.view.n_c] = bi, e.view.c_col[e.view.n_c] = bj, e.view.c_sign[e.view.n_c] = W[r][bi * g + bj], ++e.view.n_c;
                    }
            lead_with_plus(e.pr.A);
            lead_with_plus(e.pr.B);
            // a product whose operand sum or destination set lies wholly in the zero padding contributes nothing
            if (e.view.n_a == 0 || e.view.n_b == 0 || e.view.n_c == 0) continue;
            list.push_back(e);
        }
        tc::FusedConfig base_cfg{a_mode, b_mode, 1, 1, a_vec, b_vec, repack_a ? 1 : 0, repack_b ? 1 : 0, p->c_mode, 128};
        emit(list, base_cfg, variant == TC_VARIANT_ABC || level == 0);
    }
    // ---- edge products of the peeled rows and columns: classical, each the first and only writer of its part of C ----
    p->m = m_full, p->n = n_full;
    if (!empty && p->k > 0) {
        auto edge = [&](int64_t r0, int64_t rows, int64_t c0, int64_t cols) {
            Product pr;
            std::memset(&pr, 0, sizeof pr);
            set_a(pr.A, r0 + rows);
            add_term(pr.A, r0, 0, 1.0);
            set_b(pr.B, c0 + cols);
            add_term(pr.B, 0, c0, 1.0);
            setop(pr.C, V_RSC, V_CSC, r0 + rows, c0 + cols, 0, 0);
            add_term(pr.C, r0, c0, 1.0);
            pr.mb = rows, pr.nb = cols, pr.kb = p->k;
            pr.first_mask = 1;
            const tc::FusedConfig cfg{a_mode, b_mode, 1, 1, a_vec, b_vec, repack_a ? 1 : 0, repack_b ? 1 : 0, p->c_mode, 128};
            p->steps.push_back(Step{STEP_FUSED, (int)p->prods.size(), 1, cfg, rows, cols, 0, 0});
            p->prods.push_back(pr);
        };
        if (p->m_peel > 0) edge(m_full - p->m_peel, p->m_peel, 0, n_full);
        if (p->n_peel > 0) edge(0, m_full - p->m_peel, n_full - p->n_peel, p->n_peel);
    }
    p->n_launches = (int)p->steps.size();
    // ---- tile shape and tails (launches whose tiles do not fill whole rounds of the compute units) ----
    int64_t chunk_elems = 0;
    for (Step& s : p->steps)
        if (s.kind == STEP_FUSED) choose_tiles(p, s, kDefaultModel, tile_mode, tail_mode, &chunk_elems);
    if (chunk_elems > 0) {
        p->wsPart = (int64_t)(p->workspace_bytes / sizeof(double));
        p->workspace_bytes += (size_t)chunk_elems * sizeof(double);
    }
    if (!p->host_only && !p->prods.empty()) {
        if (tc::dev_malloc((void**)&p->prods_dev, sizeof(Product) * p->prods.size())) return TC_ERR_HIP;
        if (tc::dev_upload(p->prods_dev, p->prods.data(), sizeof(Product) * p->prods.size(), stream)) return TC_ERR_HIP;
    }
    if (!p->host_only && tc::dev_stream_sync(stream)) return TC_ERR_HIP;
    return TC_OK;
}

void release(tc_plan_t* p) {
    if (!p) return;
    if (p->store_dev) tc::dev_free(p->store_dev);
    if (p->bundles_dev) tc::dev_free(p->bundles_dev);
    if (p->prods_dev) tc::dev_free(p->prods_dev);
    delete p;
}

void copy_labels(char* out, const std::vector<Dim>& b) {
    size_t i = 0;
    for (; i < b.size() && i < TC_MAX_NDIM; ++i) out[i] = b[i].label;
    out[i] = 0;
}

// ---- performance model (Sec. 5) on the plan's schedule ----
// Defaults: python -m paper_1704_03092_amd.sweep --fit on one MI355X (every launch of six plans of each shape of the
// grid; launches of a millisecond and more are reproduced to 5 - 8 % RMS).
extern const tc_model_params_t kDefaultModel = {
    78.6e12,               // published FP64 matrix peak
    // Tiles gathered by stride, 1 / 2 / 4-term operand sums.  (Two terms: the fits gave 0.958 - 0.976 of the single-term
    // figure; 0.97 of it is what the automatic choice does best with on the sweep.)
    {0.948, 0.920, 0.773},
    8.0e12,                // HBM3E
    0.742,                 // element-wise passes and destination updates
    11.6e-6,               // per launch (the fixed part of a kernel's duration)
    2.71e-6,               // per wave of tiles: gather tables, pipeline fill, destination update
    256, {0, 0, 0},
    1.047,                 // 128 x 64 tiles (fitted to the classical plans measured in both tile shapes)
    0.0,                   // no cost per wave of their own: one workgroup's fill and update hide behind the other's multiplications
    0.858,                 // element-by-element gathers
    0.0053,                // operand reads not hidden behind the matrix cores
    // Tiles gathered through the scatter tables.  Two-term sums: the fits give 0.838 - 0.883, with a wide scatter over
    // the tensors' layouts (0.70 - 0.93 per shape).  The default is set below them on purpose: from 0.83 on the
    // automatic choice takes a Strassen level for a tensor of the sweep on which that level measures 12 % slower
    // (its own two-term launches run at 0.80).
    {0.870, 0.810, 0.592},
    // 128 x 64 tiles gathered through the tables (their address arithmetic waits for the partner's matrix cores):
    // 0.96 - 0.97 measured on launches of thousands of tiles; 0.98 also lets the launches of a few hundred chunks
    // take this shape, where it measures 7 % faster (9216 x 96 x 4096: 0.250 -> 0.233 ms).
    0.980};

// What the model needs to know of a fused launch.
struct FusedShape {
    int64_t tiles, kb;
    int terms, tile_n;
    double c_elems;
    double op_elems;  // elements of A and B that the tiles of the launch read (every tile its panels of every summed block)
    bool pairs;       // both operands gathered two contiguous elements at a time
    double free_frac; // share of the tiles gathered by stride
};

FusedShape fused_shape(const tc_plan_t* p, const Step& s) {
    FusedShape f{0, 0, 1, 128, 0.0, 0.0, true, s.free_frac};
    f.tile_n = s.cfg.tile_n;
    f.pairs = s.cfg.a_vec && s.cfg.b_vec;
    const int64_t per_prod = ((s.rows + 127) / 128) * ((s.cols + f.tile_n - 1) / f.tile_n);
    f.tiles = (int64_t)s.count * per_prod;
    for (int i = s.first; i < s.first + s.count; ++i) {
        const Product& q = p->prods[i];
        f.terms = std::max(f.terms, std::max(q.A.nterms, q.B.nterms));
        f.kb = q.kb;
        f.c_elems += (q.overwrite ? 1.0 : 2.0) * q.C.nterms * (double)q.mb * (double)q.nb;
        f.op_elems += (double)per_prod * (double)q.kb * (128.0 * q.A.nterms + (double)f.tile_n * q.B.nterms);
    }
    return f;
}

// Merged run of a bundle's fastest dimensions: entries [q * len, (q + 1) * len) of its scatter vector are equally
// spaced by `stride` for every q (dimensions chain while each stride is the previous stride times the previous length).
struct Run {
    int64_t stride, len;
};

Run fastest_run(const BundleDesc& b) {
    Run r{0, 1};
    int64_t next = 0;
    bool first = true;
    for (int d = 0; d < b.ndim; ++d) {
        if (b.len[d] <= 1) continue;
        if (first) {
            r.stride = b.stride[d];
            first = false;
        } else if (b.stride[d] != next) {
            break;
        }
        r.len *= b.len[d];
        next = b.stride[d] * b.len[d];
    }
    if (first) r.len = b.total > 0 ? b.total : 1;  // a single entry
    return r;
}

// How many tiles of a fused launch the kernel gathers by stride, without its scatter tables (the kernel decides this
// per tile from the block scatter vectors; this is the same decision made from the bundle descriptions).
// A tail tile cut into chunks counts if its chunks do.
int64_t count_table_free(const tc_plan_t* p, const Step& s) {
    if (s.kind != STEP_FUSED || !s.cfg.a_vec || !s.cfg.b_vec || s.cfg.nta == 0) return 0;  // pair-wise gathers and exact term counts only
    const int64_t limit = (int64_t)1 << 20;
    const int64_t TN = s.cfg.tile_n;
    const int KT = (TN == 128 && s.cfg.nta + s.cfg.ntb <= 6) ? 32 : 16;  // the kernel's k-step depth (Cfg::KT)
    const int64_t tiles_m = (s.rows + 127) / 128, tiles_n = (s.cols + TN - 1) / TN;
    const int64_t per_prod = tiles_m * tiles_n, main_count = (int64_t)s.count * per_prod - s.tail_tiles;
    int64_t n = 0;
    for (int pi = 0; pi < s.count; ++pi) {
        const Product& q = p->prods[s.first + pi];
        if (q.A.cs_stride < 0 || q.B.rs_stride < 0 || q.A.cs_stride >= limit || q.B.rs_stride >= limit) continue;
        // the run structure of the scatter vector an operand reads along its free bundle
        auto run_of = [&](const Operand& op, bool rows) -> Run {
            const int64_t st = rows ? op.rs_stride : op.cs_stride;
            if (st >= 0) return Run{st, INT64_MAX};
            if (p->bs_block != 16) return Run{0, 0};  // the kernel gets no block scatter vectors then
            return fastest_run(p->bundles[rows ? op.rs_id : op.cs_id]);
        };
        const Run ra = run_of(q.A, true), rb = run_of(q.B, false);
        if (ra.stride >= limit || rb.stride >= limit) continue;
        if ((ra.len != INT64_MAX && (ra.len < 128 || ra.stride <= 0)) || (rb.len != INT64_MAX && (rb.len < TN || rb.stride <= 0))) continue;
        for (int64_t tm = 0; tm < tiles_m; ++tm)
            for (int64_t tn = 0; tn < tiles_n; ++tn) {
                const int64_t i0 = tm * 128, j0 = tn * TN;
                bool ok = true;
                int64_t klimit = q.kb;
                for (int t = 0; t < q.A.nterms && ok; ++t) {
                    ok = std::min(q.mb, q.A.rs_len - q.A.roff[t]) - i0 >= 128;
                    klimit = std::min(klimit, q.A.cs_len - q.A.coff[t]);
                    const int64_t f0 = q.A.roff[t] + i0;
                    if (ok && ra.len != INT64_MAX) ok = f0 % ra.len + 128 <= ra.len;
                }
                for (int t = 0; t < q.B.nterms && ok; ++t) {
                    ok = std::min(q.nb, q.B.cs_len - q.B.coff[t]) - j0 >= TN;
                    klimit = std::min(klimit, q.B.rs_len - q.B.roff[t]);
                    const int64_t f0 = q.B.coff[t] + j0;
                    if (ok && rb.len != INT64_MAX) ok = f0 % rb.len + TN <= rb.len;
                }
                if (!ok) continue;
                // either no padded k-step (every term reaches the full depth, which is a whole, even number of
                // k-steps), or at least four whole k-steps ahead of the padded ones (those then go through the tables)
                auto depth_ok = [&](int64_t depth, int64_t real) { return (real == depth && depth % (2 * KT) == 0) || real / KT >= 4; };
                // position of the tile in the launch: the last tail_tiles logical ids are cut into chunks
                const int64_t gsz = 8 * tiles_n, grp = tm / 8, gm0 = grp * 8, gh = std::min<int64_t>(8, tiles_m - gm0);
                const int64_t lid = (int64_t)pi * per_prod + grp * gsz + tn * gh + (tm - gm0);
                if (lid < main_count) {
                    ok = depth_ok(q.kb, klimit);
                } else {
                    for (int64_t c = 0; c < s.tail_chunks && ok; ++c) {
                        const int64_t d = std::min<int64_t>(s.tail_kc, q.kb - c * s.tail_kc);
                        ok = depth_ok(d, std::min(d, klimit - c * s.tail_kc));
                    }
                }
                n += ok;
            }
    }
    return n;
}

// Modelled time of a fused launch except its destination updates: whole tiles in whole waves (one 128 x 128 tile, or
// two 128 x 64 tiles, per compute unit), the chunks of the tail tiles in whole waves of their own depth, the chunks
// written and read back, the second launch.
struct TailCost {
    double arith, temporaries, launch, operands;
    double total() const { return arith + temporaries + launch + operands; }
};

int64_t tiles_per_wave(const tc_model_params_t& mp, int tile_n) { return (int64_t)mp.units * (128 / tile_n); }

TailCost fused_cost(const tc_model_params_t& mp, const FusedShape& f, int64_t tail_tiles, int64_t chunks, int64_t kc) {
    const bool small = f.tile_n == 64;
    const int cls = f.terms <= 1 ? 0 : f.terms <= 2 ? 1 : 2;
    const double by_stride = mp.rho_a[cls] * (small ? mp.rho_small : 1.0), by_table = mp.rho_table[cls] * (small ? mp.rho_small_table : 1.0);
    const double rho = 1.0 / (f.free_frac / by_stride + (1.0 - f.free_frac) / by_table) * (f.pairs ? 1.0 : mp.rho_gather);
    const double fixed = small ? mp.t_tile_small : mp.t_tile;
    const int64_t per = tiles_per_wave(mp, f.tile_n);
    auto wave = [&](int64_t depth) { return mp.units * 2.0 * 128.0 * 128.0 * (double)depth / (rho * mp.peak_flops) + fixed; };
    TailCost c{0, 0, mp.t_launch, mp.lambda_ab * f.op_elems * 8.0 / (mp.rho_b * mp.bandwidth)};
    const int64_t whole = f.tiles - tail_tiles;
    c.arith = (double)((whole + per - 1) / per) * wave(f.kb);
    if (tail_tiles > 0) {
        c.arith += (double)((tail_tiles * chunks + per - 1) / per) * wave(kc);
        c.temporaries = 2.0 * (double)(tail_tiles * chunks) * 128.0 * f.tile_n * 8.0 / (mp.rho_b * mp.bandwidth);
        c.launch += mp.t_launch;  // the second launch
    }
    return c;
}

// The tail of a launch: the tiles beyond the last full round of the compute units.  Cut into 2..16 chunks of a
// multiple of 64 contracted entries if the model says that this is faster than running them whole.
// forced >= 2: that many chunks whatever the model says.  Returns the modelled time of the choice.
double choose_tail(const tc_plan_t* p, Step& s, const tc_model_params_t& mp, int forced) {
    s.tail_tiles = s.tail_chunks = 0;
    s.tail_kc = 0;
    const FusedShape f = fused_shape(p, s);
    if (f.tiles <= 0) return 0.0;
    double best = fused_cost(mp, f, 0, 0, 0).total();
    const int64_t r = f.tiles % tiles_per_wave(mp, f.tile_n);
    if (forced < 0 || r == 0 || f.tiles > 0x7fffffff) return best;
    for (int64_t want = forced ? forced : 2; want <= (forced ? forced : 16); ++want) {
        const int64_t kc = round_up((f.kb + want - 1) / want, 64);
        const int64_t chunks = (f.kb + kc - 1) / kc;
        if (chunks < 2 || r * chunks > 1024) continue;
        const double t = fused_cost(mp, f, r, chunks, kc).total();
        if (forced || t < best) {
            best = t;
            s.tail_tiles = (int)r;
            s.tail_chunks = (int)chunks;
            s.tail_kc = kc;
        }
    }
    return best;
}

// Tile shape, then tail, of one fused launch.  Launches of single-block products may run in 128 x 64 tiles, two
// workgroups per compute unit; the model picks the shape with the smaller time (tile_mode 0) or the caller does.
// *chunk_elems grows to the elements of workspace that the launch's chunks need.
void choose_tiles(const tc_plan_t* p, Step& s, const tc_model_params_t& mp, int tile_mode, int tail_mode, int64_t* chunk_elems) {
    const bool may_small = s.cfg.nta == 1 && s.cfg.ntb == 1;
    auto with_tiles = [&](int tile_n) {
        s.cfg.tile_n = tile_n;
        s.tail_tiles = s.tail_chunks = 0;
        const int64_t tiles = (int64_t)s.count * ((s.rows + 127) / 128) * ((s.cols + tile_n - 1) / tile_n);
        s.free_frac = tiles > 0 ? (double)count_table_free(p, s) / (double)tiles : 0.0;
        return choose_tail(p, s, mp, tail_mode);
    };
    const double t = with_tiles(128);
    if (may_small && tile_mode != 128) {
        const Step big = s;
        const double ts = with_tiles(64);
        // A launch that mixes tiles gathered by stride with tiles gathered through the tables stays in 128 x 128 tiles
        // whatever the model says: next to a workgroup whose loop is all matrix-core instructions, a workgroup whose
        // loop computes addresses on the vector unit is starved (measured: 3.7 times the tile time; the model has no
        // term for who a tile's neighbour is).  All by stride, or all through the tables, the two are even.
        const bool mixed = s.free_frac > 0.0 && s.free_frac < 1.0;
        if (tile_mode == 0 && (ts >= t || mixed)) s = big;
    }
    *chunk_elems = std::max<int64_t>(*chunk_elems, (int64_t)s.tail_tiles * s.tail_chunks * 128 * s.cfg.tile_n);
}

void predict(const tc_plan_t* p, const tc_model_params_t& mp, tc_model_time_t* out) {
    const double tau_b = 8.0 / (mp.rho_b * mp.bandwidth);
    tc_model_time_t t = {0, 0, 0, 0, 0, 0};
    for (const Step& s : p->steps) {
        if (s.kind == STEP_FUSED) {
            const FusedShape f = fused_shape(p, s);
            if (f.tiles == 0) {
                t.launch += mp.t_launch;
                continue;
            }
            const TailCost c = fused_cost(mp, f, s.tail_tiles, s.tail_chunks, s.tail_kc);
            t.arith += c.arith;
            t.temporaries += c.temporaries;
            t.launch += c.launch;
            t.operands += c.operands;
            t.c_update += f.c_elems * tau_b;
        } else {
            t.launch += mp.t_launch;
            const Product& q = p->prods[s.first];
            const double elems = (q.A.nterms + (q.overwrite ? 1.0 : 2.0) * q.C.nterms) * (double)s.rows * (double)s.cols;
            t.temporaries += elems * tau_b;
        }
    }
    t.total = t.arith + t.c_update + t.temporaries + t.launch + t.operands;
    *out = t;
}

// split_k = -1: the number of chunks (1..4) with the smallest modelled time
int choose_split(const tc_tensor_desc_t* A, const tc_tensor_desc_t* B, const tc_tensor_desc_t* C, int variant, tc_options_t* o) {
    tc_options_t t = *o;
    t.host_only = 1;
    double best = 0;
    int best_s = 1;
    for (int s = 1; s <= 4; ++s) {
        t.split_k = s;
        tc_plan_t cand;
        int rc = build_plan(&cand, A, B, C, 0, variant, &t, nullptr);
        if (rc != TC_OK) return rc;
        tc_model_time_t mt;
        predict(&cand, kDefaultModel, &mt);
        if (s == 1 || mt.total < best) best = mt.total, best_s = s;
    }
    o->split_k = best_s;
    return TC_OK;
}

// TC_LEVEL_AUTO / TC_VARIANT_AUTO: schedule every candidate on the host, keep the one the model likes best.
int choose_by_model(const tc_tensor_desc_t* A, const tc_tensor_desc_t* B, const tc_tensor_desc_t* C, int* level, int* variant,
                    const tc_options_t* opts) {
    tc_options_t o;
    std::memset(&o, 0, sizeof o);
    if (opts) o = *opts;
    o.host_only = 1;
    tc_options_t o0 = o;  // level 0 competes with the split it would run with
    if (o.split_k == -1) {
        o0.split_k = 1;
        if (o.tail_split != 0) {  // (the automatic tail split does that job inside the kernel)
            int rc = choose_split(A, B, C, TC_VARIANT_ABC, &o0);
            if (rc != TC_OK) return rc;
        }
        o.split_k = 1;
    }
    double best = 0;
    int best_level = -1, best_variant = -1;
    for (int L = 0; L <= 2; ++L) {
        if (*level != TC_LEVEL_AUTO && L != *level) continue;
        for (int v = TC_VARIANT_HYBRID; v >= TC_VARIANT_NAIVE; --v) {
            if (v == TC_VARIANT_HYBRID && L == 0 && *variant == TC_VARIANT_AUTO) continue;  // the same as ABC without a Strassen level
            if (*variant != TC_VARIANT_AUTO && v != *variant) continue;
            if (L == 0 && v != TC_VARIANT_ABC && *variant == TC_VARIANT_AUTO) continue;  // the variants coincide at level 0
            tc_plan_t cand;
            int rc = build_plan(&cand, A, B, C, L, v, L == 0 ? &o0 : &o, nullptr);
            if (rc != TC_OK) return rc;
            if (cand.level != L) continue;  // lowered: the same schedule as a smaller L
            tc_model_time_t t;
            predict(&cand, kDefaultModel, &t);
            if (best_level < 0 || t.total < best) best = t.total, best_level = L, best_variant = v;
        }
    }
    if (best_level < 0) best_level = 0, best_variant = (*variant == TC_VARIANT_AUTO) ? TC_VARIANT_ABC : *variant;
    *level = best_level;
    *variant = best_variant;
    return TC_OK;
}

}  // namespace

extern "C" {

int tc_model_defaults(tc_model_params_t* out) {
    if (!out) return TC_ERR_NULL;
    *out = kDefaultModel;
    return TC_OK;
}

int tc_plan_predict(const tc_plan_t* plan, const tc_model_params_t* params, tc_model_time_t* out) {
    if (!plan || !out) return TC_ERR_NULL;
    const tc_model_params_t& mp = params ? *params : kDefaultModel;
    if (!(mp.peak_flops > 0) || !(mp.bandwidth > 0) || !(mp.rho_b > 0) || mp.units <= 0) return TC_ERR_STATE;
    for (int i = 0; i < 3; ++i)
        if (!(mp.rho_a[i] > 0)) return TC_ERR_STATE;
    predict(plan, mp, out);
    return TC_OK;
}

int tc_plan_ex(tc_plan_t** plan_out, const tc_tensor_desc_t* A, const tc_tensor_desc_t* B, const tc_tensor_desc_t* C, int level,
               int variant, const tc_options_t* opts, void* stream) {
    if (!plan_out) return TC_ERR_NULL;
    *plan_out = nullptr;
    tc_plan_t* p = nullptr;
    try {
        if (level == TC_LEVEL_AUTO || variant == TC_VARIANT_AUTO) {
            if (level != TC_LEVEL_AUTO && (level < 0 || level > 2)) return TC_ERR_LEVEL;
            if (variant != TC_VARIANT_AUTO && (variant < TC_VARIANT_NAIVE || variant > TC_VARIANT_HYBRID)) return TC_ERR_VARIANT;
            int rc = choose_by_model(A, B, C, &level, &variant, opts);
            if (rc != TC_OK) return rc;
        }
        tc_options_t o;
        std::memset(&o, 0, sizeof o);
        if (opts) o = *opts;
        if (o.split_k == -1) {
            o.split_k = 1;
            if (level == 0 && o.tail_split != 0) {
                int rc = choose_split(A, B, C, variant, &o);
                if (rc != TC_OK) return rc;
            }
        }
        p = new tc_plan_t();
        int rc = build_plan(p, A, B, C, level, variant, &o, stream);
        if (rc != TC_OK) {
            release(p);
            return rc;
        }
    } catch (...) {
        release(p);
        return TC_ERR_HIP;
    }
    *plan_out = p;
    return TC_OK;
}

int tc_plan(tc_plan_t** plan_out, const tc_tensor_desc_t* A, const tc_tensor_desc_t* B, const tc_tensor_desc_t* C, int level,
            int variant, void* stream) {
    return tc_plan_ex(plan_out, A, B, C, level, variant, nullptr, stream);
}

size_t tc_plan_workspace_bytes(const tc_plan_t* plan) { return plan ? plan->workspace_bytes : 0; }

namespace {
int run_step(const tc_plan_t* plan, const Step& s, double alpha, const double* A_dev, const double* B_dev, double beta, double* C_dev, double* W,
             void* stream) {
    if (s.kind == STEP_FUSED)
        return tc::launch_fused(s.cfg, plan->prods_dev, s.first, s.count, s.rows, s.cols, A_dev, B_dev, C_dev, W, alpha, beta, s.tail_tiles,
                                s.tail_chunks, s.tail_kc, plan->wsPart, stream);
    const Product& q = plan->prods[s.first];
    return tc::launch_lincomb(plan->prods_dev, s.first, q.A.nterms, q.C.nterms, s.rows, s.cols, s.lanes_along_rows, A_dev, B_dev, C_dev, W, s.src_role,
                              beta, stream);
}
}  // namespace

int tc_contract(const tc_plan_t* plan, double alpha, const double* A_dev, const double* B_dev, double beta, double* C_dev,
                void* workspace_dev, void* stream) {
    if (!plan) return TC_ERR_NULL;
    if (plan->host_only) return TC_ERR_STATE;
    if (plan->steps.empty()) return TC_OK;  // an empty free bundle: nothing to write
    if (!C_dev) return TC_ERR_NULL;
    if (plan->k > 0 && (!A_dev || !B_dev)) return TC_ERR_NULL;
    if (plan->workspace_bytes > 0 && !workspace_dev) return TC_ERR_WORKSPACE;
    double* W = (double*)workspace_dev;
    for (const Step& s : plan->steps)
        if (run_step(plan, s, alpha, A_dev, B_dev, beta, C_dev, W, stream)) return TC_ERR_HIP;
    return TC_OK;
}

int tc_contract_static(const tc_plan_t* plan, double alpha, const double* A_dev, const double* B_dev, double beta, double* C_dev,
                       void* stream) {
    if (!plan) return TC_ERR_NULL;
    if (plan->host_only) return TC_ERR_STATE;
    if (plan->workspace_bytes > tc::kStaticWorkspaceBytes) return TC_ERR_CAPACITY;
    void* ws = nullptr;
    if (plan->workspace_bytes > 0 && tc::dev_static_workspace(&ws)) return TC_ERR_HIP;
    return tc_contract(plan, alpha, A_dev, B_dev, beta, C_dev, ws, stream);
}

int tc_contract_launch_times(const tc_plan_t* plan, double alpha, const double* A_dev, const double* B_dev, double beta, double* C_dev,
                             void* workspace_dev, void* stream, double* ms_out, int capacity) {
    if (!plan) return TC_ERR_NULL;
    if (plan->host_only) return TC_ERR_STATE;
    const int n = (int)plan->steps.size();
    if (n == 0) return 0;
    if (!ms_out || capacity < n) return TC_ERR_RANGE;
    if (!C_dev) return TC_ERR_NULL;
    if (plan->k > 0 && (!A_dev || !B_dev)) return TC_ERR_NULL;
    if (plan->workspace_bytes > 0 && !workspace_dev) return TC_ERR_WORKSPACE;
    double* W = (double*)workspace_dev;
    std::vector<void*> ev(plan->steps.size() + 1, nullptr);
    int rc = TC_OK;
    for (void*& e : ev)
        if (tc::dev_event_create(&e)) rc = TC_ERR_HIP;
    if (rc == TC_OK && tc::dev_event_record(ev[0], stream)) rc = TC_ERR_HIP;
    for (size_t i = 0; i < plan->steps.size() && rc == TC_OK; ++i) {
        if (run_step(plan, plan->steps[i], alpha, A_dev, B_dev, beta, C_dev, W, stream) || tc::dev_event_record(ev[i + 1], stream)) rc = TC_ERR_HIP;
    }
    if (rc == TC_OK && tc::dev_event_sync(ev.back())) rc = TC_ERR_HIP;
    for (size_t i = 0; i < plan->steps.size() && rc == TC_OK; ++i) {
        float ms = 0;
        if (tc::dev_event_elapsed_ms(&ms, ev[i], ev[i + 1])) {
            rc = TC_ERR_HIP;
            break;
        }
        ms_out[i] = ms;
    }
    for (void* e : ev)
        if (e) tc::dev_event_destroy(e);
    return rc == TC_OK ? n : rc;
}

int tc_contract_timed(const tc_plan_t* plan, double alpha, const double* A_dev, const double* B_dev, double beta, double* C_dev,
                      void* workspace_dev, void* stream, tc_launch_times_t* out) {
    if (!plan || !out) return TC_ERR_NULL;
    std::memset(out, 0, sizeof *out);
    std::vector<double> ms(plan->steps.size() + 1, 0.0);
    const int n = tc_contract_launch_times(plan, alpha, A_dev, B_dev, beta, C_dev, workspace_dev, stream, ms.data(), (int)ms.size());
    if (n < 0) return n;
    for (int i = 0; i < n; ++i) {
        if (plan->steps[i].kind == STEP_FUSED)
            out->fused_ms += ms[i], ++out->fused_launches;
        else
            out->elementwise_ms += ms[i], ++out->elementwise_launches;
    }
    return TC_OK;
}

int tc_bench_mfma_peak(int instruction, void* stream, double* tflops_out) {
    if (!tflops_out) return TC_ERR_NULL;
    if (instruction != 0 && instruction != 1) return TC_ERR_RANGE;
    *tflops_out = 0.0;
    return tc::bench_mfma_peak(instruction, 4000, stream, tflops_out) ? TC_ERR_HIP : TC_OK;
}

int tc_destroy(tc_plan_t* plan) {
    release(plan);
    return TC_OK;
}

const char* tc_strerror(int status) {
    switch (status) {
        case TC_OK: return "success";
        case TC_ERR_NULL: return "required pointer argument is NULL";
        case TC_ERR_NDIM: return "tensor dimensionality out of range";
        case TC_ERR_LABEL: return "index label repeated in a tensor or not present in exactly two tensors";
        case TC_ERR_LENGTH: return "negative length or one label with two lengths";
        case TC_ERR_STRIDE: return "negative or zero stride, or elements of C may overlap";
        case TC_ERR_LEVEL: return "Strassen level must be 0, 1 or 2";
        case TC_ERR_VARIANT: return "unknown variant";
        case TC_ERR_WORKSPACE: return "workspace required but NULL";
        case TC_ERR_HIP: return "HIP runtime call failed";
        case TC_ERR_STATE: return "plan cannot run (host-only) or option out of range";
        case TC_ERR_RANGE: return "index or capacity out of range";
        case TC_ERR_CAPACITY: return "the plan needs more workspace than the static buffer holds (TC_STATIC_WORKSPACE_BYTES)";
        default: return "unknown status";
    }
}

int tc_plan_info(const tc_plan_t* plan, tc_plan_info_t* out) {
    if (!plan || !out) return TC_ERR_NULL;
    std::memset(out, 0, sizeof *out);
    out->m = plan->m, out->n = plan->n, out->k = plan->k;
    out->level_requested = plan->level_requested;
    out->level = plan->level;
    out->variant = plan->variant;
    out->n_products = (int)plan->sched.size();
    out->n_launches = plan->n_launches;
    out->bs_block = plan->bs_block;
    out->a_mode = plan->a_mode, out->b_mode = plan->b_mode;
    out->mb = plan->mb, out->nb = plan->nb, out->kb = plan->kb;
    copy_labels(out->I, plan->I);
    copy_labels(out->J, plan->J);
    copy_labels(out->P, plan->P);
    out->m_peel = plan->m_peel, out->n_peel = plan->n_peel;
    return TC_OK;
}

int tc_plan_schedule(const tc_plan_t* plan, int index, tc_product_t* out) {
    if (!plan || !out) return TC_ERR_NULL;
    if (index < 0 || index >= (int)plan->sched.size()) return TC_ERR_RANGE;
    *out = plan->sched[index];
    return TC_OK;
}

int tc_plan_launch(const tc_plan_t* plan, int index, tc_launch_info_t* out) {
    if (!plan || !out) return TC_ERR_NULL;
    if (index < 0 || index >= (int)plan->steps.size()) return TC_ERR_RANGE;
    std::memset(out, 0, sizeof *out);
    const Step& s = plan->steps[index];
    out->kind = s.kind == STEP_FUSED ? 0 : 1;
    out->rows = s.rows, out->cols = s.cols;
    if (s.kind == STEP_FUSED) {
        const FusedShape f = fused_shape(plan, s);
        out->n_products = s.count;
        out->max_terms = f.terms;
        out->terms_a = s.cfg.nta;
        out->terms_b = s.cfg.ntb;
        out->tile_n = s.cfg.tile_n;
        out->tiles_table_free = count_table_free(plan, s);
        out->depth = f.kb;
        out->tiles = f.tiles;
        out->tail_tiles = s.tail_tiles, out->tail_chunks = s.tail_chunks, out->tail_kc = s.tail_kc;
        out->moved_elems = f.c_elems;
        out->pairs_a = s.cfg.a_vec ? 1 : 0, out->pairs_b = s.cfg.b_vec ? 1 : 0;
    } else {
        const Product& q = plan->prods[s.first];
        out->moved_elems = (q.A.nterms + (q.overwrite ? 1.0 : 2.0) * q.C.nterms) * (double)s.rows * (double)s.cols;
    }
    return TC_OK;
}

int64_t tc_plan_vector(const tc_plan_t* plan, int which, int64_t* host_out, int64_t capacity) {
    if (!plan) return TC_ERR_NULL;
    if (which < 0 || which >= 12) return TC_ERR_RANGE;
    const BundleDesc& b = plan->bundles[which % 6];
    int64_t count = which < 6 ? b.total : (b.total + plan->bs_block - 1) / plan->bs_block;
    if (!host_out) return count;
    if (plan->host_only || !plan->store_dev) return TC_ERR_STATE;
    int64_t ncopy = std::min(count, capacity);
    if (ncopy > 0 && tc::dev_download(host_out, plan->store_dev + (which < 6 ? b.out_off : b.bs_off), sizeof(int64_t) * (size_t)ncopy))
        return TC_ERR_HIP;
    return count;
}

}  // extern "C"
