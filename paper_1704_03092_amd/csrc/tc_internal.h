// Internal interface between the host planner (tc_host.cpp) and the device code (tc_device.hip).
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace tc {

constexpr int kMaxTerms = 4;  // 2^L blocks per operand at L = 2
// Scatter-table entry for a row/column that lies outside the matrix (zero padding of a Strassen block, ragged
// tile edge).  rscat + cscat of a real element is >= 0; with one or two sentinels the sum stays negative and
// cannot overflow (-2^62 - 2^62 = -2^63).
constexpr int64_t kSentinel = INT64_MIN / 2;

// One side of the general primitive M = alpha (X + dY)(V + eW); C += g0 M; D += g1 M  (Sec. 3, first display),
// extended to up to four signed blocks: a linear combination of blocks of one matrix view.
struct Operand {
    const int64_t* rs;  // row scatter vector of the whole matrix view (device memory)
    const int64_t* cs;  // column scatter vector
    int64_t rs_len;     // entries in rs: rows at or beyond it read as zero / are not written
    int64_t cs_len;
    int32_t space;      // 0: the caller's tensor (A, B or C by role); 1: the workspace
    int32_t nterms;
    int32_t rs_id, cs_id;  // which of the plan's vectors rs and cs are (host-side bookkeeping)
    int64_t base_off;   // element offset of the matrix view inside its space
    int64_t rs_stride;  // >= 0: rs[i] == i * rs_stride for every i (the bundle is one run of a constant stride); -1 otherwise
    int64_t cs_stride;
    const int64_t* rbs; // block scatter vectors of rs and cs (Sec. 2.3): stride of each block of 16 entries, 0 = irregular;
    const int64_t* cbs; // nullptr where the plan's block size is not 16 (the kernel then decides by rs_stride / cs_stride alone)
    int64_t roff[kMaxTerms];  // first row of each block
    int64_t coff[kMaxTerms];  // first column of each block
    double coef[kMaxTerms];   // +1 / -1
};

struct Product {
    Operand A, B, C;
    int64_t mb, nb, kb;   // extents of the product (block extents of the Strassen partition)
    uint32_t first_mask;  // bit d set: destination d has not been written before, so it takes beta instead of 1
    int32_t overwrite;    // 1: destinations are plain stores (dense temporary), beta is ignored
};

// Vector generation request for the planner kernel: scatter vector of one bundle of one tensor.
struct BundleDesc {
    int32_t ndim;
    int32_t pad;
    int64_t total;        // product of lengths = number of entries
    int64_t out_off;      // where the vector starts inside the plan's vector store (in entries)
    int64_t bs_off;       // where its block scatter vector starts
    int64_t len[16];
    int64_t stride[16];
};

struct FusedConfig {
    int a_mode, b_mode;   // 0: lanes run along the free bundle when gathering, 1: along the contracted bundle
    int nta, ntb;         // terms of the A and B sums if every product of the launch has exactly that many (1 or 2 each);
                          // 0, 0: up to four terms, counted at run time
    int a_vec, b_vec;     // consecutive entry pairs along the lane direction are contiguous and evenly placed
    int a_space, b_space; // 0: caller's tensor, 1: workspace
    int c_mode;           // 0: the destination is contiguous along its rows (free bundle I), 1: along its columns
    int tile_n;           // tile columns: 128 (512 threads, one workgroup per compute unit) or 64 (256 threads, two per
                          // compute unit; single-term products only)
};

// Size of the per-GPU array that stands in for the caller's workspace in tc_contract_static
// (= TC_STATIC_WORKSPACE_BYTES of the public header).
constexpr size_t kStaticWorkspaceBytes = (size_t)32 << 20;

// ---- device entry points (tc_device.hip); each returns a hipError_t cast to int ----
// Device address of the current GPU's static workspace array (looked up on the first call per device, then cached).
int dev_static_workspace(void** ptr);
// MFMA-only loop (kind 0: v_mfma_f64_4x4x4_4b_f64, 1: v_mfma_f64_16x16x4_f64); blocks until done; TFLOP/s achieved
int bench_mfma_peak(int kind, int iters, void* stream, double* tflops_out);
int dev_malloc(void** p, size_t bytes);
int dev_free(void* p);
int dev_upload(void* dst, const void* src, size_t bytes, void* stream);
int dev_download(void* dst, const void* src, size_t bytes);
int dev_stream_sync(void* stream);
int dev_event_create(void** e);
int dev_event_record(void* e, void* stream);
int dev_event_sync(void* e);
int dev_event_elapsed_ms(float* ms, void* a, void* b);
int dev_event_destroy(void* e);

// scatter + block scatter vectors for `nvec` bundles described in device array `descs`
int launch_planner(const BundleDesc* descs_dev, int nvec, int64_t max_total, int bs_block, int64_t* store_dev, void* stream);

// products [first, first + count) of the device schedule, all with the same extents, in one launch.
// tail_tiles > 0: the last tail_tiles tiles of the launch are cut along the contracted bundle into tail_chunks chunks
// of tail_kc entries (a multiple of 64), computed by one workgroup each into W + partial_off (tail_tiles * tail_chunks
// dense 128 x tile_n tiles), and a second kernel adds the chunks and updates the destinations.
int launch_fused(const FusedConfig& cfg, const Product* prods_dev, int first, int count, int64_t mb, int64_t nb,
                 const double* A, const double* B, double* C, double* W, double alpha, double beta, int tail_tiles, int tail_chunks,
                 int64_t tail_kc, int64_t partial_off, void* stream);

// element-wise: v = sum_t coefA_t * srcA_t;  for each destination d: dst_d = coefC_d * v + f_d * dst_d
// (Product::B is ignored; extents mb x nb).  lanes_along_rows picks the coalesced direction.  n_src, n_dst: the
// product's numbers of sources and destinations (they select the kernel instantiation).
int launch_lincomb(const Product* prods_dev, int index, int n_src, int n_dst, int64_t mb, int64_t nb, int lanes_along_rows, const double* A,
                   const double* B, double* C, double* W, int src_role, double beta, void* stream);

}  // namespace tc
