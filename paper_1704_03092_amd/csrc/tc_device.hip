// Device side of libstrassen_tc (gfx950 / CDNA4 only), except the fused kernel (tc_fused.h; its launchers are
// instantiated one family per translation unit, tc_fused_*.hip).
//
//  planner kernels   scatter vectors and block scatter vectors of the matrix view (Sec. 2.3)
//  lincomb kernel    element-wise  dst_d = g_d * (sum_t c_t src_t) + f_d * dst_d  on matrix views; used for
//                    the dense operand sums of the Naive variant and to accumulate a dense product M into the
//                    blocks of C (AB and Naive variants), Sec. 4.1.
//  launchers         thin host wrappers the planner code in tc_host.cpp calls
#include <hip/hip_runtime.h>

#include <mutex>

#include "tc_fused.h"
#include "tc_fused_small.h"
#include "tc_internal.h"

// ---------------------------------------------------------------------------------------------------------
// workspace for callers that cannot allocate (tc_contract_static)
// ---------------------------------------------------------------------------------------------------------
// One array per GPU, held from the moment the library's code object is loaded on that GPU until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address differs per GPU and is
// looked up once per device, with that device current; kernels, copies and fills only ever see the looked-up pointer.
static __device__ __align__(256) unsigned char scratch[tc::kStaticWorkspaceBytes];

namespace tc {

namespace {

// ---------------------------------------------------------------------------------------------------------
// element-wise linear combination on matrix views
// ---------------------------------------------------------------------------------------------------------
// A workgroup covers 256 * LC_FPT entries of the fast direction (LC_FPT per thread, 256 apart) and slow_per_block of
// the slow one, in chunks of LC_SLOW.  The scatter entries of a chunk's slow direction are staged in LDS first (they
// are the same for every thread), and every thread issues the loads of a batch of elements together before it
// stores.  Measured on 8192 x 8192 blocks: with the entries fetched from global memory inside the loop, one slow entry
// at a time, every entry pays the latency of its fetch, its loads and its store in turn (3.4 TB/s); many slow entries
// in flight per workgroup open as many DRAM pages at once and cost bandwidth again, hence few slow entries and
// several fast ones per thread.
constexpr int LC_SLOW = 2, LC_FPT = 2;  // measured best of {1, 2, 4, 8, 16} x {1, 2, 4}: 5.8 TB/s

// NS, ND: upper bounds (1, 2 or 4) of the numbers of sources and destinations; they size the register arrays.
template <bool ROWS_FAST, int NS, int ND>
__global__ __launch_bounds__(256) void lincomb_kernel(const Product* __restrict__ prods, int index, const double* __restrict__ srcU,
                                                      double* __restrict__ Cu, double* __restrict__ W, double beta, int slow_per_block) {
    constexpr int CAP = 48 / ((NS + ND) * LC_FPT);  // slow entries per batch: at most 48 elements in registers
    constexpr int LC_BATCH = CAP >= LC_SLOW ? LC_SLOW : (CAP >= 4 ? 4 : (CAP >= 2 ? 2 : 1));
    static_assert(LC_SLOW % LC_BATCH == 0, "batches tile the chunk");
    __shared__ int64_t s_off[2][kMaxTerms][LC_SLOW];  // [0]: sources, [1]: destinations
    const Product& P = prods[index];
    const int tid = threadIdx.x;
    const int64_t fast0 = (int64_t)blockIdx.x * (256 * LC_FPT) + tid;
    const int64_t nfast = ROWS_FAST ? P.mb : P.nb, nslow = ROWS_FAST ? P.nb : P.mb;
    const int64_t slow0 = (int64_t)blockIdx.y * slow_per_block;
    const int64_t slow_end = slow0 + slow_per_block < nslow ? slow0 + slow_per_block : nslow;
    const double* src = (P.A.space == 0 ? srcU : W) + P.A.base_off;
    double* dst = (P.C.space == 0 ? Cu : W) + P.C.base_off;
    const int nS = P.A.nterms, nD = P.C.nterms;
    int64_t sfix[LC_FPT][NS], dfix[LC_FPT][ND];  // kSentinel: the entry does not exist
    double cs[NS], gd[ND], fd[ND];
#pragma unroll
    for (int t = 0; t < NS; ++t) {
        cs[t] = t < nS ? P.A.coef[t] : 0.0;
#pragma unroll
        for (int i = 0; i < LC_FPT; ++i) {
            sfix[i][t] = kSentinel;
            const int64_t fast = fast0 + 256 * i;
            if (t < nS && fast < nfast) {
                const int64_t g = (ROWS_FAST ? P.A.roff[t] : P.A.coff[t]) + fast;
                if (g < (ROWS_FAST ? P.A.rs_len : P.A.cs_len)) sfix[i][t] = (ROWS_FAST ? P.A.rs : P.A.cs)[g];
            }
        }
    }
#pragma unroll
    for (int t = 0; t < ND; ++t) {
        gd[t] = t < nD ? P.C.coef[t] : 0.0;
        fd[t] = (t >= nD || P.overwrite) ? 0.0 : (((P.first_mask >> t) & 1u) ? beta : 1.0);
#pragma unroll
        for (int i = 0; i < LC_FPT; ++i) {
            dfix[i][t] = kSentinel;
            const int64_t fast = fast0 + 256 * i;
            if (t < nD && fast < nfast) {
                const int64_t g = (ROWS_FAST ? P.C.roff[t] : P.C.coff[t]) + fast;
                if (g < (ROWS_FAST ? P.C.rs_len : P.C.cs_len)) dfix[i][t] = (ROWS_FAST ? P.C.rs : P.C.cs)[g];
            }
        }
    }
    for (int64_t base = slow0; base < slow_end; base += LC_SLOW) {
        __syncthreads();  // the previous chunk's entries have been used
        if (tid < 2 * kMaxTerms * LC_SLOW) {
            const int which = tid / (kMaxTerms * LC_SLOW), t = (tid / LC_SLOW) % kMaxTerms, e = tid % LC_SLOW;
            const Operand& op = which ? P.C : P.A;
            int64_t val = kSentinel;
            if (base + e < slow_end && t < op.nterms) {
                const int64_t g = (ROWS_FAST ? op.coff[t] : op.roff[t]) + base + e;
                if (g < (ROWS_FAST ? op.cs_len : op.rs_len)) val = (ROWS_FAST ? op.cs : op.rs)[g];
            }
            s_off[which][t][e] = val;
        }
        __syncthreads();
#pragma unroll 1
        for (int e0 = 0; e0 < LC_SLOW; e0 += LC_BATCH) {
            double x[LC_BATCH][LC_FPT][NS], cur[LC_BATCH][LC_FPT][ND];
#pragma unroll
            for (int b = 0; b < LC_BATCH; ++b)
#pragma unroll
                for (int i = 0; i < LC_FPT; ++i) {
#pragma unroll
                    for (int t = 0; t < NS; ++t) {
                        x[b][i][t] = 0.0;
                        const int64_t a = sfix[i][t] + s_off[0][t][e0 + b];  // negative if either entry does not exist
                        if (a >= 0) x[b][i][t] = src[a];
                    }
#pragma unroll
                    for (int t = 0; t < ND; ++t) {
                        cur[b][i][t] = 0.0;
                        const int64_t o = dfix[i][t] + s_off[1][t][e0 + b];
                        if (o >= 0 && fd[t] != 0.0) cur[b][i][t] = dst[o];
                    }
                }
#pragma unroll
            for (int b = 0; b < LC_BATCH; ++b)
#pragma unroll
                for (int i = 0; i < LC_FPT; ++i) {
                    double v = 0.0;
#pragma unroll
                    for (int t = 0; t < NS; ++t)
                        if (t < nS) v = __builtin_fma(cs[t], x[b][i][t], v);  // (an absent element counts as zero)
#pragma unroll
                    for (int d = 0; d < ND; ++d) {
                        const int64_t o = dfix[i][d] + s_off[1][d][e0 + b];
                        const double gv = gd[d] * v;
                        if (o >= 0) dst[o] = (fd[d] == 0.0) ? gv : __builtin_fma(fd[d], cur[b][i][d], gv);
                    }
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

}  // namespace

// ---- static workspace: device address per GPU ----
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

int dev_static_workspace(void** ptr) {
    *ptr = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(::scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return 0;
}

// ---------------------------------------------------------------------------------------------------------
// matrix-core ceiling: nothing but dependent-free FP64 MFMA instructions (benchmark tool)
// ---------------------------------------------------------------------------------------------------------
namespace {
typedef double double4_t __attribute__((ext_vector_type(4)));
constexpr int kPeakBlocks = 2048, kPeakThreads = 512, kPeakChains = 32;

// KIND 0: v_mfma_f64_4x4x4_4b_f64 (512 flops per wave and instruction), KIND 1: v_mfma_f64_16x16x4_f64 (2048).
// Every wave keeps kPeakChains (KIND 0) or kPeakChains / 4 (KIND 1) independent accumulator chains going.
template <int KIND>
__global__ __launch_bounds__(kPeakThreads) void mfma_peak_kernel(double* __restrict__ out, int iters) {
    const double a = 1.0 + 1e-9 * threadIdx.x, b = 1.0 - 1e-9 * threadIdx.x;
    double r = 0.0;
    if constexpr (KIND == 0) {
        double acc[kPeakChains];
#pragma unroll
        for (int j = 0; j < kPeakChains; ++j) acc[j] = j;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int j = 0; j < kPeakChains; ++j) acc[j] = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kPeakChains; ++j) r += acc[j];
    } else {
        double4_t acc[kPeakChains / 4];
#pragma unroll
        for (int j = 0; j < kPeakChains / 4; ++j) acc[j] = double4_t{(double)j, 0.0, 0.0, 0.0};
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int j = 0; j < kPeakChains / 4; ++j) acc[j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < kPeakChains / 4; ++j) r += acc[j].x + acc[j].y + acc[j].z + acc[j].w;
    }
    out[(size_t)blockIdx.x * kPeakThreads + threadIdx.x] = r;
}
}  // namespace

int bench_mfma_peak(int kind, int iters, void* stream, double* tflops_out) {
    static_assert((size_t)kPeakBlocks * kPeakThreads * sizeof(double) <= kStaticWorkspaceBytes, "the results fit the static workspace");
    void* out = nullptr;
    int rc = dev_static_workspace(&out);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return (int)hipErrorUnknown;
    float ms = 0;
    for (int pass = 0; pass < 2; ++pass) {  // the first pass warms up
        hipEventRecord(e0, st);
        if (kind == 0)
            hipLaunchKernelGGL(mfma_peak_kernel<0>, dim3(kPeakBlocks), dim3(kPeakThreads), 0, st, (double*)out, iters);
        else
            hipLaunchKernelGGL(mfma_peak_kernel<1>, dim3(kPeakBlocks), dim3(kPeakThreads), 0, st, (double*)out, iters);
        hipEventRecord(e1, st);
        hipError_t e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) {
            hipEventDestroy(e0);
            hipEventDestroy(e1);
            return (int)e;
        }
    }
    hipEventDestroy(e0);
    hipEventDestroy(e1);
    const double per_instr = kind == 0 ? 512.0 : 2048.0, chains = kind == 0 ? kPeakChains : kPeakChains / 4;
    const double flops = per_instr * chains * (double)iters * (kPeakThreads / 64) * (double)kPeakBlocks;
    *tflops_out = flops / (ms * 1e-3) * 1e-12;
    return 0;
}

int dev_malloc(void** p, size_t bytes) { return (int)hipMalloc(p, bytes); }
int dev_free(void* p) { return (int)hipFree(p); }
int dev_upload(void* dst, const void* src, size_t bytes, void* stream) {
    // the source is pageable host memory owned by the plan: the copy is complete when this returns
    (void)stream;
    return (int)hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice);
}
int dev_download(void* dst, const void* src, size_t bytes) { return (int)hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost); }
int dev_stream_sync(void* stream) { return (int)hipStreamSynchronize((hipStream_t)stream); }
int dev_event_create(void** e) { return (int)hipEventCreate((hipEvent_t*)e); }
int dev_event_record(void* e, void* stream) { return (int)hipEventRecord((hipEvent_t)e, (hipStream_t)stream); }
int dev_event_sync(void* e) { return (int)hipEventSynchronize((hipEvent_t)e); }
int dev_event_elapsed_ms(float* ms, void* a, void* b) { return (int)hipEventElapsedTime(ms, (hipEvent_t)a, (hipEvent_t)b); }
int dev_event_destroy(void* e) { return (int)hipEventDestroy((hipEvent_t)e); }

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
                 const double* B, double* C, double* W, double alpha, double beta, int tail_tiles, int tail_chunks, int64_t tail_kc,
                 int64_t partial_off, void* stream) {
    const bool small = cfg.tile_n == fused_small::TN;
    if (!small && cfg.tile_n != fused::TN) return (int)hipErrorInvalidValue;
    const int64_t tiles_m = (mb + fused::TM - 1) / fused::TM, tiles_n = (nb + cfg.tile_n - 1) / cfg.tile_n;
    if (tiles_m <= 0 || tiles_n <= 0 || tiles_m > (1 << 20) || tiles_n > (1 << 20)) return (int)hipErrorInvalidValue;
    if (tail_tiles < 0 || tail_kc < 0 || tail_kc > 0x7fffffff || (tail_tiles > 0 && !W)) return (int)hipErrorInvalidValue;
    hipStream_t st = (hipStream_t)stream;
    const int vec = (cfg.a_vec ? 1 : 0) | (cfg.b_vec ? 2 : 0);  // pair-wise gathers (pairs are 8-byte aligned)
    const int tm = (int)tiles_m, tn = (int)tiles_n;
    double* partial = tail_tiles > 0 ? W + partial_off : nullptr;
    const int main_count = (int)((int64_t)count * tm * tn - tail_tiles);
    if (small) {
        // the small geometry exists for single-term products only
        if (cfg.nta != 1 || cfg.ntb != 1) return (int)hipErrorInvalidValue;
        const fused_small::TailSplit tail{tail_tiles, tail_chunks, (int)tail_kc, partial};
        const int err = fused_small::launch_family<1, 1, true>(cfg.a_mode, cfg.b_mode, vec, cfg.c_mode, prods_dev, first, count, tm, tn, A, B, C,
                                                               W, alpha, beta, tail, st);
        if (err || tail_tiles == 0) return err;
        return fused_small::launch_tail_fixup(cfg.c_mode == 0, prods_dev, first, tm, tn, main_count, tail_tiles, tail_chunks, partial, C, W,
                                              alpha, beta, st);
    }
    const fused::TailSplit tail{tail_tiles, tail_chunks, (int)tail_kc, partial};
    int err = (int)hipErrorInvalidValue;
#define TC_FAMILY(NA, NB, EX)                                                                                                             \
    err = fused::launch_family<NA, NB, EX>(cfg.a_mode, cfg.b_mode, vec, cfg.c_mode, prods_dev, first, count, tm, tn, A, B, C, W, alpha, beta, \
                                           tail, st);                                                                                      \
    break
    switch (cfg.nta * 8 + cfg.ntb) {
        case 0: TC_FAMILY(4, 4, false);
        case 1 * 8 + 1: TC_FAMILY(1, 1, true);
        case 1 * 8 + 2: TC_FAMILY(1, 2, true);
        case 2 * 8 + 1: TC_FAMILY(2, 1, true);
        case 2 * 8 + 2: TC_FAMILY(2, 2, true);
        case 1 * 8 + 4: TC_FAMILY(1, 4, true);
        case 4 * 8 + 1: TC_FAMILY(4, 1, true);
        case 2 * 8 + 4: TC_FAMILY(2, 4, true);
        case 4 * 8 + 2: TC_FAMILY(4, 2, true);
        case 4 * 8 + 4: TC_FAMILY(4, 4, true);
        default: break;
    }
#undef TC_FAMILY
    if (err || tail_tiles == 0) return err;
    return fused::launch_tail_fixup(cfg.c_mode == 0, prods_dev, first, tm, tn, main_count, tail_tiles, tail_chunks, partial, C, W, alpha, beta, st);
}

namespace {
template <bool ROWS_FAST>
void launch_lincomb_sized(int ns, int nd, dim3 grid, hipStream_t st, const Product* prods_dev, int index, const double* src, double* C, double* W,
                          double beta, int per) {
#define TC_LC(NS, ND)                                                                                                               \
    hipLaunchKernelGGL((lincomb_kernel<ROWS_FAST, NS, ND>), grid, dim3(256), 0, st, prods_dev, index, src, C, W, beta, per); \
    return
    switch (ns * 8 + nd) {
        case 1 * 8 + 1: TC_LC(1, 1);
        case 1 * 8 + 2: TC_LC(1, 2);
        case 1 * 8 + 4: TC_LC(1, 4);
        case 2 * 8 + 1: TC_LC(2, 1);
        case 2 * 8 + 2: TC_LC(2, 2);
        case 2 * 8 + 4: TC_LC(2, 4);
        case 4 * 8 + 1: TC_LC(4, 1);
        case 4 * 8 + 2: TC_LC(4, 2);
        default: TC_LC(4, 4);
    }
#undef TC_LC
}
}  // namespace

int launch_lincomb(const Product* prods_dev, int index, int n_src, int n_dst, int64_t mb, int64_t nb, int lanes_along_rows, const double* A,
                   const double* B, double* C, double* W, int src_role, double beta, void* stream) {
    hipStream_t st = (hipStream_t)stream;
    const double* src = src_role == 0 ? A : B;
    const int64_t nfast = lanes_along_rows ? mb : nb, nslow = lanes_along_rows ? nb : mb;
    if (nfast <= 0 || nslow <= 0) return 0;
    if (n_src < 0 || n_src > kMaxTerms || n_dst < 0 || n_dst > kMaxTerms) return (int)hipErrorInvalidValue;
    int64_t per = LC_SLOW;
    while ((nslow + per - 1) / per > 65535) per *= 2;
    const int64_t gx = (nfast + 256 * LC_FPT - 1) / (256 * LC_FPT), gy = (nslow + per - 1) / per;
    if (gx > 0x7fffffff || per > (1 << 30)) return (int)hipErrorInvalidValue;
    const int ns = n_src <= 1 ? 1 : n_src <= 2 ? 2 : 4, nd = n_dst <= 1 ? 1 : n_dst <= 2 ? 2 : 4;  // register-array sizes
    const dim3 grid((unsigned)gx, (unsigned)gy);
    if (lanes_along_rows)
        launch_lincomb_sized<true>(ns, nd, grid, st, prods_dev, index, src, C, W, beta, (int)per);
    else
        launch_lincomb_sized<false>(ns, nd, grid, st, prods_dev, index, src, C, W, beta, (int)per);
    return (int)hipGetLastError();
}

}  // namespace tc
