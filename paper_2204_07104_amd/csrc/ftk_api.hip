// C ABI of the ftk library (see include/ftk.h for the contract of every entry point).
// Host side only: argument checks, ownership, the call-order state machine, kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <numeric>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <utility>
#include <limits>
#include <vector>

#include "../../include/ftk.h"
#include "ftk_kernels_generic.hpp"
#include "ftk_kernels_mfma16.hpp"
#include "ftk_kernels_tiled.hpp"
#define FTK_INSTANCES_EXTERN
#include "ftk_instances.hpp"   // the matrix-core kernel instances are compiled in translation units of their own

using namespace ftk;

// Scratch memory of ftk_sgd_step_noalloc: the per-workgroup partial tables of one step (factor-row sums,
// then core-gradient sums).  A device global, so no allocation call is ever needed for it; every GPU the
// library's code is loaded on holds its own copy until the process ends.  Host code never uses this name
// as an address: the per-device address comes from hipGetSymbolAddress (scratch_address below).
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) float scratch[kScratchBytes / sizeof(float)];

namespace {

thread_local std::string g_create_error;

enum Variant { V_GENERIC = 0, V_MFMA16 = 1, V_TILED = 2 };
const char* const kVariantNames[] = {"generic", "mfma16", "tiled"};

struct TimingSlot {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pending;
    double total_ms = 0.0;
    int64_t launches = 0;
};

}  // namespace

struct ftk_ctx {
    int order = 0;
    int64_t dims[kMaxOrder] = {};
    int64_t nnz = 0;
    Layout L = {};           // the library's own copy of the parameters: J[n], R are the PADDED ranks
    int J_user[kMaxOrder] = {};   // ranks as the caller gave them (equal to L.J / L.R unless padded)
    int R_user = 0;
    long long A_total = 0;   // floats in the packed A (and dA) allocation, multiple of 64

    uint32_t* d_rec = nullptr;               // the tensor: one record per stored entry (see struct Coo)
    int rec_words = 4;
    int32_t* d_new_of_old[kMaxOrder] = {};   // internal row number of every caller row
    float* d_stage = nullptr;                // staging for ftk_get/set_factors (largest I_n * J_n floats)
    float* d_A = nullptr;
    float* d_dA = nullptr;
    float* d_B = nullptr;
    float* d_GB = nullptr;
    double* d_sums = nullptr;
    unsigned int* d_flag = nullptr;

    uint32_t* d_pos = nullptr;
    int32_t* d_bidx = nullptr;
    float* d_bval = nullptr;
    long long cap = 0;
    long long n_samples = 0;      // |Psi| of the current sample set (0: none drawn yet)
    uint64_t sample_seed = 0;
    bool batch_valid = false;     // d_pos / d_bidx / d_bval hold the current Psi

    hipStream_t stream = nullptr;
    int device = 0;
    int num_cu = 1;
    int max_lds = 65536;
    int mode = FTK_SYNC;

    int variant = V_GENERIC;
    int gen_threads = 0;     // block size of grad_generic for this shape (0: does not fit)
    int gen_b_in_lds = 0;
    size_t gen_lds_bytes = 0;

    // frequently hit rows: rows [0, hot_K[n]) of mode n (internal numbering) are accumulated in LDS
    bool mfma16_ok = false;
    bool tiled_ok = false;    // general matrix-core kernel: J_n, R <= 64
    int tiled_P = 1;          // ranks padded to 16 * tiled_P
    int tiled_waves = 8;
    bool tiled_x4 = false;    // every J_n is a multiple of four: rows are fetched 16 bytes per lane
    size_t tiled_lds_bytes = 0;
    int sampling = FTK_SAMPLE_ENTRIES;
    uint32_t* d_rec_tiles = nullptr;   // the records in the order of the tile-sampling rule (built on first use)
    uint64_t tile_a = 1, tile_b = 0;
    int hot_K[kMaxOrder] = {};
    int hot_top[kMaxOrder] = {};   // 16 where rows 0..15 of the mode go through the one-hot matrix product, else 0
    int hot_off[kMaxOrder] = {};
    int hot_H = 0;            // rows in the LDS table for the current |Psi|
    int hot_H_max = 0;        // rows the LDS budget allows (partial tables are sized for this)
    long long hot_for_M = -1; // |Psi| the current choice was made for
    std::vector<std::vector<unsigned int>> sorted_counts;   // per mode: occurrence counts, descending
    int mfma_grid = 0;                // workgroups of the persistent gradient kernels for the current |Psi|
    int mfma_grid_max = 0;            // what the partial tables are sized for (one workgroup per CU)
    size_t mfma_lds_bytes = 0;
    float* d_hot_partial = nullptr;   // [mfma_grid][hot_H][16]
    // Ranks above 32 (tiled kernel, P = 4): A, dA and the workgroups' tables of the frequent rows are ONE allocation
    // (d_A its start), because there the table rows are added by the same buffer atomics as the rows of dA (or of A,
    // in-place mode) and must be within reach of the same 32-bit offsets.  The tables are zero between steps.
    int sort_mode = -1;       // tiled kernel, ranks up to 32: samples of a group sorted by their route in this mode (see pick_hot_rows)
    float* d_arena = nullptr;
    float* d_wide_tables = nullptr;   // [mfma_grid][hot_H][16 P], behind dA; NULL: no such tables (K[n] = top[n])
    float* d_gb_partial = nullptr;    // [mfma_grid][B_total]
    // "rows" form of the tiled variant: rows outside the tables are appended to per-workgroup lists and summed by
    // row-owning workgroups (ftk_kernels_tiled.hpp, ROWS)
    bool pair_turns = false;         // J = R = 16 kernel: turns in pairs that share their Philox blocks (large |Psi|, entry rule)
    bool rows_ok = false;            // the shape has a bucket plan (set at create)
    bool rows = false;               // in use (only with variant == V_TILED)
    bool rows_tight = false;         // list capacities at half the expected counts: lists fill up all the time (for tests)
    int rows_shift[kMaxOrder] = {};  // rows per bucket of mode n = 1 << shift
    int rows_bucket0[kMaxOrder] = {};
    int rows_n_buckets = 0;          // for the current tables (K_n) and |Psi|
    int rows_max_buckets = 0;        // with no table rows at all: what LDS and the device tables are sized for
    unsigned int rows_list_words = 0;
    size_t rows_apply_lds = 0;
    std::vector<std::vector<unsigned long long>> count_prefix;   // per mode: prefix sums of sorted_counts
    float* d_lists = nullptr;
    size_t lists_bytes = 0;
    unsigned int* d_list_fill = nullptr;
    uint2* d_bucket_info = nullptr;
    int4* d_bucket_rows = nullptr;
    unsigned int* d_overflow = nullptr;
    float* use_hot_partial = nullptr; // the partial tables of the step being enqueued: the two above, or the
    float* use_gb_partial = nullptr;  // library's static scratch array (ftk_sgd_step_noalloc)

    bool timing = false;
    bool no_events = false;   // set while ftk_sgd_step_noalloc enqueues: no event is created even if timing is on
    bool prepare_only = false;   // the launch functions stop after raising the kernel's LDS limit
    TimingSlot slots[FTK_K_COUNT];
    std::vector<const void*> lds_limit_raised;   // kernels whose dynamic-LDS limit this context has raised

    std::string err;
};

namespace {

int fail(ftk_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c)
        c->err = buf;
    else
        g_create_error = buf;
    return code;
}

int step_impl(ftk_ctx* c, float lr_A, float lr_B, float lambda_A, float lambda_B);
int prepare_variant(ftk_ctx* c);

#define FTK_HIP(c, call)                                                                         \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail((c), e_ == hipErrorOutOfMemory ? FTK_ENOMEM : FTK_EDEVICE, "%s: %s", #call, \
                        hipGetErrorString(e_));                                                  \
    } while (0)

inline int blocks_for(long long work, int threads, int cap_blocks) {
    long long b = (work + threads - 1) / threads;
    if (b < 1) b = 1;
    if (b > cap_blocks) b = cap_blocks;
    return (int)b;
}

// Every pointer the context holds belongs to the device that was current in ftk_create.
int check_device(ftk_ctx* c) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return fail(c, FTK_EDEVICE, "hipGetDevice failed");
    if (dev != c->device)
        return fail(c, FTK_ESTATE, "current HIP device is %d, the context was created on device %d", dev, c->device);
    return FTK_OK;
}

// Address of the static scratch array on the current device (which must be c->device): looked up once
// per device, at the first ftk_create on it.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

int scratch_setup(ftk_ctx* c) {
    if (c->device < 0 || c->device >= kMaxDevices) return FTK_OK;   // ftk_sgd_step_noalloc will refuse
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[c->device]) return FTK_OK;
    float* ptr = nullptr;
    FTK_HIP(c, hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(c, FTK_EDEVICE, "hipGetSymbolAddress returned no address for the scratch array");
    g_scratch_ptr[c->device] = ptr;
    return FTK_OK;
}

float* scratch_address(const ftk_ctx* c) {
    if (c->device < 0 || c->device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[c->device];
}

// Raise a kernel's dynamic-LDS limit to the device maximum, once per context and kernel (the limit is
// a property of the kernel on this device, so raising it again is harmless but costs a runtime call
// per step).  Always the device's maximum, so that contexts of different shapes cannot lower it for
// each other.
int raise_lds_limit(ftk_ctx* c, const void* kernel, int bytes) {
    for (const void* k : c->lds_limit_raised)
        if (k == kernel) return FTK_OK;
    FTK_HIP(c, hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    try {
        c->lds_limit_raised.push_back(kernel);
    } catch (...) {   // not remembered: the next launch sets it again
    }
    return FTK_OK;
}

// event bracket around one kernel launch when timing is on
struct Bracket {
    ftk_ctx* c;
    int slot;
    hipEvent_t a = nullptr, b = nullptr;
    bool on = false;
    Bracket(ftk_ctx* ctx, int s) : c(ctx), slot(s) {
        if (!c->timing || c->no_events) return;
        if (hipEventCreate(&a) != hipSuccess) return;
        if (hipEventCreate(&b) != hipSuccess) {
            hipEventDestroy(a);
            return;
        }
        on = hipEventRecord(a, c->stream) == hipSuccess;
        if (!on) {
            hipEventDestroy(a);
            hipEventDestroy(b);
        }
    }
    ~Bracket() {
        if (!on) return;
        if (hipEventRecord(b, c->stream) == hipSuccess)
            c->slots[slot].pending.emplace_back(a, b);
        else {
            hipEventDestroy(a);
            hipEventDestroy(b);
        }
    }
};

void drop_pending(ftk_ctx* c) {
    for (auto& s : c->slots) {
        for (auto& p : s.pending) {
            hipEventDestroy(p.first);
            hipEventDestroy(p.second);
        }
        s.pending.clear();
    }
}

void pick_generic_config(ftk_ctx* c) {
    const long long NR = (long long)c->order * c->L.R, BT = c->L.B_total;
    c->gen_threads = 0;
    for (int T : {256, 128, 64})
        for (int b : {1, 0}) {
            const long long bytes = 4LL * (2 * NR * T + (T / 64) * BT + (b ? BT : 0));
            if (bytes <= c->max_lds) {
                c->gen_threads = T;
                c->gen_b_in_lds = b;
                c->gen_lds_bytes = (size_t)bytes;
                return;
            }
        }
}

// The sampling rule in force and the record array it reads.
SampleRule sample_rule(const ftk_ctx* c) {
    SampleRule r;
    r.nnz = (uint64_t)c->nnz;
    r.n_runs = c->sampling == FTK_SAMPLE_TILES ? ((uint64_t)c->nnz + 63) / 64 : 0;
    r.a = c->tile_a;
    r.b = c->tile_b;
    return r;
}
Coo sampled_records(const ftk_ctx* c) {
    return Coo{c->sampling == FTK_SAMPLE_TILES ? c->d_rec_tiles : c->d_rec, c->rec_words};
}

int launch_grad_generic(ftk_ctx* c, float lambda_A, float lr_A, bool modewise = false) {
    const bool in_place = c->mode == FTK_HOGWILD;
    GradArgs g;
    g.L = c->L;
    g.batch = Batch{c->d_bidx, c->d_bval, c->n_samples, c->cap};
    g.A = c->d_A;
    g.B = c->d_B;
    g.dA = in_place ? c->d_A : c->d_dA;
    g.GB = c->d_GB;
    g.lambda_A = lambda_A;
    g.scale = in_place ? -lr_A : 1.0f;
    g.b_in_lds = c->gen_b_in_lds;
    g.core_only = modewise ? 1 : 0;
    if (c->gen_threads == 0)
        return fail(c, FTK_EUNSUPPORTED, "generic gradient kernel: N*R = %d and sum J_n R = %d exceed the LDS budget",
                    c->order * c->L.R, c->L.B_total);
    const int T = c->gen_threads;
    const int grid = blocks_for(c->n_samples, T, c->num_cu * 4);
    if (c->gen_lds_bytes > 65536) {
        if (const int rc = raise_lds_limit(c, reinterpret_cast<const void*>(grad_generic_kernel), c->max_lds)) return rc;
        if (const int rc = raise_lds_limit(c, reinterpret_cast<const void*>(factor_phase_generic_kernel), c->max_lds)) return rc;
    }
    if (c->prepare_only) return FTK_OK;
    Bracket t(c, FTK_K_GRAD);
    if (modewise) {
        // Algorithm 1 as printed: the factor phase changes A in place, then the core gradient is
        // taken over the same samples at the rows it left
        hipLaunchKernelGGL(factor_phase_generic_kernel, dim3(grid), dim3(T), c->gen_lds_bytes, c->stream, g, c->d_A, lr_A);
        FTK_HIP(c, hipGetLastError());
    }
    hipLaunchKernelGGL(grad_generic_kernel, dim3(grid), dim3(T), c->gen_lds_bytes, c->stream, g);
    FTK_HIP(c, hipGetLastError());
    return FTK_OK;
}

template <int N, bool TILES, int MODE>
int launch_mfma16_ntm(ftk_ctx* c, const Mfma16Args& g) {
    if (const int rc = raise_lds_limit(c, reinterpret_cast<const void*>(grad_mfma16_kernel<N, TILES, MODE>), c->max_lds)) return rc;
    if (c->prepare_only) return FTK_OK;
    Bracket t(c, FTK_K_GRAD);
    hipLaunchKernelGGL((grad_mfma16_kernel<N, TILES, MODE>), dim3(c->mfma_grid), dim3(kMfmaThreads), c->mfma_lds_bytes,
                       c->stream, g);
    FTK_HIP(c, hipGetLastError());
    return FTK_OK;
}

template <int N, bool TILES>
int launch_mfma16_nt(ftk_ctx* c, const Mfma16Args& g, int pass) {
    switch (pass) {
        case kSyncPass: return launch_mfma16_ntm<N, TILES, kSyncPass>(c, g);
        case kInPlacePass: return launch_mfma16_ntm<N, TILES, kInPlacePass>(c, g);
        case kFactorPhase: return launch_mfma16_ntm<N, TILES, kFactorPhase>(c, g);
        default: return launch_mfma16_ntm<N, TILES, kCorePhase>(c, g);
    }
}

template <int N>
int launch_mfma16_n(ftk_ctx* c, const Mfma16Args& g, int pass) {
    return c->sampling == FTK_SAMPLE_TILES ? launch_mfma16_nt<N, true>(c, g, pass) : launch_mfma16_nt<N, false>(c, g, pass);
}

// pass: kSyncPass / kInPlacePass by the context's mode (pass < 0), or one of the two phases of the mode-by-mode order
int launch_grad_mfma16(ftk_ctx* c, float lambda_A, float lr_A, int pass = -1) {
    if (pass < 0) pass = c->mode == FTK_HOGWILD ? kInPlacePass : kSyncPass;
    const bool in_place = pass == kInPlacePass || pass == kFactorPhase;
    Mfma16Args g;
    g.coo = sampled_records(c);
    g.rule = sample_rule(c);
    g.seed = c->sample_seed;
    g.M = c->n_samples;
    g.A = c->d_A;
    g.B = c->d_B;
    g.dA = in_place ? c->d_A : c->d_dA;
    g.scale = in_place ? -lr_A : 1.0f;
    g.pair_turns = c->pair_turns ? 1 : 0;
    {
        const long long T = (c->n_samples + 15) / 16;
        if (T / c->mfma_grid >= (1LL << 27)) return fail(c, FTK_EUNSUPPORTED, "mfma16 kernel: more than 2^31 samples per workgroup");
        g.tiles_each = (int)(T / c->mfma_grid);
        g.tiles_more = (int)(T % c->mfma_grid);
    }
    for (int n = 0; n < kMfma16MaxOrder; ++n) {
        g.A_off[n] = c->L.A_off[n];
        g.B_off[n] = c->L.B_off[n];
        g.K[n] = c->hot_K[n];
        g.top[n] = c->hot_top[n];
        g.row_bytes[n] = (unsigned int)(c->dims[n] * 64);
        g.hot_off[n] = c->hot_off[n];
        g.first_row[n] = (unsigned int)(c->L.A_off[n] / 16);
    }
    g.all_bytes = (unsigned int)(c->A_total * 4);
    g.H = c->hot_H;
    g.hot_partial = c->use_hot_partial;
    g.gb_partial = c->use_gb_partial;
    g.lambda_A = lambda_A;
    // what the kernel assumes: 16-float rows, records of 4 * ceil((N + 1) / 4) words, partial
    // tables sized for the grid, an LDS table of hot_H rows
    if (!c->mfma16_ok || c->rec_words != 4 * ((c->order + 1 + 3) / 4) || !c->use_hot_partial || !c->use_gb_partial)
        return fail(c, FTK_EUNSUPPORTED, "mfma16 kernel is not available for this shape");
    switch (c->order) {
        case 1: return launch_mfma16_n<1>(c, g, pass);
        case 2: return launch_mfma16_n<2>(c, g, pass);
        case 3: return launch_mfma16_n<3>(c, g, pass);
        case 4: return launch_mfma16_n<4>(c, g, pass);
        case 5: return launch_mfma16_n<5>(c, g, pass);
        case 6: return launch_mfma16_n<6>(c, g, pass);
        default: return fail(c, FTK_EUNSUPPORTED, "mfma16 kernel is built for order <= 6");
    }
}

template <int N, int P, int WAVES, bool X4, bool ROWS, int MODE = kSyncPass>
int launch_tiled_npwxr(ftk_ctx* c, const TiledArgs& g) {
    if (const int rc = raise_lds_limit(c, reinterpret_cast<const void*>(grad_tiled_kernel<N, P, WAVES, X4, ROWS, MODE>), c->max_lds)) return rc;
    if (c->prepare_only) return FTK_OK;
    Bracket t(c, FTK_K_GRAD);
    hipLaunchKernelGGL((grad_tiled_kernel<N, P, WAVES, X4, ROWS, MODE>), dim3(c->mfma_grid), dim3(WAVES * 64), c->tiled_lds_bytes,
                       c->stream, g);
    FTK_HIP(c, hipGetLastError());
    return FTK_OK;
}

// The mode-by-mode order runs on both matrix-core kernels (the row-owner form of the tiled kernel serves the synchronous
// step only), else on the one-lane-per-sample kernels.
inline bool tiled_modewise_ok(const ftk_ctx* c) { return c->variant == V_TILED && !c->rows; }
inline bool modewise_on_matrix_cores(const ftk_ctx* c) { return c->variant == V_MFMA16 || tiled_modewise_ok(c); }

template <int N, int P, int WAVES>
int launch_tiled_npw(ftk_ctx* c, const TiledArgs& g, int pass) {
    if (pass == kFactorPhase || pass == kCorePhase) {
        if (!tiled_modewise_ok(c)) return fail(c, FTK_EUNSUPPORTED, "the mode-by-mode order is not built for the rows form of the tiled kernel");
        if (c->tiled_x4)
            return pass == kFactorPhase ? launch_tiled_npwxr<N, P, WAVES, true, false, kFactorPhase>(c, g)
                                        : launch_tiled_npwxr<N, P, WAVES, true, false, kCorePhase>(c, g);
        return pass == kFactorPhase ? launch_tiled_npwxr<N, P, WAVES, false, false, kFactorPhase>(c, g)
                                    : launch_tiled_npwxr<N, P, WAVES, false, false, kCorePhase>(c, g);
    }
    // the rows form is built for rows fetched 16 bytes per lane (every J_n a multiple of four) only
    if (c->rows) {
        // the row owners' table (up to 64 KB, dynamic) sits next to 4 KB of static LDS
        if (const int rc = raise_lds_limit(c, reinterpret_cast<const void*>(rows_apply_kernel), 65536)) return rc;
        return c->tiled_x4 ? launch_tiled_npwxr<N, P, WAVES, true, true>(c, g) : fail(c, FTK_EUNSUPPORTED, "rows needs every J_n to be a multiple of 4");
    }
    return c->tiled_x4 ? launch_tiled_npwxr<N, P, WAVES, true, false>(c, g) : launch_tiled_npwxr<N, P, WAVES, false, false>(c, g);
}

template <int N>
int launch_tiled_n(ftk_ctx* c, const TiledArgs& g, int pass) {
    switch (c->tiled_P) {
        case 1: return launch_tiled_npw<N, 1, 8>(c, g, pass);
        case 2: return launch_tiled_npw<N, 2, 8>(c, g, pass);
        default: return launch_tiled_npw<N, 4, 4>(c, g, pass);
    }
}

// Ranks above 32 on the tiled kernel: the workgroups' tables of the frequent rows are the ones behind dA, filled by atomics.
inline bool wide_tables(const ftk_ctx* c) { return c->variant == V_TILED && c->tiled_P == 4 && c->d_wide_tables != nullptr; }

// pass: the synchronous or the fused in-place pass by the context's mode (pass < 0), or one of the two phases of the
// mode-by-mode order
int launch_grad_tiled(ftk_ctx* c, float lambda_A, float lr_A, int pass = -1) {
    const bool in_place = c->mode == FTK_HOGWILD || pass == kFactorPhase || pass == kCorePhase;
    TiledArgs g;
    g.coo = sampled_records(c);
    g.rule = sample_rule(c);
    g.seed = c->sample_seed;
    g.M = c->n_samples;
    g.A = c->d_A;
    g.B = c->d_B;
    g.dA = in_place ? c->d_A : c->d_dA;
    g.scale = in_place ? -lr_A : 1.0f;
    g.R = c->L.R;
    for (int n = 0; n < kMaxOrder; ++n) {
        g.A_off[n] = c->L.A_off[n];
        g.B_off[n] = c->L.B_off[n];
        g.J[n] = c->L.J[n];
        g.K[n] = c->hot_K[n];
        g.top[n] = c->hot_top[n];
        g.hot_off[n] = c->hot_off[n];
        g.mode_bytes[n] = (unsigned int)(c->dims[n] * c->L.J[n] * 4);
    }
    g.H = c->hot_H;
    g.hot_partial = wide_tables(c) ? c->d_wide_tables : c->use_hot_partial;
    g.table_stride = (unsigned int)((size_t)c->hot_H * 16 * c->tiled_P * sizeof(float));
    for (int n = 0; n < kMaxOrder; ++n) {
        g.table_off[n] = 0;
        g.dA_bytes[n] = g.mode_bytes[n];
        if (wide_tables(c) && n < c->order) {
            // from row 0 of mode n in the array the atomics go to, to the tables and to their end
            const size_t to_tables = (size_t)(c->d_wide_tables - (g.dA + c->L.A_off[n])) * sizeof(float);
            const size_t to_end = to_tables + (size_t)c->mfma_grid * g.table_stride;
            if (to_end >= (1ull << 30)) return fail(c, FTK_EUNSUPPORTED, "tiled kernel: the workgroups' tables are out of the atomics' reach");
            g.table_off[n] = (unsigned int)to_tables;
            g.dA_bytes[n] = (unsigned int)to_end;
        }
    }
    g.gb_partial = c->use_gb_partial;
    g.B_total = c->L.B_total;
    g.lambda_A = lambda_A;
    g.sort_mode = c->sort_mode;
    {
        const long long T = (c->n_samples + 15) / 16;
        if (T / c->mfma_grid >= (1LL << 27)) return fail(c, FTK_EUNSUPPORTED, "tiled kernel: more than 2^31 samples per workgroup");
        g.tiles_each = (int)(T / c->mfma_grid);
        g.tiles_more = (int)(T % c->mfma_grid);
    }
    g.lists = c->d_lists;
    g.list_fill = c->d_list_fill;
    g.bucket_info = c->d_bucket_info;
    g.overflow = c->d_overflow;
    g.list_words = c->rows_list_words;
    g.n_buckets = c->rows ? c->rows_n_buckets : 0;
    for (int n = 0; n < kMaxOrder; ++n) {
        g.bucket0[n] = c->rows_bucket0[n];
        g.bucket_shift[n] = c->rows_shift[n];
    }
    if (c->rows && !c->prepare_only &&
        (in_place || !c->d_lists || !c->d_list_fill || !c->d_bucket_info || !c->d_overflow || c->rows_n_buckets < 1 ||
         (size_t)c->mfma_grid * c->rows_list_words * sizeof(float) > c->lists_bytes))
        return fail(c, FTK_EUNSUPPORTED, "the rows form of the tiled kernel is not set up for this step");
    // what the kernel assumes: padded ranks 16 P, records of 4 * ceil((N + 1) / 4) words, an LDS
    // table that fits, partial tables sized for grid x waves
    if (!c->tiled_ok || c->rec_words != 4 * ((c->order + 1 + 3) / 4) || !g.hot_partial || !c->use_gb_partial ||
        (size_t)c->mfma_grid * g.table_stride > (size_t)c->num_cu * (size_t)c->max_lds ||
        c->tiled_lds_bytes > (size_t)c->max_lds || (size_t)c->hot_H * 64 * c->tiled_P > (size_t)c->max_lds)
        return fail(c, FTK_EUNSUPPORTED, "tiled kernel is not available for this shape");
    switch (c->order) {
        case 1: return launch_tiled_n<1>(c, g, pass);
        case 2: return launch_tiled_n<2>(c, g, pass);
        case 3: return launch_tiled_n<3>(c, g, pass);
        case 4: return launch_tiled_n<4>(c, g, pass);
        case 5: return launch_tiled_n<5>(c, g, pass);
        case 6: return launch_tiled_n<6>(c, g, pass);
        case 7: return launch_tiled_n<7>(c, g, pass);
        case 8: return launch_tiled_n<8>(c, g, pass);
        // orders 9 and 10 (the paper's sweep ends at 10) are built for ranks up to 16 only
        case 9: return launch_tiled_npw<9, 1, 8>(c, g, pass);
        default: return launch_tiled_npw<10, 1, 8>(c, g, pass);
    }
}

// Psi as arrays (positions, row numbers, values): needed by the generic kernel and ftk_get_samples
int ensure_batch(ftk_ctx* c) {
    if (c->batch_valid) return FTK_OK;
    const long long n_samples = c->n_samples;
    if (n_samples > c->cap) {
        FTK_HIP(c, hipStreamSynchronize(c->stream));
        if (c->d_pos) hipFree(c->d_pos);
        if (c->d_bidx) hipFree(c->d_bidx);
        if (c->d_bval) hipFree(c->d_bval);
        c->d_pos = nullptr;
        c->d_bidx = nullptr;
        c->d_bval = nullptr;
        c->cap = 0;
        const long long cap = ((n_samples + 255) / 256) * 256;
        FTK_HIP(c, hipMalloc(&c->d_pos, (size_t)cap * sizeof(uint32_t)));
        FTK_HIP(c, hipMalloc(&c->d_bidx, (size_t)cap * c->order * sizeof(int32_t)));
        FTK_HIP(c, hipMalloc(&c->d_bval, (size_t)cap * sizeof(float)));
        c->cap = cap;
    }
    {
        Bracket t(c, FTK_K_SAMPLE);
        hipLaunchKernelGGL(sample_gather_kernel, dim3((unsigned)((n_samples + 255) / 256)), dim3(256), 0, c->stream,
                           sampled_records(c), c->order, sample_rule(c), c->sample_seed, (long long)n_samples, c->cap,
                           c->d_pos, c->d_bidx, c->d_bval);
    }
    FTK_HIP(c, hipGetLastError());
    c->batch_valid = true;
    return FTK_OK;
}

template <int N>
void launch_errors_mfma16_n(ftk_ctx* c, const Coo& coo, long long nnz) {
    const long long groups = (nnz + 63) / 64;
    const int grid = blocks_for(groups, 4, c->num_cu * 8);
    ModeBytes row_bytes = {};
    for (int n = 0; n < N; ++n) row_bytes.v[n] = (unsigned int)(c->dims[n] * 64);
    hipLaunchKernelGGL(errors_mfma16_kernel<N>, dim3(grid), dim3(256), 0, c->stream, coo, (uint64_t)nnz,
                       (const float*)c->d_A, (const float*)c->d_B, c->L, row_bytes, c->d_sums);
}

template <int N, int P, bool X4>
int launch_errors_tiled_npx(ftk_ctx* c, const Coo& coo, long long nnz) {
    const long long groups = (nnz + 63) / 64;
    const int grid = blocks_for(groups, 4, c->num_cu * 8);
    const size_t lds = 4 * ((size_t)N * 256 * P * P + 4 * (size_t)tiled_wave_scratch(N, P));
    TiledModeBytes mode_bytes = {};
    for (int n = 0; n < N; ++n) mode_bytes.v[n] = (unsigned int)(c->dims[n] * c->L.J[n] * 4);
    // the kernel also has 64 bytes of static LDS
    if (const int rc = raise_lds_limit(c, reinterpret_cast<const void*>(errors_tiled_kernel<N, P, X4>), c->max_lds - 1024)) return rc;
    hipLaunchKernelGGL((errors_tiled_kernel<N, P, X4>), dim3(grid), dim3(256), lds, c->stream, coo, (uint64_t)nnz,
                       (const float*)c->d_A, (const float*)c->d_B, c->L, mode_bytes, c->d_sums);
    return FTK_OK;
}

template <int N>
int launch_errors_tiled_n(ftk_ctx* c, const Coo& coo, long long nnz) {
    const bool x4 = c->tiled_x4;
    switch (c->tiled_P) {
        case 1: return x4 ? launch_errors_tiled_npx<N, 1, true>(c, coo, nnz) : launch_errors_tiled_npx<N, 1, false>(c, coo, nnz);
        case 2: return x4 ? launch_errors_tiled_npx<N, 2, true>(c, coo, nnz) : launch_errors_tiled_npx<N, 2, false>(c, coo, nnz);
        default: return x4 ? launch_errors_tiled_npx<N, 4, true>(c, coo, nnz) : launch_errors_tiled_npx<N, 4, false>(c, coo, nnz);
    }
}

// Sums of squared and absolute errors over `nnz` packed records (internal row numbers).
int launch_errors(ftk_ctx* c, Coo coo, long long nnz, double* host_sums) {
    FTK_HIP(c, hipMemsetAsync(c->d_sums, 0, 2 * sizeof(double), c->stream));
    if (c->variant == V_MFMA16 && c->rec_words == 4 * ((c->order + 1 + 3) / 4)) {
        switch (c->order) {
            case 1: launch_errors_mfma16_n<1>(c, coo, nnz); break;
            case 2: launch_errors_mfma16_n<2>(c, coo, nnz); break;
            case 3: launch_errors_mfma16_n<3>(c, coo, nnz); break;
            case 4: launch_errors_mfma16_n<4>(c, coo, nnz); break;
            case 5: launch_errors_mfma16_n<5>(c, coo, nnz); break;
            default: launch_errors_mfma16_n<6>(c, coo, nnz); break;
        }
    } else if (c->variant == V_TILED && c->rec_words == 4 * ((c->order + 1 + 3) / 4)) {
        int rc = FTK_OK;
        switch (c->order) {
            case 1: rc = launch_errors_tiled_n<1>(c, coo, nnz); break;
            case 2: rc = launch_errors_tiled_n<2>(c, coo, nnz); break;
            case 3: rc = launch_errors_tiled_n<3>(c, coo, nnz); break;
            case 4: rc = launch_errors_tiled_n<4>(c, coo, nnz); break;
            case 5: rc = launch_errors_tiled_n<5>(c, coo, nnz); break;
            case 6: rc = launch_errors_tiled_n<6>(c, coo, nnz); break;
            case 7: rc = launch_errors_tiled_n<7>(c, coo, nnz); break;
            case 8: rc = launch_errors_tiled_n<8>(c, coo, nnz); break;
            case 9:
                rc = c->tiled_x4 ? launch_errors_tiled_npx<9, 1, true>(c, coo, nnz) : launch_errors_tiled_npx<9, 1, false>(c, coo, nnz);
                break;
            default:
                rc = c->tiled_x4 ? launch_errors_tiled_npx<10, 1, true>(c, coo, nnz) : launch_errors_tiled_npx<10, 1, false>(c, coo, nnz);
                break;
        }
        if (rc != FTK_OK) return rc;
    } else {
        const int b_in_lds = (size_t)c->L.B_total * 4 <= 65536 - 256;
        const size_t lds = b_in_lds ? (size_t)c->L.B_total * 4 : 0;
        const int grid = blocks_for(nnz, 256, c->num_cu * 8);
        hipLaunchKernelGGL(errors_generic_kernel, dim3(grid), dim3(256), lds, c->stream, coo, c->L, (uint64_t)nnz,
                           (const float*)c->d_A, (const float*)c->d_B, b_in_lds, c->d_sums);
    }
    FTK_HIP(c, hipGetLastError());
    FTK_HIP(c, hipMemcpyAsync(host_sums, c->d_sums, 2 * sizeof(double), hipMemcpyDeviceToHost, c->stream));
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    return FTK_OK;
}

void release(ftk_ctx* c) {
    if (!c) return;
    hipStreamSynchronize(c->stream);
    drop_pending(c);
    for (int n = 0; n < kMaxOrder; ++n)
        if (c->d_new_of_old[n]) hipFree(c->d_new_of_old[n]);
    if (c->d_arena) c->d_A = c->d_dA = nullptr;   // parts of the arena
    void* ptrs[] = {c->d_arena, c->d_rec, c->d_rec_tiles, c->d_stage, c->d_A, c->d_dA, c->d_B, c->d_GB, c->d_sums, c->d_flag,
                    c->d_pos, c->d_bidx, c->d_bval, c->d_hot_partial, c->d_gb_partial, c->d_lists, c->d_list_fill,
                    c->d_bucket_info, c->d_bucket_rows, c->d_overflow};
    for (void* p : ptrs)
        if (p) hipFree(p);
    delete c;
}

// Choose which rows are accumulated in LDS for a sample set of n_samples entries: most frequent
// first, down to a fraction of an expected hit per workgroup and step, as many as the LDS budget
// allows.  Rows are already sorted by count within a mode, so this is a merge of sorted lists.
int plan_rows(ftk_ctx* c, long long n_samples);

int pick_hot_rows(ftk_ctx* c, long long n_samples) {
    const int N = c->order;
    // One workgroup per CU, but no more than there are tiles of 16 samples to give every wave
    // one: every workgroup writes (and the update pass reads) a whole partial table.
    {
        const long long waves = c->variant == V_TILED ? c->tiled_waves : kMfmaWaves;
        // turns in pairs that share their Philox blocks (J = R = 16 kernel, entry-sampling rule) only where every
        // wave of a full launch has at least two groups of 64 anyway
        c->pair_turns = c->variant == V_MFMA16 && c->sampling == FTK_SAMPLE_ENTRIES &&
                        (n_samples + 63) / 64 >= 2LL * c->mfma_grid_max * kMfmaWaves;
        const long long tiles = (n_samples + 15) / 16;
        c->mfma_grid = (int)std::max<long long>(1, std::min<long long>(c->mfma_grid_max, (tiles + waves - 1) / waves));
    }
    long long rows_total = 0;
    for (int n = 0; n < N; ++n) rows_total += c->dims[n];
    // LDS left for the table once the kernel's fixed needs are met, in table rows
    long long budget_bytes, row_bytes;
    if (c->variant == V_TILED) {
        budget_bytes = (long long)c->max_lds - 4LL * (long long)tiled_lds_floats(N, c->tiled_P, c->tiled_waves, 0) - 1024;
        if (c->rows) budget_bytes -= 4LL * (long long)tiled_rows_lds_words(N, c->tiled_waves, c->rows_max_buckets);
        row_bytes = 64LL * c->tiled_P;
    } else {
        budget_bytes = (long long)c->max_lds - 4LL * (kMfmaWaves * mfma16_wave_scratch(N) + N * 256 + kSinkRows * 16) - 1024;
        row_bytes = 64;
    }
    c->hot_H_max = (int)std::max(1LL, budget_bytes / row_bytes);
    const int H = (int)std::min<long long>(c->hot_H_max, rows_total);
    // A table row saves its workgroup one global atomic per hit (~12 ns of a per-CU unit that is the
    // kernel's bottleneck) and costs one 64-byte store and one read at the end of the step: worth
    // it from a fraction of an expected hit per workgroup and step.
    double min_count = 0.25 * (double)c->mfma_grid * (double)c->nnz / (double)std::max<long long>(n_samples, 1);
    // Ranks above 32: the pass is bound by matrix-instruction issue and the atomic unit has room, so the
    // table rows are added by atomics as well (to per-workgroup tables in global memory, see the kernel)
    // and save no atomic.  What they are for is to keep a frequent row from queueing on ONE address across
    // all workgroups: float atomics on one address retire at ~41 ns each, so a row is worth a table row
    // (which the update pass has to sum over all workgroups) when its hits would keep that queue busy for
    // a good part of the pass, which takes about twice its matrix time.
    if (c->variant == V_TILED && c->tiled_P == 4) {
        const double width = 16.0 * c->tiled_P;
        const double pass_seconds = (double)n_samples * 6.0 * N * width * width / (0.5 * 157.3e12);
        const double min_hits = 0.35 * pass_seconds / 41e-9;
        min_count = std::max(min_count, min_hits * (double)c->nnz / (double)std::max<long long>(n_samples, 1));
        // (no tables behind dA: only the rows of the one-hot product are summed per workgroup)
        if (!c->d_wide_tables) min_count = std::numeric_limits<double>::infinity();
    }
    // the 16 most frequent rows of a mode, where they go through the one-hot product (decided below), are
    // summed without a swap: they are taken whatever their count
    bool top_ok[kMaxOrder] = {};
    for (int n = 0; n < N; ++n) {
        double top_hits = 0.0;
        for (int r = 0; r < 16 && r < (int)c->dims[n]; ++r) top_hits += (double)c->sorted_counts[n][r];
        top_ok[n] = c->dims[n] >= 16 && top_hits * 8.0 >= (double)c->nnz;
    }
    int taken[kMaxOrder] = {};
    bool no_table[kMaxOrder] = {};
    auto take_rows = [&]() {
        for (int n = 0; n < N; ++n) taken[n] = 0;
        for (int t = 0; t < H; ++t) {
            int best = -1;
            unsigned int best_count = 0;
            for (int n = 0; n < N; ++n)
                if (!no_table[n] && taken[n] < c->dims[n] &&
                    ((double)c->sorted_counts[n][taken[n]] >= min_count || (top_ok[n] && taken[n] < 16))) {
                    const unsigned int cnt = c->sorted_counts[n][taken[n]];
                    if (best < 0 || cnt > best_count) {
                        best = n;
                        best_count = cnt;
                    }
                }
            if (best < 0) break;
            taken[best] += 1;
        }
    };
    take_rows();
    // Tiled kernel with LDS tables: a tile pays for a mode's table swaps as soon as ONE of its 16 samples has a table row
    // in that mode, and an atomic instruction costs the same with one request as with four.  A mode without frequent
    // rows whose table would hold only a small share of the samples (below a quarter: the swaps then run in nearly
    // every tile and empty hardly any atomic instruction) gets no table; its LDS goes to the other modes.
    // (C3's third mode, 3 000 rows of which 407 fitted, 14 % of the samples: 0.859 -> 0.841 ms per launch without.)
    if (c->variant == V_TILED && c->tiled_P <= 2) {
        bool again = false;
        for (int n = 0; n < N; ++n) {
            if (top_ok[n] || taken[n] == 0 || taken[n] == (int)c->dims[n]) continue;
            double share = 0.0;
            for (int r = 0; r < taken[n]; ++r) share += (double)c->sorted_counts[n][r];
            if (share < 0.25 * (double)c->nnz) {
                no_table[n] = true;
                again = true;
            }
        }
        if (again) take_rows();
    }
    int off = 0;
    for (int n = 0; n < N; ++n) {
        c->hot_K[n] = taken[n];
        c->hot_off[n] = off;
        off += taken[n];
        // The 16 most frequent rows go through a one-hot matrix product (four more matrix
        // instructions per tile and mode) only where they collect a fair share of the samples:
        // at least two of a tile's 16 on average.  Elsewhere they are ordinary table rows.
        c->hot_top[n] = (taken[n] >= 16 && top_ok[n]) ? 16 : 0;
    }
    // Tiled kernel, ranks up to 32: the samples of a group of 64 are parked sorted by the route of their row in ONE
    // mode, the one in which the routes are most mixed (share p of the samples summed per workgroup, p (1 - p)
    // largest).  C3: 0.875 -> 0.855 ms per launch; sorting by two modes gains nothing more; at ranks above 32
    // (no table swaps to skip) it costs 2 %.
    c->sort_mode = -1;
    if (c->variant == V_TILED && c->tiled_P <= 2) {
        double best = 0.05;   // below this the routes are too uniform for the sort to pay
        for (int n = 0; n < N; ++n) {
            double on_chip = 0.0;
            for (int r = 0; r < c->hot_K[n]; ++r) on_chip += (double)c->sorted_counts[n][r];
            const double p = on_chip / (double)c->nnz;
            if (p * (1.0 - p) > best) {
                best = p * (1.0 - p);
                c->sort_mode = n;
            }
        }
    }
    c->hot_H = std::max(off, 1);
    c->mfma_lds_bytes = 4 * ((size_t)(c->hot_H + kSinkRows) * 16 + kMfmaWaves * mfma16_wave_scratch(N) + N * 256);
    c->tiled_lds_bytes = 4 * tiled_lds_floats(N, c->tiled_P, c->tiled_waves, c->hot_H);
    c->hot_for_M = n_samples;
    if (c->variant == V_TILED && c->rows) return plan_rows(c, n_samples);
    return FTK_OK;
}

// The rows form of the tiled kernel: buckets of the rows outside the tables, one list per (gradient
// workgroup, bucket) with room for the expected number of entries plus slack, and the device tables
// that describe them.  Called whenever the tables or |Psi| change (never while a step is being enqueued).
int plan_rows(ftk_ctx* c, long long n_samples) {
    const int N = c->order;
    std::vector<uint2> info;
    std::vector<int4> rows;
    unsigned long long words = 0;
    size_t lds_cells = 0;
    try {
        for (int n = 0; n < N; ++n) {
            c->rows_bucket0[n] = (int)info.size();
            const long long per_bucket = 1LL << c->rows_shift[n];
            const std::vector<unsigned long long>& prefix = c->count_prefix[n];
            for (long long lo = c->hot_K[n]; lo < c->dims[n]; lo += per_bucket) {
                const long long hi = std::min<long long>(lo + per_bucket, c->dims[n]);
                // expected entries of this bucket in one workgroup's list
                const double expect = (double)(prefix[(size_t)hi] - prefix[(size_t)lo]) / (double)c->nnz * (double)n_samples /
                                      (double)c->mfma_grid;
                const double cap = c->rows_tight ? std::max(1.0, std::floor(0.5 * expect)) : std::ceil(expect + 6.0 * std::sqrt(expect) + 8.0);
                if (cap * (double)c->mfma_grid_max > 2e9 || words > 0x07ffffffull) return fail(c, FTK_EUNSUPPORTED, "rows: the lists of one workgroup exceed 2^27 words");
                info.push_back(make_uint2((unsigned int)words, (unsigned int)cap));
                rows.push_back(make_int4(n, (int)lo, (int)(hi - lo), 0));
                words += (unsigned long long)cap * (unsigned long long)rows_entry_words(c->L.J[n]);
                lds_cells = std::max(lds_cells, (size_t)(hi - lo) * (size_t)c->L.J[n]);
            }
        }
    } catch (...) {
        return fail(c, FTK_ENOMEM, "host allocation failed");
    }
    if (words > 0x07ffffffull) return fail(c, FTK_EUNSUPPORTED, "rows: the lists of one workgroup exceed 2^27 words");
    if (info.empty()) {   // every row is in a table: one empty bucket keeps the launches well formed
        info.push_back(make_uint2(0u, 0u));
        rows.push_back(make_int4(0, (int)c->dims[0], 0, 0));
    }
    if (c->mfma_grid_max > kRowsApplyMaxSources) return fail(c, FTK_EUNSUPPORTED, "rows: more than %d gradient workgroups", kRowsApplyMaxSources);
    if ((int)info.size() > c->rows_max_buckets) return fail(c, FTK_EUNSUPPORTED, "rows: internal error, more buckets than planned for");
    const size_t need = (size_t)c->mfma_grid_max * std::max<unsigned long long>(words, 1) * sizeof(float);
    if (need > ((size_t)8 << 30)) return fail(c, FTK_EUNSUPPORTED, "rows: the lists would need %zu bytes (limit 8 GiB)", need);
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    if (need > c->lists_bytes) {
        if (c->d_lists) hipFree(c->d_lists);
        c->d_lists = nullptr;
        c->lists_bytes = 0;
        FTK_HIP(c, hipMalloc(&c->d_lists, need));
        c->lists_bytes = need;
    }
    FTK_HIP(c, hipMemcpy(c->d_bucket_info, info.data(), info.size() * sizeof(uint2), hipMemcpyHostToDevice));
    FTK_HIP(c, hipMemcpy(c->d_bucket_rows, rows.data(), rows.size() * sizeof(int4), hipMemcpyHostToDevice));
    c->rows_n_buckets = (int)info.size();
    c->rows_list_words = (unsigned int)std::max<unsigned long long>(words, 1);
    c->rows_apply_lds = std::max<size_t>(lds_cells, 1) * sizeof(float);
    c->tiled_lds_bytes += 4 * tiled_rows_lds_words(N, c->tiled_waves, c->rows_n_buckets);
    return FTK_OK;
}

int create_impl(ftk_ctx* c, const int64_t* dims, const int32_t* const* idx, const float* vals, uint64_t init_seed,
                uint32_t flags) {
    const int N = c->order;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return fail(c, FTK_EDEVICE, "no HIP device available");
    FTK_HIP(c, hipGetDevice(&c->device));
    FTK_HIP(c, hipDeviceGetAttribute(&c->num_cu, hipDeviceAttributeMultiprocessorCount, c->device));
    FTK_HIP(c, hipDeviceGetAttribute(&c->max_lds, hipDeviceAttributeMaxSharedMemoryPerBlock, c->device));
    if (c->num_cu < 1) c->num_cu = 1;
    if (c->max_lds < 65536) c->max_lds = 65536;

    // packed parameter layout: every mode starts on a 256-byte boundary
    long long a_off = 0, stage = 0;
    int b_off = 0;
    for (int n = 0; n < N; ++n) {
        c->L.A_off[n] = a_off;
        c->L.B_off[n] = b_off;
        a_off += ((dims[n] * c->L.J[n] + 16 + 63) / 64) * 64;   // >= 16 floats of slack after every mode
        b_off += c->L.J[n] * c->L.R;
        stage = std::max(stage, (long long)dims[n] * c->J_user[n]);
    }
    c->A_total = a_off;
    c->L.B_total = b_off;
    pick_generic_config(c);
    c->mfma16_ok = c->L.R == 16 && N <= 6 && c->max_lds >= 131072;
    for (int n = 0; n < N; ++n)   // 16-float rows whose byte offset inside a mode fits 30 bits
        c->mfma16_ok = c->mfma16_ok && c->L.J[n] == 16 && dims[n] < (1LL << 24);
    // the whole packed array is one buffer for the kernel's atomics: 31-bit byte offsets
    c->mfma16_ok = c->mfma16_ok && c->A_total * 4 < 0x7fffffc0LL;
    {
        int pm = c->L.R;
        c->tiled_ok = N <= kTiledMaxOrder && c->L.R <= 64 && c->max_lds >= 131072;
        c->tiled_x4 = true;
        for (int n = 0; n < N; ++n) {
            pm = std::max(pm, c->L.J[n]);
            c->tiled_x4 = c->tiled_x4 && c->L.J[n] % 4 == 0;
            c->tiled_ok = c->tiled_ok && c->L.J[n] <= 64 && dims[n] * c->L.J[n] < (1LL << 28);   // a mode's rows end below 2^30 bytes
        }
        c->tiled_P = pm <= 16 ? 1 : pm <= 32 ? 2 : 4;
        if (N > 8 && c->tiled_P != 1) c->tiled_ok = false;   // orders 9, 10: instances for ranks up to 16 only
        c->tiled_waves = c->tiled_P == 4 ? 4 : 8;
        if (4LL * (long long)tiled_lds_floats(N, c->tiled_P, c->tiled_waves, 16) + 1024 > c->max_lds) c->tiled_ok = false;
    }
    if (c->gen_threads == 0 && !c->mfma16_ok && !c->tiled_ok)
        return fail(c, FTK_EUNSUPPORTED, "N*R = %d with sum J_n R = %d exceeds the kernels' LDS budget", N * c->L.R,
                    c->L.B_total);

    // ---- the tensor: range check, per-mode row frequencies, renumbering, record packing ----
    const hipMemcpyKind kind = (flags & FTK_PTRS_DEVICE) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    const int scan_blocks = blocks_for(c->nnz, 256, c->num_cu * 8);
    c->rec_words = record_words(N);
    FTK_HIP(c, hipMalloc(&c->d_flag, sizeof(unsigned int)));
    FTK_HIP(c, hipMalloc(&c->d_rec, (size_t)c->nnz * c->rec_words * sizeof(uint32_t)));
    if (c->rec_words != N + 1) FTK_HIP(c, hipMemset(c->d_rec, 0, (size_t)c->nnz * c->rec_words * sizeof(uint32_t)));
    uint32_t* d_col = nullptr;        // one caller column at a time
    unsigned int* d_counts = nullptr;
    struct Guard {
        uint32_t*& a;
        unsigned int*& b;
        ~Guard() {
            if (a) hipFree(a);
            if (b) hipFree(b);
        }
    } guard{d_col, d_counts};
    FTK_HIP(c, hipMalloc(&d_col, (size_t)c->nnz * sizeof(uint32_t)));
    std::vector<std::vector<unsigned int>>& sorted_counts = c->sorted_counts;
    sorted_counts.assign(N, {});
    for (int n = 0; n < N; ++n) {
        FTK_HIP(c, hipMemcpy(d_col, idx[n], (size_t)c->nnz * sizeof(int32_t), kind));
        FTK_HIP(c, hipMemset(c->d_flag, 0, sizeof(unsigned int)));
        hipLaunchKernelGGL(check_range_kernel, dim3(scan_blocks), dim3(256), 0, c->stream, (const int32_t*)d_col,
                           (uint64_t)c->nnz, (int32_t)dims[n], c->d_flag);
        FTK_HIP(c, hipGetLastError());
        unsigned int bad = 0;
        FTK_HIP(c, hipMemcpy(&bad, c->d_flag, sizeof bad, hipMemcpyDeviceToHost));
        if (bad) return fail(c, FTK_EINVAL, "idx[%d] holds %u entries outside [0, %lld)", n, bad, (long long)dims[n]);

        FTK_HIP(c, hipMalloc(&d_counts, (size_t)dims[n] * sizeof(unsigned int)));
        FTK_HIP(c, hipMemset(d_counts, 0, (size_t)dims[n] * sizeof(unsigned int)));
        hipLaunchKernelGGL(histogram_kernel, dim3(scan_blocks), dim3(256), 0, c->stream, (const int32_t*)d_col,
                           (uint64_t)c->nnz, d_counts);
        FTK_HIP(c, hipGetLastError());
        std::vector<unsigned int> counts((size_t)dims[n]);
        FTK_HIP(c, hipMemcpy(counts.data(), d_counts, counts.size() * sizeof(unsigned int), hipMemcpyDeviceToHost));
        FTK_HIP(c, hipFree(d_counts));
        d_counts = nullptr;

        // internal row number = rank by descending count (ties: ascending caller row number)
        std::vector<int32_t> order_rows((size_t)dims[n]);
        for (size_t i = 0; i < order_rows.size(); ++i) order_rows[i] = (int32_t)i;
        std::stable_sort(order_rows.begin(), order_rows.end(),
                         [&](int32_t x, int32_t y) { return counts[(size_t)x] > counts[(size_t)y]; });
        std::vector<int32_t> new_of_old((size_t)dims[n]);
        sorted_counts[n].resize((size_t)dims[n]);
        for (size_t r = 0; r < order_rows.size(); ++r) {
            new_of_old[(size_t)order_rows[r]] = (int32_t)r;
            sorted_counts[n][r] = counts[(size_t)order_rows[r]];
        }
        FTK_HIP(c, hipMalloc(&c->d_new_of_old[n], (size_t)dims[n] * sizeof(int32_t)));
        FTK_HIP(c, hipMemcpy(c->d_new_of_old[n], new_of_old.data(), new_of_old.size() * sizeof(int32_t),
                             hipMemcpyHostToDevice));
        hipLaunchKernelGGL(pack_records_kernel, dim3(scan_blocks), dim3(256), 0, c->stream, (const uint32_t*)d_col,
                           (uint64_t)c->nnz, (const int32_t*)c->d_new_of_old[n], c->d_rec, c->rec_words, n);
        FTK_HIP(c, hipGetLastError());
        FTK_HIP(c, hipStreamSynchronize(c->stream));
    }
    FTK_HIP(c, hipMemcpy(d_col, vals, (size_t)c->nnz * sizeof(float), kind));
    hipLaunchKernelGGL(pack_records_kernel, dim3(scan_blocks), dim3(256), 0, c->stream, (const uint32_t*)d_col,
                       (uint64_t)c->nnz, (const int32_t*)nullptr, c->d_rec, c->rec_words, N);
    FTK_HIP(c, hipGetLastError());
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    FTK_HIP(c, hipFree(d_col));
    d_col = nullptr;

    // ---- parameters ----
    {
        // the tables never outgrow what the LDS of a CU holds per workgroup (the kernels' table rows are sized for that)
        const size_t table_floats = (size_t)c->num_cu * (size_t)c->max_lds / sizeof(float);
        const size_t arena_floats = 2 * (size_t)c->A_total + table_floats;
        // every offset the atomics use stays below the out-of-range marker of the kernel (2^30) with room to spare
        if (c->tiled_ok && c->tiled_P == 4 && arena_floats * sizeof(float) < (1ull << 30) - (1ull << 20)) {
            FTK_HIP(c, hipMalloc(&c->d_arena, arena_floats * sizeof(float)));
            c->d_A = c->d_arena;
            c->d_dA = c->d_A + c->A_total;
            c->d_wide_tables = c->d_dA + c->A_total;
            FTK_HIP(c, hipMemset(c->d_wide_tables, 0, table_floats * sizeof(float)));
        } else {
            FTK_HIP(c, hipMalloc(&c->d_A, (size_t)c->A_total * sizeof(float)));
            FTK_HIP(c, hipMalloc(&c->d_dA, (size_t)c->A_total * sizeof(float)));
        }
    }
    FTK_HIP(c, hipMalloc(&c->d_B, (size_t)c->L.B_total * sizeof(float)));
    FTK_HIP(c, hipMalloc(&c->d_GB, (size_t)c->L.B_total * sizeof(float)));
    FTK_HIP(c, hipMalloc(&c->d_stage, (size_t)stage * sizeof(float)));
    FTK_HIP(c, hipMalloc(&c->d_sums, 2 * sizeof(double)));
    FTK_HIP(c, hipMemset(c->d_A, 0, (size_t)c->A_total * sizeof(float)));
    FTK_HIP(c, hipMemset(c->d_dA, 0, (size_t)c->A_total * sizeof(float)));
    FTK_HIP(c, hipMemset(c->d_B, 0, (size_t)c->L.B_total * sizeof(float)));
    FTK_HIP(c, hipMemset(c->d_GB, 0, (size_t)c->L.B_total * sizeof(float)));
    for (int n = 0; n < N; ++n) {
        const long long na = dims[n] * c->J_user[n], nb = (long long)c->J_user[n] * c->R_user;
        hipLaunchKernelGGL(init_factor_kernel, dim3(blocks_for(na, 256, c->num_cu * 8)), dim3(256), 0, c->stream,
                           c->d_A + c->L.A_off[n], (long long)dims[n], c->J_user[n], c->L.J[n],
                           (const int32_t*)c->d_new_of_old[n], init_seed, (uint32_t)n);
        hipLaunchKernelGGL(init_uniform_kernel, dim3(blocks_for(nb, 256, c->num_cu * 8)), dim3(256), 0, c->stream,
                           c->d_B + c->L.B_off[n], (long long)c->J_user[n], c->R_user, c->L.R, init_seed, (uint32_t)(N + n));
    }
    FTK_HIP(c, hipGetLastError());

    // ---- kernel variant ----
    // At order 6 the J = R = 16 kernel's register tiles spill and the general matrix-core kernel is the faster
    // one (10 000^6, |Psi| = 1e6: 0.38 ms against 0.44 ms per step); it stays available by name.
    const bool prefer_mfma16 = c->mfma16_ok && (N <= 5 || !c->tiled_ok);
    c->variant = prefer_mfma16 ? V_MFMA16 : c->tiled_ok ? V_TILED : c->mfma16_ok ? V_MFMA16 : V_GENERIC;
    if (c->mfma16_ok || c->tiled_ok) {
        c->mfma_grid_max = c->num_cu;
        c->mfma_grid = c->mfma_grid_max;
        // per-workgroup tables of the frequently hit rows: never more than the LDS can hold; per-workgroup
        // tables of the core gradient
        FTK_HIP(c, hipMalloc(&c->d_hot_partial, (size_t)c->mfma_grid_max * c->max_lds));
        FTK_HIP(c, hipMalloc(&c->d_gb_partial, (size_t)c->mfma_grid_max * c->L.B_total * sizeof(float)));
        // the rows form of the tiled kernel: bucket sizes follow from the shape alone
        if (c->tiled_ok && c->tiled_x4) {
            c->count_prefix.assign(N, {});
            for (int n = 0; n < N; ++n) {
                std::vector<unsigned long long>& pre = c->count_prefix[n];
                pre.resize((size_t)dims[n] + 1);
                pre[0] = 0;
                for (size_t r = 0; r < (size_t)dims[n]; ++r) pre[r + 1] = pre[r] + c->sorted_counts[n][r];
                // a bucket's rows fit a 64 KB LDS table of the row-owner kernel ...
                int shift = 8;
                while (shift < 20 && (2LL << shift) * c->L.J[n] * 4 <= 65536) ++shift;
                c->rows_shift[n] = shift;
            }
            auto count_buckets = [&]() {
                long long total = 0;
                for (int n = 0; n < N; ++n) total += (dims[n] + (1LL << c->rows_shift[n]) - 1) >> c->rows_shift[n];
                return total;
            };
            // ... and there are at least four buckets per CU (the owners then spread evenly) where the shape allows it (down to 256 rows a bucket)
            for (bool changed = true; changed && count_buckets() < 4LL * c->num_cu;) {
                changed = false;
                for (int n = 0; n < N; ++n)
                    if (c->rows_shift[n] > 8 && (dims[n] >> c->rows_shift[n]) > 0) {
                        c->rows_shift[n] -= 1;
                        changed = true;
                    }
            }
            const long long max_buckets = std::max<long long>(count_buckets(), 1);
            bool fits = max_buckets <= 4096;
            for (int n = 0; n < N; ++n) fits = fits && (1LL << c->rows_shift[n]) * c->L.J[n] * 4 <= 65536;
            fits = fits && 4LL * ((long long)tiled_lds_floats(N, c->tiled_P, c->tiled_waves, 16) +
                                  (long long)tiled_rows_lds_words(N, c->tiled_waves, (int)max_buckets)) + 1024 <= c->max_lds;
            if (fits) {
                c->rows_max_buckets = (int)max_buckets;
                FTK_HIP(c, hipMalloc(&c->d_bucket_info, (size_t)max_buckets * sizeof(uint2)));
                FTK_HIP(c, hipMalloc(&c->d_bucket_rows, (size_t)max_buckets * sizeof(int4)));
                FTK_HIP(c, hipMalloc(&c->d_list_fill, (size_t)c->mfma_grid_max * max_buckets * sizeof(unsigned int)));
                FTK_HIP(c, hipMalloc(&c->d_overflow, sizeof(unsigned int)));
                FTK_HIP(c, hipMemset(c->d_overflow, 0, sizeof(unsigned int)));
                c->rows_ok = true;
            }
        }
        if (const int rc = pick_hot_rows(c, 1LL << 20)) return rc;
    }
    if (const int rc = scratch_setup(c)) return rc;
    if (const int rc = prepare_variant(c)) return rc;
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    return FTK_OK;
}

}  // namespace

extern "C" {

int ftk_create(ftk_ctx** out, int32_t order, const int64_t* dims, int64_t nnz, const int32_t* const* idx,
               const float* vals, const int32_t* J, int32_t R, uint64_t init_seed, uint32_t flags) {
    if (!out) return fail(nullptr, FTK_EINVAL, "out is NULL");
    *out = nullptr;
    if (order < 1 || order > FTK_MAX_ORDER) return fail(nullptr, FTK_EINVAL, "order %d outside 1..%d", order, FTK_MAX_ORDER);
    if (!dims || !idx || !vals || !J) return fail(nullptr, FTK_EINVAL, "NULL argument");
    if (nnz < 1 || nnz >= (1LL << 32)) return fail(nullptr, FTK_EINVAL, "nnz %lld outside 1..2^32-1", (long long)nnz);
    if (R < 1 || R > 1024) return fail(nullptr, FTK_EINVAL, "R %d outside 1..1024", R);
    if (flags & ~(uint32_t)(FTK_PTRS_DEVICE | FTK_LAYOUT_EXACT)) return fail(nullptr, FTK_EINVAL, "unknown flag bits 0x%x", flags);
    for (int n = 0; n < order; ++n) {
        if (dims[n] < 1 || dims[n] >= (1LL << 31))
            return fail(nullptr, FTK_EINVAL, "dims[%d] = %lld outside 1..2^31-1", n, (long long)dims[n]);
        if (J[n] < 1 || J[n] > 1024) return fail(nullptr, FTK_EINVAL, "J[%d] = %d outside 1..1024", n, J[n]);
        if (!idx[n]) return fail(nullptr, FTK_EINVAL, "idx[%d] is NULL", n);
    }
    ftk_ctx* c = new (std::nothrow) ftk_ctx();
    if (!c) return fail(nullptr, FTK_ENOMEM, "host allocation failed");
    c->order = order;
    c->nnz = nnz;
    c->L.order = order;
    c->L.R = R;
    c->R_user = R;
    for (int n = 0; n < order; ++n) {
        c->dims[n] = dims[n];
        c->L.J[n] = J[n];
        c->J_user[n] = J[n];
    }
    // Ranks up to 16 are held zero-padded to 16 (rows of 64 bytes, 16 x 16 core factors) where that
    // puts the shape on the J_n = R = 16 kernel.  Padding is inert: a padded component of a row is 0
    // and meets a zero row of B^(n), so its gradient is 0; a padded r has c^(k)_r = 0 in every mode,
    // so with two or more modes its leave-one-out products, its share of the prediction and its core
    // gradient are 0.
    // Up to order 5, where that kernel is the faster one (measured: order 5 0.28 ms against 0.32 ms per step on
    // the general matrix-core kernel, order 6 0.44 ms against 0.37 ms: its register tiles spill there).
    if (!(flags & FTK_LAYOUT_EXACT) && order >= 2 && order <= 5 && R <= 16) {
        bool pad = true, all16 = R == 16;
        long long bytes = 0;
        for (int n = 0; n < order; ++n) {
            pad = pad && J[n] <= 16 && dims[n] < (1LL << 24);
            all16 = all16 && J[n] == 16;
            bytes += ((dims[n] * 16 + 16 + 63) / 64) * 64 * 4;
        }
        if (pad && !all16 && bytes < 0x7fffffc0LL) {
            c->L.R = 16;
            for (int n = 0; n < order; ++n) c->L.J[n] = 16;
        }
    }
    int rc;
    try {
        rc = create_impl(c, dims, idx, vals, init_seed, flags);
    } catch (...) {
        rc = fail(c, FTK_ENOMEM, "host allocation failed");
    }
    if (rc != FTK_OK) {
        g_create_error = c->err;
        release(c);
        return rc;
    }
    *out = c;
    return FTK_OK;
}

void ftk_destroy(ftk_ctx* ctx) { release(ctx); }

int ftk_sample(ftk_ctx* c, uint64_t seed, int64_t n_samples) {
    if (!c) return FTK_EINVAL;
    if (n_samples < 1 || n_samples >= (1LL << 31))
        return fail(c, FTK_EINVAL, "n_samples %lld outside 1..2^31-1", (long long)n_samples);
    // Psi is a pure function of (seed, k): the fused kernel regenerates positions in registers,
    // so nothing is launched here; the arrays are only materialised for callers that need them.
    c->sample_seed = seed;
    c->n_samples = n_samples;
    c->batch_valid = false;
    if (c->variant != V_GENERIC && c->hot_for_M != n_samples) {
        if (c->rows)   // the lists are re-planned (and possibly re-allocated) on the device
            if (const int rc_dev = check_device(c)) return rc_dev;
        if (const int rc = pick_hot_rows(c, n_samples)) {
            c->n_samples = 0;   // no usable Psi
            return rc;
        }
    }
    return FTK_OK;
}

int ftk_get_samples(ftk_ctx* c, int64_t* pos_out) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (!pos_out) return fail(c, FTK_EINVAL, "pos_out is NULL");
    if (c->n_samples < 1) return fail(c, FTK_ESTATE, "ftk_get_samples before ftk_sample");
    {
        const int rc = ensure_batch(c);
        if (rc != FTK_OK) return rc;
    }
    try {
        std::vector<uint32_t> tmp((size_t)c->n_samples);
        FTK_HIP(c, hipMemcpyAsync(tmp.data(), c->d_pos, tmp.size() * sizeof(uint32_t), hipMemcpyDeviceToHost, c->stream));
        FTK_HIP(c, hipStreamSynchronize(c->stream));
        for (size_t k = 0; k < tmp.size(); ++k) pos_out[k] = (int64_t)tmp[k];
    } catch (...) {
        return fail(c, FTK_ENOMEM, "host allocation failed");
    }
    return FTK_OK;
}

int ftk_sgd_step(ftk_ctx* c, float lr_A, float lr_B, float lambda_A, float lambda_B) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (c->n_samples < 1) return fail(c, FTK_ESTATE, "ftk_sgd_step before ftk_sample");
    c->use_hot_partial = c->d_hot_partial;
    c->use_gb_partial = c->d_gb_partial;
    return step_impl(c, lr_A, lr_B, lambda_A, lambda_B);
}

int ftk_sgd_step_noalloc(ftk_ctx* c, float lr_A, float lr_B, float lambda_A, float lambda_B) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (c->n_samples < 1) return fail(c, FTK_ESTATE, "ftk_sgd_step_noalloc before ftk_sample");
    if (c->mode == FTK_HOGWILD_MODEWISE)
        return fail(c, FTK_EUNSUPPORTED, "ftk_sgd_step_noalloc serves the one-pass modes (FTK_SYNC, FTK_HOGWILD) only");
    if (c->variant == V_GENERIC)
        return fail(c, FTK_EUNSUPPORTED, "ftk_sgd_step_noalloc runs on the matrix-core kernels only: the one-lane-per-sample "
                                         "kernels keep Psi in arrays that are allocated on demand");
    if (c->rows) return fail(c, FTK_EUNSUPPORTED, "ftk_sgd_step_noalloc does not serve the \"rows\" kernel (its lists are allocated buffers)");
    float* base = scratch_address(c);
    if (!base) return fail(c, FTK_EUNSUPPORTED, "no static scratch array on device %d", c->device);
    // the partial tables of this step: [grid][H][row floats], then [grid x parts][B_total]
    const bool tiled = c->variant == V_TILED;
    // (ranks above 32: the tables of the frequent rows sit behind dA, allocated with it)
    const size_t hot_floats = wide_tables(c) ? 0 : (((size_t)c->mfma_grid * c->hot_H * (tiled ? 16 * c->tiled_P : 16)) + 63) / 64 * 64;
    const size_t gb_floats = (size_t)c->mfma_grid * c->L.B_total;
    const size_t need = (hot_floats + gb_floats) * sizeof(float);
    if (need > kScratchBytes)
        return fail(c, FTK_EUNSUPPORTED, "this shape and |Psi| need %zu bytes of partial tables, the static scratch array holds %zu",
                    need, kScratchBytes);
    c->use_hot_partial = base;
    c->use_gb_partial = base + hot_floats;
    c->no_events = true;
    const int rc = step_impl(c, lr_A, lr_B, lambda_A, lambda_B);
    c->no_events = false;
    return rc;
}

}  // extern "C"

namespace {

// The update pass after a matrix-core gradient pass, in parts: `hot` adds the workgroups' tables of the frequent
// rows to A (scaled by -lr_A; -1 where the tables already hold -lr_A x gradient), `core` updates B from the
// workgroups' core-gradient tables.
int launch_apply_parts(ftk_ctx* c, bool hot, bool core, float lr_A, float lr_B, float lambda_B) {
    ApplyArgs p = {};
    p.A = c->d_A;
    p.dA = c->d_dA;
    p.n4 = c->A_total / 4;
    p.dense_blocks = 0;
    if (hot) {
        // tables behind dA were filled by atomics: cleared as they are read, for the next step
        p.hot_clear = wide_tables(c);
        p.hot_partial = p.hot_clear ? c->d_wide_tables : c->use_hot_partial;
        p.hot_parts = c->mfma_grid;
        p.H = c->hot_H;
        p.J = c->variant == V_TILED ? 16 * c->tiled_P : 16;
        p.hot_blocks = (c->hot_H * p.J + 63) / 64;
        p.order = c->order;
        for (int n = 0; n < kMaxOrder; ++n) {
            p.Jn[n] = c->L.J[n];
            p.K[n] = c->hot_K[n];
            p.hot_off[n] = c->hot_off[n];
            p.A_off[n] = c->L.A_off[n];
        }
    }
    p.B = c->d_B;
    p.GB = c->use_gb_partial;
    p.B_total = c->L.B_total;
    p.gb_parts = c->mfma_grid;
    p.gb_clear = 0;
    p.lr_A = lr_A;
    p.lr_B = lr_B;
    p.lambda_B = lambda_B;
    p.inv_M = 1.0f / (float)c->n_samples;
    const int b_blocks = core ? (c->L.B_total + 63) / 64 : 0;
    if (p.hot_blocks + b_blocks < 1) return FTK_OK;
    Bracket t(c, FTK_K_APPLY);
    hipLaunchKernelGGL(apply_kernel, dim3(p.hot_blocks + b_blocks), dim3(256), 0, c->stream, p);
    FTK_HIP(c, hipGetLastError());
    return FTK_OK;
}

// Algorithm 1 in the order it is printed, on the matrix cores (J_n = R = 16 kernel or tiled kernel): the factor
// phase (lines 1-16: the modes of a sample in turn, rows changed in place), the tables of the frequent rows added
// to A, then the core phase (lines 17-39) over the same Psi at the rows the factor phase left, and one update of B.
int step_modewise_matrix_cores(ftk_ctx* c, float lr_A, float lr_B, float lambda_A, float lambda_B) {
    const bool tiled = c->variant == V_TILED;
    if (int rc = tiled ? launch_grad_tiled(c, lambda_A, lr_A, kFactorPhase) : launch_grad_mfma16(c, lambda_A, lr_A, kFactorPhase)) return rc;
    if (int rc = launch_apply_parts(c, true, false, -1.0f, lr_B, lambda_B)) return rc;
    if (int rc = tiled ? launch_grad_tiled(c, lambda_A, lr_A, kCorePhase) : launch_grad_mfma16(c, lambda_A, lr_A, kCorePhase)) return rc;
    return launch_apply_parts(c, false, true, -1.0f, lr_B, lambda_B);
}

// One step over the current Psi with the partial tables c->use_hot_partial / c->use_gb_partial.
int step_impl(ftk_ctx* c, float lr_A, float lr_B, float lambda_A, float lambda_B) {
    // the mode-by-mode in-place order: on the matrix cores where a kernel is built for it, else on the one-lane-per-sample kernels
    const bool modewise = c->mode == FTK_HOGWILD_MODEWISE;
    if (modewise && modewise_on_matrix_cores(c)) return step_modewise_matrix_cores(c, lr_A, lr_B, lambda_A, lambda_B);
    const bool mfma = c->variant != V_GENERIC && !modewise;   // a matrix-core variant: per-workgroup tables
    const bool tiled = c->variant == V_TILED && !modewise;
    const bool in_place = c->mode != FTK_SYNC;
    int rc = mfma ? FTK_OK : ensure_batch(c);
    if (rc != FTK_OK) return rc;
    rc = tiled ? launch_grad_tiled(c, lambda_A, lr_A)
               : mfma ? launch_grad_mfma16(c, lambda_A, lr_A) : launch_grad_generic(c, lambda_A, lr_A, modewise);
    if (rc != FTK_OK) return rc;
    {
        ApplyArgs p = {};
        p.A = c->d_A;
        p.dA = c->d_dA;
        p.n4 = c->A_total / 4;
        const bool rows = tiled && c->rows;
        if (rows) {
            // the row-owning workgroups: every bucket's lists summed on chip, its rows of A updated with plain stores
            RowsApplyArgs r = {};
            r.lists = c->d_lists;
            r.list_fill = c->d_list_fill;
            r.bucket_info = c->d_bucket_info;
            r.bucket_rows = c->d_bucket_rows;
            r.list_words = c->rows_list_words;
            r.n_buckets = c->rows_n_buckets;
            r.n_sources = c->mfma_grid;
            r.A = c->d_A;
            r.dA = c->d_dA;
            for (int n = 0; n < kMaxOrder; ++n) {
                r.A_off[n] = c->L.A_off[n];
                r.J[n] = c->L.J[n];
            }
            r.overflow = c->d_overflow;
            r.lr_A = lr_A;
            Bracket t(c, FTK_K_APPLY);
            hipLaunchKernelGGL(rows_apply_kernel, dim3(c->rows_n_buckets), dim3(kRowsApplyThreads), c->rows_apply_lds, c->stream, r);
            FTK_HIP(c, hipGetLastError());
            p.clear_word = c->d_overflow;
        }
        // in-place mode: the gradient pass already added -lr_A * gradient to A (and to the workgroup
        // tables), so there is no accumulator to scan and the tables are added as they are; rows form:
        // the row owners above have done the accumulator's part
        p.dense_blocks = (in_place || rows) ? 0 : blocks_for(p.n4, 256, c->num_cu * 16);
        if (mfma) {
            // tables behind dA were filled by atomics: cleared as they are read, for the next step
            p.hot_clear = tiled && wide_tables(c);
            p.hot_partial = p.hot_clear ? c->d_wide_tables : c->use_hot_partial;
            p.hot_parts = c->mfma_grid;
            p.H = c->hot_H;
            p.J = tiled ? 16 * c->tiled_P : 16;
            p.hot_blocks = (c->hot_H * p.J + 63) / 64;
            p.order = c->order;
            for (int n = 0; n < kMaxOrder; ++n) {
                p.Jn[n] = c->L.J[n];
                p.K[n] = c->hot_K[n];
                p.hot_off[n] = c->hot_off[n];
                p.A_off[n] = c->L.A_off[n];
            }
        }
        p.B = c->d_B;
        p.GB = mfma ? c->use_gb_partial : c->d_GB;
        p.B_total = c->L.B_total;
        p.gb_parts = mfma ? c->mfma_grid : 1;
        p.gb_clear = mfma ? 0 : 1;
        p.lr_A = in_place ? -1.0f : lr_A;
        p.lr_B = lr_B;
        p.lambda_B = lambda_B;
        p.inv_M = 1.0f / (float)c->n_samples;
        const int b_blocks = (c->L.B_total + 63) / 64;
        Bracket t(c, FTK_K_APPLY);
        hipLaunchKernelGGL(apply_kernel, dim3(p.dense_blocks + p.hot_blocks + b_blocks), dim3(256), 0, c->stream, p);
    }
    FTK_HIP(c, hipGetLastError());
    return FTK_OK;
}

// Everything a step of the current variant and mode needs set up on the host side, so that the step
// itself only launches: today, the kernels' dynamic-LDS limits.
int prepare_variant(ftk_ctx* c) {
    c->prepare_only = true;
    c->use_hot_partial = c->d_hot_partial;
    c->use_gb_partial = c->d_gb_partial;
    const bool modewise = c->mode == FTK_HOGWILD_MODEWISE;
    int rc;
    if (modewise && c->variant == V_MFMA16) {
        rc = launch_grad_mfma16(c, 0.0f, 0.0f, kFactorPhase);
        if (rc == FTK_OK) rc = launch_grad_mfma16(c, 0.0f, 0.0f, kCorePhase);
    } else if (modewise && tiled_modewise_ok(c)) {
        rc = launch_grad_tiled(c, 0.0f, 0.0f, kFactorPhase);
        if (rc == FTK_OK) rc = launch_grad_tiled(c, 0.0f, 0.0f, kCorePhase);
    } else {
        rc = (c->variant == V_TILED && !modewise) ? launch_grad_tiled(c, 0.0f, 0.0f)
             : (c->variant == V_MFMA16 && !modewise) ? launch_grad_mfma16(c, 0.0f, 0.0f)
                                                     : launch_grad_generic(c, 0.0f, 0.0f, modewise);
    }
    c->prepare_only = false;
    return rc;
}

}  // namespace

extern "C" {

int ftk_rmse(ftk_ctx* c, double* out) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (!out) return fail(c, FTK_EINVAL, "out is NULL");
    double s[2] = {0.0, 0.0};
    int rc = launch_errors(c, Coo{c->d_rec, c->rec_words}, c->nnz, s);
    if (rc != FTK_OK) return rc;
    *out = sqrt(s[0] / (double)c->nnz);
    return FTK_OK;
}

int ftk_mae(ftk_ctx* c, double* out) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (!out) return fail(c, FTK_EINVAL, "out is NULL");
    double s[2] = {0.0, 0.0};
    int rc = launch_errors(c, Coo{c->d_rec, c->rec_words}, c->nnz, s);
    if (rc != FTK_OK) return rc;
    *out = s[1] / (double)c->nnz;
    return FTK_OK;
}

int ftk_evaluate(ftk_ctx* c, int64_t n_eval, const int32_t* const* idx, const float* vals, uint32_t flags,
                 double* rmse_out, double* mae_out) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (n_eval < 1 || n_eval >= (1LL << 32)) return fail(c, FTK_EINVAL, "n_eval %lld outside 1..2^32-1", (long long)n_eval);
    if (!idx || !vals) return fail(c, FTK_EINVAL, "NULL argument");
    if (flags & ~(uint32_t)FTK_PTRS_DEVICE) return fail(c, FTK_EINVAL, "unknown flag bits 0x%x", flags);
    const int N = c->order;
    for (int n = 0; n < N; ++n)
        if (!idx[n]) return fail(c, FTK_EINVAL, "idx[%d] is NULL", n);
    const hipMemcpyKind kind = (flags & FTK_PTRS_DEVICE) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    uint32_t* d_rec = nullptr;
    uint32_t* d_col = nullptr;
    struct Guard {
        uint32_t*& a;
        uint32_t*& b;
        ~Guard() {
            if (a) hipFree(a);
            if (b) hipFree(b);
        }
    } guard{d_rec, d_col};
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    FTK_HIP(c, hipMalloc(&d_rec, (size_t)n_eval * c->rec_words * sizeof(uint32_t)));
    FTK_HIP(c, hipMalloc(&d_col, (size_t)n_eval * sizeof(uint32_t)));
    if (c->rec_words != N + 1) FTK_HIP(c, hipMemset(d_rec, 0, (size_t)n_eval * c->rec_words * sizeof(uint32_t)));
    const int scan_blocks = blocks_for(n_eval, 256, c->num_cu * 8);
    for (int n = 0; n <= N; ++n) {
        FTK_HIP(c, hipMemcpy(d_col, n < N ? (const void*)idx[n] : (const void*)vals, (size_t)n_eval * sizeof(uint32_t), kind));
        if (n < N) {
            FTK_HIP(c, hipMemset(c->d_flag, 0, sizeof(unsigned int)));
            hipLaunchKernelGGL(check_range_kernel, dim3(scan_blocks), dim3(256), 0, c->stream, (const int32_t*)d_col,
                               (uint64_t)n_eval, (int32_t)c->dims[n], c->d_flag);
            FTK_HIP(c, hipGetLastError());
            unsigned int bad = 0;
            FTK_HIP(c, hipMemcpy(&bad, c->d_flag, sizeof bad, hipMemcpyDeviceToHost));
            if (bad) return fail(c, FTK_EINVAL, "idx[%d] holds %u entries outside [0, %lld)", n, bad, (long long)c->dims[n]);
        }
        // row numbers go through the same renumbering as the stored entries; values are copied as bits
        hipLaunchKernelGGL(pack_records_kernel, dim3(scan_blocks), dim3(256), 0, c->stream, (const uint32_t*)d_col,
                           (uint64_t)n_eval, n < N ? (const int32_t*)c->d_new_of_old[n] : (const int32_t*)nullptr, d_rec,
                           c->rec_words, n);
        FTK_HIP(c, hipGetLastError());
        FTK_HIP(c, hipStreamSynchronize(c->stream));
    }
    double s[2] = {0.0, 0.0};
    int rc = launch_errors(c, Coo{d_rec, c->rec_words}, n_eval, s);
    if (rc != FTK_OK) return rc;
    if (rmse_out) *rmse_out = sqrt(s[0] / (double)n_eval);
    if (mae_out) *mae_out = s[1] / (double)n_eval;
    return FTK_OK;
}

double ftk_step_size(double alpha, double beta, int64_t t) {
    if (t < 0) return NAN;
    const double denom = 1.0 + beta * pow((double)t, 1.5);
    if (!(denom > 0.0)) return NAN;
    return alpha / denom;
}

int ftk_get_factors(ftk_ctx* c, float* const* A_out, float* const* B_out) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    for (int n = 0; n < c->order; ++n) {
        if (A_out && A_out[n]) {
            const long long na = c->dims[n] * c->J_user[n];
            hipLaunchKernelGGL(permute_rows_kernel, dim3(blocks_for(na, 256, c->num_cu * 8)), dim3(256), 0, c->stream,
                               (const float*)(c->d_A + c->L.A_off[n]), c->d_stage, (const int32_t*)c->d_new_of_old[n],
                               (long long)c->dims[n], c->J_user[n], c->L.J[n], 0);
            FTK_HIP(c, hipGetLastError());
            FTK_HIP(c, hipMemcpyAsync(A_out[n], c->d_stage, (size_t)na * sizeof(float), hipMemcpyDeviceToHost, c->stream));
            FTK_HIP(c, hipStreamSynchronize(c->stream));
        }
        if (B_out && B_out[n])   // J_n rows of R floats out of rows of (padded) L.R floats
            FTK_HIP(c, hipMemcpy2DAsync(B_out[n], (size_t)c->R_user * sizeof(float), c->d_B + c->L.B_off[n],
                                        (size_t)c->L.R * sizeof(float), (size_t)c->R_user * sizeof(float),
                                        (size_t)c->J_user[n], hipMemcpyDeviceToHost, c->stream));
    }
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    return FTK_OK;
}

int ftk_set_factors(ftk_ctx* c, const float* const* A_in, const float* const* B_in) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    for (int n = 0; n < c->order; ++n) {
        if (A_in && A_in[n]) {
            const long long na = c->dims[n] * c->J_user[n];
            FTK_HIP(c, hipMemcpyAsync(c->d_stage, A_in[n], (size_t)na * sizeof(float), hipMemcpyHostToDevice, c->stream));
            hipLaunchKernelGGL(permute_rows_kernel, dim3(blocks_for(na, 256, c->num_cu * 8)), dim3(256), 0, c->stream,
                               (const float*)c->d_stage, c->d_A + c->L.A_off[n], (const int32_t*)c->d_new_of_old[n],
                               (long long)c->dims[n], c->J_user[n], c->L.J[n], 1);
            FTK_HIP(c, hipGetLastError());
            FTK_HIP(c, hipStreamSynchronize(c->stream));
        }
        if (B_in && B_in[n])
            FTK_HIP(c, hipMemcpy2DAsync(c->d_B + c->L.B_off[n], (size_t)c->L.R * sizeof(float), B_in[n],
                                        (size_t)c->R_user * sizeof(float), (size_t)c->R_user * sizeof(float),
                                        (size_t)c->J_user[n], hipMemcpyHostToDevice, c->stream));
    }
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    return FTK_OK;
}

int ftk_set_sampling(ftk_ctx* c, int rule) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (rule != FTK_SAMPLE_ENTRIES && rule != FTK_SAMPLE_TILES) return fail(c, FTK_EINVAL, "unknown sampling rule %d", rule);
    if (rule == FTK_SAMPLE_TILES && !c->d_rec_tiles) {
        // first use: the order pi(q) = (a q + b) mod nnz and a second copy of the records in it
        uint64_t a = (uint64_t)c->nnz * 618034ull / 1000000ull;
        if (a < 1) a = 1;
        while (a > 1 && std::gcd(a, (uint64_t)c->nnz) != 1) --a;
        c->tile_a = a;
        c->tile_b = (uint64_t)c->nnz / 3;
        FTK_HIP(c, hipStreamSynchronize(c->stream));
        uint32_t* d = nullptr;
        FTK_HIP(c, hipMalloc(&d, (size_t)c->nnz * c->rec_words * sizeof(uint32_t)));
        hipLaunchKernelGGL(reorder_records_kernel, dim3(blocks_for(c->nnz, 256, c->num_cu * 8)), dim3(256), 0, c->stream,
                           (const uint32_t*)c->d_rec, d, (uint64_t)c->nnz, c->rec_words, c->tile_a, c->tile_b);
        if (hipGetLastError() != hipSuccess || hipStreamSynchronize(c->stream) != hipSuccess) {
            hipFree(d);
            return fail(c, FTK_EDEVICE, "reordering the records failed");
        }
        c->d_rec_tiles = d;
    }
    if (rule != c->sampling) c->batch_valid = false;
    c->sampling = rule;
    if (c->variant != V_GENERIC)
        if (const int rc = pick_hot_rows(c, std::max<long long>(c->n_samples, 1))) return rc;
    return prepare_variant(c);
}

int ftk_set_mode(ftk_ctx* c, int mode) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    if (mode != FTK_SYNC && mode != FTK_HOGWILD && mode != FTK_HOGWILD_MODEWISE)
        return fail(c, FTK_EINVAL, "unknown mode %d", mode);
    if (mode != FTK_SYNC && c->rows)
        return fail(c, FTK_EUNSUPPORTED, "the \"rows\" kernel serves the synchronous step only");
    if (mode == FTK_HOGWILD_MODEWISE && !modewise_on_matrix_cores(c) && c->gen_threads == 0)
        return fail(c, FTK_EUNSUPPORTED, "the mode-by-mode order runs on the matrix-core kernels or on the one-lane-per-sample kernels, which do not fit this shape");
    const int old_mode = c->mode;
    c->mode = mode;
    const int rc = prepare_variant(c);
    if (rc != FTK_OK) c->mode = old_mode;
    return rc;
}

int ftk_set_stream(ftk_ctx* c, void* hip_stream) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    drop_pending(c);
    c->stream = (hipStream_t)hip_stream;
    return FTK_OK;
}

int ftk_set_timing(ftk_ctx* c, int enabled) {
    if (!c) return FTK_EINVAL;
    if (const int rc_dev = check_device(c)) return rc_dev;
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    drop_pending(c);
    for (auto& s : c->slots) {
        s.total_ms = 0.0;
        s.launches = 0;
    }
    c->timing = enabled != 0;
    return FTK_OK;
}

int ftk_get_timing(ftk_ctx* c, int which, double* total_ms, int64_t* launches, int reset) {
    if (!c) return FTK_EINVAL;
    if (which < 0 || which >= FTK_K_COUNT) return fail(c, FTK_EINVAL, "unknown kernel slot %d", which);
    if (const int rc_dev = check_device(c)) return rc_dev;
    FTK_HIP(c, hipStreamSynchronize(c->stream));
    for (auto& s : c->slots) {
        for (auto& p : s.pending) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, p.first, p.second) == hipSuccess) {
                s.total_ms += (double)ms;
                s.launches += 1;
            }
            hipEventDestroy(p.first);
            hipEventDestroy(p.second);
        }
        s.pending.clear();
    }
    if (total_ms) *total_ms = c->slots[which].total_ms;
    if (launches) *launches = c->slots[which].launches;
    if (reset) {
        c->slots[which].total_ms = 0.0;
        c->slots[which].launches = 0;
    }
    return FTK_OK;
}

int ftk_set_kernel(ftk_ctx* c, const char* name) {
    if (!c) return FTK_EINVAL;
    if (!name) return fail(c, FTK_EINVAL, "name is NULL");
    if (const int rc_dev = check_device(c)) return rc_dev;
    // the accumulators of both variants are clean between steps, so switching is always safe
    if (!strcmp(name, "auto"))
        name = (c->mfma16_ok && (c->order <= 5 || !c->tiled_ok)) ? "mfma16" : c->tiled_ok ? "tiled" : c->mfma16_ok ? "mfma16" : "generic";
    if (!strcmp(name, "rows") || !strcmp(name, "rows:tight")) {
        if (!c->rows_ok)
            return fail(c, FTK_EUNSUPPORTED, "rows needs the tiled kernel's shapes with every J_n a multiple of 4 and at most 4096 buckets of rows");
        if (c->mode != FTK_SYNC) return fail(c, FTK_EUNSUPPORTED, "the \"rows\" kernel serves the synchronous step only");
        const int old_variant = c->variant;
        const bool old_rows = c->rows, old_tight = c->rows_tight;
        c->variant = V_TILED;
        c->rows = true;
        c->rows_tight = name[4] == ':';
        int rc = pick_hot_rows(c, std::max<long long>(c->n_samples, 1));
        if (rc == FTK_OK) rc = prepare_variant(c);
        if (rc != FTK_OK) {   // back to what was in use
            c->variant = old_variant;
            c->rows = old_rows;
            c->rows_tight = old_tight;
            if (c->variant != V_GENERIC) pick_hot_rows(c, std::max<long long>(c->n_samples, 1));
        }
        return rc;
    }
    c->rows = false;
    if (!strcmp(name, "generic")) {
        if (c->gen_threads == 0) return fail(c, FTK_EUNSUPPORTED, "the generic kernel does not fit this shape");
        c->variant = V_GENERIC;
        return prepare_variant(c);
    }
    if (!strcmp(name, "mfma16")) {
        if (!c->mfma16_ok) return fail(c, FTK_EUNSUPPORTED, "mfma16 needs J_n = R = 16 and order <= 6");
        c->variant = V_MFMA16;
        if (const int rc = pick_hot_rows(c, std::max<long long>(c->n_samples, 1))) return rc;
        return prepare_variant(c);
    }
    if (!strcmp(name, "tiled")) {
        if (!c->tiled_ok) return fail(c, FTK_EUNSUPPORTED, "tiled needs order <= 8 with J_n, R <= 64 (order 9, 10: <= 16) and padded core factors that fit LDS twice");
        c->variant = V_TILED;
        if (const int rc = pick_hot_rows(c, std::max<long long>(c->n_samples, 1))) return rc;
        return prepare_variant(c);
    }
    return fail(c, FTK_EUNSUPPORTED, "no kernel variant named '%s'", name);
}

const char* ftk_kernel_name(const ftk_ctx* c) {
    if (!c) return "none";
    return (c->variant == V_TILED && c->rows) ? "rows" : kVariantNames[c->variant];
}

int ftk_get_table_rows(ftk_ctx* c, int32_t* K_out, int32_t* top_out) {
    if (!c) return FTK_EINVAL;
    const bool table = c->variant != V_GENERIC;
    for (int n = 0; n < c->order; ++n) {
        if (K_out) K_out[n] = table ? c->hot_K[n] : 0;
        if (top_out) top_out[n] = table ? c->hot_top[n] : 0;
    }
    return FTK_OK;
}

const char* ftk_last_error(const ftk_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
