// libnomad: C ABI over the gfx950 kernels in nomad_kernels.h.  Host code only sequences kernel
// launches on the context's stream and moves buffers; every step of the epoch runs on the GPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "nomad.h"
#include "nomad_kernels.h"

using namespace nomad;

struct KernelTimer {
    std::vector<hipEvent_t> begin, end;   // events borrowed from the context's pool
};

struct nomad_ctx {
    nomad_config cfg{};
    hipStream_t stream = nullptr;
    float noise_count = 0.f;
    std::string err;
    bool has_graph = false, has_theta = false, has_grad = false;
    int64_t n = 0, E = 0;
    int32_t R = 0;
    bool grouped = false;
    int lpr = 16;
    // graph
    int32_t *row_ptr = nullptr, *col = nullptr, *cluster_of = nullptr, *group_of_cluster = nullptr;
    float* pe = nullptr;
    // partition tables
    uint32_t *counts = nullptr, *gbase = nullptr, *gcount = nullptr, *chunk_start = nullptr;
    float* gomega = nullptr;
    float4* hinfo = nullptr;
    int32_t *gmembers = nullptr, *cmembers = nullptr;
    MeanChunk* chunks = nullptr;
    uint32_t n_chunks = 0;
    double2* mean_partial = nullptr;
    float omega0 = 0.f;
    // state
    float2 *theta = nullptr, *g = nullptr, *ghead = nullptr, *mu = nullptr, *B = nullptr;
    float4* cinfo = nullptr;
    int32_t* cell_slot = nullptr;   // grouped: slot of each cell in the group-ordered cell table
    int2* group_slots = nullptr;    // grouped: slot range [lo, hi) of each group's cells
    float* A = nullptr;
    unsigned long long* gfix = nullptr;
    // gradient through the means (opt-in, grouped graphs)
    bool through_means = false;
    float *cS = nullptr, *chead = nullptr;   // 2 p_e / S_e per edge, its row sums
    unsigned long long* Gfix = nullptr;      // [2 R] fixed-point sums over the heads, per cell
    float2* gmean = nullptr;                 // [R] what every member of a cell adds to its gradient
    // binned deterministic scatter
    bool binned = false;
    int n_wg = 0, bin_block = 1024;
    int pool_rounds = 0;            // > 0: the pooled edge pass runs, pool_block = bin_block * pool_rounds
    bool sorted_records = true;     // the binned edge pass counting-sorts a round's records by tile before writing them
    int flush_rounds = 1;           // unsorted form: rounds between two flushes of the records (1 or 2)
    std::vector<int64_t> batch_row, batch_edge;   // [B + 1] first head / first CSR position of every sub-step
    uint32_t n_bins = 0, max_chunks = 0;
    int tile_bits = kMaxTileBits;
    uint32_t *pool = nullptr, *chunk_prev = nullptr, *chain_head = nullptr, *chain_fill = nullptr, *wg_pool_begin = nullptr;
    int32_t* head = nullptr;
    int* overflow = nullptr;
    double *loss_partial = nullptr, *loss_out = nullptr;
    uint32_t edge_grid = 0;
    int* flags = nullptr;
    // launch-shape knobs (nomad_tune) and what set_graph made of them
    int tune_edge_block = 0, tune_wg_per_cu = 0, tune_path = 0, tune_pool_kernel = 1, tune_phases = 0, tune_record_sort = 0, tune_flush_rounds = 0;
    int path = 0;                   // NOMAD_PATH_* in use
    int phases = 1;                 // record phases of the binned edge pass
    unsigned long long* carry = nullptr;   // [2 n] fixed-point sums carried from phase to phase (phases > 1)
    uint32_t* pool_keys = nullptr;  // stratified pools: the keys of the epoch whose kernels run next on the stream
    bool distinct_kernel = false;   // the pooled edge pass is the one for distinct picks
    uint32_t pool_blocks = 1;       // distinct picks: number of blocks
    std::unordered_map<const void*, size_t> allocations;   // device memory held, by pointer
    int64_t device_bytes = 0;
    // timing
    bool profiling = false;
    KernelTimer timers[NOMAD_K_COUNT];
    std::vector<hipEvent_t> event_pool;   // created when timing is switched on, so that a timed launch only records
    size_t event_next = 0;
};

namespace {

int fail(nomad_ctx* c, int code, const char* fmt, ...) {
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof(buf), fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return code;
}

#define HIP_TRY(c, call)                                                                                   \
    do {                                                                                                   \
        hipError_t e_ = (call);                                                                            \
        if (e_ != hipSuccess)                                                                              \
            return fail((c), e_ == hipErrorOutOfMemory ? NOMAD_E_OOM : NOMAD_E_HIP, "%s: %s", #call,       \
                        hipGetErrorString(e_));                                                            \
    } while (0)

template <typename T>
int dev_alloc(nomad_ctx* c, T** p, size_t count) {
    *p = nullptr;
    const size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
    HIP_TRY(c, hipMalloc((void**)p, bytes));
    c->allocations[*p] = bytes;
    c->device_bytes += (int64_t)bytes;
    return NOMAD_OK;
}

template <typename T>
void dev_free(nomad_ctx* c, T*& p) {
    if (p) {
        auto it = c->allocations.find(p);
        if (it != c->allocations.end()) { c->device_bytes -= (int64_t)it->second; c->allocations.erase(it); }
        (void)hipFree(p);
    }
    p = nullptr;
}

void free_graph(nomad_ctx* c) {
    dev_free(c, c->row_ptr); dev_free(c, c->col); dev_free(c, c->cluster_of); dev_free(c, c->group_of_cluster);
    dev_free(c, c->pe); dev_free(c, c->counts); dev_free(c, c->gbase); dev_free(c, c->gcount); dev_free(c, c->chunk_start);
    dev_free(c, c->gomega); dev_free(c, c->hinfo); dev_free(c, c->gmembers); dev_free(c, c->cmembers); dev_free(c, c->chunks); dev_free(c, c->mean_partial);
    dev_free(c, c->theta); dev_free(c, c->g); dev_free(c, c->ghead); dev_free(c, c->mu); dev_free(c, c->B); dev_free(c, c->cinfo);
    dev_free(c, c->cell_slot); dev_free(c, c->group_slots);
    dev_free(c, c->A); dev_free(c, c->gfix); dev_free(c, c->loss_partial); dev_free(c, c->loss_out);
    dev_free(c, c->cS); dev_free(c, c->chead); dev_free(c, c->Gfix); dev_free(c, c->gmean);
    c->through_means = false;
    dev_free(c, c->flags);
    dev_free(c, c->pool); dev_free(c, c->chunk_prev); dev_free(c, c->chain_head); dev_free(c, c->chain_fill); dev_free(c, c->wg_pool_begin);
    dev_free(c, c->head); dev_free(c, c->overflow); dev_free(c, c->carry); dev_free(c, c->pool_keys);
    c->phases = 1;
    c->binned = false;
    c->pool_rounds = 0;
    c->distinct_kernel = false;
    c->path = 0;
    c->has_graph = c->has_theta = c->has_grad = false;
    c->E = 0;
}

hipMemcpyKind in_kind(int mem) { return mem == NOMAD_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice; }
hipMemcpyKind out_kind(int mem) { return mem == NOMAD_DEVICE ? hipMemcpyDeviceToDevice : hipMemcpyDeviceToHost; }

inline uint32_t blocks_for(int64_t items, int per_block = kBlock) { return (uint32_t)((items + per_block - 1) / per_block); }

bool grow_event_pool(nomad_ctx* c, size_t count) {
    for (size_t k = 0; k < count; ++k) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return false;
        c->event_pool.push_back(e);
    }
    return true;
}

hipEvent_t take_event(nomad_ctx* c) {
    if (c->event_next == c->event_pool.size() && !grow_event_pool(c, 1024)) return nullptr;
    return c->event_pool[c->event_next++];
}

struct Timed {  // records a begin/end event pair around one launch when timing is on
    nomad_ctx* c; int kind; hipEvent_t e1 = nullptr;
    Timed(nomad_ctx* ctx, int k) : c(ctx), kind(k) {
        if (!c->profiling) return;
        hipEvent_t e0 = take_event(c);
        e1 = take_event(c);
        if (!e0 || !e1) { e1 = nullptr; return; }
        (void)hipEventRecord(e0, c->stream);
        c->timers[kind].begin.push_back(e0);
    }
    ~Timed() {
        if (!e1) return;
        (void)hipEventRecord(e1, c->stream);
        c->timers[kind].end.push_back(e1);
    }
};

void clear_timers(nomad_ctx* c) {
    for (auto& t : c->timers) {
        t.begin.clear();
        t.end.clear();
    }
    c->event_next = 0;
}

void destroy_event_pool(nomad_ctx* c) {
    clear_timers(c);
    for (auto e : c->event_pool) (void)hipEventDestroy(e);
    c->event_pool.clear();
}

inline bool is_power_of_two(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
inline uint32_t log2_of(int64_t v) { uint32_t b = 0; while (((int64_t)1 << (b + 1)) <= v) ++b; return b; }

EdgeArgs edge_args(nomad_ctx* c, uint32_t t) {
    EdgeArgs a{};
    a.row_ptr = c->row_ptr; a.col = c->col; a.pe = c->pe; a.theta = c->theta;
    a.cluster_of = c->cluster_of; a.group_of_cluster = c->grouped ? c->group_of_cluster : nullptr;
    a.gbase = c->gbase; a.gcount = c->gcount; a.gomega = c->gomega; a.gmembers = c->gmembers; a.hinfo = c->hinfo;
    a.A = c->A; a.B = c->B;
    a.mu = c->mu; a.far = (c->grouped && c->cfg.far_field == NOMAD_FAR_FIELD_SAMPLED) ? 1 : 0;
    a.noise_count = c->noise_count; a.omega0 = c->omega0;
    a.key0 = (uint32_t)c->cfg.seed; a.key1 = (uint32_t)(c->cfg.seed >> 32); a.epoch = t;
    a.pool_size = (uint32_t)c->cfg.pool_size; a.pool_block = (uint32_t)c->cfg.pool_block;
    a.pool_mode = (uint32_t)c->cfg.pool_mode;
    a.pool_line_bits = log2_of(c->cfg.pool_line); a.pool_segment_bits = log2_of(c->cfg.pool_segment);
    a.pool_blocks = c->pool_blocks;
    a.pool_keys = c->pool_keys;
    if (c->cfg.pool_mode == NOMAD_POOL_STRATIFIED)   // the keys of epoch t, ahead of the kernels that read them on the same stream
        hipLaunchKernelGGL(k_pool_keys, dim3(1), dim3(64), 0, c->stream, a.key0, a.key1, t, (uint32_t)c->n, c->pool_keys);
    a.s = c->cfg.n_neg; a.n = c->n; a.row_begin = 0; a.row_end = c->n;
    a.g = c->g; a.ghead = c->ghead; a.gfix = c->gfix; a.loss_partial = c->loss_partial;
    a.cS = nullptr;   // set by nomad_epoch when the gradient flows through the means
    return a;
}

template <int MODE, int LPR>
void launch_edges_s(nomad_ctx* c, const EdgeArgs& a) {
    const dim3 grid(c->edge_grid), block(kBlock);
    switch (c->cfg.n_neg) {
#define NOMAD_CASE(S) case S: hipLaunchKernelGGL((k_edges<S, MODE, LPR>), grid, block, 0, c->stream, a); break;
        NOMAD_CASE(1) NOMAD_CASE(2) NOMAD_CASE(3) NOMAD_CASE(4) NOMAD_CASE(5) NOMAD_CASE(6) NOMAD_CASE(7) NOMAD_CASE(8)
#undef NOMAD_CASE
        default: hipLaunchKernelGGL((k_edges<0, MODE, LPR>), grid, block, 0, c->stream, a); break;
    }
}

template <int MODE>
void launch_edges(nomad_ctx* c, const EdgeArgs& a) {
    launch_edges_s<MODE, 16>(c, a);
}

BinArgs bin_args(nomad_ctx* c) {
    BinArgs q{};
    q.head = c->head; q.pool = c->pool; q.chunk_prev = c->chunk_prev; q.chain_head = c->chain_head; q.chain_fill = c->chain_fill;
    q.wg_pool_begin = c->wg_pool_begin; q.ghead = c->ghead; q.E = c->E; q.e_begin = 0; q.e_end = c->E;
    q.max_chunks = c->max_chunks; q.n_bins = c->n_bins;
    q.tile_bits = c->tile_bits; q.overflow = c->overflow;
    return q;
}


size_t edge_pass_lds_bytes(const nomad_ctx* c) {
    if (c->pool_rounds && c->distinct_kernel)
        return distinct_lds_bytes(c->n_bins, (uint32_t)c->cfg.pool_size, (uint32_t)(c->cfg.pool_size / c->cfg.pool_line), c->pool_rounds);
    return c->pool_rounds ? pooled_lds_bytes(c->n_bins, c->cfg.pool_block, (uint32_t)c->cfg.pool_size)
                          : binned_lds_bytes(c->n_bins, c->cfg.n_neg, c->bin_block, c->sorted_records);
}

// Calls `fn(kernel)` with the edge-pass kernel that matches the context: number of negatives, sampler, launch shape.
using EdgePassKernel = void (*)(const EdgeArgs, const BinArgs);

template <int S, typename Fn>
void with_edge_pass_kernel_s(const nomad_ctx* c, Fn fn) {
    EdgePassKernel k = k_edges_binned<S, 1024>;
    if (c->distinct_kernel && c->pool_rounds == 1) k = k_edges_pooled_distinct<S, 1>;
    else if (c->distinct_kernel && c->pool_rounds == 2) k = k_edges_pooled_distinct<S, 2>;
    else if (c->distinct_kernel && c->pool_rounds == 4) k = k_edges_pooled_distinct<S, 4>;
    else if (c->distinct_kernel && c->pool_rounds == 8) k = k_edges_pooled_distinct<S, 8>;
    else if (c->pool_rounds == 1) k = k_edges_pooled<S, 1, 1024>;
    else if (c->pool_rounds == 2) k = k_edges_pooled<S, 2, 1024>;
    else if (c->pool_rounds == 4) k = k_edges_pooled<S, 4, 1024>;
    else if (c->pool_rounds == 8) k = k_edges_pooled<S, 8, 1024>;
    else if (c->bin_block == 512) k = c->sorted_records ? k_edges_binned<S, 512, true> : k_edges_binned<S, 512, false>;
    else if (!c->sorted_records && c->flush_rounds == 2) k = k_edges_binned<S, 1024, false, 2>;
    else if (!c->sorted_records) k = k_edges_binned<S, 1024, false, 1>;
    fn(k);
}

template <typename Fn>
bool with_edge_pass_kernel(const nomad_ctx* c, Fn fn) {
    switch (c->cfg.n_neg) {
        case 0: with_edge_pass_kernel_s<0>(c, fn); return true;
        case 1: with_edge_pass_kernel_s<1>(c, fn); return true;
        case 2: with_edge_pass_kernel_s<2>(c, fn); return true;
        case 3: with_edge_pass_kernel_s<3>(c, fn); return true;
        case 4: with_edge_pass_kernel_s<4>(c, fn); return true;
        case 5: with_edge_pass_kernel_s<5>(c, fn); return true;
        case 6: with_edge_pass_kernel_s<6>(c, fn); return true;
        case 7: with_edge_pass_kernel_s<7>(c, fn); return true;
        case 8: with_edge_pass_kernel_s<8>(c, fn); return true;
    }
    return false;
}

int prepare_binned(nomad_ctx* c) {
    HIP_TRY(c, hipFuncSetAttribute((const void*)k_tile_accumulate, hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)(sizeof(unsigned long long) * 2 << c->tile_bits)));
    hipError_t err = hipErrorInvalidValue;
    const int lds = (int)edge_pass_lds_bytes(c);
    with_edge_pass_kernel(c, [&](EdgePassKernel kernel) {
        err = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    HIP_TRY(c, err);
    return NOMAD_OK;
}

void launch_edges_binned(nomad_ctx* c, const EdgeArgs& a, int64_t e_begin, int64_t e_end) {
    BinArgs q = bin_args(c);
    q.e_begin = e_begin;
    q.e_end = e_end;
    const dim3 grid(c->n_wg), block(c->bin_block);
    const size_t lds = edge_pass_lds_bytes(c);
    with_edge_pass_kernel(c, [&](EdgePassKernel kernel) { hipLaunchKernelGGL(kernel, grid, block, lds, c->stream, a, q); });
}

// cell means of the current embedding -> mu, cinfo
int run_means(nomad_ctx* c) {
    Timed tm(c, NOMAD_K_MEANS);
    if (c->n_chunks)
        hipLaunchKernelGGL(k_mean_chunks, dim3(c->n_chunks), dim3(kBlock), 0, c->stream, c->theta, c->cmembers, c->chunks,
                           c->mean_partial);
    hipLaunchKernelGGL(k_mean_finish, dim3(blocks_for((int64_t)c->R * 64)), dim3(kBlock), 0, c->stream, c->mean_partial,
                       c->chunk_start, c->counts, c->grouped ? c->group_of_cluster : nullptr, c->grouped ? c->cell_slot : nullptr,
                       c->R, 1.0 / (double)c->n, c->mu, c->cinfo);
    return NOMAD_OK;
}

// mean-field sums of the heads row_begin .. row_end-1
int run_mean_field(nomad_ctx* c, int64_t row_begin, int64_t row_end) {
    if (!c->grouped || row_end <= row_begin || c->cfg.far_field == NOMAD_FAR_FIELD_SAMPLED) return NOMAD_OK;
    Timed tm(c, NOMAD_K_MEANFIELD);
    hipLaunchKernelGGL(k_mean_field, dim3(blocks_for(row_end - row_begin, kMeanFieldBlock * kMeanFieldHeads)), dim3(kMeanFieldBlock), 0,
                       c->stream, c->theta, c->cluster_of, c->group_of_cluster, c->cinfo, c->group_slots, c->R, row_begin, row_end,
                       c->A, c->B);
    return NOMAD_OK;
}

// Gradient through the means: c_i of the heads of this step from the edge pass's per-edge values, the sum over
// those heads for every cell, and the vector every member of a cell adds to its gradient.
int run_mean_gradient(nomad_ctx* c, int64_t row_begin, int64_t row_end) {
    if (!c->through_means) return NOMAD_OK;
    Timed tm(c, NOMAD_K_MEANGRAD);
    if (row_end > row_begin) {
        hipLaunchKernelGGL(k_head_coefficients, dim3(blocks_for(row_end - row_begin)), dim3(kBlock), 0, c->stream, c->row_ptr, c->cS,
                           row_begin, row_end, c->chead);
        const dim3 grid(blocks_for(c->R), blocks_for(row_end - row_begin, kMeanGradHeads));
        hipLaunchKernelGGL(k_mean_gradient, grid, dim3(kBlock), 0, c->stream, c->theta, c->chead, c->hinfo, c->mu, c->group_of_cluster,
                           c->R, row_begin, row_end, c->Gfix);
    }
    hipLaunchKernelGGL(k_mean_gradient_finish, dim3(blocks_for(c->R)), dim3(kBlock), 0, c->stream, c->Gfix, c->counts, c->R,
                       (double)c->noise_count / (double)c->n, c->gmean);
    return NOMAD_OK;
}

int check_ready(nomad_ctx* c, bool need_theta) {
    if (!c) return NOMAD_E_INVALID_ARG;
    if (!c->has_graph) return fail(c, NOMAD_E_ORDER, "no graph: call nomad_set_graph first");
    if (need_theta && !c->has_theta) return fail(c, NOMAD_E_ORDER, "no embedding: call nomad_set_embedding first");
    return NOMAD_OK;
}

int copy_out(nomad_ctx* c, void* dst, const void* src, size_t bytes, int mem) {
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->overflow) {
        int ov = 0;
        HIP_TRY(c, hipMemcpy(&ov, c->overflow, sizeof(int), hipMemcpyDeviceToHost));
        if (ov) return fail(c, NOMAD_E_HIP, "internal error: record pool bound exceeded");
    }
    HIP_TRY(c, hipMemcpy(dst, src, bytes, out_kind(mem)));
    return NOMAD_OK;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

int nomad_create(const nomad_config* cfg, nomad_ctx** out) {
    if (!cfg || !out) return NOMAD_E_INVALID_ARG;
    if (cfg->struct_size != sizeof(nomad_config)) return NOMAD_E_INVALID_ARG;
    if (cfg->n_points < 1 || cfg->n_clusters < 1 || cfg->n_neg < 0 || cfg->n_neg > NOMAD_MAX_NEG || cfg->n_epochs < 1 ||
        cfg->batches_per_epoch < 1 || cfg->batches_per_epoch > NOMAD_MAX_BATCHES || !(cfg->lr0 >= 0.f) || !std::isfinite(cfg->lr0) || !std::isfinite(cfg->noise_count) ||
        (cfg->scatter_mode != NOMAD_SCATTER_DETERMINISTIC && cfg->scatter_mode != NOMAD_SCATTER_ATOMIC) || cfg->device < 0)
        return NOMAD_E_INVALID_ARG;
    if (cfg->pool_size < 0 || cfg->pool_size > NOMAD_MAX_POOL || cfg->pool_block < 0 || (cfg->pool_size == 0) != (cfg->pool_block == 0))
        return NOMAD_E_INVALID_ARG;
    if ((cfg->far_field != NOMAD_FAR_FIELD_EXACT && cfg->far_field != NOMAD_FAR_FIELD_SAMPLED) ||
        (cfg->far_field == NOMAD_FAR_FIELD_SAMPLED && cfg->pool_size > 0))
        return NOMAD_E_INVALID_ARG;
    if (cfg->pool_mode != NOMAD_POOL_PICKS16 && cfg->pool_mode != NOMAD_POOL_DISTINCT && cfg->pool_mode != NOMAD_POOL_STRATIFIED)
        return NOMAD_E_INVALID_ARG;
    if (cfg->pool_mode == NOMAD_POOL_PICKS16 && (cfg->pool_line > 1 || cfg->pool_line < 0 || cfg->pool_segment < 0)) return NOMAD_E_INVALID_ARG;
    if (cfg->pool_mode == NOMAD_POOL_DISTINCT || cfg->pool_mode == NOMAD_POOL_STRATIFIED) {
        const int line = cfg->pool_line ? cfg->pool_line : 1, seg = cfg->pool_segment ? cfg->pool_segment : 64;
        // (a line is at most the whole point set: its points are start, start + 1, ... taken modulo n with one subtraction)
        if (cfg->pool_size < 2 || !is_power_of_two(cfg->pool_size) || !is_power_of_two(line) || line > cfg->pool_size ||
            line > cfg->n_points || cfg->n_neg > cfg->pool_size / line || seg < 64 || !is_power_of_two(seg) ||
            cfg->pool_block % seg != 0 || cfg->batches_per_epoch != 1)
            return NOMAD_E_INVALID_ARG;
    }
    if (cfg->edge_weights != NOMAD_WEIGHTS_GIVEN && cfg->edge_weights != NOMAD_WEIGHTS_INVERSE_RANK) return NOMAD_E_INVALID_ARG;
    if ((cfg->mean_gradient != 0 && cfg->mean_gradient != 1) ||
        (cfg->mean_gradient && (cfg->far_field == NOMAD_FAR_FIELD_SAMPLED || cfg->batches_per_epoch > 1)))
        return NOMAD_E_INVALID_ARG;
    if (cfg->n_points >= ((int64_t)1 << 31) || cfg->n_clusters > cfg->n_points) return cfg->n_points >= ((int64_t)1 << 31) ? NOMAD_E_TOO_LARGE : NOMAD_E_INVALID_ARG;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device >= ndev) return NOMAD_E_HIP;
    nomad_ctx* c = new (std::nothrow) nomad_ctx();
    if (!c) return NOMAD_E_OOM;
    c->cfg = *cfg;
    if (c->cfg.pool_line == 0) c->cfg.pool_line = 1;
    if (c->cfg.pool_segment == 0) c->cfg.pool_segment = 64;
    c->stream = (hipStream_t)cfg->stream;
    c->n = cfg->n_points;
    c->R = cfg->n_clusters;
    c->noise_count = cfg->noise_count > 0.f ? cfg->noise_count : (float)cfg->n_neg;
    *out = c;
    return NOMAD_OK;
}

void nomad_destroy(nomad_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->cfg.device);
    (void)hipStreamSynchronize(c->stream);
    destroy_event_pool(c);
    free_graph(c);
    delete c;
}

const char* nomad_last_error(const nomad_ctx* c) { return c ? c->err.c_str() : "null context"; }

int64_t nomad_num_edges(const nomad_ctx* c) { return c ? c->E : 0; }

int nomad_set_graph(nomad_ctx* c, const int32_t* row_ptr, const int32_t* col_idx, const float* weights,
                    const int32_t* cluster_of, const int32_t* cluster_group, int mem) {
    if (!c) return NOMAD_E_INVALID_ARG;
    if (!row_ptr || !cluster_of || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return fail(c, NOMAD_E_INVALID_ARG, "null pointer or bad mem");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    free_graph(c);
    const int64_t n = c->n;
    const int32_t R = c->R;
    hipStream_t st = c->stream;
    int rc;
    std::string fallback_note;
#define TRY(x) do { rc = (x); if (rc != NOMAD_OK) { free_graph(c); return rc; } } while (0)
#define HTRY(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { free_graph(c); return fail(c, e_ == hipErrorOutOfMemory ? NOMAD_E_OOM : NOMAD_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); } } while (0)

    // ---- copy the CSR offsets, learn E
    TRY(dev_alloc(c, &c->row_ptr, (size_t)n + 1));
    HTRY(hipMemcpy(c->row_ptr, row_ptr, sizeof(int32_t) * ((size_t)n + 1), in_kind(mem)));
    int32_t E32 = 0;
    HTRY(hipMemcpy(&E32, c->row_ptr + n, sizeof(int32_t), hipMemcpyDeviceToHost));
    if (E32 < 0) { free_graph(c); return fail(c, NOMAD_E_BAD_GRAPH, "row_ptr[n] is negative"); }
    const int64_t E = E32;
    if (E > 0 && !col_idx) { free_graph(c); return fail(c, NOMAD_E_INVALID_ARG, "col_idx is null"); }
    c->E = E;
    {   // sub-steps of an epoch: consecutive head ranges and the CSR positions they own
        const int B = c->cfg.batches_per_epoch;
        c->batch_row.assign((size_t)B + 1, 0);
        c->batch_edge.assign((size_t)B + 1, 0);
        for (int b = 0; b <= B; ++b) {
            c->batch_row[b] = n * (int64_t)b / B;
            int32_t off = 0;
            HTRY(hipMemcpy(&off, c->row_ptr + c->batch_row[b], sizeof(int32_t), hipMemcpyDeviceToHost));
            c->batch_edge[b] = off;
        }
    }
    TRY(dev_alloc(c, &c->col, (size_t)E));
    if (E) HTRY(hipMemcpy(c->col, col_idx, sizeof(int32_t) * (size_t)E, in_kind(mem)));
    TRY(dev_alloc(c, &c->cluster_of, (size_t)n));
    HTRY(hipMemcpy(c->cluster_of, cluster_of, sizeof(int32_t) * (size_t)n, in_kind(mem)));
    float* wdev = nullptr;
    const bool by_rank = c->cfg.edge_weights == NOMAD_WEIGHTS_INVERSE_RANK;
    if (by_rank && weights) { free_graph(c); return fail(c, NOMAD_E_INVALID_ARG, "edge_weights = NOMAD_WEIGHTS_INVERSE_RANK takes no weights array"); }
    if (by_rank) TRY(dev_alloc(c, &c->pe, (size_t)E));
    if (weights) {
        TRY(dev_alloc(c, &c->pe, (size_t)E));
        TRY(dev_alloc(c, &wdev, (size_t)E));
        hipError_t e_ = E ? hipMemcpy(wdev, weights, sizeof(float) * (size_t)E, in_kind(mem)) : hipSuccess;
        if (e_ != hipSuccess) { dev_free(c, wdev); free_graph(c); return fail(c, NOMAD_E_HIP, "copy of weights: %s", hipGetErrorString(e_)); }
    }
    std::vector<int32_t> hgroup;
    c->grouped = false;
    if (cluster_group) {
        hgroup.resize(R);
        hipError_t e_ = hipMemcpy(hgroup.data(), cluster_group, sizeof(int32_t) * (size_t)R,
                                  mem == NOMAD_DEVICE ? hipMemcpyDeviceToHost : hipMemcpyHostToHost);
        if (e_ != hipSuccess) { dev_free(c, wdev); free_graph(c); return fail(c, NOMAD_E_HIP, "copy of cluster_group: %s", hipGetErrorString(e_)); }
        for (int32_t r = 0; r < R; ++r)
            if (hgroup[r] < 0 || hgroup[r] >= R) { dev_free(c, wdev); free_graph(c); return fail(c, NOMAD_E_BAD_GRAPH, "cluster_group[%d] = %d is outside 0..|R|-1", r, hgroup[r]); }
        for (int32_t r = 1; r < R; ++r)
            if (hgroup[r] != hgroup[0]) c->grouped = true;   // one label everywhere == nothing approximated
        if (c->grouped && c->cfg.pool_size > 0) { dev_free(c, wdev); free_graph(c); return fail(c, NOMAD_E_INVALID_ARG, "the pooled sampler needs a single sampling population (cluster_group = NULL)"); }
        if (c->grouped) {
            rc = dev_alloc(c, &c->group_of_cluster, (size_t)R);
            if (rc == NOMAD_OK && hipMemcpy(c->group_of_cluster, hgroup.data(), sizeof(int32_t) * (size_t)R, hipMemcpyHostToDevice) != hipSuccess) rc = fail(c, NOMAD_E_HIP, "upload of cluster_group failed");
            if (rc != NOMAD_OK) { dev_free(c, wdev); free_graph(c); return rc; }
        }
    }

    // ---- validate on the device
    rc = dev_alloc(c, &c->flags, kFlagCount);
    uint32_t *first = nullptr, *gfirst = nullptr;
    unsigned long long* boundaries = nullptr;
    if (rc == NOMAD_OK) rc = dev_alloc(c, &c->counts, (size_t)R);
    if (rc == NOMAD_OK) rc = dev_alloc(c, &first, (size_t)R);
    if (rc == NOMAD_OK) rc = dev_alloc(c, &gfirst, (size_t)R);
    if (rc == NOMAD_OK) rc = dev_alloc(c, &boundaries, 2);
    auto cleanup_tmp = [&]() { dev_free(c, wdev); dev_free(c, first); dev_free(c, gfirst); dev_free(c, boundaries); };
    if (rc != NOMAD_OK) { cleanup_tmp(); free_graph(c); return rc; }
#define HTRY2(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { cleanup_tmp(); free_graph(c); return fail(c, e_ == hipErrorOutOfMemory ? NOMAD_E_OOM : NOMAD_E_HIP, "%s: %s", #call, hipGetErrorString(e_)); } } while (0)
    HTRY2(hipMemsetAsync(c->flags, 0, sizeof(int) * kFlagCount, st));
    HTRY2(hipMemsetAsync(c->counts, 0, sizeof(uint32_t) * (size_t)R, st));
    HTRY2(hipMemsetAsync(first, 0xFF, sizeof(uint32_t) * (size_t)R, st));
    HTRY2(hipMemsetAsync(gfirst, 0xFF, sizeof(uint32_t) * (size_t)R, st));
    HTRY2(hipMemsetAsync(boundaries, 0, sizeof(unsigned long long) * 2, st));
    hipLaunchKernelGGL(k_check_row_ptr, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->row_ptr, n, c->flags);
    int hflags[kFlagCount];
    HTRY2(hipMemcpyAsync(hflags, c->flags, sizeof(hflags), hipMemcpyDeviceToHost, st));
    HTRY2(hipStreamSynchronize(st));
    if (hflags[kFlagRowPtr]) { cleanup_tmp(); free_graph(c); return fail(c, NOMAD_E_BAD_GRAPH, "row_ptr must start at 0 and be non-decreasing"); }
    hipLaunchKernelGGL(k_check_rows, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->row_ptr, c->col, wdev, c->pe, n, by_rank ? 1 : 0, c->flags);
    hipLaunchKernelGGL(k_cluster_census, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->cluster_of,
                       c->grouped ? c->group_of_cluster : nullptr, n, R, c->counts, first, gfirst, boundaries, c->flags);
    HTRY2(hipMemcpyAsync(hflags, c->flags, sizeof(hflags), hipMemcpyDeviceToHost, st));
    HTRY2(hipStreamSynchronize(st));
    const char* what = hflags[kFlagCol] ? "col_idx entry outside 0..n-1" : hflags[kFlagSelfLoop] ? "self loop in the graph"
                     : hflags[kFlagWeight] ? "weights must be finite, >= 0, with a positive sum on every non-empty row"
                     : hflags[kFlagCluster] ? "cluster_of entry outside 0..|R|-1" : nullptr;
    if (what) { cleanup_tmp(); free_graph(c); return fail(c, NOMAD_E_BAD_GRAPH, "%s", what); }
    dev_free(c, wdev);

    // ---- partition tables (host arithmetic on |R|-sized arrays only)
    std::vector<uint32_t> hcounts(R), hfirst(R), hgfirst(R);
    unsigned long long hb[2];
    HTRY2(hipMemcpy(hcounts.data(), c->counts, sizeof(uint32_t) * (size_t)R, hipMemcpyDeviceToHost));
    HTRY2(hipMemcpy(hfirst.data(), first, sizeof(uint32_t) * (size_t)R, hipMemcpyDeviceToHost));
    HTRY2(hipMemcpy(hgfirst.data(), gfirst, sizeof(uint32_t) * (size_t)R, hipMemcpyDeviceToHost));
    HTRY2(hipMemcpy(hb, boundaries, sizeof(hb), hipMemcpyDeviceToHost));
    cleanup_tmp();
    int64_t nonempty = 0;
    for (int32_t r = 0; r < R; ++r) nonempty += hcounts[r] > 0;
    const bool clusters_contiguous = (int64_t)hb[0] == nonempty - 1;
    std::vector<int32_t> hcluster;   // host copy of cluster_of, fetched only if a member list is needed
    auto fetch_clusters = [&]() -> int {
        if (!hcluster.empty()) return NOMAD_OK;
        hcluster.resize((size_t)n);
        hipError_t e_ = hipMemcpy(hcluster.data(), c->cluster_of, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost);
        return e_ == hipSuccess ? NOMAD_OK : fail(c, NOMAD_E_HIP, "download of cluster_of: %s", hipGetErrorString(e_));
    };
    // member order of the cells for the mean reduction
    std::vector<uint32_t> cstart(R + 1, 0);
    if (clusters_contiguous) {
        for (int32_t r = 0; r < R; ++r) cstart[r] = hcounts[r] ? hfirst[r] : 0;   // start in index space
    } else {
        TRY(fetch_clusters());
        for (int32_t r = 0; r < R; ++r) cstart[r + 1] = cstart[r] + hcounts[r];
        std::vector<uint32_t> cur(cstart.begin(), cstart.end() - 1);
        std::vector<int32_t> mem_list((size_t)n);
        for (int64_t i = 0; i < n; ++i) mem_list[cur[hcluster[i]]++] = (int32_t)i;
        TRY(dev_alloc(c, &c->cmembers, (size_t)n));
        HTRY(hipMemcpy(c->cmembers, mem_list.data(), sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
    }
    {
        constexpr uint32_t kChunk = 2048;
        std::vector<MeanChunk> chunks;
        std::vector<uint32_t> chunk_start(R + 1, 0);
        for (int32_t r = 0; r < R; ++r) {
            chunk_start[r] = (uint32_t)chunks.size();
            for (uint32_t o = 0; o < hcounts[r]; o += kChunk)
                chunks.push_back(MeanChunk{r, cstart[r] + o, cstart[r] + std::min(hcounts[r], o + kChunk)});
        }
        chunk_start[R] = (uint32_t)chunks.size();
        c->n_chunks = (uint32_t)chunks.size();
        TRY(dev_alloc(c, &c->chunks, chunks.size()));
        TRY(dev_alloc(c, &c->chunk_start, (size_t)R + 1));
        TRY(dev_alloc(c, &c->mean_partial, chunks.size()));
        HTRY(hipMemcpy(c->chunks, chunks.data(), sizeof(MeanChunk) * chunks.size(), hipMemcpyHostToDevice));
        HTRY(hipMemcpy(c->chunk_start, chunk_start.data(), sizeof(uint32_t) * ((size_t)R + 1), hipMemcpyHostToDevice));
    }
    // sampling populations
    const double Mn = (double)c->noise_count;
    const int s = c->cfg.n_neg;
    c->omega0 = s > 0 ? (float)(Mn / (double)s) : 0.f;
    if (c->grouped) {
        std::vector<uint32_t> gcount(R, 0), gbase(R, 0);
        std::vector<float> gomega(R, 0.f);
        for (int32_t r = 0; r < R; ++r) gcount[hgroup[r]] += hcounts[r];
        int64_t ngroups = 0;
        for (int32_t g = 0; g < R; ++g) ngroups += gcount[g] > 0;
        const bool groups_contiguous = (int64_t)hb[1] == ngroups - 1;
        if (groups_contiguous) {
            for (int32_t g = 0; g < R; ++g) gbase[g] = gcount[g] ? hgfirst[g] : 0;
        } else {
            TRY(fetch_clusters());
            uint32_t run = 0;
            for (int32_t g = 0; g < R; ++g) { gbase[g] = run; run += gcount[g]; }
            std::vector<uint32_t> cur(gbase);
            std::vector<int32_t> mem_list((size_t)n);
            for (int64_t i = 0; i < n; ++i) mem_list[cur[hgroup[hcluster[i]]]++] = (int32_t)i;   // ascending inside each group
            TRY(dev_alloc(c, &c->gmembers, (size_t)n));
            HTRY(hipMemcpy(c->gmembers, mem_list.data(), sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice));
        }
        for (int32_t g = 0; g < R; ++g) gomega[g] = s > 0 ? (float)(Mn * ((double)gcount[g] / (double)n) / (double)s) : 0.f;
        TRY(dev_alloc(c, &c->gbase, (size_t)R));
        TRY(dev_alloc(c, &c->gcount, (size_t)R));
        TRY(dev_alloc(c, &c->gomega, (size_t)R));
        HTRY(hipMemcpy(c->gbase, gbase.data(), sizeof(uint32_t) * (size_t)R, hipMemcpyHostToDevice));
        HTRY(hipMemcpy(c->gcount, gcount.data(), sizeof(uint32_t) * (size_t)R, hipMemcpyHostToDevice));
        HTRY(hipMemcpy(c->gomega, gomega.data(), sizeof(float) * (size_t)R, hipMemcpyHostToDevice));
        TRY(dev_alloc(c, &c->hinfo, (size_t)n));
        hipLaunchKernelGGL(k_head_info, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->cluster_of, c->group_of_cluster, c->gbase,
                           c->gcount, c->gomega, n, c->hinfo);
        TRY(dev_alloc(c, &c->A, (size_t)n));
        TRY(dev_alloc(c, &c->B, (size_t)n));
        if (c->cfg.mean_gradient) {
            c->through_means = true;
            TRY(dev_alloc(c, &c->cS, (size_t)E));
            TRY(dev_alloc(c, &c->chead, (size_t)n));
            TRY(dev_alloc(c, &c->Gfix, (size_t)R * 2));
            TRY(dev_alloc(c, &c->gmean, (size_t)R));
            HTRY(hipMemsetAsync(c->Gfix, 0, sizeof(unsigned long long) * 2 * (size_t)R, st));
            HTRY(hipMemsetAsync(c->cS, 0, sizeof(float) * (size_t)std::max<int64_t>(E, 1), st));
        }
        // cell table ordered group by group (stable in the cell id): the mean-field pass skips a head's own
        // group as one slot range
        std::vector<int32_t> gcells(R, 0), slot(R);
        std::vector<int2> gslots(R);
        for (int32_t r = 0; r < R; ++r) gcells[hgroup[r]]++;
        int32_t run_slot = 0;
        for (int32_t g = 0; g < R; ++g) { gslots[g] = make_int2(run_slot, run_slot + gcells[g]); run_slot += gcells[g]; }
        std::vector<int32_t> next_slot(R);
        for (int32_t g = 0; g < R; ++g) next_slot[g] = gslots[g].x;
        for (int32_t r = 0; r < R; ++r) slot[r] = next_slot[hgroup[r]]++;
        TRY(dev_alloc(c, &c->cell_slot, (size_t)R));
        TRY(dev_alloc(c, &c->group_slots, (size_t)R));
        HTRY(hipMemcpy(c->cell_slot, slot.data(), sizeof(int32_t) * (size_t)R, hipMemcpyHostToDevice));
        HTRY(hipMemcpy(c->group_slots, gslots.data(), sizeof(int2) * (size_t)R, hipMemcpyHostToDevice));
    }

    c->pool_blocks = 1;
    if (c->cfg.pool_mode != NOMAD_POOL_PICKS16) {   // blocks of the pooled sampler with distinct picks: NB = ceil(NS / Q)
        if (c->cfg.pool_mode == NOMAD_POOL_STRATIFIED) TRY(dev_alloc(c, &c->pool_keys, 8));
        const int64_t seg = c->cfg.pool_segment, NS = (E + seg - 1) / seg, Qs = c->cfg.pool_block / seg;
        c->pool_blocks = (uint32_t)std::max<int64_t>(1, (NS + Qs - 1) / Qs);
    }

    // ---- state buffers
    c->edge_grid = (blocks_for(n, kBlock / c->lpr) + 7u) & ~7u;
    TRY(dev_alloc(c, &c->theta, (size_t)n));
    TRY(dev_alloc(c, &c->g, (size_t)n));
    TRY(dev_alloc(c, &c->mu, (size_t)R));
    TRY(dev_alloc(c, &c->cinfo, (size_t)R));
    TRY(dev_alloc(c, &c->loss_partial, (size_t)c->edge_grid));
    TRY(dev_alloc(c, &c->loss_out, 1));
    if (c->cfg.scatter_mode == NOMAD_SCATTER_DETERMINISTIC) {
        TRY(dev_alloc(c, &c->ghead, (size_t)n));
        // Binned scatter of the tail and negative forces: needs a compile-time s and per-tile tables
        // that fit LDS; if its record pool cannot be allocated, fixed-point global atomics remain
        // as the fallback.
        EdgePlanRequest want_plan;
        want_plan.n = n; want_plan.E = E; want_plan.s = s;
        want_plan.pool_size = c->cfg.pool_size; want_plan.pool_block = c->cfg.pool_block; want_plan.pool_line = std::max(1, c->cfg.pool_line);
        want_plan.pool_distinct = c->cfg.pool_mode != NOMAD_POOL_PICKS16;
        want_plan.tune_edge_block = c->tune_edge_block; want_plan.tune_wg_per_cu = c->tune_wg_per_cu;
        want_plan.tune_pool_kernel = c->tune_pool_kernel; want_plan.tune_record_sort = c->tune_record_sort;
        want_plan.tune_flush_rounds = c->tune_flush_rounds;
        const EdgePlan plan = plan_edge_pass(want_plan);   // tile size, kernel, launch shape (edge_plan.h)
        const int tile_bits = plan.tile_bits, bin_block = plan.bin_block, wg_per_cu = plan.wg_per_cu, pool_rounds = plan.pool_rounds;
        const uint32_t n_bins = plan.n_bins;
        const bool sorted = plan.sorted, distinct = plan.distinct_kernel;
        std::string why;   // why the fallback path is in use, if it is
        if (c->tune_path == NOMAD_PATH_FIXED_ATOMICS) why = "the fixed-point atomics path was asked for (nomad_tune)";
        else if (s > 8) why = "more than 8 negatives per edge: the binned edge pass is built for s <= 8";
        else if (!bin_block) why = "the per-tile tables of the binned edge pass do not fit LDS at this number of points";
        if (E > 0 && why.empty()) {
            hipDeviceProp_t prop;
            HTRY(hipGetDeviceProperties(&prop, c->cfg.device));
            c->bin_block = bin_block;
            c->sorted_records = sorted;
            c->flush_rounds = plan.flush_rounds;
            c->pool_rounds = pool_rounds;
            c->distinct_kernel = distinct;
            c->n_wg = std::max(1, prop.multiProcessorCount) * wg_per_cu;
            c->n_bins = n_bins;
            c->tile_bits = tile_bits;
            unsigned long long* total_dev = nullptr;
            unsigned long long want = 0;
            bool ok = dev_alloc(c, &c->wg_pool_begin, (size_t)c->n_wg + 1) == NOMAD_OK && dev_alloc(c, &total_dev, 1) == NOMAD_OK;
            if (ok) {
                if (c->pool_rounds && distinct)
                    hipLaunchKernelGGL(k_wg_pools_distinct, dim3(1), dim3(64), 0, st, c->pool_blocks, c->n_wg, (int64_t)c->cfg.pool_block,
                                       (uint32_t)c->cfg.pool_size, n_bins, c->wg_pool_begin, total_dev);
                else if (c->pool_rounds)
                    hipLaunchKernelGGL(k_wg_pools_pooled, dim3(1), dim3(64), 0, st, E, c->n_wg, (int64_t)c->cfg.pool_block,
                                       (uint32_t)c->cfg.pool_size, n_bins, c->wg_pool_begin, total_dev);
                else {
                    c->phases = plan_record_phases(E, s, c->bin_block, c->tune_phases);   // edge_plan.h
                    const int64_t per_phase = (E + c->phases - 1) / c->phases + c->bin_block;   // ranges are cut at multiples of the block
                    hipLaunchKernelGGL(k_wg_pools, dim3(1), dim3(64), 0, st, std::min<int64_t>(E, per_phase), c->n_wg, s + 1, c->bin_block, n_bins,
                                       c->wg_pool_begin, total_dev);
                }
                ok = hipMemcpyAsync(&want, total_dev, sizeof(want), hipMemcpyDeviceToHost, st) == hipSuccess &&
                     hipStreamSynchronize(st) == hipSuccess;
            }
            dev_free(c, total_dev);
            if (ok && want < (1ull << 31)) {
                c->max_chunks = (uint32_t)want;
                const size_t chains = (size_t)c->n_wg * n_bins;
                ok = dev_alloc(c, &c->pool, (size_t)c->max_chunks * kChunk * 3) == NOMAD_OK &&
                     dev_alloc(c, &c->chunk_prev, c->max_chunks) == NOMAD_OK && dev_alloc(c, &c->chain_head, chains) == NOMAD_OK &&
                     dev_alloc(c, &c->chain_fill, chains) == NOMAD_OK && dev_alloc(c, &c->head, (size_t)E) == NOMAD_OK &&
                     dev_alloc(c, &c->overflow, 1) == NOMAD_OK && (c->phases == 1 || dev_alloc(c, &c->carry, (size_t)n * 2) == NOMAD_OK);
                if (ok) ok = prepare_binned(c) == NOMAD_OK;
                if (ok) {
                    HTRY(hipMemsetAsync(c->overflow, 0, sizeof(int), st));
                    hipLaunchKernelGGL(k_edge_heads, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->row_ptr, n, c->head);
                    hipLaunchKernelGGL(k_zero_f2, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->ghead, n);
                    c->binned = true;
                }
            } else {
                ok = false;
            }
            if (!ok) {
                char buf[256];
                snprintf(buf, sizeof(buf), "the record pool of the binned edge pass (%.1f GB) could not be set up (%s)",
                         (double)want * kChunk * 12 / 1e9, c->err.empty() ? "size out of range" : c->err.c_str());
                why = buf;
                (void)hipGetLastError();
                dev_free(c, c->pool); dev_free(c, c->chunk_prev); dev_free(c, c->chain_head); dev_free(c, c->chain_fill); dev_free(c, c->wg_pool_begin);
                dev_free(c, c->head); dev_free(c, c->overflow); dev_free(c, c->carry);
                c->phases = 1;
                c->pool_rounds = 0;
                c->distinct_kernel = false;
            }
        }
        if (!c->binned && E > 0) fallback_note = "deterministic scatter on the fixed-point atomics path: " + why;
        if (!c->binned) {
            TRY(dev_alloc(c, &c->gfix, (size_t)n * 2));
            hipLaunchKernelGGL(k_zero_u64, dim3(blocks_for(n * 2)), dim3(kBlock), 0, st, c->gfix, n * 2);
            hipLaunchKernelGGL(k_zero_f2, dim3(blocks_for(n)), dim3(kBlock), 0, st, c->ghead, n);
        }
    }
    HTRY(hipStreamSynchronize(st));
    HTRY(hipGetLastError());
#undef TRY
#undef HTRY
#undef HTRY2
    c->has_graph = true;
    c->path = c->cfg.scatter_mode == NOMAD_SCATTER_ATOMIC ? NOMAD_PATH_ATOMIC_FP32
              : !c->binned ? NOMAD_PATH_FIXED_ATOMICS : c->pool_rounds ? NOMAD_PATH_BINNED_POOLED : NOMAD_PATH_BINNED;
    c->err = fallback_note;   // empty unless a slower path had to be taken
    return NOMAD_OK;
}

int nomad_scatter_path(const nomad_ctx* c) { return c ? c->path : 0; }

int64_t nomad_device_bytes(const nomad_ctx* c) { return c ? c->device_bytes : 0; }

int nomad_tune(nomad_ctx* c, int knob, int value) {
    if (!c) return NOMAD_E_INVALID_ARG;
    if (c->has_graph) return fail(c, NOMAD_E_ORDER, "nomad_tune has to come before nomad_set_graph");
    switch (knob) {
        case NOMAD_TUNE_EDGE_BLOCK:
            if (value != 1024 && value != 512) break;
            c->tune_edge_block = value; return NOMAD_OK;
        case NOMAD_TUNE_WORKGROUPS_PER_CU:
            if (value < 1 || value > 8) break;
            c->tune_wg_per_cu = value; return NOMAD_OK;
        case NOMAD_TUNE_SCATTER_PATH:
            if (value != 0 && value != NOMAD_PATH_FIXED_ATOMICS) break;
            c->tune_path = value; return NOMAD_OK;
        case NOMAD_TUNE_POOL_KERNEL:
            if (value != 0 && value != 1) break;
            c->tune_pool_kernel = value; return NOMAD_OK;
        case NOMAD_TUNE_RECORD_PHASES:
            if (value < 0 || value > 64) break;
            c->tune_phases = value; return NOMAD_OK;
        case NOMAD_TUNE_RECORD_SORT:
            if (value < 0 || value > 2) break;
            c->tune_record_sort = value; return NOMAD_OK;
        case NOMAD_TUNE_FLUSH_ROUNDS:
            if (value < 0 || value > 2) break;
            c->tune_flush_rounds = value; return NOMAD_OK;
    }
    return fail(c, NOMAD_E_INVALID_ARG, "nomad_tune: unknown knob %d or value %d out of range", knob, value);
}

int nomad_set_embedding(nomad_ctx* c, const float* theta, int mem) {
    int rc = check_ready(c, false);
    if (rc) return rc;
    if (!theta || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return fail(c, NOMAD_E_INVALID_ARG, "null pointer or bad mem");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    // on the context's own stream (which may not synchronise with the null stream), and complete on return
    HIP_TRY(c, hipMemcpyAsync(c->theta, theta, sizeof(float2) * (size_t)c->n, in_kind(mem), c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->has_theta = true;   // the stored gradient stays that of the most recent epoch
    return NOMAD_OK;
}

int nomad_epoch(nomad_ctx* c, int32_t t) {
    int rc = check_ready(c, true);
    if (rc) return rc;
    if (t < 0 || t >= c->cfg.n_epochs) return fail(c, NOMAD_E_INVALID_ARG, "epoch index %d outside 0..T-1", t);
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    const int64_t n = c->n;
    if (c->grouped) run_means(c);   // constants of the epoch, also across its sub-steps; unused when no cell is approximated
    const float eta = (float)((double)c->cfg.lr0 * (1.0 - (double)t / (double)c->cfg.n_epochs));
    const int B = c->cfg.batches_per_epoch;
    for (int b = 0; b < B; ++b) {
        const int64_t r0 = c->batch_row[b], r1 = c->batch_row[b + 1], e0 = c->batch_edge[b], e1 = c->batch_edge[b + 1];
        if (e1 == e0) {   // no edge in this sub-step: nothing moves; the stored gradient is that of the last sub-step
            if (b == B - 1 && B > 1)
                hipLaunchKernelGGL(k_zero_f2, dim3(blocks_for(n)), dim3(kBlock), 0, c->stream, c->g, n);
            if (B > 1) continue;
        }
        run_mean_field(c, r0, r1);
        EdgeArgs a = edge_args(c, (uint32_t)t);
        a.row_begin = r0;
        a.row_end = r1;
        if (c->through_means) a.cS = c->cS;
        if (c->cfg.scatter_mode == NOMAD_SCATTER_DETERMINISTIC && c->binned) {
            // the positions of this step in `phases` ranges cut at multiples of the workgroup size; every range's
            // records are accumulated before the next range reuses the pool, the last accumulation takes the step
            const int phases = c->pool_rounds ? 1 : (int)std::max<int64_t>(1, std::min<int64_t>(c->phases, (e1 - e0 + c->bin_block - 1) / c->bin_block));
            for (int ph = 0; ph < phases; ++ph) {
                const int64_t blocks = (e1 - e0 + c->bin_block - 1) / c->bin_block;
                const int64_t p0 = e0 + blocks * ph / phases * c->bin_block, p1 = ph + 1 == phases ? e1 : e0 + blocks * (ph + 1) / phases * c->bin_block;
                { Timed tm(c, NOMAD_K_EDGES);
                  launch_edges_binned(c, a, p0, p1); }
                const bool last = ph + 1 == phases;
                if (last) run_mean_gradient(c, r0, r1);
                const int kind = phases == 1 ? kPhaseOnly : ph == 0 ? kPhaseFirst : last ? kPhaseLast : kPhaseMiddle;
                Timed tm(c, NOMAD_K_TILES);   // accumulates the records of every tile; the last one takes the SGD step for its points
                hipLaunchKernelGGL(k_tile_accumulate, dim3(c->n_bins), dim3(kBinBlock), sizeof(unsigned long long) * 2 << c->tile_bits,
                                   c->stream, bin_args(c), (uint32_t)c->n_wg, c->g, n, c->theta, eta,
                                   c->through_means ? c->cluster_of : nullptr, c->through_means ? c->gmean : nullptr, c->carry, kind);
            }
            continue;
        }
        if (c->cfg.scatter_mode == NOMAD_SCATTER_ATOMIC) {
            { Timed tm(c, NOMAD_K_ZERO);
              hipLaunchKernelGGL(k_zero_f2, dim3(blocks_for(n)), dim3(kBlock), 0, c->stream, c->g, n); }
            { Timed tm(c, NOMAD_K_EDGES);
              launch_edges<kModeAtomic>(c, a); }
        } else {
            { Timed tm(c, NOMAD_K_EDGES);
              launch_edges<kModeDet>(c, a); }
            { Timed tm(c, NOMAD_K_SCATTER);
              hipLaunchKernelGGL(k_combine_fixed, dim3(blocks_for(n)), dim3(kBlock), 0, c->stream, c->ghead, c->gfix, c->g, n); }
        }
        if (c->through_means) {
            run_mean_gradient(c, r0, r1);
            Timed tm(c, NOMAD_K_MEANGRAD);
            hipLaunchKernelGGL(k_add_mean_gradient, dim3(blocks_for(n)), dim3(kBlock), 0, c->stream, c->g, c->cluster_of, c->gmean, n);
        }
        { Timed tm(c, NOMAD_K_UPDATE);
          hipLaunchKernelGGL(k_update, dim3(blocks_for(n)), dim3(kBlock), 0, c->stream, c->theta, c->g, eta, n); }
    }
    HIP_TRY(c, hipGetLastError());
    c->has_grad = true;
    return NOMAD_OK;
}

int nomad_loss(nomad_ctx* c, int32_t t_sample, double* out_host) {
    int rc = check_ready(c, true);
    if (rc) return rc;
    if (!out_host || t_sample < 0) return fail(c, NOMAD_E_INVALID_ARG, "null output or negative epoch index");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    run_means(c);
    run_mean_field(c, 0, c->n);
    const EdgeArgs a = edge_args(c, (uint32_t)t_sample);
    { Timed tm(c, NOMAD_K_LOSS);
      launch_edges<kModeLoss>(c, a);
      hipLaunchKernelGGL(k_loss_finish, dim3(1), dim3(kBlock), 0, c->stream, c->loss_partial, c->edge_grid, 1.0 / (double)c->n,
                         c->loss_out); }
    HIP_TRY(c, hipGetLastError());
    return copy_out(c, out_host, c->loss_out, sizeof(double), NOMAD_HOST);
}

int nomad_get_embedding(nomad_ctx* c, float* out, int mem) {
    int rc = check_ready(c, true);
    if (rc) return rc;
    if (!out || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return fail(c, NOMAD_E_INVALID_ARG, "null pointer or bad mem");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    return copy_out(c, out, c->theta, sizeof(float2) * (size_t)c->n, mem);
}

int nomad_get_gradient(nomad_ctx* c, float* out, int mem) {
    int rc = check_ready(c, true);
    if (rc) return rc;
    if (!c->has_grad) return fail(c, NOMAD_E_ORDER, "no gradient yet: call nomad_epoch first");
    if (!out || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return fail(c, NOMAD_E_INVALID_ARG, "null pointer or bad mem");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    return copy_out(c, out, c->g, sizeof(float2) * (size_t)c->n, mem);
}

int nomad_get_negatives(nomad_ctx* c, int32_t t, int64_t e_begin, int64_t e_end, int32_t* out, int mem) {
    int rc = check_ready(c, false);
    if (rc) return rc;
    if (t < 0 || e_begin < 0 || e_end < e_begin || e_end > c->E || (mem != NOMAD_HOST && mem != NOMAD_DEVICE))
        return fail(c, NOMAD_E_INVALID_ARG, "bad edge range or epoch index");
    const int64_t cnt = e_end - e_begin;
    const int s = c->cfg.n_neg;
    if (cnt == 0 || s == 0) return NOMAD_OK;
    if (!out) return fail(c, NOMAD_E_INVALID_ARG, "null output");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    int32_t* dst = out;
    int32_t* tmp = nullptr;
    if (mem == NOMAD_HOST) {
        rc = dev_alloc(c, &tmp, (size_t)cnt * s);
        if (rc) return rc;
        dst = tmp;
    }
    const EdgeArgs a = edge_args(c, (uint32_t)t);
    hipLaunchKernelGGL(k_negatives, dim3(blocks_for(cnt)), dim3(kBlock), 0, c->stream, a, e_begin, e_end, dst);
    hipError_t e_ = hipStreamSynchronize(c->stream);
    if (e_ == hipSuccess && tmp) e_ = hipMemcpy(out, tmp, sizeof(int32_t) * (size_t)cnt * s, hipMemcpyDeviceToHost);
    dev_free(c, tmp);
    if (e_ != hipSuccess) return fail(c, NOMAD_E_HIP, "negatives: %s", hipGetErrorString(e_));
    return NOMAD_OK;
}

int nomad_get_means(nomad_ctx* c, float* mu, int64_t* counts, int mem) {
    int rc = check_ready(c, true);
    if (rc) return rc;
    if ((!mu && !counts) || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return fail(c, NOMAD_E_INVALID_ARG, "null pointer or bad mem");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    run_means(c);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (mu) HIP_TRY(c, hipMemcpy(mu, c->mu, sizeof(float2) * (size_t)c->R, out_kind(mem)));
    if (counts) {
        std::vector<uint32_t> h32(c->R);
        std::vector<int64_t> h64(c->R);
        HIP_TRY(c, hipMemcpy(h32.data(), c->counts, sizeof(uint32_t) * (size_t)c->R, hipMemcpyDeviceToHost));
        for (int32_t r = 0; r < c->R; ++r) h64[r] = (int64_t)h32[r];
        HIP_TRY(c, hipMemcpy(counts, h64.data(), sizeof(int64_t) * (size_t)c->R,
                             mem == NOMAD_DEVICE ? hipMemcpyHostToDevice : hipMemcpyHostToHost));
    }
    return NOMAD_OK;
}

int nomad_get_mean_field(nomad_ctx* c, float* A, float* B, int mem) {
    int rc = check_ready(c, true);
    if (rc) return rc;
    if (!A || !B || (mem != NOMAD_HOST && mem != NOMAD_DEVICE)) return fail(c, NOMAD_E_INVALID_ARG, "null pointer or bad mem");
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    if (!c->grouped || c->cfg.far_field == NOMAD_FAR_FIELD_SAMPLED) {
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        if (mem == NOMAD_DEVICE) {
            HIP_TRY(c, hipMemset(A, 0, sizeof(float) * (size_t)c->n));
            HIP_TRY(c, hipMemset(B, 0, sizeof(float2) * (size_t)c->n));
        } else {
            memset(A, 0, sizeof(float) * (size_t)c->n);
            memset(B, 0, sizeof(float2) * (size_t)c->n);
        }
        return NOMAD_OK;
    }
    run_means(c);
    run_mean_field(c, 0, c->n);
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    HIP_TRY(c, hipMemcpy(A, c->A, sizeof(float) * (size_t)c->n, out_kind(mem)));
    HIP_TRY(c, hipMemcpy(B, c->B, sizeof(float2) * (size_t)c->n, out_kind(mem)));
    return NOMAD_OK;
}

int nomad_profile(nomad_ctx* c, int enable) {
    if (!c) return NOMAD_E_INVALID_ARG;
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    clear_timers(c);
    if (enable && c->event_pool.empty() && !grow_event_pool(c, 4096)) return fail(c, NOMAD_E_HIP, "hipEventCreate failed");
    c->profiling = enable != 0;
    return NOMAD_OK;
}

int nomad_profile_read(nomad_ctx* c, int kind, double* total_ms, int64_t* launches) {
    if (!c || kind < 0 || kind >= NOMAD_K_COUNT || !total_ms || !launches) return NOMAD_E_INVALID_ARG;
    HIP_TRY(c, hipSetDevice(c->cfg.device));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const KernelTimer& t = c->timers[kind];
    double tot = 0.0;
    const size_t cnt = std::min(t.begin.size(), t.end.size());
    for (size_t k = 0; k < cnt; ++k) {
        float ms = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&ms, t.begin[k], t.end[k]));
        tot += (double)ms;
    }
    *total_ms = tot;
    *launches = (int64_t)cnt;
    return NOMAD_OK;
}

}  // extern "C"
#pragma GCC visibility pop
